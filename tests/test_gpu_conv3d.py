"""GPU parity of Convolution over three spatial axes (ngc_conv3d_*) against the fp64 oracle
(oracle/conv3d_oracle.py), through the C ABI.  Tolerances as for the rank-2 ops: 1e-5 (fp32),
2e-2 (bf16), max-normalised."""
import numpy as np
import pytest
import torch

import oracle
import paper_1801_08058_amd as ng
import synth_inputs
from oracle import Attrs3
from gpu_util import bound, Run3, attrs3_of, desc3_of, dev, encode, host, stream

pytestmark = pytest.mark.gpu
NCHW, BLK = ng.NGC_NCHW, ng.NGC_NCHW16C
OPS = (ng.NGC_OP_FWD, ng.NGC_OP_BWD_DATA, ng.NGC_OP_BWD_FILTERS)


def _tensors3(a: Attrs3, dtype: str, seed: int):
    L = synth_inputs.Conv3dLayer("t", a.n, a.c, a.d, a.h, a.w, a.k, a.t, a.r, a.s, (a.sd, a.sh, a.sw), (a.dd, a.dh, a.dw),
                                 (a.pbd, a.pbh, a.pbw), (a.pad, a.pah, a.paw), dtype=dtype, seed=seed)
    t = synth_inputs.layer3_tensors(L)
    return t["x"], t["w"], t["bias"], t["dy"]


def _check3(a: Attrs3, dtype: str, xl: int, yl: int, pre: bool, seed: int, expect=None):
    print(f"case attrs={a} dtype={dtype} xl={xl} yl={yl} pre={pre} seed={seed}", flush=True)
    x, w, b, dy = _tensors3(a, dtype, seed)
    run = Run3(a, dtype, xl, yl, pre)
    tol = bound(dtype, "act")
    y = run.fwd(x, w, bias=b, relu=True)
    if expect:
        assert ng.ngc_conv3d_variant(run.last_desc, ng.NGC_OP_FWD).startswith(expect[0]), ng.ngc_conv3d_variant(run.last_desc, 0)
    e = oracle.max_normalised_error(y, oracle.conv3d_fwd(a, x, w, bias=b, relu=True))
    assert e <= tol, f"fwd+bias+relu err {e}"
    e = oracle.max_normalised_error(run.fwd(x, w), oracle.conv3d_fwd(a, x, w))
    assert e <= tol, f"fwd err {e}"
    dx = run.bwd_data(dy, w)
    if expect:
        assert ng.ngc_conv3d_variant(run.last_desc, ng.NGC_OP_BWD_DATA).startswith(expect[1]), ng.ngc_conv3d_variant(run.last_desc, 1)
    ref_dx = oracle.conv3d_bwd_data(a, dy, w)
    e = oracle.max_normalised_error(dx, ref_dx)
    assert e <= tol, f"bwd_data err {e}"
    # the backward compounds: ReLU backprop of the data input (x doubles as that input: about half of it is <= 0),
    # the channel sums of the dx the device stored, and the bias gradient
    dxr = run.bwd_data_relu(dy, w, x)
    e = oracle.max_normalised_error(dxr, oracle.relu_bwd_mask(ref_dx, x))
    assert e <= tol, f"bwd_data_relu err {e}"
    blocked = ~(x > 0)
    assert np.all(dxr[blocked] == 0) and not np.signbit(dxr[blocked]).any(), "gradient leaked through x_in <= 0"
    dx2, dbp = run.bwd_data_relu(dy, w, x, with_db=True)
    assert np.array_equal(dx2, dxr)
    e = oracle.max_normalised_error(dbp, oracle.bias_grad(dxr.reshape(a.n, a.c, a.d * a.h, a.w)))
    assert e <= 1e-5, f"bwd_data_relu_db err {e}"
    db = run.bias_grad(dy)
    e = oracle.max_normalised_error(db, oracle.bias_grad(dy.reshape(a.n, a.k, -1, dy.shape[-1])))
    assert e <= 1e-5, f"bias_grad err {e}"
    dw = run.bwd_filters(x, dy)
    if expect:
        assert ng.ngc_conv3d_variant(run.last_desc, ng.NGC_OP_BWD_FILTERS).startswith(expect[2]), ng.ngc_conv3d_variant(run.last_desc, 2)
    e = oracle.max_normalised_error(dw, oracle.conv3d_bwd_filters(a, x, dy))
    assert e <= bound(dtype, "dw"), f"bwd_filters err {e}"


def _expect_blocked(a: Attrs3, strip=True):
    """Kernel names for bf16 blocked tensors: the strip kernel takes windows of 2..25 taps in (h, w) with up to 7
    depth taps and channel multiples of 16, the gather kernel reductions over multiples of 32 channels into
    multiples of 64, the per-tap backprop-filters GEMM multiples of 16."""
    s3 = strip and 2 <= a.r * a.s <= 25 and a.t <= 7 and a.c % 16 == 0 and a.k % 16 == 0
    fwd = "strip3" if s3 else ("igemm3" if a.c % 32 == 0 and a.k % 64 == 0 else "direct3")
    bwd = "strip3" if s3 else ("igemm3" if a.k % 32 == 0 and a.c % 64 == 0 and a.sd * a.sh * a.sw <= 16 else "direct3")
    return fwd, bwd, "wgrad_gemm3" if a.c % 16 == 0 and a.k % 16 == 0 else "direct3"


# the video configuration at a quarter of the clip length / image side, batch 2: several tiles, ragged tails
@pytest.mark.parametrize("i", range(7))
@pytest.mark.parametrize("pre", [False, True])
@pytest.mark.parametrize("strip", [True, False])
def test_video_layers_reduced(i, pre, strip, monkeypatch):
    if not strip:
        monkeypatch.setenv("NGC_CONV3D_STRIP", "0")          # the gather kernel with a depth axis instead
    L = synth_inputs.video_layers(2, scale=4)[i]
    a = attrs3_of(L)
    expect = ("rank2", "rank2", "rank2") if L.name in ("v_3x1x1_c128k64", "v_1x1x1_c256k64") else _expect_blocked(a, strip)
    _check3(a, "bf16", BLK, BLK, pre, L.seed, expect)


GATHER_CASES = [
    # n  c   d  h  w   k   t  r  s  strides    dilation   pad below  pad above
    (1, 32, 5, 9, 11, 64, 3, 3, 3, (1, 1, 1), (1, 1, 1), (1, 1, 1), (1, 1, 1)),
    (2, 64, 4, 7, 9, 128, 2, 3, 1, (1, 2, 1), (1, 1, 1), (0, 1, 0), (1, 0, 0)),
    (1, 96, 6, 6, 6, 192, 3, 1, 3, (2, 1, 2), (1, 1, 2), (1, 0, 2), (0, 0, 1)),
    (3, 64, 7, 5, 8, 64, 1, 3, 3, (1, 1, 1), (1, 2, 1), (0, 2, 1), (0, 2, 1)),
    (1, 128, 9, 8, 7, 128, 3, 3, 3, (2, 2, 2), (1, 1, 1), (1, 1, 1), (1, 1, 1)),
    (2, 64, 8, 9, 10, 64, 4, 2, 2, (3, 2, 2), (1, 1, 1), (0, 0, 0), (0, 0, 0)),       # stride > window on depth: untouched voxels
    (1, 64, 3, 4, 5, 64, 3, 3, 3, (1, 1, 1), (2, 2, 2), (3, 3, 3), (3, 3, 3)),       # windows mostly in the padding
    (1, 64, 6, 6, 6, 64, 1, 1, 1, (2, 2, 2), (1, 1, 1), (0, 0, 0), (0, 0, 0)),       # 1x1x1 strided: 7 of 8 classes without taps
]


@pytest.mark.parametrize("case", GATHER_CASES)
@pytest.mark.parametrize("strip", [True, False])
def test_mfma_kernels_with_depth(case, strip, monkeypatch):
    if not strip:
        monkeypatch.setenv("NGC_CONV3D_STRIP", "0")
    n, c, d, h, w, k, t, r, s, st, dil, pb, pa = case
    a = Attrs3(n, c, d, h, w, k, t, r, s, *st, *dil, *pb, *pa)
    _check3(a, "bf16", BLK, BLK, False, 300 + c + d, _expect_blocked(a, strip))


# channel counts the gather kernel does not take: the strip kernel (multiples of 16), without it the direct
# kernels; backprop-filters on the per-tap GEMM (multiples of 16)
@pytest.mark.parametrize("ck", [(16, 48), (48, 80), (80, 16)])
def test_channel_multiples_of_16(ck, monkeypatch):
    c, k = ck
    a = Attrs3(2, c, 4, 6, 7, k, 3, 2, 3, 1, 1, 2, 1, 1, 1, 1, 0, 1, 1, 1, 1)
    _check3(a, "bf16", BLK, BLK, False, 400 + c, ("strip3", "strip3", "wgrad_gemm3"))
    monkeypatch.setenv("NGC_CONV3D_STRIP", "0")
    _check3(a, "bf16", BLK, BLK, False, 400 + c, ("direct3", "direct3", "wgrad_gemm3"))


DIRECT_CASES = [("f32", NCHW, NCHW), ("f32", BLK, BLK), ("bf16", NCHW, NCHW), ("bf16", NCHW, BLK), ("f32", BLK, NCHW)]


@pytest.mark.parametrize("dtype,xl,yl", DIRECT_CASES)
def test_direct_kernels(dtype, xl, yl):
    a = Attrs3(2, 5, 4, 6, 5, 7, 2, 3, 2, 1, 2, 1, 2, 1, 1, 1, 0, 1, 0, 1, 0)
    _check3(a, dtype, xl, yl, False, 500, ("direct3",) * 3)
    a = Attrs3(1, 20, 3, 5, 6, 18, 3, 1, 3, 2, 1, 1, 1, 1, 1, 1, 0, 1, 1, 0, 1)
    _check3(a, dtype, xl, yl, False, 501, ("direct3",) * 3)


# windows that move over one group of adjacent axes: the rank-2 kernels on the reshaped tensor, and the
# same node forced onto the rank-3 kernels (NGC_CONV3D_RANK2=0) gives the same tensors
RANK2_CASES = [
    (2, 64, 6, 5, 7, 64, 3, 1, 1, (1, 1, 1), (1, 1, 1), (1, 0, 0), (1, 0, 0)),
    (2, 64, 9, 4, 4, 128, 3, 1, 1, (2, 1, 1), (2, 1, 1), (2, 0, 0), (1, 0, 0)),
    (1, 128, 4, 6, 8, 64, 1, 1, 1, (1, 1, 1), (1, 1, 1), (0, 0, 0), (0, 0, 0)),
    (2, 64, 3, 5, 12, 64, 1, 1, 5, (1, 1, 2), (1, 1, 1), (0, 0, 2), (0, 0, 1)),
]


@pytest.mark.parametrize("case", RANK2_CASES)
@pytest.mark.parametrize("layouts", [(BLK, BLK), (NCHW, NCHW)])
def test_windows_that_reduce_to_rank2(case, layouts, monkeypatch):
    n, c, d, h, w, k, t, r, s, st, dil, pb, pa = case
    a = Attrs3(n, c, d, h, w, k, t, r, s, *st, *dil, *pb, *pa)
    _check3(a, "bf16", layouts[0], layouts[1], False, 600 + d, ("rank2",) * 3)
    monkeypatch.setenv("NGC_CONV3D_RANK2", "0")
    native = _expect_blocked(a) if layouts == (BLK, BLK) else ("direct3",) * 3
    _check3(a, "bf16", layouts[0], layouts[1], False, 600 + d, native)


def test_random_descriptors():
    """Randomised attributes on the MFMA kernels (channel multiples of 32 / 64) and on the direct kernels."""
    g = np.random.default_rng(20180126)
    done = 0
    while done < 40:
        mf = done % 4 != 3
        t, r, s = (int(v) for v in g.integers(1, 4, size=3))
        st = tuple(int(v) for v in g.integers(1, 3, size=3))
        dil = tuple(int(v) for v in g.integers(1, 3, size=3))
        pb = tuple(int(v) for v in g.integers(0, 3, size=3))
        pa = tuple(int(v) for v in g.integers(0, 3, size=3))
        d, h, w = (int(v) for v in g.integers(2, 9, size=3))
        c = int(g.choice([32, 64, 96])) if mf else int(g.integers(1, 24))
        k = int(g.choice([64, 128])) if mf else int(g.integers(1, 24))
        a = Attrs3(int(g.integers(1, 3)), c, d, h, w, k, t, r, s, *st, *dil, *pb, *pa)
        if min((d + pb[0] + pa[0] - dil[0] * (t - 1) - 1), (h + pb[1] + pa[1] - dil[1] * (r - 1) - 1),
               (w + pb[2] + pa[2] - dil[2] * (s - 1) - 1)) < 0:
            continue
        dtype = "bf16" if mf else ("f32" if done % 8 == 3 else "bf16")
        _check3(a, dtype, BLK if mf else (NCHW if done % 8 == 3 else BLK), BLK if mf else NCHW, bool(done % 2), 700 + done)
        done += 1


def test_random_descriptors_gather_kernel(monkeypatch):
    """The same draw of MFMA descriptors with the strip kernel switched off."""
    monkeypatch.setenv("NGC_CONV3D_STRIP", "0")
    g = np.random.default_rng(20180127)
    done = 0
    while done < 20:
        t, r, s = (int(v) for v in g.integers(1, 4, size=3))
        st = tuple(int(v) for v in g.integers(1, 3, size=3))
        dil = tuple(int(v) for v in g.integers(1, 3, size=3))
        pb = tuple(int(v) for v in g.integers(0, 3, size=3))
        pa = tuple(int(v) for v in g.integers(0, 3, size=3))
        d, h, w = (int(v) for v in g.integers(2, 9, size=3))
        a = Attrs3(int(g.integers(1, 3)), 64, d, h, w, int(g.choice([64, 128])), t, r, s, *st, *dil, *pb, *pa)
        if min(oracle.out_shape3(a)) < 1:
            continue
        _check3(a, "bf16", BLK, BLK, bool(done % 2), 800 + done)
        done += 1


def test_filter_convert_is_the_stated_layout():
    a = Attrs3(1, 40, 3, 3, 3, 24, 2, 3, 2)
    g = np.random.default_rng(3)
    bits = g.integers(1, 0xFFFF, size=(a.k, a.c, a.t, a.r, a.s), dtype=np.uint16)
    src = dev(bits)
    for layout in (ng.NGC_BLOCKED_FWD, ng.NGC_BLOCKED_BWD):
        d = desc3_of(a, "bf16", BLK, BLK, layout)
        dst = torch.full((ng.ngc_conv3d_filter_elems(d, layout),), -1, dtype=torch.int16, device="cuda")
        ng.ngc_conv3d_filter_convert(d, src, dst, layout, stream())
        torch.cuda.synchronize()
        got = host(dst, np.uint16)
        if layout == ng.NGC_BLOCKED_FWD:
            pad = np.zeros((a.k, 48, a.t, a.r, a.s), np.uint16); pad[:, :a.c] = bits
            want = pad.reshape(a.k, 3, 16, a.t, a.r, a.s).transpose(3, 4, 5, 1, 0, 2)
        else:
            pad = np.zeros((32, a.c, a.t, a.r, a.s), np.uint16); pad[:a.k] = bits
            want = pad.reshape(2, 16, a.c, a.t, a.r, a.s).transpose(3, 4, 5, 0, 2, 1)
        assert np.array_equal(got, np.ascontiguousarray(want).reshape(-1))


@pytest.mark.parametrize("i", [0, 2, 6])
def test_video_layers_full_size_sampled(i):
    """The timed shapes (batch 8): 256 sampled elements per op against the oracle's per-element routines, and
    every element of the outputs finite (the buffers start poisoned)."""
    L = synth_inputs.video_layers()[i]
    a = attrs3_of(L)
    print(f"case {L.name}", flush=True)
    t = synth_inputs.layer3_tensors(L)
    run = Run3(a, "bf16", BLK, BLK, True)
    g = np.random.default_rng(L.seed)
    O, P, Q = oracle.out_shape3(a)
    y = run.fwd(t["x"], t["w"], bias=t["bias"], relu=True)
    assert np.isfinite(y).all()
    idx = g.integers(0, y.size, size=256)
    ref = oracle.conv3d_fwd_at(a, t["x"], t["w"], idx, bias=t["bias"], relu=True)
    scale = max(np.abs(ref).max(), np.abs(y).max() * 0.25)
    assert np.abs(y.reshape(-1)[idx] - ref).max() / scale <= bound("bf16", "act")
    del y
    dx = run.bwd_data(t["dy"], t["w"])
    assert np.isfinite(dx).all()
    idx = g.integers(0, dx.size, size=256)
    ref = oracle.conv3d_bwd_data_at(a, t["dy"], t["w"], idx)
    scale = max(np.abs(ref).max(), np.abs(dx).max() * 0.25)
    assert np.abs(dx.reshape(-1)[idx] - ref).max() / scale <= bound("bf16", "act")
    del dx
    dw = run.bwd_filters(t["x"], t["dy"])
    assert np.isfinite(dw).all()
    idx = g.integers(0, dw.size, size=64)
    ref = oracle.conv3d_bwd_filters_at(a, t["x"], t["dy"], idx)
    scale = max(np.abs(ref).max(), np.abs(dw).max() * 0.25)
    assert np.abs(dw.reshape(-1)[idx] - ref).max() / scale <= bound("bf16", "dw")


def test_temporal_window_on_large_slices_runs_on_the_strip_kernel():
    """A (3,1,1) window is the rank-2 node over (D, H*W); rows of H*W = 1600 pixels are cut into column tiles."""
    a = Attrs3(2, 64, 6, 40, 40, 64, 3, 1, 1, 1, 1, 1, 1, 1, 1, 1, 0, 0, 1, 0, 0)
    _check3(a, "bf16", BLK, BLK, True, 900, ("rank2:strip", "rank2:strip", "rank2:"))


FALLBACK_CASES = [
    # more depth taps than the strip kernel holds -> gather kernel; more taps than that holds -> direct kernels
    (Attrs3(1, 64, 12, 6, 5, 64, 9, 3, 1, 1, 1, 1, 1, 1, 1, 4, 1, 0, 4, 1, 0), ("igemm3", "igemm3", "wgrad_gemm3")),
    (Attrs3(1, 32, 10, 6, 6, 64, 9, 3, 3, 1, 1, 1, 1, 1, 1, 4, 1, 1, 4, 1, 1), ("direct3", "direct3", "direct3")),
    # more residue classes of the strides than either MFMA kernel holds -> direct backprop-data
    (Attrs3(1, 64, 9, 9, 8, 64, 3, 3, 3, 3, 3, 2, 1, 1, 1, 1, 1, 1, 1, 1, 1), ("strip3", "direct3", "wgrad_gemm3")),
]


@pytest.mark.parametrize("a,expect", FALLBACK_CASES)
def test_kernel_limits_fall_back(a, expect):
    _check3(a, "bf16", BLK, BLK, False, 950 + a.t + a.sd, expect)


@pytest.mark.parametrize("a", [
    Attrs3(1, 32, 3, 5, 1000, 64, 3, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1),       # slices 1000 pixels wide
    Attrs3(1, 64, 4, 4, 2001, 64, 2, 3, 3, 2, 1, 2, 1, 1, 1, 0, 1, 1, 1, 1, 1),       # strided: one launch per class
])
def test_strip_kernel_with_depth_and_column_tiles(a):
    _check3(a, "bf16", BLK, BLK, True, 980 + a.w, ("strip3", "strip3", "wgrad_gemm3"))
