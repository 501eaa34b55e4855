"""GPU parity tests: the HIP path (through the C ABI) against the fp64 CPU oracle, element
by element, on seeded inputs.  Tolerances (max normalised error, L-inf / L-inf):
1e-5 for fp32, 2e-2 for bf16 data; layout transforms bit exact."""
import numpy as np
import pytest
import torch

import oracle
import paper_1801_08058_amd as ng
import synth_inputs
from oracle import Attrs
from gpu_util import (TOL, bound, Run, attrs_of, data_to_device, desc_of, dev, encode, filter_blocked_host, host,
                      out_tensor, stream, workspace)

pytestmark = pytest.mark.gpu

NCHW, BLK = ng.NGC_NCHW, ng.NGC_NCHW16C


def _tensors(a: Attrs, dtype: str, seed: int):
    P, Q = oracle.out_shape(a)
    x = synth_inputs.normal(seed, 0, (a.n, a.c, a.h, a.w), 0.0, 1.0)
    w = synth_inputs.normal(seed, 1, (a.k, a.c, a.r, a.s), 0.0, (2.0 / (a.c * a.r * a.s)) ** 0.5)
    b = synth_inputs.uniform(seed, 2, (a.k,), -0.1, 0.1)
    dy = synth_inputs.normal(seed, 3, (a.n, a.k, P, Q), 0.0, 0.1)
    if dtype == "bf16":
        rt = lambda t: synth_inputs.bf16_bits_to_f32(synth_inputs.f32_to_bf16_bits(t))
        x, w, dy = rt(x), rt(w), rt(dy)
    return x, w, b, dy


def _check_backward_compounds(run, a, x_in, w, dy, ref_dx, tol):
    """Backprop-data compounded with the ReLU backprop of its data input (x_in doubles as the forward
    input of the node: about half of its elements are <= 0), and the bias gradient."""
    dxr = run.bwd_data_relu(dy, w, x_in)
    ref = oracle.relu_bwd_mask(ref_dx, x_in)
    e = oracle.max_normalised_error(dxr, ref)
    assert e <= tol, f"bwd_data_relu err {e}"
    blocked = ~(x_in > 0)
    assert np.all(dxr[blocked] == 0) and not np.signbit(dxr[blocked]).any(), "gradient leaked through x_in <= 0"
    # the same compound returning the bias gradient of the producing layer as well: dx identical, db = channel
    # sums of the dx the device stored (its own rounded output is what the next op reads)
    dx2, dbp = run.bwd_data_relu_db(dy, w, x_in)
    assert np.array_equal(dx2, dxr), "fused channel sums changed dx"
    e = oracle.max_normalised_error(dbp, oracle.bias_grad(dxr))
    assert e <= 1e-5, f"bwd_data_relu_db err {e}"
    db = run.bias_grad(dy)
    assert ng.ngc_conv_variant(run.last_desc, ng.NGC_OP_BIAS_GRAD).startswith("bias_grad")
    e = oracle.max_normalised_error(db, oracle.bias_grad(dy))
    assert e <= 1e-5, f"bias_grad err {e}"


def _check_all(a: Attrs, dtype: str, xl: int, yl: int, pre: bool, seed: int, expect_variant=None):
    print(f"case attrs={a} dtype={dtype} xl={xl} yl={yl} pre={pre} seed={seed}", flush=True)
    x, w, b, dy = _tensors(a, dtype, seed)
    run = Run(a, dtype, xl, yl, pre)
    tol = bound(dtype, "act")
    y = run.fwd(x, w, bias=b, relu=True)
    if expect_variant:
        assert ng.ngc_conv_variant(run.last_desc, ng.NGC_OP_FWD).startswith(expect_variant[0]), \
            ng.ngc_conv_variant(run.last_desc, ng.NGC_OP_FWD)
    e = oracle.max_normalised_error(y, oracle.conv_fwd(a, x, w, bias=b, relu=True))
    assert e <= tol, f"fwd+bias+relu err {e}"
    y0 = run.fwd(x, w)
    e = oracle.max_normalised_error(y0, oracle.conv_fwd(a, x, w))
    assert e <= tol, f"fwd err {e}"
    dx = run.bwd_data(dy, w)
    if expect_variant:
        assert ng.ngc_conv_variant(run.last_desc, ng.NGC_OP_BWD_DATA).startswith(expect_variant[1]), \
            ng.ngc_conv_variant(run.last_desc, ng.NGC_OP_BWD_DATA)
    ref_dx = oracle.conv_bwd_data(a, dy, w)
    e = oracle.max_normalised_error(dx, ref_dx)
    assert e <= tol, f"bwd_data err {e}"
    _check_backward_compounds(run, a, x, w, dy, ref_dx, tol)
    dw = run.bwd_filters(x, dy)
    if expect_variant:
        assert ng.ngc_conv_variant(run.last_desc, ng.NGC_OP_BWD_FILTERS).startswith(expect_variant[2])
    e = oracle.max_normalised_error(dw, oracle.conv_bwd_filters(a, x, dy))
    assert e <= bound(dtype, "dw"), f"bwd_filters err {e}"


# ------------------------------------------------------------------ layout conversion (bit exact)
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("shape", [(2, 16, 8, 8), (3, 40, 7, 7), (2, 3, 14, 14), (1, 17, 5, 3), (2, 64, 56, 56),
                                   (1, 33, 30, 31), (2, 256, 9, 30)])
def test_layout_convert_bit_exact(dtype, shape):
    n, c, h, w = shape
    rng = np.random.default_rng(1234 + c * h)
    if dtype == "bf16":
        bits = rng.integers(1, 0xFFFF, size=shape, dtype=np.uint16)
    else:
        bits = rng.integers(1, 0xFFFFFFFF, size=shape, dtype=np.uint32)
    code = ng.NGC_BF16 if dtype == "bf16" else ng.NGC_F32
    src = dev(bits)
    cb = (c + 15) // 16
    dst = torch.full((n * cb * h * w * 16,), -1, dtype=src.dtype, device="cuda")
    ng.ngc_layout_convert(code, n, c, h, w, src, NCHW, dst, BLK, stream())
    torch.cuda.synchronize()
    got = host(dst, bits.dtype).reshape(n, cb, h, w, 16)
    assert np.array_equal(got, oracle.nchw_to_blocked16(bits))           # includes +0 tail lanes
    back = torch.full((n * c * h * w,), -1, dtype=src.dtype, device="cuda")
    ng.ngc_layout_convert(code, n, c, h, w, dst, BLK, back, NCHW, stream())
    torch.cuda.synchronize()
    assert np.array_equal(host(back, bits.dtype).reshape(shape), bits)
    # same-layout call is a copy
    cp = torch.full((n * c * h * w,), -1, dtype=src.dtype, device="cuda")
    ng.ngc_layout_convert(code, n, c, h, w, src, NCHW, cp, NCHW, stream())
    torch.cuda.synchronize()
    assert np.array_equal(host(cp, bits.dtype).reshape(shape), bits)


@pytest.mark.parametrize("kcrs", [(64, 32, 3, 3), (20, 17, 1, 2), (128, 64, 1, 1)])
def test_filter_convert_bit_exact(kcrs):
    K, C, R, S = kcrs
    rng = np.random.default_rng(99)
    bits = rng.integers(1, 0xFFFF, size=kcrs, dtype=np.uint16)
    d = ng.make_desc(1, C, 8, 8, K, R, S, pad_below=(R // 2, S // 2), pad_above=(R // 2, S // 2))
    for layout in (ng.NGC_BLOCKED_FWD, ng.NGC_BLOCKED_BWD):
        exp = filter_blocked_host(bits, layout)
        assert ng.ngc_filter_elems(d, layout) == exp.size
        dst = torch.full((exp.size,), -1, dtype=torch.int16, device="cuda")
        ng.ngc_filter_convert(d, dev(bits), dst, layout, stream())
        torch.cuda.synchronize()
        assert np.array_equal(host(dst, np.uint16).reshape(exp.shape), exp)


# ------------------------------------------------------------------ configuration 1 (fp32, exact shape)
def test_cfg1_fp32():
    L = synth_inputs.config_layers(1)[0]
    a = attrs_of(L)
    t = synth_inputs.layer_tensors(L)
    run = Run(a, "f32", NCHW, NCHW, False)
    y = run.fwd(t["x"], t["w"], bias=t["bias"], relu=True)
    assert oracle.max_normalised_error(y, oracle.conv_fwd(a, t["x"], t["w"], bias=t["bias"], relu=True)) <= 1e-5
    dx = run.bwd_data(t["dy"], t["w"])
    assert oracle.max_normalised_error(dx, oracle.conv_bwd_data(a, t["dy"], t["w"])) <= 1e-5
    dw = run.bwd_filters(t["x"], t["dy"])
    assert oracle.max_normalised_error(dw, oracle.conv_bwd_filters(a, t["x"], t["dy"])) <= 1e-5


# ------------------------------------------------------------------ direct kernels: every attribute
DIRECT_CASES = [
    Attrs(2, 5, 9, 8, 7, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1),
    Attrs(1, 3, 11, 13, 4, 3, 2, 2, 3, 1, 2, 2, 0, 1, 3),        # stride, dilation, asymmetric pads
    Attrs(2, 17, 6, 6, 19, 1, 1, 2, 2, 1, 1, 0, 0, 0, 0),        # 1x1 stride 2, channel tails
    Attrs(1, 4, 10, 10, 6, 5, 5, 1, 1, 2, 2, 4, 4, 4, 4),        # dilation 2
    Attrs(3, 2, 7, 5, 3, 7, 3, 3, 1, 1, 1, 3, 1, 3, 1),
]


@pytest.mark.parametrize("case", range(len(DIRECT_CASES)))
@pytest.mark.parametrize("dtype,xl,yl", [("f32", NCHW, NCHW), ("bf16", NCHW, NCHW), ("bf16", BLK, BLK),
                                         ("f32", BLK, NCHW), ("bf16", NCHW, BLK)])
def test_direct_kernels(case, dtype, xl, yl):
    _check_all(DIRECT_CASES[case], dtype, xl, yl, False, 1000 + case, ("direct", "direct", "direct"))


def test_blocked_output_tail_lanes_are_zero():
    a = Attrs(1, 5, 6, 6, 20, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1)
    x, w, b, dy = _tensors(a, "bf16", 7)
    run = Run(a, "bf16", BLK, BLK, False)
    run.fwd(x, w, bias=b, relu=False)
    raw = host(run.last_raw, np.uint16).reshape(1, 2, 6, 6, 16)
    assert np.all(raw[:, 1, :, :, 4:] == 0)
    run.bwd_data(dy, w)
    raw = host(run.last_raw, np.uint16).reshape(1, 1, 6, 6, 16)
    assert np.all(raw[..., 5:] == 0)


# ------------------------------------------------------------------ MFMA kernels, small multi-tile shapes
MFMA_CASES = [
    # n  c   h   w   k   r  s  sh sw dh dw pbh pbw pah paw
    Attrs(3, 64, 13, 13, 64, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1),      # 507 positions: 2 tiles of 256 + ragged tail
    Attrs(2, 32, 12, 10, 128, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1),     # 128x128 tile variant fwd; bwd -> direct (c%64)
    Attrs(2, 128, 9, 11, 64, 1, 1, 1, 1, 1, 1, 0, 0, 0, 0),      # 1x1
    Attrs(2, 64, 14, 14, 128, 3, 3, 2, 2, 1, 1, 1, 1, 1, 1),     # 3x3 stride 2 (bwd-data parity classes)
    Attrs(2, 128, 14, 14, 256, 1, 1, 2, 2, 1, 1, 0, 0, 0, 0),    # 1x1 stride 2 projection (empty classes)
    Attrs(1, 64, 15, 9, 64, 3, 3, 2, 1, 2, 1, 2, 0, 1, 1),       # mixed stride / dilation / asymmetric pads
    Attrs(5, 64, 7, 7, 192, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1),       # 7x7 images, several per tile; K=192 -> 256x64 tile
    Attrs(1, 64, 16, 16, 64, 5, 5, 1, 1, 1, 1, 2, 2, 2, 2),      # 5x5
    Attrs(2, 64, 9, 9, 64, 3, 3, 3, 3, 1, 1, 1, 1, 1, 1),        # stride 3 (9 classes)
    Attrs(2, 48, 56, 56, 64, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1),      # 14-row strips of a 56x56 image, C = 3 chunks
    Attrs(9, 64, 14, 14, 128, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1),     # several whole images per strip, ragged last group
    Attrs(1, 32, 30, 20, 64, 3, 2, 1, 1, 2, 1, 3, 0, 1, 1),      # dilation / asymmetric pads, ragged last strip
    Attrs(3, 64, 56, 56, 64, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1),      # all-taps wgrad: row strips + 4-row stages
    Attrs(5, 128, 20, 9, 64, 3, 3, 1, 1, 2, 2, 2, 2, 2, 2),      # all-taps wgrad: dilation 2, two c tiles, odd width
    Attrs(70, 64, 7, 7, 64, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1),       # many small images
]


@pytest.fixture
def strip_nf(monkeypatch):
    """NGC_STRIP_NF: 0 = gather kernel only, 7/4/2 = force a strip size, unset = dispatcher's choice."""
    def set_(v):
        if v is None:
            monkeypatch.delenv("NGC_STRIP_NF", raising=False)
        else:
            monkeypatch.setenv("NGC_STRIP_NF", str(v))
    return set_


@pytest.mark.parametrize("case", range(len(MFMA_CASES)))
@pytest.mark.parametrize("pre", [True, False])
@pytest.mark.parametrize("nf", [None, 0, 7, 4])
def test_mfma_kernels_small(case, pre, nf, strip_nf):
    a = MFMA_CASES[case]
    if nf in (7, 4) and ((a.sh, a.sw) != (1, 1) or a.r * a.s == 1 or not pre):  # forced sizes: stride-1 shapes only
        pytest.skip("strip kernel covers stride-1 multi-tap shapes; one filter-layout mode is enough for forced sizes")
    strip_nf(nf)
    # multi-tap layers go through the strip kernel: forward with any stride, backprop-data one launch per
    # residue class of the stride (case 5: no tap reaches the odd rows of dx, which are cleared first)
    strip_ok = a.r * a.s > 1 and nf != 0
    bwd_strip_ok = strip_ok
    one_tap = a.r * a.s == 1 and a.c % 16 == 0 and a.k % 16 == 0
    fwd_v = "strip" if (strip_ok and a.c % 16 == 0 and a.k % 16 == 0) else "gemm1x1" if one_tap else \
        "igemm" if (a.c % 32 == 0 and a.k % 64 == 0) else "direct"
    bwd_v = "strip" if (bwd_strip_ok and a.k % 16 == 0 and a.c % 16 == 0) else "gemm1x1" if one_tap else \
        "igemm" if (a.k % 32 == 0 and a.c % 64 == 0) else "direct"
    wg_v = "wgrad" if (a.c % 16 == 0 and a.k % 16 == 0) else "direct"
    _check_all(a, "bf16", BLK, BLK, pre, 2000 + case, (fwd_v, bwd_v, wg_v))


@pytest.mark.parametrize("case", [0, 9, 10, 11])
def test_wgrad_per_tap_kernel_still_matches(case, monkeypatch):
    """3x3 stride-1 shapes through the per-tap split kernel (the all-taps kernel switched off)."""
    monkeypatch.setenv("NGC_WGRAD_STRIP", "0")
    monkeypatch.setenv("NGC_WGRAD_GEMM", "0")
    a = MFMA_CASES[case]
    if a.c % 64 or a.k % 64:
        pytest.skip("per-tap MFMA kernel needs C, K multiples of 64")
    x, w, b, dy = _tensors(a, "bf16", 3000 + case)
    run = Run(a, "bf16", BLK, BLK, True)
    dw = run.bwd_filters(x, dy)
    assert ng.ngc_conv_variant(run.last_desc, ng.NGC_OP_BWD_FILTERS) == "wgrad_bf16_64x64"
    assert oracle.max_normalised_error(dw, oracle.conv_bwd_filters(a, x, dy)) <= bound("bf16", "dw")


@pytest.mark.parametrize("case", [12, 13, 14])
@pytest.mark.parametrize("ncq,ring,late", [(1, 3, None), (2, 3, None), (4, 3, None), (2, 2, None), (2, 3, "0"), (2, 2, "0xFF"),
                                           (4, 3, "0x5A")])
def test_wgrad_all_taps_channel_group_variants(case, ncq, ring, late, monkeypatch):
    """Channel-group splits, LDS ring depths (3 buffers are used when they fit, 2 otherwise / when forced) and
    which waves issue their loads after their MFMAs (default: waves 4-7)."""
    monkeypatch.setenv("NGC_WGRAD_NCQ", str(ncq))
    monkeypatch.setenv("NGC_WGRAD_RING", str(ring))
    if late is not None:
        monkeypatch.setenv("NGC_WGRAD_LATE", late)
    a = MFMA_CASES[case]
    x, w, b, dy = _tensors(a, "bf16", 4000 + case)
    run = Run(a, "bf16", BLK, BLK, True)
    dw = run.bwd_filters(x, dy)
    assert ng.ngc_conv_variant(run.last_desc, ng.NGC_OP_BWD_FILTERS) == "wgrad_strip_bf16"
    assert oracle.max_normalised_error(dw, oracle.conv_bwd_filters(a, x, dy)) <= bound("bf16", "dw")


SMALL_IMAGE_WGRAD_CASES = [
    # n   c    h  w  k    r  s  sh sw dh dw pbh pbw pah paw
    Attrs(70, 64, 7, 7, 64, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1),       # 4 images per stage, ragged last stage
    Attrs(33, 128, 7, 7, 64, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1),      # two c tiles
    Attrs(21, 64, 9, 5, 128, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1),      # 9x5 images (45 positions), two k tiles
    Attrs(13, 64, 6, 10, 64, 3, 3, 1, 1, 2, 1, 2, 1, 2, 1),      # dilation 2 in h: 3 images of 60 positions
    Attrs(9, 64, 3, 3, 64, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1),        # 3x3 images: 24 per stage, fewer than that exist
]


@pytest.mark.parametrize("case", range(len(SMALL_IMAGE_WGRAD_CASES)))
@pytest.mark.parametrize("g1", [False, True])
def test_wgrad_all_taps_small_images(case, g1, monkeypatch):
    """Stages of several whole images (g1: forced back to one image per stage)."""
    if g1:
        monkeypatch.setenv("NGC_WGRAD_G1", "1")
    a = SMALL_IMAGE_WGRAD_CASES[case]
    x, w, b, dy = _tensors(a, "bf16", 9000 + case)
    run = Run(a, "bf16", BLK, BLK, True)
    dw = run.bwd_filters(x, dy)
    assert ng.ngc_conv_variant(run.last_desc, ng.NGC_OP_BWD_FILTERS) == "wgrad_strip_bf16"
    assert oracle.max_normalised_error(dw, oracle.conv_bwd_filters(a, x, dy)) <= bound("bf16", "dw")


@pytest.mark.parametrize("case", [0, 2, 3, 4, 5, 6, 8, 13])
@pytest.mark.parametrize("sp", [0, 64, 128])
def test_wgrad_gemm_kernel(case, sp, monkeypatch):
    """Per-tap GEMM backprop-filters (the all-taps kernel switched off so that 3x3 shapes reach it too);
    sp = positions per LDS stage (0: the dispatcher's choice)."""
    monkeypatch.setenv("NGC_WGRAD_STRIP", "0")
    if sp:
        monkeypatch.setenv("NGC_WGG_SP", str(sp))
    a = MFMA_CASES[case]
    x, w, b, dy = _tensors(a, "bf16", 6000 + case)
    run = Run(a, "bf16", BLK, BLK, True)
    dw = run.bwd_filters(x, dy)
    assert ng.ngc_conv_variant(run.last_desc, ng.NGC_OP_BWD_FILTERS) == "wgrad_gemm_bf16"
    assert oracle.max_normalised_error(dw, oracle.conv_bwd_filters(a, x, dy)) <= bound("bf16", "dw")


GEMM1X1_CASES = [
    # n  c    h   w   k    r  s  sh sw dh dw pbh pbw pah paw
    Attrs(3, 64, 13, 13, 128, 1, 1, 1, 1, 1, 1, 0, 0, 0, 0),     # one 64-channel stage, ragged position tail
    Attrs(2, 192, 17, 9, 256, 1, 1, 1, 1, 1, 1, 0, 0, 0, 0),     # 3 stages = ring depth
    Attrs(2, 320, 12, 12, 64, 1, 1, 1, 1, 1, 1, 0, 0, 0, 0),     # 5 stages; 64 outputs fwd (512x64 tile), 320 bwd
    Attrs(5, 128, 15, 14, 256, 1, 1, 2, 2, 1, 1, 0, 0, 0, 0),    # stride-2 projection, odd height
    Attrs(2, 64, 11, 12, 128, 1, 1, 2, 3, 1, 1, 1, 2, 1, 0),     # mixed strides with padding (tap class offset != 0)
    Attrs(1, 64, 9, 9, 64, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1),        # padded 1x1: border outputs see no input
    Attrs(40, 128, 14, 14, 128, 1, 1, 1, 1, 1, 1, 0, 0, 0, 0),   # 7840 positions: all 8 XCD slots, several m groups
    Attrs(2, 64, 3, 3, 64, 1, 1, 4, 4, 1, 1, 0, 0, 0, 0),        # stride larger than the image: single output pixel
]


@pytest.mark.parametrize("case", range(len(GEMM1X1_CASES)))
@pytest.mark.parametrize("pre,variant", [(True, 0), (False, 0), (True, 1), (True, 2), (True, 3), (True, 4), (True, 5), (True, 6)])
def test_gemm1x1_kernel(case, pre, variant, monkeypatch):
    """variant 0 = the dispatcher's tile, stage size and ring depth; 1..5 = forced tile / stage / ring choices (5 = the large-layer default)."""
    monkeypatch.setenv("NGC_G1_VARIANT", str(variant))
    a = GEMM1X1_CASES[case]
    _check_all(a, "bf16", BLK, BLK, pre, 7000 + case, ("gemm1x1", "gemm1x1", "wgrad"))


CHANNEL_TAIL_CASES = [
    # n  c    h   w   k    r  s  sh sw dh dw pads      channel counts that are multiples of 16 but not of 64
    Attrs(2, 48, 14, 14, 96, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1),      # strip: second 64-channel tile half empty
    Attrs(3, 80, 9, 9, 16, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1),        # one output block of a 64-channel tile
    Attrs(2, 16, 12, 12, 48, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1),      # one input chunk
    Attrs(2, 48, 16, 16, 80, 3, 3, 2, 2, 1, 1, 1, 1, 1, 1),      # strided: per-class backprop-data launches
    Attrs(2, 48, 8, 8, 96, 1, 1, 1, 1, 1, 1, 0, 0, 0, 0),        # 1x1: partial last stage (48 = 32 + 16) and tile
    Attrs(3, 80, 10, 10, 16, 1, 1, 1, 1, 1, 1, 0, 0, 0, 0),      # 1x1: 16 outputs of a 64-channel tile
    Attrs(2, 144, 7, 7, 208, 1, 1, 1, 1, 1, 1, 0, 0, 0, 0),      # 1x1: 128-wide tiles, the second 80 / 128 full
    Attrs(2, 96, 8, 8, 48, 1, 1, 2, 2, 1, 1, 0, 0, 0, 0),        # 1x1 stride 2
    Attrs(2, 112, 12, 12, 160, 5, 5, 1, 1, 1, 1, 2, 2, 2, 2),    # 5x5, both channel counts partial
]


@pytest.mark.parametrize("case", range(len(CHANNEL_TAIL_CASES)))
@pytest.mark.parametrize("pre", [True, False])
def test_channel_counts_not_multiples_of_64(case, pre):
    a = CHANNEL_TAIL_CASES[case]
    fb = "gemm1x1" if a.r * a.s == 1 else "strip"
    _check_all(a, "bf16", BLK, BLK, pre, 7500 + case, (fb, fb, "wgrad_gemm"))


STRIDED_1X1_CASES = [
    # 1x1 windows with strides: backprop-data computes one pixel per stride block and writes zeros to the rest
    Attrs(2, 64, 7, 7, 64, 1, 1, 2, 2, 1, 1, 0, 0, 0, 0),        # odd image: the last block row / column is cut
    Attrs(2, 32, 9, 12, 64, 1, 1, 2, 1, 1, 1, 0, 0, 0, 0),       # stride (2, 1)
    Attrs(3, 64, 8, 9, 32, 1, 1, 1, 2, 1, 1, 0, 0, 0, 0),        # stride (1, 2), odd width
    Attrs(2, 64, 10, 10, 64, 1, 1, 3, 3, 1, 1, 0, 0, 0, 0),      # 9 pixels per block: fill pass
    Attrs(2, 64, 9, 9, 64, 1, 1, 2, 2, 1, 1, 1, 1, 1, 1),        # padding: the lattice starts at pixel (1, 1): fill pass
    Attrs(1, 64, 3, 3, 64, 1, 1, 4, 4, 1, 1, 0, 0, 0, 0),        # stride beyond the image: one position
    Attrs(4, 128, 28, 28, 256, 1, 1, 2, 2, 1, 1, 0, 0, 0, 0),    # several position tiles
]


@pytest.mark.parametrize("case", range(len(STRIDED_1X1_CASES)))
@pytest.mark.parametrize("pre", [True, False])
def test_strided_1x1_backprop_data_writes_every_pixel(case, pre):
    """The output tensor starts as NaN bit patterns (out_tensor), so a pixel that neither the computed class nor the
    zeros next to it (or the fill pass) reach fails the comparison; the ReLU-mask and channel-sum compounds run on the
    same launches."""
    _check_all(STRIDED_1X1_CASES[case], "bf16", BLK, BLK, pre, 7700 + case, ("gemm1x1", "gemm1x1", "wgrad"))


@pytest.mark.parametrize("case", range(len(CHANNEL_TAIL_CASES)))
def test_channel_tail_loads_never_look_behind_the_filter_tensor(case):
    """Filter rows past Cout and channel blocks past Cin of a partial tile / stage must read as zeros, not whatever
    lies behind the filter tensor: here the blocked filters sit at the front of a larger allocation whose remainder
    holds NaN bit patterns (all accesses stay inside that allocation, so nothing can fault).  A NaN picked up there
    would reach real outputs through 0 * NaN."""
    a = CHANNEL_TAIL_CASES[case]
    x, w, b, dy = _tensors(a, "bf16", 7700 + case)
    wbits = encode(w, "bf16")
    st = stream()
    P, Q = oracle.out_shape(a)

    def fenced(layout):
        blk = filter_blocked_host(wbits, layout).reshape(-1)
        big = torch.full((blk.size + 64 * 1024,), 0x7FC0, dtype=torch.int16, device="cuda")
        big[:blk.size] = dev(blk)
        return big

    d_f = desc_of(a, "bf16", BLK, BLK, ng.NGC_BLOCKED_FWD, ng.NGC_EPI_BIAS | ng.NGC_EPI_RELU)
    d_b = desc_of(a, "bf16", BLK, BLK, ng.NGC_BLOCKED_BWD)
    wf, wb = fenced(ng.NGC_BLOCKED_FWD), fenced(ng.NGC_BLOCKED_BWD)
    y, dx = out_tensor(d_f, 1, "bf16"), out_tensor(d_b, 0, "bf16")
    ng.ngc_conv_fwd(d_f, data_to_device(x, "bf16", BLK), wf, dev(np.asarray(b, dtype=np.float32)), y, workspace(d_f, ng.NGC_OP_FWD), st)
    ng.ngc_conv_bwd_data(d_b, data_to_device(dy, "bf16", BLK), wb, dx, workspace(d_b, ng.NGC_OP_BWD_DATA), st)
    torch.cuda.synchronize()
    from gpu_util import data_from_device
    yh = data_from_device(y, "bf16", BLK, (a.n, a.k, P, Q))
    dxh = data_from_device(dx, "bf16", BLK, (a.n, a.c, a.h, a.w))
    assert np.isfinite(yh).all() and np.isfinite(dxh).all()
    assert oracle.max_normalised_error(yh, oracle.conv_fwd(a, x, w, bias=b, relu=True)) <= bound("bf16", "act")
    assert oracle.max_normalised_error(dxh, oracle.conv_bwd_data(a, dy, w)) <= bound("bf16", "act")


@pytest.mark.parametrize("xl,yl", [(NCHW, BLK), (BLK, NCHW), (NCHW, NCHW)])
def test_channel_tails_with_nchw_tensors(xl, yl):
    _check_all(CHANNEL_TAIL_CASES[4], "bf16", xl, yl, True, 7600, ("gemm1x1", "gemm1x1", "wgrad_gemm"))
    _check_all(Attrs(2, 80, 4, 6, 208, 1, 1, 1, 1, 1, 1, 0, 0, 0, 0), "bf16", xl, yl, True, 7601,
               ("gemm1x1", "gemm1x1", "wgrad_gemm"))


@pytest.mark.parametrize("case,cases", [(0, "mfma"), (3, "mfma"), (2, "mfma"), (4, "mfma"), (0, "tail"), (6, "tail")])
def test_channel_sums_second_pass_matches_fused(case, cases, monkeypatch):
    """NGC_DB_FUSE=0: the channel sums come from a second pass over dx instead of the backprop-data workgroups."""
    a = (MFMA_CASES if cases == "mfma" else CHANNEL_TAIL_CASES)[case]
    x, w, b, dy = _tensors(a, "bf16", 7700 + case)
    run = Run(a, "bf16", BLK, BLK, True)
    dx1, db1 = run.bwd_data_relu_db(dy, w, x)
    ws_fused = ng.ngc_conv_workspace_bytes(run.last_desc, ng.NGC_OP_BWD_DATA_DB)
    monkeypatch.setenv("NGC_DB_FUSE", "0")
    dx0, db0 = run.bwd_data_relu_db(dy, w, x)
    assert np.array_equal(dx0, dx1)
    assert oracle.max_normalised_error(db1, db0) <= 1e-6                 # same values, different summation order
    assert oracle.max_normalised_error(db0, oracle.bias_grad(dx0)) <= 1e-5
    assert ws_fused > 0 and ng.ngc_conv_workspace_bytes(run.last_desc, ng.NGC_OP_BWD_DATA_DB) > 0


NCHW_1X1_CASES = [
    # n  c    h   w   k    r  s  sh sw dh dw pads      stride 1, no padding, H*W % 8 == 0
    Attrs(2, 128, 8, 12, 64, 1, 1, 1, 1, 1, 1, 0, 0, 0, 0),      # 192 positions: one ragged tile
    Attrs(3, 64, 16, 16, 128, 1, 1, 1, 1, 1, 1, 0, 0, 0, 0),     # 768 positions, tiles straddle images
    Attrs(5, 256, 8, 8, 64, 1, 1, 1, 1, 1, 1, 0, 0, 0, 0),       # 320 positions of a 512-position tile; 8 stages
    Attrs(2, 64, 28, 28, 256, 1, 1, 1, 1, 1, 1, 0, 0, 0, 0),     # 1568 positions, ragged last tile
    Attrs(9, 192, 4, 6, 320, 1, 1, 1, 1, 1, 1, 0, 0, 0, 0),      # 24-position images: 10.7 images per 256-position tile
]


@pytest.mark.parametrize("case", range(len(NCHW_1X1_CASES)))
@pytest.mark.parametrize("xl,yl", [(NCHW, BLK), (BLK, NCHW), (NCHW, NCHW)])
@pytest.mark.parametrize("pre,variant", [(True, 0), (False, 0), (True, 3)])
def test_gemm1x1_reads_and_writes_nchw(case, xl, yl, pre, variant, monkeypatch):
    """Layout propagation: the 1x1 GEMM reads its activations from / writes its result to NCHW tensors."""
    monkeypatch.setenv("NGC_G1_VARIANT", str(variant))
    a = NCHW_1X1_CASES[case]
    _check_all(a, "bf16", xl, yl, pre, 7300 + case, ("gemm1x1", "gemm1x1", "wgrad_gemm"))


def test_nchw_1x1_outside_the_in_place_path_runs_on_blocked_copies():
    a = Attrs(2, 64, 7, 7, 64, 1, 1, 1, 1, 1, 1, 0, 0, 0, 0)       # 49 positions per image: not a multiple of 8
    _check_all(a, "bf16", NCHW, BLK, False, 7400, ("staged:gemm1x1", "staged:gemm1x1", "staged:wgrad_gemm"))
    b = Attrs(2, 64, 8, 8, 64, 1, 1, 2, 2, 1, 1, 0, 0, 0, 0)       # stride 2
    _check_all(b, "bf16", BLK, NCHW, False, 7401, ("staged:gemm1x1", "staged:gemm1x1", "staged:"))


@pytest.mark.parametrize("case", [0, 3, 4, 5])
def test_one_tap_gather_kernel_still_matches(case, monkeypatch):
    """1x1 shapes through the gather implicit-GEMM kernel (the pipelined GEMM switched off)."""
    monkeypatch.setenv("NGC_GEMM1X1", "0")
    a = GEMM1X1_CASES[case]
    _check_all(a, "bf16", BLK, BLK, True, 7100 + case, ("igemm", "igemm", "wgrad"))


STRIDED_STRIP_CASES = [
    # n  c    h   w   k    r  s  sh sw dh dw pbh pbw pah paw
    Attrs(3, 128, 56, 56, 128, 3, 3, 2, 2, 1, 1, 1, 1, 1, 1),    # ResNet stage transition: row strips of a 57-wide patch
    Attrs(5, 64, 28, 28, 64, 3, 3, 2, 2, 1, 1, 1, 1, 1, 1),      # whole 14x14 outputs, one image per strip
    Attrs(9, 64, 14, 14, 128, 3, 3, 2, 2, 1, 1, 1, 1, 1, 1),     # several 7x7 outputs per strip, ragged last group
    Attrs(2, 64, 17, 23, 64, 5, 3, 2, 3, 1, 1, 2, 1, 2, 1),      # 5x3 taps, strides (2,3), odd sizes
    Attrs(2, 64, 20, 20, 64, 3, 3, 2, 2, 1, 1, 0, 0, 0, 0),      # no padding: the last input row / column is never read
    Attrs(1, 64, 9, 9, 64, 2, 2, 2, 2, 1, 1, 0, 0, 1, 1),        # 2x2 taps, stride 2: every class has exactly one tap
]


@pytest.mark.parametrize("case", range(len(STRIDED_STRIP_CASES)))
@pytest.mark.parametrize("pre", [True, False])
def test_strided_strip_kernel(case, pre):
    a = STRIDED_STRIP_CASES[case]
    _check_all(a, "bf16", BLK, BLK, pre, 8000 + case, ("strip", "strip", "wgrad"))


@pytest.mark.parametrize("case", range(len(STRIDED_STRIP_CASES)))
def test_strided_strip_one_launch_per_class(case, monkeypatch):
    """NGC_STRIP_MERGE=0: the residue classes of backprop-data as separate launches instead of one grid."""
    monkeypatch.setenv("NGC_STRIP_MERGE", "0")
    _check_all(STRIDED_STRIP_CASES[case], "bf16", BLK, BLK, True, 8050 + case, ("strip", "strip", "wgrad"))


@pytest.mark.parametrize("case", [0, 3])
def test_strided_gather_kernel_still_matches(case, monkeypatch):
    """Strided multi-tap shapes through the gather implicit-GEMM kernel (strided strips switched off)."""
    monkeypatch.setenv("NGC_STRIP_STRIDED", "0")
    a = STRIDED_STRIP_CASES[case]
    _check_all(a, "bf16", BLK, BLK, True, 8100 + case, ("igemm", "igemm", "wgrad"))


def test_run_to_run_identical():
    a = MFMA_CASES[0]
    x, w, b, dy = _tensors(a, "bf16", 5)
    run = Run(a, "bf16", BLK, BLK, True)
    outs = []
    for _ in range(2):
        run.fwd(x, w, bias=b, relu=True); r1 = run.last_raw.clone()
        run.bwd_data(dy, w); r2 = run.last_raw.clone()
        run.bwd_filters(x, dy); r3 = run.last_raw.clone()
        outs.append((r1, r2, r3))
    for t0, t1 in zip(*outs):
        assert torch.equal(t0.view(torch.int32) if t0.dtype == torch.float32 else t0,
                           t1.view(torch.int32) if t1.dtype == torch.float32 else t1)


# ------------------------------------------------------------------ benchmark configurations
def _sampled_layer_check(L, n_y=100_000, n_dw=2048, convert_x_on_device=False):
    """Full-size launch configuration; oracle evaluated at sampled output elements."""
    print(f"layer {L.name} n={L.n}", flush=True)
    a = attrs_of(L)
    t = synth_inputs.layer_tensors(L)
    P, Q = oracle.out_shape(a)
    rng = np.random.default_rng(L.seed % (2 ** 32))
    blocked_ok = L.c % 16 == 0
    xl = BLK if blocked_ok else NCHW
    run = Run(a, "bf16", xl, BLK, True if blocked_ok else False)
    x64, w64, dy64 = (t[k].astype(np.float64) for k in ("x", "w", "dy"))
    bias = t["bias"] if L.bias_relu else None
    if "fwd" in L.ops:
        y = run.fwd(t["x"], t["w"], bias=bias, relu=L.bias_relu)
        idx = rng.integers(0, y.size, n_y)
        ref = oracle.conv_fwd_at(a, x64, w64, idx, bias=bias, relu=L.bias_relu)
        assert oracle.max_normalised_error(y.reshape(-1)[idx], ref) <= bound("bf16", "act"), "fwd"
        assert np.isfinite(y).all()
    if "bwd_data" in L.ops:
        dx = run.bwd_data(t["dy"], t["w"])
        idx = rng.integers(0, dx.size, n_y)
        ref = oracle.conv_bwd_data_at(a, dy64, w64, idx)
        assert oracle.max_normalised_error(dx.reshape(-1)[idx], ref) <= bound("bf16", "act"), "bwd_data"
        assert np.isfinite(dx).all()
        dxr = run.bwd_data_relu(t["dy"], t["w"], t["x"])
        xs = x64.reshape(-1)[idx]
        assert oracle.max_normalised_error(dxr.reshape(-1)[idx], oracle.relu_bwd_mask(ref, xs)) <= bound("bf16", "act"), "bwd_data_relu"
        keep = t["x"] > 0
        assert np.array_equal(dxr[keep], dx[keep]) and not dxr[~keep].any(), "mask applied to the same gradient"
        dx2, dbp = run.bwd_data_relu_db(t["dy"], t["w"], t["x"])
        assert np.array_equal(dx2, dxr) and oracle.max_normalised_error(dbp, oracle.bias_grad(dxr)) <= 1e-5, "bwd_data_relu_db"
        db = run.bias_grad(t["dy"])
        assert oracle.max_normalised_error(db, oracle.bias_grad(dy64)) <= 1e-5, "bias_grad"
    if "bwd_filters" in L.ops:
        dw = run.bwd_filters(t["x"], t["dy"])
        idx = rng.integers(0, dw.size, min(n_dw, dw.size))
        ref = oracle.conv_bwd_filters_at(a, x64, dy64, idx)
        assert oracle.max_normalised_error(dw.reshape(-1)[idx], ref) <= bound("bf16", "dw"), "bwd_filters"
        assert np.isfinite(dw).all()
    if ("bwd_data" in L.ops and "bwd_filters" in L.ops and blocked_ok and
            ng.ngc_conv_variant(desc_of(a, "bf16", BLK, BLK, ng.NGC_BLOCKED_BWD), ng.NGC_OP_BWD_DATA_FILTERS) == "bwd1x1_fused_bf16"):
        # both derivative ops in one pass over dy, at the launch configuration `bench.py --fused-backward` times
        dxf, dwf = run.bwd_data_filters(t["x"], t["dy"], t["w"])
        idx = rng.integers(0, dxf.size, n_y)
        assert oracle.max_normalised_error(dxf.reshape(-1)[idx], oracle.conv_bwd_data_at(a, dy64, w64, idx)) <= bound("bf16", "act"), "fused dx"
        idx = rng.integers(0, dwf.size, min(n_dw, dwf.size))
        assert oracle.max_normalised_error(dwf.reshape(-1)[idx], oracle.conv_bwd_filters_at(a, x64, dy64, idx)) <= bound("bf16", "dw"), "fused dw"
        assert np.isfinite(dxf).all() and np.isfinite(dwf).all()


def test_cfg2_full_size_sampled():
    _sampled_layer_check(synth_inputs.config_layers(2)[0])


def test_cfg2_reduced_batch_full_tensors():
    L = synth_inputs.config_layers(2, batch=2)[0]
    a = attrs_of(L)
    t = synth_inputs.layer_tensors(L)
    run = Run(a, "bf16", BLK, BLK, True)
    y = run.fwd(t["x"], t["w"], bias=t["bias"], relu=True)
    assert oracle.max_normalised_error(y, oracle.conv_fwd(a, t["x"], t["w"], bias=t["bias"], relu=True)) <= bound("bf16", "act")
    dx = run.bwd_data(t["dy"], t["w"])
    assert oracle.max_normalised_error(dx, oracle.conv_bwd_data_gather(a, t["dy"], t["w"])) <= bound("bf16", "act")
    dw = run.bwd_filters(t["x"], t["dy"])
    assert oracle.max_normalised_error(dw, oracle.conv_bwd_filters(a, t["x"], t["dy"])) <= bound("bf16", "dw")


def test_cfg3_full_size_with_device_layout_conversion():
    """1x1 bottleneck: x arrives in NCHW, is converted on the device (bit exact), then the
    three ops run on the blocked tensor."""
    L = synth_inputs.config_layers(3)[0]
    a = attrs_of(L)
    t = synth_inputs.layer_tensors(L)
    xbits = encode(t["x"], "bf16")
    x_nchw = dev(xbits)
    xb = torch.empty(L.n * (L.c // 16) * L.h * L.w * 16, dtype=torch.int16, device="cuda")
    ng.ngc_layout_convert(ng.NGC_BF16, L.n, L.c, L.h, L.w, x_nchw, NCHW, xb, BLK, stream())
    torch.cuda.synchronize()
    got = host(xb, np.uint16).reshape(L.n, L.c // 16, L.h, L.w, 16)
    exp = xbits.reshape(L.n, L.c // 16, 16, L.h, L.w).transpose(0, 1, 3, 4, 2)
    assert np.array_equal(got, exp)
    del got, exp
    _sampled_layer_check(L)


STEM_CASES = [
    Attrs(2, 3, 38, 40, 64, 7, 7, 2, 2, 1, 1, 3, 3, 3, 3),       # ragged last tile (P = 19), Q = 20
    Attrs(1, 2, 23, 16, 128, 7, 7, 2, 2, 1, 1, 2, 3, 4, 2),      # C = 2, asymmetric pads, two k tiles
    Attrs(3, 1, 64, 64, 64, 7, 7, 2, 2, 1, 1, 3, 3, 3, 3),       # C = 1
    Attrs(2, 3, 50, 48, 64, 7, 7, 2, 2, 1, 1, 3, 3, 3, 3),       # Q = 24: 4-row stages, ragged last stage (P = 25)
    Attrs(5, 3, 30, 80, 128, 7, 7, 2, 2, 1, 1, 1, 3, 2, 3),      # Q = 40, two k tiles, asymmetric pad_h
]


@pytest.mark.parametrize("case", range(len(STEM_CASES)))
@pytest.mark.parametrize("bh", [0, 2])
def test_stem_kernels_small(case, bh, monkeypatch):
    """bh: rows per sub-pixel block of the backprop-data formulation (0: the dispatcher's 4 x 2 blocks, 2: 2 x 2)."""
    if bh:
        monkeypatch.setenv("NGC_STEM_BH", str(bh))
    a = STEM_CASES[case]
    _check_all(a, "bf16", NCHW, BLK, False, 5000 + case, ("stem_fwd", "", ""))


@pytest.mark.parametrize("tp", [1, 5, 11, 14, 16])
def test_stem_forward_tile_heights(tp, monkeypatch):
    """Output rows per workgroup of the low-channel forward kernel (the dispatcher picks 4..16 by the number of
    workgroup rounds; forced here): ragged last tiles, tiles taller than the image part left, one row."""
    monkeypatch.setenv("NGC_STEM_TP", str(tp))
    for case in (0, 4):
        a = STEM_CASES[case]
        x, w, b, dy = _tensors(a, "bf16", 5200 + case)
        run = Run(a, "bf16", NCHW, BLK, False)
        y = run.fwd(x, w, bias=b, relu=True)
        assert ng.ngc_conv_variant(run.last_desc, ng.NGC_OP_FWD) == "stem_fwd_bf16"
        e = oracle.max_normalised_error(y, oracle.conv_fwd(a, x, w, bias=b, relu=True))
        assert e <= bound("bf16", "act"), f"tp {tp} case {case} err {e}"


@pytest.mark.parametrize("case", [1, 2, 3, 4])                       # the cases whose Q is a multiple of 8
def test_stem_backprop_filters_two_buffer_form(case, monkeypatch):
    """The low-channel backprop-filters kernel with two stage buffers and the input rows through registers (the form
    taken when three buffers plus the staging area do not fit the LDS; forced here)."""
    monkeypatch.setenv("NGC_WSTEM_RING", "2")
    a = STEM_CASES[case]
    x, w, b, dy = _tensors(a, "bf16", 5300 + case)
    run = Run(a, "bf16", NCHW, BLK, False)
    dw = run.bwd_filters(x, dy)
    assert ng.ngc_conv_variant(run.last_desc, ng.NGC_OP_BWD_FILTERS) == "wgrad_stem_bf16"
    e = oracle.max_normalised_error(dw, oracle.conv_bwd_filters(a, x, dy))
    assert e <= bound("bf16", "dw"), f"err {e}"


def test_stem_backprop_data_unstaged_store():
    """Width not a multiple of 8: the sub-pixel store cannot go through whole 16-byte row pieces."""
    a = Attrs(2, 3, 30, 44, 64, 7, 7, 2, 2, 1, 1, 3, 3, 3, 3)
    _check_all(a, "bf16", NCHW, BLK, False, 5100, ("", "stem_bwd", ""))


def test_cfg4_stem_full_size_sampled():
    _sampled_layer_check(synth_inputs.config_layers(4)[0], n_y=50_000, n_dw=512)


def test_cfg4_stem_reduced_batch():
    L = synth_inputs.config_layers(4, batch=4)[0]
    _sampled_layer_check(L, n_y=50_000, n_dw=512)


@pytest.mark.parametrize("idx", range(23))
def test_cfg5_shapes_full_batch(idx):
    """Batch 128, i.e. the launch configurations the benchmark times: tile shapes, stage sizes, position
    chunks and images per stage depend on the batch."""
    L = synth_inputs.config_layers(5)[idx]
    _sampled_layer_check(L, n_y=20_000, n_dw=256)


@pytest.mark.parametrize("idx", range(23))
def test_cfg5_shapes_reduced_batch(idx):
    L = synth_inputs.config_layers(5, batch=4)[idx]
    _sampled_layer_check(L, n_y=20_000, n_dw=256)


# ------------------------------------------------------------------ general-attribute layers (dilation, padding
# below != above, 5x5 / 1x7 / 7x1 / 2x2 windows, per-axis strides) at the sizes bench.py --workload cfg6 times
@pytest.mark.parametrize("idx", range(8))
def test_general_attribute_layers_full_batch(idx):
    L = synth_inputs.config_layers(6)[idx]
    _sampled_layer_check(L, n_y=20_000, n_dw=256)
    d = Run(attrs_of(L), "bf16", BLK, BLK, True)
    assert L.p == d.P and L.q == d.Q


@pytest.mark.parametrize("idx", range(8))
def test_general_attribute_layers_whole_tensors(idx):
    L = synth_inputs.config_layers(6, batch=2)[idx]
    _check_all(attrs_of(L), "bf16", BLK, BLK, True, 9000 + idx, ("strip", "strip", "wgrad"))


# ------------------------------------------------------------------ randomized descriptors (seeded)
def _random_attrs(rng, channel_step):
    while True:
        r, s = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        sh, sw = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        dh, dw = int(rng.integers(1, 3)), int(rng.integers(1, 3))
        h, w = int(rng.integers(1, 21)), int(rng.integers(1, 21))
        pbh, pah = int(rng.integers(0, 4)), int(rng.integers(0, 4))
        pbw, paw = int(rng.integers(0, 4)), int(rng.integers(0, 4))
        a = Attrs(int(rng.integers(1, 5)), channel_step * int(rng.integers(1, 11)), h, w,
                  channel_step * int(rng.integers(1, 11)), r, s, sh, sw, dh, dw, pbh, pbw, pah, paw)
        P, Q = oracle.out_shape(a)
        if P >= 1 and Q >= 1:
            return a


@pytest.mark.parametrize("seed", range(150))
def test_random_descriptors_blocked_bf16(seed):
    """Whatever kernel the dispatcher picks for a random node (window, strides, dilation, one-sided padding,
    channel counts that are multiples of 16): all ops and backward compounds against the oracle."""
    rng = np.random.default_rng(424200 + seed)
    a = _random_attrs(rng, 16)
    _check_all(a, "bf16", BLK, BLK, bool(seed & 1), 9100 + seed)


@pytest.mark.parametrize("seed", range(40))
def test_random_descriptors_other_types_and_layouts(seed):
    """fp32 / NCHW / odd channel counts: the direct kernels (and the NCHW 1x1 paths where they apply)."""
    rng = np.random.default_rng(434300 + seed)
    a = _random_attrs(rng, 1 if seed % 2 else 16)
    dtype = "f32" if seed % 4 == 0 else "bf16"
    xl, yl = [(NCHW, NCHW), (NCHW, BLK), (BLK, NCHW), (BLK, BLK)][(seed // 2) % 4]
    _check_all(a, dtype, xl, yl, False, 9200 + seed)


@pytest.mark.parametrize("seed", range(60))
def test_random_descriptors_larger_images(seed):
    """Images of up to 64 x 64 pixels, batch up to 8: several tiles, strips, stages and position chunks per launch."""
    rng = np.random.default_rng(444400 + seed)
    while True:
        r, s = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        a = Attrs(int(rng.integers(1, 9)), 16 * int(rng.integers(1, 5)), int(rng.integers(8, 65)), int(rng.integers(8, 65)),
                  16 * int(rng.integers(1, 5)), r, s, int(rng.integers(1, 3)), int(rng.integers(1, 3)),
                  int(rng.integers(1, 3)), int(rng.integers(1, 3)), *(int(v) for v in rng.integers(0, 3, 4)))
        P, Q = oracle.out_shape(a)
        if P >= 1 and Q >= 1:
            break
    _check_all(a, "bf16", BLK, BLK, bool(seed & 1), 9300 + seed)


@pytest.mark.parametrize("a", [Attrs(3, 128, 17, 17, 192, 1, 7, 1, 1, 1, 1, 0, 3, 0, 3),
                               Attrs(4, 128, 20, 20, 128, 3, 3, 2, 2, 1, 1, 0, 0, 1, 1),
                               Attrs(2, 48, 9, 11, 80, 2, 3, 1, 2, 2, 1, 1, 0, 0, 2)])
def test_per_tap_backprop_filters_xcd_ordered_grid(a, monkeypatch):
    """NGC_WGG_XCD=1 forces what large multi-tap layers get by default: the one-dimensional grid of the per-tap
    kernel with the workgroups of a position chunk on one XCD, chunk count in multiples of 8."""
    monkeypatch.setenv("NGC_WGG_XCD", "1")
    x, w, b, dy = _tensors(a, "bf16", 9100 + a.c)
    run = Run(a, "bf16", BLK, BLK, True)
    dw = run.bwd_filters(x, dy)
    assert ng.ngc_conv_variant(run.last_desc, ng.NGC_OP_BWD_FILTERS) == "wgrad_gemm_bf16"
    assert oracle.max_normalised_error(dw, oracle.conv_bwd_filters(a, x, dy)) <= bound("bf16", "dw")


def test_strip_two_dimensional_grid_switch(monkeypatch):
    """NGC_STRIP_XCD=0: the strip kernel's launches with several output-channel tiles on the two-dimensional grid
    (default: one-dimensional, the tiles of a strip on one XCD)."""
    monkeypatch.setenv("NGC_STRIP_XCD", "0")
    a = Attrs(5, 64, 19, 21, 192, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1)
    _check_all(a, "bf16", BLK, BLK, True, 9200, ("strip", "strip", "wgrad"))


STRIP_PATH_CASES = [
    # n  c   h   w   k   r  s  sh sw dh dw pbh pbw pah paw
    Attrs(2, 64, 56, 56, 64, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1),       # 14-row strips: 25 fragments, the last one shared (r = 1)
    Attrs(2, 64, 14, 14, 64, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1),       # two images per strip: 13 fragments, shared (r = 5)
    Attrs(4, 80, 14, 14, 64, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1),       # 5 chunks: two per stage leaves the last stage half full
    Attrs(6, 128, 14, 14, 128, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1),     # 8 chunks, two output-channel tiles
    Attrs(10, 64, 7, 7, 64, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1),        # one fragment per wave
    Attrs(3, 96, 20, 24, 80, 3, 3, 1, 1, 2, 2, 2, 2, 2, 2),       # dilated window: backprop-filters without the shared row addresses
]


@pytest.mark.parametrize("switch", [None, ("NGC_STRIP_TAIL", "0"), ("NGC_STRIP_SPLIT", "0"), ("NGC_STRIP_CPS", "1"),
                                    ("NGC_WGRAD_NT", "0"), ("NGC_WGRAD_NT", "1")])
@pytest.mark.parametrize("a", STRIP_PATH_CASES)
def test_strip_epilogue_split_and_stage_paths(a, switch, monkeypatch):
    """The strip kernel's store path with the epilogues inside the last chunk, the shared last fragment and two
    chunks per LDS stage, and each of them switched off (the paths the other launches take); the backprop-filters
    partial stores in both forms.  Forward with and without bias + ReLU, backprop-data bare and with the ReLU-backprop
    mask, backprop-filters: all against the oracle."""
    if switch:
        monkeypatch.setenv(*switch)
    _check_all(a, "bf16", BLK, BLK, True, 9250 + a.c + a.h, ("strip", "strip", "wgrad"))


@pytest.mark.parametrize("a,variant", [
    (Attrs(2, 64, 12, 12, 64, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1), "strip"),
    (Attrs(2, 64, 12, 12, 64, 1, 1, 1, 1, 1, 1, 0, 0, 0, 0), "gemm1x1"),
    (Attrs(2, 64, 12, 12, 64, 3, 3, 2, 2, 1, 1, 1, 1, 1, 1), "strip"),
])
@pytest.mark.filterwarnings("ignore:invalid value encountered")          # the signalling NaN among the patterns
def test_relu_backprop_mask_special_values(a, variant):
    """The ReLU-backprop mask is `x_in > 0` as a comparison of floats: +0, -0, negative values (denormals and -inf
    included) and NaNs of either sign block, positive denormals and +inf pass.  x_in carries each of those bit patterns
    at seeded places; everything else about the call is the ordinary parity case."""
    x, w, b, dy = _tensors(a, "bf16", 9700 + a.r + a.sh)
    specials = np.array([0x0000, 0x8000, 0x0001, 0x8001, 0x007F, 0x7F80, 0xFF80, 0x7FC0, 0xFFC0, 0x7F81, 0x3F80, 0xBF80],
                        dtype=np.uint16)
    vals = (specials.astype(np.uint32) << 16).view(np.float32)
    rng = np.random.default_rng(9700)
    x_in = np.array(x, dtype=np.float32, copy=True)
    flat = x_in.reshape(-1)
    idx = rng.choice(flat.size, size=flat.size // 3, replace=False)
    flat[idx] = vals[rng.integers(0, len(vals), size=idx.size)]
    run = Run(a, "bf16", BLK, BLK, True)
    dxr = run.bwd_data_relu(dy, w, x_in)
    assert ng.ngc_conv_variant(run.last_desc, ng.NGC_OP_BWD_DATA).startswith(variant)
    ref = oracle.relu_bwd_mask(oracle.conv_bwd_data(a, dy, w), x_in)
    assert oracle.max_normalised_error(dxr, ref) <= bound("bf16", "act")
    with np.errstate(invalid="ignore"):
        blocked = ~(x_in > 0)
    assert np.all(dxr[blocked] == 0) and not np.signbit(dxr[blocked]).any()
    passed = dxr[~blocked]
    assert np.count_nonzero(passed) > 0.9 * passed.size            # positive denormals and +inf let the gradient through


WIDE_ROW_CASES = [
    # n  c   h   w     k   r  s  sh sw dh dw pbh pbw pah paw      rows wider than a strip holds: column tiles
    Attrs(1, 32, 5, 1000, 64, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1),
    Attrs(2, 64, 12, 3136, 64, 3, 1, 1, 1, 1, 1, 1, 0, 1, 0),     # a 3x1x1 temporal window seen as a rank-2 node
    Attrs(1, 64, 9, 1500, 128, 3, 3, 2, 2, 1, 1, 1, 1, 1, 1),     # stride 2: four residue classes, ragged last tile
    Attrs(1, 48, 4, 2051, 80, 1, 5, 1, 1, 1, 2, 0, 4, 0, 4),      # odd width, dilated 1x5, channel tails
    Attrs(1, 64, 30, 901, 64, 5, 5, 1, 1, 1, 1, 2, 2, 2, 2),      # one column past a strip, 25 taps
    Attrs(1, 64, 3, 700, 64, 3, 3, 1, 1, 1, 40, 1, 40, 1, 40),    # patch wider than LDS holds although 700 positions fit
]


@pytest.mark.parametrize("a", WIDE_ROW_CASES)
def test_strip_column_tiles(a):
    _check_all(a, "bf16", BLK, BLK, True, 9300 + a.w, ("strip", "strip", "wgrad"))


def test_strip_column_tiles_strided_classes_and_channel_sums():
    """Lattice rows of a strided backprop-data that are wider than a strip: one launch per residue class (no shared
    grid), and the channel sums of ngc_conv_bwd_data_relu_db come from the second pass."""
    a = Attrs(1, 64, 6, 2000, 64, 3, 3, 2, 2, 1, 1, 1, 1, 1, 1)
    _check_all(a, "bf16", BLK, BLK, True, 9400, ("strip", "strip", "wgrad"))


def test_random_wide_row_descriptors():
    """Randomised windows, strides, dilation and padding on images 900-2600 pixels wide (column tiles, residue classes
    with and without shared grids, channel tails)."""
    g = np.random.default_rng(20180128)
    done = 0
    while done < 24:
        r, s = (int(v) for v in g.integers(1, 6, size=2))
        sh, sw = (int(v) for v in g.integers(1, 4, size=2))
        dh, dw = (int(v) for v in g.integers(1, 4, size=2))
        pb = [int(v) for v in g.integers(0, 4, size=4)]
        a = Attrs(int(g.integers(1, 3)), int(g.choice([16, 48, 64, 128])), int(g.integers(1, 10)), int(g.integers(900, 2600)),
                  int(g.choice([16, 64, 96, 128])), r, s, sh, sw, dh, dw, *pb)
        P, Q = oracle.out_shape(a)
        if P < 1 or Q < 1 or a.n * a.c * a.h * a.w > 5e6:
            continue
        _check_all(a, "bf16", BLK, BLK, bool(done % 2), 9500 + done)
        done += 1


# ------------------------------------------------------------------ epilogue order and rounding, bit for bit
EPILOGUE_BIT_CASES = [
    # attrs                                                       x layout, y layout, tap (r0, s0), kernel
    (Attrs(2, 16, 9, 12, 16, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1), BLK, BLK, (1, 1), "strip_bf16"),
    (Attrs(2, 64, 14, 14, 64, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1), BLK, BLK, (0, 2), "strip_bf16"),
    (Attrs(3, 16, 8, 8, 16, 1, 1, 1, 1, 1, 1, 0, 0, 0, 0), BLK, BLK, (0, 0), "gemm1x1_bf16"),
    (Attrs(2, 32, 8, 8, 48, 1, 1, 1, 1, 1, 1, 0, 0, 0, 0), NCHW, NCHW, (0, 0), "gemm1x1_bf16"),
    (Attrs(2, 32, 9, 9, 64, 6, 6, 1, 1, 1, 1, 2, 2, 3, 3), BLK, BLK, (2, 2), "igemm_bf16"),
    (Attrs(2, 3, 32, 32, 64, 7, 7, 2, 2, 1, 1, 3, 3, 3, 3), NCHW, BLK, (3, 3), "stem_fwd_bf16"),
    (Attrs(2, 5, 7, 6, 7, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1), NCHW, NCHW, (1, 1), "direct"),
]


@pytest.mark.parametrize("case", range(len(EPILOGUE_BIT_CASES)))
def test_epilogue_bias_relu_single_rne_rounding_bit_exact(case, expect=None):
    """Bias, then ReLU, then exactly one round-to-nearest-even conversion of the fp32 value.  The filter is a single
    tap of ones on c == k mod C, so the fp32 accumulator of every kernel equals one input element exactly; the input
    values and the fp32 biases are chosen so that x + b lands on exact ties of the bf16 grid (both parities of the kept
    bit), a few fp32 ulps to either side of them, and on ordinary values.  The device bits must equal the oracle's RNE
    conversion of relu(fp32(x) + b) - truncation, round-half-up, rounding before the bias or before the ReLU all
    differ on these values."""
    a, xl, yl, (r0, s0), variant = EPILOGUE_BIT_CASES[case]
    P, Q = oracle.out_shape(a)
    rng = np.random.default_rng(777 + case)
    # bf16 inputs: 8 significant bits, binades [0.5, 4), both signs, a few zeros
    xbits = (rng.integers(0x3F00, 0x4080, size=(a.n, a.c, a.h, a.w)).astype(np.uint16)
             | (rng.integers(0, 2, size=(a.n, a.c, a.h, a.w)).astype(np.uint16) << 15))
    xbits[rng.random(xbits.shape) < 0.05] = 0
    x = oracle.bf16_bits_to_f64(xbits).astype(np.float32)
    u = np.float32(2.0) ** -23
    ties = [2.0 ** -8, 2.0 ** -8 + 2.0 ** -22, 2.0 ** -8 - 2.0 ** -22, 2.0 ** -9, 2.0 ** -9 + 2.0 ** -23, 2.0 ** -7 - 2.0 ** -21,
            -2.0 ** -8, 2.0 ** -7, -2.0 ** -9, 3 * 2.0 ** -9, -(2.0 ** -8 + 2.0 ** -22), 0.1, -0.1, 1e-3, 5 * 2.0 ** -10, 0.0]
    b = np.array([ties[k % len(ties)] for k in range(a.k)], dtype=np.float32)
    w = np.zeros((a.k, a.c, a.r, a.s), dtype=np.float32)
    for k in range(a.k):
        w[k, k % a.c, r0, s0] = 1.0
    run = Run(a, "bf16", xl, yl, True)
    run.fwd(x, w, bias=b, relu=True)
    assert ng.ngc_conv_variant(run.last_desc, ng.NGC_OP_FWD).startswith(expect or variant), ng.ngc_conv_variant(run.last_desc, ng.NGC_OP_FWD)
    raw = host(run.last_raw, np.uint16)
    if yl == BLK:
        got = oracle.blocked16_to_nchw(raw.reshape(a.n, (a.k + 15) // 16, P, Q, 16), a.k)
    else:
        got = raw.reshape(a.n, a.k, P, Q)
    # the input element each output reads (zero outside the image), by explicit index arithmetic
    hh = np.arange(P) * a.sh - a.pbh + r0 * a.dh
    ww = np.arange(Q) * a.sw - a.pbw + s0 * a.dw
    okh, okw = (hh >= 0) & (hh < a.h), (ww >= 0) & (ww < a.w)
    xin = np.zeros((a.n, a.k, P, Q), dtype=np.float32)
    src = x[:, np.arange(a.k) % a.c][:, :, np.clip(hh, 0, a.h - 1)][:, :, :, np.clip(ww, 0, a.w - 1)]
    xin[:] = np.where(okh[None, None, :, None] & okw[None, None, None, :], src, np.float32(0))
    v = xin + b[None, :, None, None]                       # one fp32 addition, round-to-nearest-even
    assert v.dtype == np.float32
    v = np.where(v > 0, v, np.float32(0))                  # ReLU; written so that -0 becomes +0
    want = oracle.f32_to_bf16_bits_rne(v)
    # the chosen values do exercise the tie rule: a fair share of the sums sit exactly between two bf16 values
    frac = v.view(np.uint32) & np.uint32(0xFFFF)
    assert (frac == 0x8000).mean() > 0.02, "exact ties"
    assert ((frac > 0x8000) & (frac <= 0x8004)).any() and ((frac < 0x8000) & (frac >= 0x7FFC)).any(), "next to a tie"
    got_cmp = np.where(got == 0x8000, np.uint16(0), got)   # the sign of a ReLU zero is free (numerically equal)
    bad = np.argwhere(got_cmp != want)
    assert bad.size == 0, (f"{len(bad)} elements differ, first at {bad[0]}: got {got[tuple(bad[0])]:#06x} want "
                           f"{want[tuple(bad[0])]:#06x} from fp32 bits {v.view(np.uint32)[tuple(bad[0])]:#010x}")


# ------------------------------------------------------------------ filter-resident strip kernel (opt-in)
ROWS_CASES = [
    Attrs(3, 64, 56, 56, 64, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1),      # the headline shape: sub-strips of 8 + 8 + ... rows
    Attrs(2, 64, 30, 20, 48, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1),      # ragged fragments, partial channel tile (forward)
    Attrs(2, 32, 17, 56, 64, 3, 3, 1, 1, 1, 1, 0, 2, 2, 0),      # one-sided padding, strips that end inside a sub-strip
    Attrs(2, 16, 9, 12, 16, 3, 3, 1, 1, 2, 2, 2, 2, 2, 2),       # one chunk, dilation 2
    Attrs(5, 48, 14, 14, 64, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1),      # three chunks, small images
]


@pytest.mark.parametrize("case", range(len(ROWS_CASES)))
def test_filter_resident_strip_kernel(case, monkeypatch):
    """NGC_ROWS=1 selects the filter-resident form of the strip kernel for stride-1 3x3 nodes whose filter tile fits the
    LDS (forward and backprop-data, with the ReLU-backprop mask); everything else of the node runs as usual."""
    monkeypatch.setenv("NGC_ROWS", "1")
    _check_all(ROWS_CASES[case], "bf16", BLK, BLK, True, 9800 + case, ("strip_rows", "strip_rows", "wgrad"))


def test_filter_resident_strip_kernel_epilogue_bits(monkeypatch):
    monkeypatch.setenv("NGC_ROWS", "1")
    test_epilogue_bias_relu_single_rne_rounding_bit_exact(0, expect="strip_rows_bf16")
