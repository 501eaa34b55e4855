"""Tensors of more than 2^31 bytes (just over 10^9 elements; the boundary allows fewer than 2^31 elements): the
kernels that address with 32-bit byte offsets run forward / backprop-data over groups of images that stay below
2 GiB, backprop-filters adds up the dw of such groups; all must index past 2 GiB correctly.  The
batch is a seeded 4-image tensor repeated 17 times, so every image of the result has a twin in the first four,
which are checked against the oracle on sampled elements."""
import numpy as np
import pytest
import torch

import oracle
import paper_1801_08058_amd as ng
import synth_inputs
from oracle import Attrs
from gpu_util import bound, dev, host, stream

pytestmark = pytest.mark.gpu
BLK = ng.NGC_NCHW16C
PERIOD, REPS = 4, 17


def _bits(v):
    return synth_inputs.f32_to_bf16_bits(v)


@pytest.mark.timeout(600)
def test_three_ops_on_tensors_past_two_gib():
    n, c, h, w, k = PERIOD * REPS, 64, 500, 500, 64
    a1 = Attrs(PERIOD, c, h, w, k, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1)
    print("case 68 x 64 x 500 x 500, 3x3", flush=True)
    x1 = synth_inputs.bf16_bits_to_f32(_bits(synth_inputs.normal(77, 0, (PERIOD, c, h, w), 0.0, 1.0)))
    dy1 = synth_inputs.bf16_bits_to_f32(_bits(synth_inputs.normal(77, 3, (PERIOD, k, h, w), 0.0, 0.1)))
    wt = synth_inputs.bf16_bits_to_f32(_bits(synth_inputs.normal(77, 1, (k, c, 3, 3), 0.0, (2.0 / (c * 9)) ** 0.5)))
    bias = synth_inputs.uniform(77, 2, (k,), -0.1, 0.1)
    xb = oracle.nchw_to_blocked16(_bits(x1))                       # [4][4][500][500][16]
    dyb = oracle.nchw_to_blocked16(_bits(dy1))
    xd = dev(np.tile(xb, (REPS, 1, 1, 1, 1)))
    dyd = dev(np.tile(dyb, (REPS, 1, 1, 1, 1)))
    assert xd.numel() * 2 > (1 << 31)
    wd, bd = dev(_bits(wt)), dev(np.asarray(bias, dtype=np.float32))
    mk = lambda nn, epi=ng.NGC_EPI_NONE: ng.make_desc(nn, c, h, w, k, 3, 3, pad_below=(1, 1), pad_above=(1, 1), epilogue=epi)
    d = mk(n, ng.NGC_EPI_BIAS | ng.NGC_EPI_RELU)
    names = [ng.ngc_conv_variant(d, op) for op in (ng.NGC_OP_FWD, ng.NGC_OP_BWD_DATA, ng.NGC_OP_BWD_FILTERS)]
    print("variants", names, flush=True)
    assert names == ["sliced:strip_bf16", "sliced:strip_bf16", "sliced:wgrad_gemm_bf16"], names
    ws = lambda dd, op: torch.empty(max(ng.ngc_conv_workspace_bytes(dd, op), 16), dtype=torch.uint8, device="cuda")
    g = np.random.default_rng(5)

    def check_twins_and_samples(t, ref_at, what):
        r = host(t, np.uint16).reshape(REPS, PERIOD, -1)
        for i in range(1, REPS):
            assert np.array_equal(r[i], r[0]), f"{what}: repetition {i} differs from the first"
        first = oracle.bf16_bits_to_f64(oracle.blocked16_to_nchw(r[0].reshape(PERIOD, 4, h, w, 16), 64))
        idx = g.integers(0, first.size, size=256)
        ref = ref_at(idx)
        assert np.abs(first.reshape(-1)[idx] - ref).max() / max(np.abs(ref).max(), 1e-30) <= bound("bf16", "act"), what

    y = torch.empty(ng.ngc_data_elems(d, 1), dtype=torch.int16, device="cuda")
    ng.ngc_conv_fwd(d, xd, wd, bd, y, ws(d, ng.NGC_OP_FWD), stream())
    torch.cuda.synchronize()
    check_twins_and_samples(y, lambda idx: oracle.conv_fwd_at(a1, x1, wt, idx, bias=bias, relu=True), "fwd")
    del y
    d = mk(n)
    dx = torch.empty(ng.ngc_data_elems(d, 0), dtype=torch.int16, device="cuda")
    ng.ngc_conv_bwd_data(d, dyd, wd, dx, ws(d, ng.NGC_OP_BWD_DATA), stream())
    torch.cuda.synchronize()
    check_twins_and_samples(dx, lambda idx: oracle.conv_bwd_data_at(a1, dy1, wt, idx), "bwd_data")
    # the compound: ReLU backprop of the data input and the channel sums of the dx written (a pass over all of dx)
    db = torch.full((c,), float("nan"), dtype=torch.float32, device="cuda")
    ng.ngc_conv_bwd_data_relu_db(d, dyd, wd, xd, dx, db, ws(d, ng.NGC_OP_BWD_DATA_DB), stream())
    torch.cuda.synchronize()
    keep = (x1 > 0).reshape(-1)
    check_twins_and_samples(dx, lambda idx: oracle.conv_bwd_data_at(a1, dy1, wt, idx) * keep[idx], "bwd_data_relu")
    first = oracle.bf16_bits_to_f64(oracle.blocked16_to_nchw(host(dx, np.uint16).reshape(REPS, PERIOD, -1)[0].reshape(PERIOD, 4, h, w, 16), 64))
    want = REPS * oracle.bias_grad(first)
    assert np.abs(db.cpu().numpy() - want).max() / np.abs(want).max() <= 1e-5
    del dx
    # backprop-filters sums over the batch: 17 repetitions = 17 x the 4-image node
    dw = torch.empty(k * c * 9, dtype=torch.float32, device="cuda")
    ng.ngc_conv_bwd_filters(d, xd, dyd, dw, ws(d, ng.NGC_OP_BWD_FILTERS), stream())
    torch.cuda.synchronize()
    idx = g.integers(0, k * c * 9, size=64)
    ref = REPS * oracle.conv_bwd_filters_at(a1, x1, dy1, idx)
    got = dw.cpu().numpy().astype(np.float64)[idx]
    assert np.abs(got - ref).max() / np.abs(ref).max() <= bound("bf16", "dw")


@pytest.mark.timeout(600)
def test_rank3_ops_on_tensors_past_two_gib():
    from oracle import Attrs3
    n, c, dd, h, w, k = PERIOD * REPS, 64, 4, 250, 250, 64
    a1 = Attrs3(PERIOD, c, dd, h, w, k, 3, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1)
    print("case 68 x 64 x 4 x 250 x 250, 3x3x3", flush=True)
    x1 = synth_inputs.bf16_bits_to_f32(_bits(synth_inputs.normal(78, 0, (PERIOD, c, dd, h, w), 0.0, 1.0)))
    dy1 = synth_inputs.bf16_bits_to_f32(_bits(synth_inputs.normal(78, 3, (PERIOD, k, dd, h, w), 0.0, 0.1)))
    wt = synth_inputs.bf16_bits_to_f32(_bits(synth_inputs.normal(78, 1, (k, c, 3, 3, 3), 0.0, (2.0 / (c * 27)) ** 0.5)))
    blk = lambda v: oracle.nchw_to_blocked16(_bits(v).reshape(PERIOD, -1, dd * h, w))          # (d, h, w) stay contiguous
    xd = dev(np.tile(blk(x1), (REPS, 1, 1, 1, 1)))
    dyd = dev(np.tile(blk(dy1), (REPS, 1, 1, 1, 1)))
    assert xd.numel() * 2 > (1 << 31)
    wd = dev(_bits(wt))
    d = ng.make_desc3(n, c, dd, h, w, k, 3, 3, 3, pad_below=(1, 1, 1), pad_above=(1, 1, 1))
    names = [ng.ngc_conv3d_variant(d, op) for op in (ng.NGC_OP_FWD, ng.NGC_OP_BWD_DATA, ng.NGC_OP_BWD_FILTERS)]
    print("variants", names, flush=True)
    assert names == ["sliced:strip3_bf16", "sliced:strip3_bf16", "sliced:wgrad_gemm3_bf16"], names
    ws = lambda op: torch.empty(max(ng.ngc_conv3d_workspace_bytes(d, op), 16), dtype=torch.uint8, device="cuda")
    g = np.random.default_rng(6)

    def check_twins_and_samples(t, ref_at, what):
        r = host(t, np.uint16).reshape(REPS, PERIOD, -1)
        for i in range(1, REPS):
            assert np.array_equal(r[i], r[0]), f"{what}: repetition {i} differs from the first"
        first = oracle.bf16_bits_to_f64(oracle.blocked16_to_nchw(r[0].reshape(PERIOD, 4, dd * h, w, 16), 64))
        idx = g.integers(0, first.size, size=128)
        ref = ref_at(idx)
        assert np.abs(first.reshape(-1)[idx] - ref).max() / max(np.abs(ref).max(), 1e-30) <= bound("bf16", "act"), what

    y = torch.empty(ng.ngc_conv3d_data_elems(d, 1), dtype=torch.int16, device="cuda")
    ng.ngc_conv3d_fwd(d, xd, wd, None, y, ws(ng.NGC_OP_FWD), stream())
    torch.cuda.synchronize()
    check_twins_and_samples(y, lambda idx: oracle.conv3d_fwd_at(a1, x1, wt, idx), "fwd")
    del y
    dx = torch.empty(ng.ngc_conv3d_data_elems(d, 0), dtype=torch.int16, device="cuda")
    ng.ngc_conv3d_bwd_data(d, dyd, wd, dx, ws(ng.NGC_OP_BWD_DATA), stream())
    torch.cuda.synchronize()
    check_twins_and_samples(dx, lambda idx: oracle.conv3d_bwd_data_at(a1, dy1, wt, idx), "bwd_data")
    del dx
    dw = torch.empty(k * c * 27, dtype=torch.float32, device="cuda")
    ng.ngc_conv3d_bwd_filters(d, xd, dyd, dw, ws(ng.NGC_OP_BWD_FILTERS), stream())
    torch.cuda.synchronize()
    idx = g.integers(0, k * c * 27, size=32)
    ref = REPS * oracle.conv3d_bwd_filters_at(a1, x1, dy1, idx)
    assert np.abs(dw.cpu().numpy().astype(np.float64)[idx] - ref).max() / np.abs(ref).max() <= bound("bf16", "dw")
