"""ngc_conv_bwd_data_filters: both derivative ops of a 1x1 stride-1 node in one pass over dy, against the oracle's
two adjoints and against the library's separate entry points."""
import numpy as np
import pytest
import torch

import oracle
import paper_1801_08058_amd as ng
import synth_inputs
from oracle import Attrs
from gpu_util import Run, bound, desc_of

pytestmark = pytest.mark.gpu
BLK = ng.NGC_NCHW16C


def _attrs(n, c, hw, k, w=None):
    return Attrs(n, c, hw, w or hw, k, 1, 1, 1, 1, 1, 1, 0, 0, 0, 0)


def _tensors(a, seed):
    rt = lambda t: synth_inputs.bf16_bits_to_f32(synth_inputs.f32_to_bf16_bits(t))
    x = rt(synth_inputs.normal(seed, 0, (a.n, a.c, a.h, a.w), 0.0, 1.0))
    w = rt(synth_inputs.normal(seed, 1, (a.k, a.c, 1, 1), 0.0, (2.0 / a.c) ** 0.5))
    dy = rt(synth_inputs.normal(seed, 3, (a.n, a.k, a.h, a.w), 0.0, 0.1))
    return x, w, dy


# (n, c, hw, k[, w]): stages of 64 positions that end inside an image (7x7, 9x5), straddle images, cover several
# channel tiles, every K the kernel is built for, one stage per workgroup and many, a ragged last stage
CASES = [(3, 64, 7, 64), (2, 64, 8, 128), (5, 128, 7, 256), (1, 64, 56, 256), (4, 192, 14, 128), (3, 64, 9, 64, 5),
         (2, 256, 28, 64), (64, 64, 3, 256), (1, 64, 1, 64), (3, 128, 7, 512), (2, 64, 28, 512)]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "n%dc%dhw%dk%d" % c[:4])
def test_fused_backward_matches_the_oracle(case):
    a = _attrs(*case)
    print(f"case {a}", flush=True)
    x, w, dy = _tensors(a, 91)
    run = Run(a, "bf16", BLK, BLK, True)
    assert ng.ngc_conv_variant(desc_of(a, "bf16", BLK, BLK, ng.NGC_BLOCKED_BWD), ng.NGC_OP_BWD_DATA_FILTERS) == "bwd1x1_fused_bf16"
    dx, dw = run.bwd_data_filters(x, dy, w)
    e = oracle.max_normalised_error(dx, oracle.conv_bwd_data(a, dy, w))
    assert e <= bound("bf16", "act"), f"dx err {e}"
    e = oracle.max_normalised_error(dw, oracle.conv_bwd_filters(a, x, dy))
    assert e <= bound("bf16", "dw"), f"dw err {e}"
    # the ReLU backprop of the node's input compounded into the store: the same dx where x > 0, +0 elsewhere; dw unchanged
    raw_dw = run.last_raw[1].clone()
    dxr, dwr = run.bwd_data_filters(x, dy, w, relu=True)
    keep = x > 0
    assert np.array_equal(dxr[keep], dx[keep]) and not dxr[~keep].any() and not np.signbit(dxr[~keep]).any()
    assert torch.equal(raw_dw.view(torch.int32), run.last_raw[1].view(torch.int32))


def test_fused_backward_is_run_to_run_identical_and_agrees_with_the_separate_ops():
    a = _attrs(6, 128, 14, 256)
    x, w, dy = _tensors(a, 17)
    run = Run(a, "bf16", BLK, BLK, True)
    dx, dw = run.bwd_data_filters(x, dy, w)
    raw1 = tuple(t.clone() for t in run.last_raw)
    run.bwd_data_filters(x, dy, w)
    assert torch.equal(raw1[0], run.last_raw[0]) and torch.equal(raw1[1].view(torch.int32), run.last_raw[1].view(torch.int32))
    # dx: same fp32 sums over k up to their order, one rounding to bf16 each: at most one bf16 ulp apart
    dx_sep = run.bwd_data(dy, w)
    assert oracle.max_normalised_error(dx, dx_sep) <= 2.0 ** -7
    assert oracle.max_normalised_error(dw, run.bwd_filters(x, dy)) <= 1e-5


def test_fused_backward_refuses_what_it_is_not_built_for():
    for a, wl in ((Attrs(2, 64, 8, 8, 64, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1), ng.NGC_BLOCKED_BWD),      # 3x3
                  (Attrs(2, 64, 8, 8, 64, 1, 1, 2, 2, 1, 1, 0, 0, 0, 0), ng.NGC_BLOCKED_BWD),      # stride 2
                  (_attrs(2, 64, 8, 1024), ng.NGC_BLOCKED_BWD),                                    # K beyond the kernel
                  (_attrs(2, 48, 8, 64), ng.NGC_BLOCKED_BWD),                                      # C not a multiple of 64
                  (_attrs(2, 64, 8, 64), ng.NGC_KCRS)):                                            # filters not in the backprop-data layout
        d = desc_of(a, "bf16", BLK, BLK, wl)
        assert ng.ngc_conv_variant(d, ng.NGC_OP_BWD_DATA_FILTERS) == "unsupported"
        assert ng.ngc_conv_workspace_bytes(d, ng.NGC_OP_BWD_DATA_FILTERS) == 0
        t = torch.zeros(1 << 20, dtype=torch.int16, device="cuda")
        f = torch.zeros(1 << 20, dtype=torch.float32, device="cuda")
        assert ng.ngc_conv_bwd_data_filters(d, t, t, t, t, f, t, torch.cuda.current_stream().cuda_stream, check=False) == ng.NGC_UNSUPPORTED
    d = desc_of(_attrs(2, 64, 8, 64), "bf16", BLK, BLK, ng.NGC_BLOCKED_BWD)
    t = torch.zeros(1 << 20, dtype=torch.int16, device="cuda")
    f = torch.zeros(1 << 20, dtype=torch.float32, device="cuda")
    assert ng.ngc_conv_bwd_data_filters(d, t, t, t, t, f, None, torch.cuda.current_stream().cuda_stream, check=False) == ng.NGC_WORKSPACE_TOO_SMALL
