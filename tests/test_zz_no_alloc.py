"""ngc_conv_bwd_filters_noalloc: the entry point for callers that cannot allocate (its split-reduction partials live
in a static device array of the library).  Checked through the C ABI against ngc_conv_bwd_filters with a caller
workspace - same kernels, fixed-order reduction, so bit for bit - and against the oracle, on two calls in a row,
the second with a smaller input (the array keeps the first call's contents)."""
import numpy as np
import pytest
import torch

import oracle
import paper_1801_08058_amd as ng
from oracle import Attrs
from gpu_util import Run, bound, data_to_device, desc_of, stream, workspace

pytestmark = pytest.mark.gpu
BLK = ng.NGC_NCHW16C


def _tensors(a, seed):
    import synth_inputs
    P, Q = oracle.out_shape(a)
    rt = lambda t: synth_inputs.bf16_bits_to_f32(synth_inputs.f32_to_bf16_bits(t))
    x = rt(synth_inputs.normal(seed, 0, (a.n, a.c, a.h, a.w), 0.0, 1.0))
    dy = rt(synth_inputs.normal(seed, 3, (a.n, a.k, P, Q), 0.0, 0.1))
    return x, dy


def _both(a, seed):
    x, dy = _tensors(a, seed)
    d = desc_of(a, "bf16", BLK, BLK)
    need = ng.ngc_conv_workspace_bytes(d, ng.NGC_OP_BWD_FILTERS)
    assert 0 < need <= ng.ngc_static_scratch_bytes(), need
    xd, dyd = data_to_device(x, "bf16", BLK), data_to_device(dy, "bf16", BLK)
    n = a.k * a.c * a.r * a.s
    dw_ws = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    dw_na = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    print(f"noalloc case {a} variant {ng.ngc_conv_variant(d, ng.NGC_OP_BWD_FILTERS)} scratch {need}", flush=True)
    ng.ngc_conv_bwd_filters_noalloc(d, xd, dyd, dw_na, stream())
    ng.ngc_conv_bwd_filters(d, xd, dyd, dw_ws, workspace(d, ng.NGC_OP_BWD_FILTERS), stream())
    torch.cuda.synchronize()
    assert torch.equal(dw_na.view(torch.int32), dw_ws.view(torch.int32)), "differs from the workspace entry point"
    got = dw_na.cpu().numpy().astype(np.float64).reshape(a.k, a.c, a.r, a.s)
    e = oracle.max_normalised_error(got, oracle.conv_bwd_filters(a, x, dy))
    assert e <= bound("bf16", "dw"), e


def test_noalloc_backprop_filters_two_calls_second_smaller():
    # 3x3 stride 1 (all-taps kernel), then a smaller node of the same kind, then a 1x1 and a strided 3x3 (per-tap GEMM)
    _both(Attrs(6, 64, 28, 28, 64, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1), 31001)
    _both(Attrs(2, 64, 14, 14, 64, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1), 31002)
    _both(Attrs(4, 128, 14, 14, 64, 1, 1, 1, 1, 1, 1, 0, 0, 0, 0), 31003)
    _both(Attrs(3, 32, 15, 15, 48, 3, 3, 2, 2, 1, 1, 1, 1, 1, 1), 31004)


def test_noalloc_refuses_nodes_beyond_the_static_array():
    d = ng.make_desc(128, 512, 56, 56, 512, 3, 3, pad_below=(1, 1), pad_above=(1, 1))
    assert ng.ngc_conv_workspace_bytes(d, ng.NGC_OP_BWD_FILTERS) > ng.ngc_static_scratch_bytes()
    one = torch.zeros(16, dtype=torch.int16, device="cuda")        # never read: the size check comes first
    rc = ng.ngc_conv_bwd_filters_noalloc(d, one, one, one, stream(), check=False)
    assert rc == ng.NGC_SCRATCH_EXCEEDED
    assert "static" in ng.ngc_status_string(rc)
