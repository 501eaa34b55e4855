"""The library under HIP graph capture: it allocates nothing, never synchronises and clears memory with
kernels, so a training-step-shaped sequence of its calls can be captured once and replayed.  A two-layer
chain (3x3 with bias + ReLU -> strided 3x3; forward, then the compounded backward ops and both filter
gradients) is run eagerly, captured on a side stream, and replayed three times on fresh inputs with eager
work and synchronisations between the replays; every replay must reproduce the eager tensors bit for bit
(results are run-to-run identical by construction)."""
import numpy as np
import pytest
import torch

import paper_1801_08058_amd as ng
import synth_inputs
from gpu_util import dev

pytestmark = pytest.mark.gpu
BLK = ng.NGC_NCHW16C


def _bits(seed, tid, shape, std):
    return synth_inputs.f32_to_bf16_bits(synth_inputs.normal(seed, tid, shape, 0.0, std))


def test_captured_step_replays_bit_exact():
    n, c, hw, k1, k2 = 4, 64, 28, 128, 64
    mk = ng.make_desc
    l1 = dict(n=n, c=c, h=hw, w=hw, k=k1, r=3, s=3, pad_below=(1, 1), pad_above=(1, 1))
    l2 = dict(n=n, c=k1, h=hw, w=hw, k=k2, r=3, s=3, stride=(2, 2), pad_below=(1, 1), pad_above=(1, 1))
    d1f = mk(**l1, w_layout=ng.NGC_BLOCKED_FWD, epilogue=ng.NGC_EPI_BIAS | ng.NGC_EPI_RELU)
    d1b, d1w = mk(**l1, w_layout=ng.NGC_BLOCKED_BWD), mk(**l1)
    d2f = mk(**l2, w_layout=ng.NGC_BLOCKED_FWD, epilogue=ng.NGC_EPI_BIAS | ng.NGC_EPI_RELU)
    d2b, d2w = mk(**l2, w_layout=ng.NGC_BLOCKED_BWD), mk(**l2)
    P2, Q2 = ng.ngc_conv_out_shape(d2f)
    i16 = lambda nelem: torch.empty(nelem, dtype=torch.int16, device="cuda")
    f32 = lambda nelem: torch.empty(nelem, dtype=torch.float32, device="cuda")
    # static buffers of the graph
    x = i16(ng.ngc_data_elems(d1f, 0)); y1 = i16(ng.ngc_data_elems(d1f, 1)); y2 = i16(ng.ngc_data_elems(d2f, 1))
    dy2 = i16(ng.ngc_data_elems(d2f, 1)); dy1 = i16(ng.ngc_data_elems(d2f, 0)); dx = i16(ng.ngc_data_elems(d1f, 0))
    w1k, w2k = dev(_bits(1, 1, (k1, c, 3, 3), 0.06)), dev(_bits(2, 1, (k2, k1, 3, 3), 0.04))
    w1f, w1b = i16(ng.ngc_filter_elems(d1f, ng.NGC_BLOCKED_FWD)), i16(ng.ngc_filter_elems(d1f, ng.NGC_BLOCKED_BWD))
    w2f, w2b = i16(ng.ngc_filter_elems(d2f, ng.NGC_BLOCKED_FWD)), i16(ng.ngc_filter_elems(d2f, ng.NGC_BLOCKED_BWD))
    b1, b2 = dev(np.linspace(-0.1, 0.1, k1, dtype=np.float32)), dev(np.linspace(0.1, -0.1, k2, dtype=np.float32))
    dw1, dw2, db1, db2 = f32(k1 * c * 9), f32(k2 * k1 * 9), f32(k1), f32(k2)
    ops = ((d1f, ng.NGC_OP_FWD), (d2f, ng.NGC_OP_FWD), (d2b, ng.NGC_OP_BWD_DATA_DB), (d1b, ng.NGC_OP_BWD_DATA),
           (d1w, ng.NGC_OP_BWD_FILTERS), (d2w, ng.NGC_OP_BWD_FILTERS), (d2w, ng.NGC_OP_BIAS_GRAD))
    ws = [torch.empty(max(ng.ngc_conv_workspace_bytes(d, op), 16), dtype=torch.uint8, device="cuda") for d, op in ops]

    def step(st):
        # weights change every step in training: their re-layout is part of the captured step
        ng.ngc_filter_convert(d1f, w1k, w1f, ng.NGC_BLOCKED_FWD, st); ng.ngc_filter_convert(d1f, w1k, w1b, ng.NGC_BLOCKED_BWD, st)
        ng.ngc_filter_convert(d2f, w2k, w2f, ng.NGC_BLOCKED_FWD, st); ng.ngc_filter_convert(d2f, w2k, w2b, ng.NGC_BLOCKED_BWD, st)
        ng.ngc_conv_fwd(d1f, x, w1f, b1, y1, ws[0], st)
        ng.ngc_conv_fwd(d2f, y1, w2f, b2, y2, ws[1], st)
        # backward: dy2 is given; layer 2 backprop-data with the ReLU mask of y1 and the bias gradient of layer 1
        # (a strided layer: zero fill + one launch per residue class), then layer 1
        ng.ngc_conv_bwd_data_relu_db(d2b, dy2, w2b, y1, dy1, db1, ws[2], st)
        ng.ngc_conv_bwd_data(d1b, dy1, w1b, dx, ws[3], st)
        ng.ngc_conv_bwd_filters(d1w, x, dy1, dw1, ws[4], st)
        ng.ngc_conv_bwd_filters(d2w, y1, dy2, dw2, ws[5], st)
        ng.ngc_bias_grad(d2w, dy2, db2, ws[6], st)

    outs = (y1, y2, dy1, dx, dw1, dw2, db1, db2)

    def load_inputs(i):
        x.copy_(dev(_bits(100 + i, 0, (x.numel(),), 1.0)))
        dy2.copy_(dev(_bits(100 + i, 3, (dy2.numel(),), 0.1)))

    def poison():
        for t in outs:
            t.fill_(float("nan")) if t.dtype == torch.float32 else t.fill_(0x7FC0)

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        load_inputs(0)
        step(side.cuda_stream)                     # eager warm-up: one-time kernel attributes are set outside capture
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step(torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()

    for i in (1, 2, 3):
        load_inputs(i)
        poison()
        torch.cuda.synchronize()
        step(torch.cuda.current_stream().cuda_stream)          # eager reference on the same buffers
        torch.cuda.synchronize()
        eager = [t.clone() for t in outs]
        assert all(torch.isfinite(t).all() for t in eager if t.dtype == torch.float32)
        poison()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, a, b in zip(("y1", "y2", "dy1", "dx", "dw1", "dw2", "db1", "db2"), eager, outs):
            assert torch.equal(a, b), f"replay {i}: {name} differs from the eager run"
