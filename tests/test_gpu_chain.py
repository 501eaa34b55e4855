"""A residual-bottleneck-shaped chain (1x1 -> 3x3 -> 1x1, each with the compounded bias + ReLU) run forward
and backward through the C ABI the way a graph executor would: tensors stay on the device in the layouts
the ops produce, the first layer reads the NCHW input and writes its gradient in NCHW (layout propagation),
the backward pass uses the compounded backward ops (ReLU backprop in the backprop-data epilogue, bias
gradient of the producing layer from the same call).  Every stage is checked against the oracle applied to
the tensors the device actually fed it."""
import numpy as np
import pytest
import torch

import oracle
import paper_1801_08058_amd as ng
import synth_inputs
from oracle import Attrs
from gpu_util import bound, data_from_device, data_to_device, desc_of, dev, encode, filter_blocked_host, stream, workspace

pytestmark = pytest.mark.gpu
NCHW, BLK = ng.NGC_NCHW, ng.NGC_NCHW16C


def _bf16(t):
    return synth_inputs.bf16_bits_to_f32(synth_inputs.f32_to_bf16_bits(t))


@pytest.mark.parametrize("n,hw,c0,c1,c3", [(2, 12, 64, 32, 128), (3, 8, 128, 48, 80)])
def test_bottleneck_chain_forward_backward(n, hw, c0, c1, c3):
    layers = [  # attrs, x layout, y layout
        (Attrs(n, c0, hw, hw, c1, 1, 1, 1, 1, 1, 1, 0, 0, 0, 0), NCHW, BLK),
        (Attrs(n, c1, hw, hw, c1, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1), BLK, BLK),
        (Attrs(n, c1, hw, hw, c3, 1, 1, 1, 1, 1, 1, 0, 0, 0, 0), BLK, BLK),
    ]
    seed = 5150 + hw
    x0 = _bf16(synth_inputs.normal(seed, 0, (n, c0, hw, hw), 0.0, 1.0))
    ws_, bs_ = [], []
    for i, (a, _, _) in enumerate(layers):
        ws_.append(_bf16(synth_inputs.normal(seed, 10 + i, (a.k, a.c, a.r, a.s), 0.0, (2.0 / (a.c * a.r * a.s)) ** 0.5)))
        bs_.append(synth_inputs.uniform(seed, 20 + i, (a.k,), -0.1, 0.1))
    d3 = _bf16(synth_inputs.normal(seed, 3, (n, c3, hw, hw), 0.0, 0.1))        # delta at the last pre-activation
    st = stream()
    tol, tol_dw = bound("bf16", "act"), bound("bf16", "dw")

    # ---- forward: device tensors chained, each output checked against the oracle on the device's own input
    acts_dev = [data_to_device(x0, "bf16", NCHW)]
    acts_host = [x0.astype(np.float64)]
    wf, wb, descs = [], [], []
    for i, (a, xl, yl) in enumerate(layers):
        d_f = desc_of(a, "bf16", xl, yl, ng.NGC_BLOCKED_FWD, ng.NGC_EPI_BIAS | ng.NGC_EPI_RELU)
        wbits = encode(ws_[i], "bf16")
        wf.append(dev(filter_blocked_host(wbits, ng.NGC_BLOCKED_FWD)))
        wb.append(dev(filter_blocked_host(wbits, ng.NGC_BLOCKED_BWD)))
        descs.append((d_f, desc_of(a, "bf16", xl, yl, ng.NGC_BLOCKED_BWD), desc_of(a, "bf16", xl, yl)))
        assert ng.ngc_conv_variant(d_f, ng.NGC_OP_FWD) in ("gemm1x1_bf16", "strip_bf16", "strip_rows_bf16")
        y = torch.empty(ng.ngc_data_elems(d_f, 1), dtype=torch.int16, device="cuda")
        ng.ngc_conv_fwd(d_f, acts_dev[-1], wf[i], dev(np.asarray(bs_[i], dtype=np.float32)), y, workspace(d_f, ng.NGC_OP_FWD), st)
        torch.cuda.synchronize()
        yh = data_from_device(y, "bf16", yl, (a.n, a.k, hw, hw))
        ref = oracle.conv_fwd(a, acts_host[-1], ws_[i], bias=bs_[i], relu=True)
        assert oracle.max_normalised_error(yh, ref) <= tol, f"forward layer {i}"
        acts_dev.append(y)
        acts_host.append(yh)

    # ---- backward: delta tensors chained on the device
    delta_dev = data_to_device(d3, "bf16", BLK)
    delta_host = d3.astype(np.float64)
    for i in (2, 1, 0):
        a, xl, yl = layers[i]
        d_f, d_b, d_w = descs[i]
        x_dev, x_host = acts_dev[i], acts_host[i]
        dw = torch.empty(a.k * a.c * a.r * a.s, dtype=torch.float32, device="cuda")
        ng.ngc_conv_bwd_filters(d_w, x_dev, delta_dev, dw, workspace(d_w, ng.NGC_OP_BWD_FILTERS), st)
        db = torch.empty(a.k, dtype=torch.float32, device="cuda")
        ng.ngc_bias_grad(d_w, delta_dev, db, workspace(d_w, ng.NGC_OP_BIAS_GRAD), st)
        dx = torch.empty(ng.ngc_data_elems(d_b, 0), dtype=torch.int16, device="cuda")
        if i > 0:   # the data input is a ReLU output: mask fused, plus the bias gradient of the layer below
            db_below = torch.empty(a.c, dtype=torch.float32, device="cuda")
            ng.ngc_conv_bwd_data_relu_db(d_b, delta_dev, wb[i], x_dev, dx, db_below, workspace(d_b, ng.NGC_OP_BWD_DATA_DB), st)
        else:       # the network input: plain backprop-data, written in NCHW
            ng.ngc_conv_bwd_data(d_b, delta_dev, wb[i], dx, workspace(d_b, ng.NGC_OP_BWD_DATA), st)
        torch.cuda.synchronize()
        dwh = dw.cpu().numpy().astype(np.float64).reshape(a.k, a.c, a.r, a.s)
        assert oracle.max_normalised_error(dwh, oracle.conv_bwd_filters(a, x_host, delta_host)) <= tol_dw, f"dw layer {i}"
        assert oracle.max_normalised_error(db.cpu().numpy().astype(np.float64), oracle.bias_grad(delta_host)) <= 1e-5, f"db layer {i}"
        dxh = data_from_device(dx, "bf16", xl, (a.n, a.c, hw, hw))
        if i > 0:
            ref = oracle.conv_bwd_data_relu(a, delta_host, ws_[i], x_host)
            assert oracle.max_normalised_error(dxh, ref) <= tol, f"dx layer {i}"
            assert not dxh[~(x_host > 0)].any()
            # the fused bias gradient of the layer below equals the separate op on the delta that layer receives
            got = db_below.cpu().numpy().astype(np.float64)
            assert oracle.max_normalised_error(got, oracle.bias_grad(dxh)) <= 1e-5, f"fused db below layer {i}"
        else:
            assert oracle.max_normalised_error(dxh, oracle.conv_bwd_data(a, delta_host, ws_[i])) <= tol, "dx of the input"
        delta_dev, delta_host = dx, dxh
