"""bf16 nodes with NCHW tensors outside what the kernels read in place: several taps, strides, images whose H*W is
not a multiple of 8.  The library runs them on blocked copies in the workspace (paper Sec. 2 / Sec. 4: the layout is
the backend's choice, the conversion at the boundary its job); every op and compound is compared with the oracle on
the caller's NCHW tensors, and the kernel named must be the blocked node's, not the one-thread-per-output kernel."""
import numpy as np
import pytest
import torch

import paper_1801_08058_amd as ng
from oracle import Attrs
from gpu_util import Run, data_to_device, dev, encode, out_tensor, stream
from test_gpu_parity import _check_all, _tensors

pytestmark = pytest.mark.gpu
NCHW, BLK = ng.NGC_NCHW, ng.NGC_NCHW16C

STAGED_CASES = [
    # attrs                                                         fwd / bwd_data / bwd_filters kernel of the blocked node
    (Attrs(2, 64, 14, 14, 64, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1), ("strip", "strip", "wgrad_strip")),
    (Attrs(3, 32, 9, 11, 48, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1), ("strip", "strip", "wgrad")),          # ragged image, channel tails
    (Attrs(2, 64, 7, 7, 128, 1, 1, 1, 1, 1, 1, 0, 0, 0, 0), ("gemm1x1", "gemm1x1", "wgrad_gemm")),  # 49 positions per image
    (Attrs(2, 64, 8, 8, 64, 1, 1, 2, 2, 1, 1, 0, 0, 0, 0), ("gemm1x1", "gemm1x1", "wgrad")),        # 1x1 stride 2
    (Attrs(2, 64, 13, 13, 64, 3, 3, 2, 2, 1, 1, 1, 1, 1, 1), ("strip", "strip", "wgrad")),          # 3x3 stride 2
    (Attrs(2, 32, 10, 10, 64, 5, 5, 1, 1, 2, 2, 4, 4, 4, 4), ("", "", "")),                         # 5x5 dilation 2
]


@pytest.mark.parametrize("case", range(len(STAGED_CASES)))
@pytest.mark.parametrize("xl,yl", [(NCHW, NCHW), (NCHW, BLK), (BLK, NCHW)])
@pytest.mark.parametrize("pre", [False, True])
def test_nchw_nodes_run_on_blocked_copies(case, xl, yl, pre):
    a, kernels = STAGED_CASES[case]
    _check_all(a, "bf16", xl, yl, pre, 9100 + case, tuple("staged:" + k for k in kernels))


def test_staged_equals_blocked_node_bit_for_bit():
    """The copies change the layout only: the NCHW node's results are the blocked node's, element for element."""
    a = Attrs(2, 64, 14, 14, 64, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1)
    x, w, b, dy = _tensors(a, "bf16", 9200)
    rn, rb = Run(a, "bf16", NCHW, NCHW, False), Run(a, "bf16", BLK, BLK, False)
    assert np.array_equal(rn.fwd(x, w, bias=b, relu=True), rb.fwd(x, w, bias=b, relu=True))
    assert np.array_equal(rn.bwd_data(dy, w), rb.bwd_data(dy, w))
    assert np.array_equal(rn.bwd_filters(x, dy), rb.bwd_filters(x, dy))
    dxn, dbn = rn.bwd_data_relu_db(dy, w, x)
    dxb, dbb = rb.bwd_data_relu_db(dy, w, x)
    assert np.array_equal(dxn, dxb) and np.array_equal(dbn, dbb)


def test_first_layer_with_nchw_result():
    """Low-channel 7x7 stride-2 layer, x and y both NCHW: only y / dy get a copy, the kernels read the NCHW x."""
    a = Attrs(2, 3, 32, 32, 64, 7, 7, 2, 2, 1, 1, 3, 3, 3, 3)
    _check_all(a, "bf16", NCHW, NCHW, False, 9300, ("staged:stem_fwd", "staged:stem_bwd", "staged:wgrad_stem"))


def test_switch_restores_the_direct_kernels(monkeypatch):
    monkeypatch.setenv("NGC_STAGED", "0")
    a = Attrs(2, 64, 7, 7, 64, 1, 1, 1, 1, 1, 1, 0, 0, 0, 0)
    _check_all(a, "bf16", NCHW, BLK, False, 9400, ("direct", "direct", "direct"))


def test_too_small_workspace_is_refused():
    a = Attrs(2, 64, 14, 14, 64, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1)
    x, w, b, dy = _tensors(a, "bf16", 9500)
    run = Run(a, "bf16", NCHW, NCHW, False)
    run.fwd(x, w)
    d = run.last_desc
    need = ng.ngc_conv_workspace_bytes(d, ng.NGC_OP_FWD)
    assert need >= 2 * 2 * 64 * 14 * 14 * 2
    xd = data_to_device(x, "bf16", NCHW)
    wd = dev(encode(w, "bf16"))
    y = out_tensor(d, 1, "bf16")
    ws = torch.empty(need - 256, dtype=torch.uint8, device="cuda")
    assert ng.ngc_conv_fwd(d, xd, wd, None, y, ws, stream(), check=False) == ng.NGC_WORKSPACE_TOO_SMALL
    assert ng.ngc_conv_fwd(d, xd, wd, None, y, None, stream(), check=False) == ng.NGC_WORKSPACE_TOO_SMALL
