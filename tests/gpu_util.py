"""Helpers for the GPU parity tests: move seeded host tensors to the device in the layouts
the C ABI takes, run the HIP path, bring results back as fp64 in logical axis order.
The host-side layout permutations used to *prepare inputs and read outputs* are the
oracle's (pinned in test_oracle_pins.py); the device conversion kernels are tested
separately against them."""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_1801_08058_amd as ng
import synth_inputs
from synth_inputs import ConvLayer

TOL = {"f32": 1e-5, "bf16": 2e-2}          # the contract: max normalised error per element type of the data

# Bounds that follow from the arithmetic of the bf16 path; every parity assert uses these (they imply the contract's).
#   y, dx: the fp32 accumulator (exact bf16 products, fp32 sums: relative error ~1e-6) is rounded once to bf16, whose
#          half ulp is at most 2^-8 of the value, hence of max|ref|.  A dropped (c, r, s) term or a truncating
#          conversion (error up to 2^-7) lands above it.
#   dw:    fp32 from exact products with fp32 accumulation over N*P*Q terms in a fixed tree; observed 1e-7..5e-6 of
#          max|dw|.  A dropped 32-position step, row or image tail moves dw by 1e-3..1e-2 of its maximum.
BOUND_BF16 = {"act": 2.0 ** -8 * 1.01, "dw": 1e-4}


def bound(dtype: str, kind: str) -> float:
    """Largest max-normalised error accepted for an output of `kind` ("act": y / dx in the element type, "dw": the
    fp32 filter gradient) computed from `dtype` data."""
    b = TOL["f32"] if dtype == "f32" else BOUND_BF16[kind]
    assert b <= TOL[dtype]
    return b


def attrs_of(L: ConvLayer) -> oracle.Attrs:
    return oracle.Attrs(*L.attrs15)


def desc_of(a: oracle.Attrs, dtype: str, x_layout, y_layout, w_layout=ng.NGC_KCRS, epilogue=ng.NGC_EPI_NONE):
    return ng.make_desc(a.n, a.c, a.h, a.w, a.k, a.r, a.s, (a.sh, a.sw), (a.dh, a.dw), (a.pbh, a.pbw),
                        (a.pah, a.paw), ng.NGC_F32 if dtype == "f32" else ng.NGC_BF16, x_layout, y_layout,
                        w_layout, epilogue)


def dev(arr: np.ndarray) -> torch.Tensor:
    a = np.ascontiguousarray(arr)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).cuda()


def host(t: torch.Tensor, as_dtype) -> np.ndarray:
    a = t.cpu().numpy()
    return a.view(as_dtype)


def encode(values_f32: np.ndarray, dtype: str) -> np.ndarray:
    """fp32 host values -> element container (fp32 itself, or bf16 bits; values of bf16
    configurations are already exactly representable)."""
    if dtype == "f32":
        return np.ascontiguousarray(values_f32, dtype=np.float32)
    return synth_inputs.f32_to_bf16_bits(values_f32)


def data_to_device(values_f32: np.ndarray, dtype: str, layout: int) -> torch.Tensor:
    e = encode(values_f32, dtype)
    if layout == ng.NGC_NCHW16C:
        e = oracle.nchw_to_blocked16(e)
    return dev(e)


def data_from_device(t: torch.Tensor, dtype: str, layout: int, shape) -> np.ndarray:
    """device tensor -> fp64 array in logical [N,C,H,W] order."""
    n, c, h, w = shape
    raw = host(t, np.float32 if dtype == "f32" else np.uint16)
    if layout == ng.NGC_NCHW16C:
        raw = raw.reshape(n, (c + 15) // 16, h, w, 16)
        raw = oracle.blocked16_to_nchw(raw, c)
    else:
        raw = raw.reshape(n, c, h, w)
    if dtype == "f32":
        return raw.astype(np.float64)
    return oracle.bf16_bits_to_f64(raw)


def filter_blocked_host(w_bits: np.ndarray, layout: int) -> np.ndarray:
    """Definition of the two blocked filter layouts, stated with numpy axis moves
    (header of include/ngconv.h): FWD [r][s][cb][k][ci], BWD [r][s][kb][c][ki]."""
    K, C, R, S = w_bits.shape
    if layout == ng.NGC_BLOCKED_FWD:
        CB = (C + 15) // 16
        pad = np.zeros((K, CB * 16, R, S), dtype=w_bits.dtype); pad[:, :C] = w_bits
        return np.ascontiguousarray(pad.reshape(K, CB, 16, R, S).transpose(3, 4, 1, 0, 2))
    KB = (K + 15) // 16
    pad = np.zeros((KB * 16, C, R, S), dtype=w_bits.dtype); pad[:K] = w_bits
    return np.ascontiguousarray(pad.reshape(KB, 16, C, R, S).transpose(3, 4, 0, 2, 1))


def workspace(desc, op) -> torch.Tensor | None:
    nbytes = ng.ngc_conv_workspace_bytes(desc, op)
    if nbytes == 0:
        return None
    return torch.empty(nbytes, dtype=torch.uint8, device="cuda")


def stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def out_tensor(desc, which: int, dtype: str, fill: float | None = None) -> torch.Tensor:
    n = ng.ngc_data_elems(desc, which)
    t = torch.empty(n, dtype=torch.float32 if dtype == "f32" else torch.int16, device="cuda")
    # poison so that unwritten elements are caught
    if dtype == "f32":
        t.fill_(float("nan"))
    else:
        t.fill_(0x7FC0)
    return t


class Run:
    """Runs the three ops of one layer through the C ABI and returns fp64 results."""

    def __init__(self, a: oracle.Attrs, dtype: str, x_layout: int, y_layout: int, pre_block_filters: bool):
        self.a, self.dtype, self.xl, self.yl, self.pre = a, dtype, x_layout, y_layout, pre_block_filters
        self.P, self.Q = oracle.out_shape(a)

    def _filter(self, w_f32, layout):
        """Filters pre-converted to the op's blocked layout when asked for and when a kernel
        takes them (the direct kernels take KCRS only), else KCRS."""
        wb = encode(w_f32, self.dtype)
        op = ng.NGC_OP_FWD if layout == ng.NGC_BLOCKED_FWD else ng.NGC_OP_BWD_DATA
        if self.pre and ng.ngc_conv_variant(desc_of(self.a, self.dtype, self.xl, self.yl, layout), op) != "unsupported":
            return dev(filter_blocked_host(wb, layout)), layout
        return dev(wb), ng.NGC_KCRS

    def fwd(self, x, w, bias=None, relu=False):
        a = self.a
        epi = (ng.NGC_EPI_BIAS if bias is not None else 0) | (ng.NGC_EPI_RELU if relu else 0)
        wd, wl = self._filter(w, ng.NGC_BLOCKED_FWD)
        d = desc_of(a, self.dtype, self.xl, self.yl, wl, epi)
        xd = data_to_device(x, self.dtype, self.xl)
        bd = dev(np.asarray(bias, dtype=np.float32)) if bias is not None else None
        y = out_tensor(d, 1, self.dtype)
        ws = workspace(d, ng.NGC_OP_FWD)
        ng.ngc_conv_fwd(d, xd, wd, bd, y, ws, stream())
        torch.cuda.synchronize()
        self.last_desc, self.last_raw = d, y
        return data_from_device(y, self.dtype, self.yl, (a.n, a.k, self.P, self.Q))

    def bwd_data(self, dy, w):
        a = self.a
        wd, wl = self._filter(w, ng.NGC_BLOCKED_BWD)
        d = desc_of(a, self.dtype, self.xl, self.yl, wl)
        dyd = data_to_device(dy, self.dtype, self.yl)
        dx = out_tensor(d, 0, self.dtype)
        ws = workspace(d, ng.NGC_OP_BWD_DATA)
        ng.ngc_conv_bwd_data(d, dyd, wd, dx, ws, stream())
        torch.cuda.synchronize()
        self.last_desc, self.last_raw = d, dx
        return data_from_device(dx, self.dtype, self.xl, (a.n, a.c, a.h, a.w))

    def bwd_data_filters(self, x, dy, w, relu=False):
        """Both derivative ops of the node in one call (blocked tensors, filters in the backprop-data layout):
        (dx, dw) as fp64, and the raw device tensors in self.last_raw."""
        a = self.a
        d = desc_of(a, self.dtype, self.xl, self.yl, ng.NGC_BLOCKED_BWD)
        wd = dev(filter_blocked_host(encode(w, self.dtype), ng.NGC_BLOCKED_BWD))
        xd = data_to_device(x, self.dtype, self.xl)
        dyd = data_to_device(dy, self.dtype, self.yl)
        dx = out_tensor(d, 0, self.dtype)
        dw = torch.full((a.k * a.c * a.r * a.s,), float("nan"), dtype=torch.float32, device="cuda")
        ws = workspace(d, ng.NGC_OP_BWD_DATA_FILTERS)
        (ng.ngc_conv_bwd_data_filters_relu if relu else ng.ngc_conv_bwd_data_filters)(d, xd, dyd, wd, dx, dw, ws, stream())
        torch.cuda.synchronize()
        self.last_desc, self.last_raw = d, (dx, dw)
        return (data_from_device(dx, self.dtype, self.xl, (a.n, a.c, a.h, a.w)),
                dw.cpu().numpy().astype(np.float64).reshape(a.k, a.c, a.r, a.s))

    def bwd_data_relu(self, dy, w, x_in):
        """ConvolutionBackpropData compounded with the backprop of the ReLU that produced x_in."""
        a = self.a
        wd, wl = self._filter(w, ng.NGC_BLOCKED_BWD)
        d = desc_of(a, self.dtype, self.xl, self.yl, wl)
        dyd = data_to_device(dy, self.dtype, self.yl)
        xin = data_to_device(x_in, self.dtype, self.xl)
        dx = out_tensor(d, 0, self.dtype)
        ws = workspace(d, ng.NGC_OP_BWD_DATA)
        ng.ngc_conv_bwd_data_relu(d, dyd, wd, xin, dx, ws, stream())
        torch.cuda.synchronize()
        self.last_desc, self.last_raw = d, dx
        return data_from_device(dx, self.dtype, self.xl, (a.n, a.c, a.h, a.w))

    def bwd_data_relu_db(self, dy, w, x_in):
        """The compound above that also returns the channel sums of the dx it wrote (fp32 [C])."""
        a = self.a
        wd, wl = self._filter(w, ng.NGC_BLOCKED_BWD)
        d = desc_of(a, self.dtype, self.xl, self.yl, wl)
        dyd = data_to_device(dy, self.dtype, self.yl)
        xin = data_to_device(x_in, self.dtype, self.xl)
        dx = out_tensor(d, 0, self.dtype)
        db = torch.full((a.c,), float("nan"), dtype=torch.float32, device="cuda")
        ws = workspace(d, ng.NGC_OP_BWD_DATA_DB)
        ng.ngc_conv_bwd_data_relu_db(d, dyd, wd, xin, dx, db, ws, stream())
        torch.cuda.synchronize()
        self.last_desc, self.last_raw = d, dx
        return data_from_device(dx, self.dtype, self.xl, (a.n, a.c, a.h, a.w)), db.cpu().numpy().astype(np.float64)

    def bias_grad(self, dy):
        a = self.a
        d = desc_of(a, self.dtype, self.xl, self.yl)
        dyd = data_to_device(dy, self.dtype, self.yl)
        db = torch.full((a.k,), float("nan"), dtype=torch.float32, device="cuda")
        ws = workspace(d, ng.NGC_OP_BIAS_GRAD)
        ng.ngc_bias_grad(d, dyd, db, ws, stream())
        torch.cuda.synchronize()
        self.last_desc, self.last_raw = d, db
        return db.cpu().numpy().astype(np.float64)

    def bwd_filters(self, x, dy):
        a = self.a
        d = desc_of(a, self.dtype, self.xl, self.yl)
        xd = data_to_device(x, self.dtype, self.xl)
        dyd = data_to_device(dy, self.dtype, self.yl)
        dw = torch.full((a.k * a.c * a.r * a.s,), float("nan"), dtype=torch.float32, device="cuda")
        ws = workspace(d, ng.NGC_OP_BWD_FILTERS)
        ng.ngc_conv_bwd_filters(d, xd, dyd, dw, ws, stream())
        torch.cuda.synchronize()
        self.last_desc, self.last_raw = d, dw
        return dw.cpu().numpy().astype(np.float64).reshape(a.k, a.c, a.r, a.s)


# ---------------------------------------------------------------- convolution over three spatial axes
def attrs3_of(L: synth_inputs.Conv3dLayer) -> oracle.Attrs3:
    return oracle.Attrs3(*L.attrs21)


def desc3_of(a: oracle.Attrs3, dtype: str, x_layout, y_layout, w_layout=ng.NGC_KCRS, epilogue=ng.NGC_EPI_NONE):
    return ng.make_desc3(a.n, a.c, a.d, a.h, a.w, a.k, a.t, a.r, a.s, (a.sd, a.sh, a.sw), (a.dd, a.dh, a.dw),
                         (a.pbd, a.pbh, a.pbw), (a.pad, a.pah, a.paw), ng.NGC_F32 if dtype == "f32" else ng.NGC_BF16,
                         x_layout, y_layout, w_layout, epilogue)


def data3_to_device(values_f32: np.ndarray, dtype: str, layout: int) -> torch.Tensor:
    """[N,C,D,H,W] host values -> device tensor in `layout`; both layouts keep (d, h, w) contiguous, so the
    rank-2 permutation with D*H rows is the rank-3 one."""
    n, c, d, h, w = values_f32.shape
    return data_to_device(values_f32.reshape(n, c, d * h, w), dtype, layout)


def data3_from_device(t: torch.Tensor, dtype: str, layout: int, shape) -> np.ndarray:
    n, c, d, h, w = shape
    return data_from_device(t, dtype, layout, (n, c, d * h, w)).reshape(n, c, d, h, w)


def poisoned(nelem: int, dtype: str) -> torch.Tensor:
    t = torch.empty(nelem, dtype=torch.float32 if dtype == "f32" else torch.int16, device="cuda")
    t.fill_(float("nan") if dtype == "f32" else 0x7FC0)
    return t


class Run3:
    """Runs the three ops of one rank-3 layer through the C ABI and returns fp64 results."""

    def __init__(self, a: oracle.Attrs3, dtype: str, x_layout: int, y_layout: int, pre_block_filters: bool = False):
        self.a, self.dtype, self.xl, self.yl, self.pre = a, dtype, x_layout, y_layout, pre_block_filters
        self.O, self.P, self.Q = oracle.out_shape3(a)

    def _ws(self, d, op):
        nbytes = ng.ngc_conv3d_workspace_bytes(d, op)
        return torch.empty(nbytes, dtype=torch.uint8, device="cuda") if nbytes else None

    def _filter(self, w_f32, layout):
        """Filters through ngc_conv3d_filter_convert when asked for and a kernel takes them, else [K][C][T][R][S]."""
        wd = dev(encode(w_f32, self.dtype))
        op = ng.NGC_OP_FWD if layout == ng.NGC_BLOCKED_FWD else ng.NGC_OP_BWD_DATA
        d = desc3_of(self.a, self.dtype, self.xl, self.yl, layout)
        if self.pre and self.dtype == "bf16" and "unsupported" not in ng.ngc_conv3d_variant(d, op):
            wb = torch.empty(ng.ngc_conv3d_filter_elems(d, layout), dtype=torch.int16, device="cuda")
            ng.ngc_conv3d_filter_convert(d, wd, wb, layout, stream())
            return wb, layout
        return wd, ng.NGC_KCRS

    def fwd(self, x, w, bias=None, relu=False):
        a = self.a
        epi = (ng.NGC_EPI_BIAS if bias is not None else 0) | (ng.NGC_EPI_RELU if relu else 0)
        wd, wl = self._filter(w, ng.NGC_BLOCKED_FWD)
        d = desc3_of(a, self.dtype, self.xl, self.yl, wl, epi)
        xd = data3_to_device(x, self.dtype, self.xl)
        bd = dev(np.asarray(bias, dtype=np.float32)) if bias is not None else None
        y = poisoned(ng.ngc_conv3d_data_elems(d, 1), self.dtype)
        ng.ngc_conv3d_fwd(d, xd, wd, bd, y, self._ws(d, ng.NGC_OP_FWD), stream())
        torch.cuda.synchronize()
        self.last_desc = d
        return data3_from_device(y, self.dtype, self.yl, (a.n, a.k, self.O, self.P, self.Q))

    def bwd_data(self, dy, w):
        a = self.a
        wd, wl = self._filter(w, ng.NGC_BLOCKED_BWD)
        d = desc3_of(a, self.dtype, self.xl, self.yl, wl)
        dyd = data3_to_device(dy, self.dtype, self.yl)
        dx = poisoned(ng.ngc_conv3d_data_elems(d, 0), self.dtype)
        ng.ngc_conv3d_bwd_data(d, dyd, wd, dx, self._ws(d, ng.NGC_OP_BWD_DATA), stream())
        torch.cuda.synchronize()
        self.last_desc = d
        return data3_from_device(dx, self.dtype, self.xl, (a.n, a.c, a.d, a.h, a.w))

    def bwd_filters(self, x, dy):
        a = self.a
        d = desc3_of(a, self.dtype, self.xl, self.yl)
        xd = data3_to_device(x, self.dtype, self.xl)
        dyd = data3_to_device(dy, self.dtype, self.yl)
        dw = torch.full((a.k * a.c * a.t * a.r * a.s,), float("nan"), dtype=torch.float32, device="cuda")
        ng.ngc_conv3d_bwd_filters(d, xd, dyd, dw, self._ws(d, ng.NGC_OP_BWD_FILTERS), stream())
        torch.cuda.synchronize()
        self.last_desc = d
        return dw.cpu().numpy().astype(np.float64).reshape(a.k, a.c, a.t, a.r, a.s)


def _run3_bwd_data_relu(self, dy, w, x_in, with_db=False):
    """ConvolutionBackpropData compounded with the backprop of the ReLU that produced x_in (and, with_db, the channel
    sums of the dx written)."""
    a = self.a
    wd, wl = self._filter(w, ng.NGC_BLOCKED_BWD)
    d = desc3_of(a, self.dtype, self.xl, self.yl, wl)
    dyd = data3_to_device(dy, self.dtype, self.yl)
    xin = data3_to_device(x_in, self.dtype, self.xl)
    dx = poisoned(ng.ngc_conv3d_data_elems(d, 0), self.dtype)
    self.last_desc = d
    if with_db:
        db = torch.full((a.c,), float("nan"), dtype=torch.float32, device="cuda")
        ng.ngc_conv3d_bwd_data_relu_db(d, dyd, wd, xin, dx, db, self._ws(d, ng.NGC_OP_BWD_DATA_DB), stream())
        torch.cuda.synchronize()
        return (data3_from_device(dx, self.dtype, self.xl, (a.n, a.c, a.d, a.h, a.w)), db.cpu().numpy().astype(np.float64))
    ng.ngc_conv3d_bwd_data_relu(d, dyd, wd, xin, dx, self._ws(d, ng.NGC_OP_BWD_DATA), stream())
    torch.cuda.synchronize()
    return data3_from_device(dx, self.dtype, self.xl, (a.n, a.c, a.d, a.h, a.w))


def _run3_bias_grad(self, dy):
    a = self.a
    d = desc3_of(a, self.dtype, self.xl, self.yl)
    dyd = data3_to_device(dy, self.dtype, self.yl)
    db = torch.full((a.k,), float("nan"), dtype=torch.float32, device="cuda")
    ng.ngc_conv3d_bias_grad(d, dyd, db, self._ws(d, ng.NGC_OP_BIAS_GRAD), stream())
    torch.cuda.synchronize()
    return db.cpu().numpy().astype(np.float64)


Run3.bwd_data_relu = _run3_bwd_data_relu
Run3.bias_grad = _run3_bias_grad
