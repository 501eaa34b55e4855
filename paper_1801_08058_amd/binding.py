"""Thin ctypes binding of libngconv.so (the C ABI declared in include/ngconv.h).

Argument marshalling only: every step of the path runs in the HIP kernels.  Tensors are
passed as anything with a ``data_ptr()`` (torch tensors) or as raw integer device
addresses; the stream is a raw ``hipStream_t`` value (``torch.cuda.current_stream().cuda_stream``)
or None for the default stream.  There is no CPU fallback: if the library is missing
the import fails loudly.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libngconv.so")

# enums of include/ngconv.h
NGC_OK, NGC_BAD_ARG, NGC_BAD_SHAPE, NGC_UNSUPPORTED, NGC_WORKSPACE_TOO_SMALL, NGC_LAUNCH_FAILED = 0, -1, -2, -3, -4, -5
NGC_SCRATCH_EXCEEDED = -6
NGC_F32, NGC_BF16 = 0, 1
NGC_NCHW, NGC_NCHW16C = 0, 1
NGC_KCRS, NGC_BLOCKED_FWD, NGC_BLOCKED_BWD = 0, 1, 2
NGC_EPI_NONE, NGC_EPI_BIAS, NGC_EPI_RELU = 0, 1, 2
NGC_OP_FWD, NGC_OP_BWD_DATA, NGC_OP_BWD_FILTERS, NGC_OP_BIAS_GRAD, NGC_OP_BWD_DATA_DB, NGC_OP_BWD_DATA_FILTERS = 0, 1, 2, 3, 4, 5

EXPORTS = ("ngc_conv_out_shape", "ngc_conv_workspace_bytes", "ngc_conv_fwd", "ngc_conv_bwd_data",
           "ngc_conv_bwd_data_relu", "ngc_conv_bwd_data_relu_db", "ngc_bias_grad", "ngc_softmax", "ngc_softmax_bwd", "ngc_softmax_variant", "ngc_conv_bwd_filters", "ngc_conv_bwd_data_filters", "ngc_conv_bwd_data_filters_relu", "ngc_layout_convert", "ngc_filter_convert", "ngc_data_elems",
           "ngc_filter_elems", "ngc_conv_variant", "ngc_status_string",
           "ngc_conv3d_out_shape", "ngc_conv3d_workspace_bytes", "ngc_conv3d_fwd", "ngc_conv3d_bwd_data",
           "ngc_conv3d_bwd_filters", "ngc_conv3d_filter_convert", "ngc_conv3d_filter_elems", "ngc_conv3d_data_elems",
           "ngc_conv3d_variant", "ngc_conv3d_bwd_data_relu", "ngc_conv3d_bwd_data_relu_db", "ngc_conv3d_bias_grad",
           "ngc_conv_bwd_filters_noalloc", "ngc_static_scratch_bytes", "ngc_reload_switches")


class ngc_conv_desc(ctypes.Structure):
    """Mirror of the C struct: constant attributes of a Convolution node."""
    _fields_ = [(name, ctypes.c_int32) for name in (
        "n", "c", "h", "w", "k", "r", "s", "stride_h", "stride_w", "dil_h", "dil_w",
        "pad_below_h", "pad_below_w", "pad_above_h", "pad_above_w",
        "dtype", "x_layout", "y_layout", "w_layout", "epilogue")]

    def __repr__(self):
        return "ngc_conv_desc(" + ", ".join(f"{n}={getattr(self, n)}" for n, _ in self._fields_) + ")"


class ngc_conv3d_desc(ctypes.Structure):
    """Mirror of the C struct: constant attributes of a Convolution node over three spatial axes."""
    _fields_ = [(name, ctypes.c_int32) for name in (
        "n", "c", "d", "h", "w", "k", "t", "r", "s", "stride_d", "stride_h", "stride_w", "dil_d", "dil_h", "dil_w",
        "pad_below_d", "pad_below_h", "pad_below_w", "pad_above_d", "pad_above_h", "pad_above_w",
        "dtype", "x_layout", "y_layout", "w_layout", "epilogue")]

    def __repr__(self):
        return "ngc_conv3d_desc(" + ", ".join(f"{n}={getattr(self, n)}" for n, _ in self._fields_) + ")"


class NgcError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {ngc_status_string(status)} ({status})")


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_1801_08058_amd.build` "
            "(there is no fallback path)")
    # PyTorch supplies device memory and streams and ships its own HIP runtime under the same
    # soname as the system one; the process must end up with ONE runtime, and it has to be the
    # one torch initialises, so torch is loaded first when it is installed.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(LIB_PATH)
    D = ctypes.POINTER(ngc_conv_desc)
    vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32
    lib.ngc_conv_out_shape.argtypes = [D, ctypes.POINTER(i32), ctypes.POINTER(i32)]
    lib.ngc_conv_out_shape.restype = ctypes.c_int
    lib.ngc_conv_workspace_bytes.argtypes = [D, ctypes.c_int]
    lib.ngc_conv_workspace_bytes.restype = sz
    lib.ngc_conv_fwd.argtypes = [D, vp, vp, vp, vp, vp, sz, vp]
    lib.ngc_conv_fwd.restype = ctypes.c_int
    lib.ngc_conv_bwd_data.argtypes = [D, vp, vp, vp, vp, sz, vp]
    lib.ngc_conv_bwd_data.restype = ctypes.c_int
    lib.ngc_conv_bwd_data_relu.argtypes = [D, vp, vp, vp, vp, vp, sz, vp]
    lib.ngc_conv_bwd_data_relu.restype = ctypes.c_int
    lib.ngc_conv_bwd_data_relu_db.argtypes = [D, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.ngc_conv_bwd_data_relu_db.restype = ctypes.c_int
    lib.ngc_bias_grad.argtypes = [D, vp, vp, vp, sz, vp]
    lib.ngc_bias_grad.restype = ctypes.c_int
    lib.ngc_softmax.argtypes = [i32, ctypes.c_int64, i32, vp, vp, vp]
    lib.ngc_softmax.restype = ctypes.c_int
    lib.ngc_softmax_bwd.argtypes = [i32, ctypes.c_int64, i32, vp, vp, vp, vp]
    lib.ngc_softmax_bwd.restype = ctypes.c_int
    lib.ngc_softmax_variant.argtypes = [i32, i32, i32]
    lib.ngc_softmax_variant.restype = ctypes.c_char_p
    lib.ngc_conv_bwd_filters.argtypes = [D, vp, vp, vp, vp, sz, vp]
    lib.ngc_conv_bwd_filters.restype = ctypes.c_int
    for f in (lib.ngc_conv_bwd_data_filters, lib.ngc_conv_bwd_data_filters_relu):
        f.argtypes = [D, vp, vp, vp, vp, vp, vp, sz, vp]
        f.restype = ctypes.c_int
    lib.ngc_conv_bwd_filters_noalloc.argtypes = [D, vp, vp, vp, vp]
    lib.ngc_conv_bwd_filters_noalloc.restype = ctypes.c_int
    lib.ngc_reload_switches.argtypes = []
    lib.ngc_reload_switches.restype = None
    lib.ngc_static_scratch_bytes.argtypes = []
    lib.ngc_static_scratch_bytes.restype = sz
    lib.ngc_layout_convert.argtypes = [i32, i32, i32, i32, i32, vp, i32, vp, i32, vp]
    lib.ngc_layout_convert.restype = ctypes.c_int
    lib.ngc_filter_convert.argtypes = [D, vp, vp, i32, vp]
    lib.ngc_filter_convert.restype = ctypes.c_int
    lib.ngc_data_elems.argtypes = [D, ctypes.c_int]
    lib.ngc_data_elems.restype = sz
    lib.ngc_filter_elems.argtypes = [D, i32]
    lib.ngc_filter_elems.restype = sz
    lib.ngc_conv_variant.argtypes = [D, ctypes.c_int]
    lib.ngc_conv_variant.restype = ctypes.c_char_p
    lib.ngc_status_string.argtypes = [ctypes.c_int]
    lib.ngc_status_string.restype = ctypes.c_char_p
    D3 = ctypes.POINTER(ngc_conv3d_desc)
    lib.ngc_conv3d_out_shape.argtypes = [D3, ctypes.POINTER(i32), ctypes.POINTER(i32), ctypes.POINTER(i32)]
    lib.ngc_conv3d_out_shape.restype = ctypes.c_int
    lib.ngc_conv3d_workspace_bytes.argtypes = [D3, ctypes.c_int]
    lib.ngc_conv3d_workspace_bytes.restype = sz
    lib.ngc_conv3d_fwd.argtypes = [D3, vp, vp, vp, vp, vp, sz, vp]
    lib.ngc_conv3d_fwd.restype = ctypes.c_int
    lib.ngc_conv3d_bwd_data.argtypes = [D3, vp, vp, vp, vp, sz, vp]
    lib.ngc_conv3d_bwd_data.restype = ctypes.c_int
    lib.ngc_conv3d_bwd_filters.argtypes = [D3, vp, vp, vp, vp, sz, vp]
    lib.ngc_conv3d_bwd_filters.restype = ctypes.c_int
    lib.ngc_conv3d_filter_convert.argtypes = [D3, vp, vp, i32, vp]
    lib.ngc_conv3d_filter_convert.restype = ctypes.c_int
    lib.ngc_conv3d_filter_elems.argtypes = [D3, i32]
    lib.ngc_conv3d_filter_elems.restype = sz
    lib.ngc_conv3d_data_elems.argtypes = [D3, ctypes.c_int]
    lib.ngc_conv3d_data_elems.restype = sz
    lib.ngc_conv3d_bwd_data_relu.argtypes = [D3, vp, vp, vp, vp, vp, sz, vp]
    lib.ngc_conv3d_bwd_data_relu.restype = ctypes.c_int
    lib.ngc_conv3d_bwd_data_relu_db.argtypes = [D3, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.ngc_conv3d_bwd_data_relu_db.restype = ctypes.c_int
    lib.ngc_conv3d_bias_grad.argtypes = [D3, vp, vp, vp, sz, vp]
    lib.ngc_conv3d_bias_grad.restype = ctypes.c_int
    lib.ngc_conv3d_variant.argtypes = [D3, ctypes.c_int]
    lib.ngc_conv3d_variant.restype = ctypes.c_char_p
    return lib


_lib = _load()


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    return ctypes.c_void_p(t.data_ptr())


def _nbytes(t) -> int:
    if t is None or isinstance(t, int):
        return 0
    return t.numel() * t.element_size()


def _stream(s):
    return ctypes.c_void_p(s) if s else None


def _check(status: int, where: str, check: bool) -> int:
    if check and status != NGC_OK:
        raise NgcError(status, where)
    return status


def make_desc(n, c, h, w, k, r, s, stride=(1, 1), dilation=(1, 1), pad_below=(0, 0), pad_above=(0, 0),
              dtype=NGC_BF16, x_layout=NGC_NCHW16C, y_layout=NGC_NCHW16C, w_layout=NGC_KCRS,
              epilogue=NGC_EPI_NONE) -> ngc_conv_desc:
    return ngc_conv_desc(n, c, h, w, k, r, s, stride[0], stride[1], dilation[0], dilation[1],
                         pad_below[0], pad_below[1], pad_above[0], pad_above[1],
                         dtype, x_layout, y_layout, w_layout, epilogue)


def ngc_status_string(status: int) -> str:
    return _lib.ngc_status_string(int(status)).decode()


def ngc_conv_out_shape(desc: ngc_conv_desc, check: bool = True):
    p, q = ctypes.c_int32(0), ctypes.c_int32(0)
    st = _lib.ngc_conv_out_shape(ctypes.byref(desc), ctypes.byref(p), ctypes.byref(q))
    if st != NGC_OK:
        if check:
            raise NgcError(st, "ngc_conv_out_shape")
        return st
    return p.value, q.value


def ngc_conv_workspace_bytes(desc: ngc_conv_desc, op: int) -> int:
    return int(_lib.ngc_conv_workspace_bytes(ctypes.byref(desc), op))


def ngc_data_elems(desc: ngc_conv_desc, which: int) -> int:
    return int(_lib.ngc_data_elems(ctypes.byref(desc), which))


def ngc_filter_elems(desc: ngc_conv_desc, layout: int) -> int:
    return int(_lib.ngc_filter_elems(ctypes.byref(desc), layout))


def ngc_conv_variant(desc: ngc_conv_desc, op: int) -> str:
    return _lib.ngc_conv_variant(ctypes.byref(desc), op).decode()


def ngc_conv_fwd(desc, x, w, bias, y, ws=None, stream=None, check: bool = True) -> int:
    return _check(_lib.ngc_conv_fwd(ctypes.byref(desc), _ptr(x), _ptr(w), _ptr(bias), _ptr(y), _ptr(ws), _nbytes(ws),
                                    _stream(stream)), "ngc_conv_fwd", check)


def ngc_conv_bwd_data(desc, dy, w, dx, ws=None, stream=None, check: bool = True) -> int:
    return _check(_lib.ngc_conv_bwd_data(ctypes.byref(desc), _ptr(dy), _ptr(w), _ptr(dx), _ptr(ws), _nbytes(ws),
                                         _stream(stream)), "ngc_conv_bwd_data", check)


def ngc_conv_bwd_data_relu(desc, dy, w, x_in, dx, ws=None, stream=None, check: bool = True) -> int:
    return _check(_lib.ngc_conv_bwd_data_relu(ctypes.byref(desc), _ptr(dy), _ptr(w), _ptr(x_in), _ptr(dx), _ptr(ws),
                                              _nbytes(ws), _stream(stream)), "ngc_conv_bwd_data_relu", check)


def ngc_conv_bwd_data_relu_db(desc, dy, w, x_in, dx, db, ws=None, stream=None, check: bool = True) -> int:
    return _check(_lib.ngc_conv_bwd_data_relu_db(ctypes.byref(desc), _ptr(dy), _ptr(w), _ptr(x_in), _ptr(dx), _ptr(db),
                                                 _ptr(ws), _nbytes(ws), _stream(stream)), "ngc_conv_bwd_data_relu_db", check)


def ngc_bias_grad(desc, dy, db, ws=None, stream=None, check: bool = True) -> int:
    return _check(_lib.ngc_bias_grad(ctypes.byref(desc), _ptr(dy), _ptr(db), _ptr(ws), _nbytes(ws),
                                     _stream(stream)), "ngc_bias_grad", check)


def ngc_softmax(dtype, rows, cols, x, y, stream=None, check: bool = True) -> int:
    return _check(_lib.ngc_softmax(dtype, rows, cols, _ptr(x), _ptr(y), _stream(stream)), "ngc_softmax", check)


def ngc_softmax_bwd(dtype, rows, cols, y, dy, dx, stream=None, check: bool = True) -> int:
    return _check(_lib.ngc_softmax_bwd(dtype, rows, cols, _ptr(y), _ptr(dy), _ptr(dx), _stream(stream)),
                  "ngc_softmax_bwd", check)


def ngc_softmax_variant(dtype, cols, bwd=False) -> str:
    return _lib.ngc_softmax_variant(dtype, cols, 1 if bwd else 0).decode()


def ngc_conv_bwd_filters(desc, x, dy, dw, ws=None, stream=None, check: bool = True) -> int:
    return _check(_lib.ngc_conv_bwd_filters(ctypes.byref(desc), _ptr(x), _ptr(dy), _ptr(dw), _ptr(ws), _nbytes(ws),
                                            _stream(stream)), "ngc_conv_bwd_filters", check)


def ngc_conv_bwd_data_filters(desc, x, dy, w, dx, dw, ws=None, stream=None, check: bool = True) -> int:
    return _check(_lib.ngc_conv_bwd_data_filters(ctypes.byref(desc), _ptr(x), _ptr(dy), _ptr(w), _ptr(dx), _ptr(dw), _ptr(ws),
                                                 _nbytes(ws), _stream(stream)), "ngc_conv_bwd_data_filters", check)


def ngc_conv_bwd_data_filters_relu(desc, x, dy, w, dx, dw, ws=None, stream=None, check: bool = True) -> int:
    return _check(_lib.ngc_conv_bwd_data_filters_relu(ctypes.byref(desc), _ptr(x), _ptr(dy), _ptr(w), _ptr(dx), _ptr(dw), _ptr(ws),
                                                      _nbytes(ws), _stream(stream)), "ngc_conv_bwd_data_filters_relu", check)


def ngc_conv_bwd_filters_noalloc(desc, x, dy, dw, stream=None, check: bool = True) -> int:
    return _check(_lib.ngc_conv_bwd_filters_noalloc(ctypes.byref(desc), _ptr(x), _ptr(dy), _ptr(dw), _stream(stream)),
                  "ngc_conv_bwd_filters_noalloc", check)


def ngc_reload_switches() -> None:
    _lib.ngc_reload_switches()


def ngc_static_scratch_bytes() -> int:
    return int(_lib.ngc_static_scratch_bytes())


def ngc_layout_convert(dtype, n, c, h, w, src, src_layout, dst, dst_layout, stream=None, check: bool = True) -> int:
    return _check(_lib.ngc_layout_convert(dtype, n, c, h, w, _ptr(src), src_layout, _ptr(dst), dst_layout,
                                          _stream(stream)), "ngc_layout_convert", check)


def ngc_filter_convert(desc, w_kcrs, w_blocked, dst_layout, stream=None, check: bool = True) -> int:
    return _check(_lib.ngc_filter_convert(ctypes.byref(desc), _ptr(w_kcrs), _ptr(w_blocked), dst_layout,
                                          _stream(stream)), "ngc_filter_convert", check)


# ---- Convolution over three spatial axes

def make_desc3(n, c, d, h, w, k, t, r, s, stride=(1, 1, 1), dilation=(1, 1, 1), pad_below=(0, 0, 0), pad_above=(0, 0, 0),
               dtype=NGC_BF16, x_layout=NGC_NCHW16C, y_layout=NGC_NCHW16C, w_layout=NGC_KCRS,
               epilogue=NGC_EPI_NONE) -> ngc_conv3d_desc:
    return ngc_conv3d_desc(n, c, d, h, w, k, t, r, s, *stride, *dilation, *pad_below, *pad_above,
                           dtype, x_layout, y_layout, w_layout, epilogue)


def ngc_conv3d_out_shape(desc: ngc_conv3d_desc, check: bool = True):
    o, p, q = ctypes.c_int32(0), ctypes.c_int32(0), ctypes.c_int32(0)
    st = _lib.ngc_conv3d_out_shape(ctypes.byref(desc), ctypes.byref(o), ctypes.byref(p), ctypes.byref(q))
    if st != NGC_OK:
        if check:
            raise NgcError(st, "ngc_conv3d_out_shape")
        return st
    return o.value, p.value, q.value


def ngc_conv3d_workspace_bytes(desc: ngc_conv3d_desc, op: int) -> int:
    return int(_lib.ngc_conv3d_workspace_bytes(ctypes.byref(desc), op))


def ngc_conv3d_data_elems(desc: ngc_conv3d_desc, which: int) -> int:
    return int(_lib.ngc_conv3d_data_elems(ctypes.byref(desc), which))


def ngc_conv3d_filter_elems(desc: ngc_conv3d_desc, layout: int) -> int:
    return int(_lib.ngc_conv3d_filter_elems(ctypes.byref(desc), layout))


def ngc_conv3d_variant(desc: ngc_conv3d_desc, op: int) -> str:
    return _lib.ngc_conv3d_variant(ctypes.byref(desc), op).decode()


def ngc_conv3d_fwd(desc, x, w, bias, y, ws=None, stream=None, check: bool = True) -> int:
    return _check(_lib.ngc_conv3d_fwd(ctypes.byref(desc), _ptr(x), _ptr(w), _ptr(bias), _ptr(y), _ptr(ws), _nbytes(ws),
                                      _stream(stream)), "ngc_conv3d_fwd", check)


def ngc_conv3d_bwd_data(desc, dy, w, dx, ws=None, stream=None, check: bool = True) -> int:
    return _check(_lib.ngc_conv3d_bwd_data(ctypes.byref(desc), _ptr(dy), _ptr(w), _ptr(dx), _ptr(ws), _nbytes(ws),
                                           _stream(stream)), "ngc_conv3d_bwd_data", check)


def ngc_conv3d_bwd_filters(desc, x, dy, dw, ws=None, stream=None, check: bool = True) -> int:
    return _check(_lib.ngc_conv3d_bwd_filters(ctypes.byref(desc), _ptr(x), _ptr(dy), _ptr(dw), _ptr(ws), _nbytes(ws),
                                              _stream(stream)), "ngc_conv3d_bwd_filters", check)


def ngc_conv3d_filter_convert(desc, w_kctrs, w_blocked, dst_layout, stream=None, check: bool = True) -> int:
    return _check(_lib.ngc_conv3d_filter_convert(ctypes.byref(desc), _ptr(w_kctrs), _ptr(w_blocked), dst_layout,
                                                 _stream(stream)), "ngc_conv3d_filter_convert", check)


def ngc_conv3d_bwd_data_relu(desc, dy, w, x_in, dx, ws=None, stream=None, check: bool = True) -> int:
    return _check(_lib.ngc_conv3d_bwd_data_relu(ctypes.byref(desc), _ptr(dy), _ptr(w), _ptr(x_in), _ptr(dx), _ptr(ws),
                                                _nbytes(ws), _stream(stream)), "ngc_conv3d_bwd_data_relu", check)


def ngc_conv3d_bwd_data_relu_db(desc, dy, w, x_in, dx, db, ws=None, stream=None, check: bool = True) -> int:
    return _check(_lib.ngc_conv3d_bwd_data_relu_db(ctypes.byref(desc), _ptr(dy), _ptr(w), _ptr(x_in), _ptr(dx), _ptr(db),
                                                   _ptr(ws), _nbytes(ws), _stream(stream)), "ngc_conv3d_bwd_data_relu_db", check)


def ngc_conv3d_bias_grad(desc, dy, db, ws=None, stream=None, check: bool = True) -> int:
    return _check(_lib.ngc_conv3d_bias_grad(ctypes.byref(desc), _ptr(dy), _ptr(db), _ptr(ws), _nbytes(ws),
                                            _stream(stream)), "ngc_conv3d_bias_grad", check)
