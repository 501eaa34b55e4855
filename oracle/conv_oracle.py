"""ctypes front end of oracle/conv_ref.c (fp64 direct definitions).  TEST INFRASTRUCTURE ONLY.

The C file is the oracle; this module only marshals numpy arrays into it and
holds the error metric the parity tests use.  It imports nothing from the HIP
path.  Operation definitions: see the header of conv_ref.c (the paper's Sec. 2
fixes that an op is inputs + constant attributes; the formulas are the standard
cross-correlation convolution and its two adjoints).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv_ref.c")
_LIB = os.path.join(_HERE, "libconvref.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile conv_ref.c with gcc (-O2 -fopenmp) into oracle/libconvref.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99",
                               "-Wall", "-Wextra", "-o", _LIB, _SRC])
    return _LIB


class _CAttrs(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("n", "c", "h", "w", "k", "r", "s", "sh", "sw", "dh", "dw", "pbh", "pbw", "pah", "paw")]


@dataclass
class Attrs:
    """Constant attributes of the three ops (window strides, padding below /
    above, window dilation) plus the logical shapes [N,C,H,W] and [K,C,R,S]."""
    n: int
    c: int
    h: int
    w: int
    k: int
    r: int
    s: int
    sh: int = 1
    sw: int = 1
    dh: int = 1
    dw: int = 1
    pbh: int = 0
    pbw: int = 0
    pah: int = 0
    paw: int = 0

    def _c(self) -> _CAttrs:
        return _CAttrs(*(getattr(self, f) for f, _ in _CAttrs._fields_))


_D = np.ctypeslib.ndpointer(dtype=np.float64, flags="C_CONTIGUOUS")
_I64 = np.ctypeslib.ndpointer(dtype=np.int64, flags="C_CONTIGUOUS")


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(build())
    A = ctypes.POINTER(_CAttrs)
    lib.ref_out_dim.restype = ctypes.c_int32
    lib.ref_out_dim.argtypes = [ctypes.c_int32] * 6
    lib.ref_conv_fwd.argtypes = [A, _D, _D, ctypes.c_void_p, ctypes.c_int, _D]
    lib.ref_conv_fwd_at.argtypes = [A, _D, _D, ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, _I64, _D]
    lib.ref_conv_bwd_data.argtypes = [A, _D, _D, _D]
    lib.ref_conv_bwd_data_gather.argtypes = [A, _D, _D, _D]
    lib.ref_conv_bwd_data_at.argtypes = [A, _D, _D, ctypes.c_int64, _I64, _D]
    lib.ref_conv_bwd_filters.argtypes = [A, _D, _D, _D]
    lib.ref_conv_bwd_filters_at.argtypes = [A, _D, _D, ctypes.c_int64, _I64, _D]
    lib.ref_nchw_to_blocked16.argtypes = [ctypes.c_int32] * 5 + [ctypes.c_void_p, ctypes.c_void_p]
    lib.ref_blocked16_to_nchw.argtypes = [ctypes.c_int32] * 5 + [ctypes.c_void_p, ctypes.c_void_p]
    lib.ref_f32_bits_to_bf16_rne.restype = ctypes.c_uint16
    lib.ref_f32_bits_to_bf16_rne.argtypes = [ctypes.c_uint32]
    lib.ref_f32_to_bf16_rne_array.argtypes = [ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
    lib.ref_relu_bwd_mask.argtypes = [ctypes.c_int64, _D, _D, _D]
    lib.ref_bias_grad.argtypes = [ctypes.c_int32] * 4 + [_D, _D]
    for f in ("ref_conv_fwd", "ref_conv_fwd_at", "ref_conv_bwd_data", "ref_conv_bwd_data_gather",
              "ref_conv_bwd_data_at", "ref_conv_bwd_filters", "ref_conv_bwd_filters_at",
              "ref_nchw_to_blocked16", "ref_blocked16_to_nchw", "ref_f32_to_bf16_rne_array",
              "ref_relu_bwd_mask", "ref_bias_grad"):
        getattr(lib, f).restype = None
    _lib = lib
    return lib


def _f64(a, shape=None) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float64)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a


def out_shape(a: Attrs):
    """(P, Q): floor-mode output extents."""
    lib = _load()
    return (lib.ref_out_dim(a.h, a.pbh, a.pah, a.dh, a.r, a.sh),
            lib.ref_out_dim(a.w, a.pbw, a.paw, a.dw, a.s, a.sw))


def _bias_ptr(bias, k):
    if bias is None:
        return None, None
    b = _f64(bias, (k,))
    return b, b.ctypes.data_as(ctypes.c_void_p)


def conv_fwd(a: Attrs, x, w, bias=None, relu=False) -> np.ndarray:
    P, Q = out_shape(a)
    x = _f64(x, (a.n, a.c, a.h, a.w)); w = _f64(w, (a.k, a.c, a.r, a.s))
    keep, bp = _bias_ptr(bias, a.k)
    y = np.empty((a.n, a.k, P, Q), dtype=np.float64)
    _load().ref_conv_fwd(ctypes.byref(a._c()), x, w, bp, int(bool(relu)), y)
    return y


def conv_fwd_at(a: Attrs, x, w, flat_idx, bias=None, relu=False) -> np.ndarray:
    """Forward definition evaluated at flat indices into y[N,K,P,Q]."""
    x = _f64(x, (a.n, a.c, a.h, a.w)); w = _f64(w, (a.k, a.c, a.r, a.s))
    idx = np.ascontiguousarray(flat_idx, dtype=np.int64)
    keep, bp = _bias_ptr(bias, a.k)
    out = np.empty(idx.shape[0], dtype=np.float64)
    _load().ref_conv_fwd_at(ctypes.byref(a._c()), x, w, bp, int(bool(relu)), idx.shape[0], idx, out)
    return out


def conv_bwd_data(a: Attrs, dy, w) -> np.ndarray:
    """Scatter form."""
    P, Q = out_shape(a)
    dy = _f64(dy, (a.n, a.k, P, Q)); w = _f64(w, (a.k, a.c, a.r, a.s))
    dx = np.empty((a.n, a.c, a.h, a.w), dtype=np.float64)
    _load().ref_conv_bwd_data(ctypes.byref(a._c()), dy, w, dx)
    return dx


def conv_bwd_data_gather(a: Attrs, dy, w) -> np.ndarray:
    P, Q = out_shape(a)
    dy = _f64(dy, (a.n, a.k, P, Q)); w = _f64(w, (a.k, a.c, a.r, a.s))
    dx = np.empty((a.n, a.c, a.h, a.w), dtype=np.float64)
    _load().ref_conv_bwd_data_gather(ctypes.byref(a._c()), dy, w, dx)
    return dx


def conv_bwd_data_at(a: Attrs, dy, w, flat_idx) -> np.ndarray:
    P, Q = out_shape(a)
    dy = _f64(dy, (a.n, a.k, P, Q)); w = _f64(w, (a.k, a.c, a.r, a.s))
    idx = np.ascontiguousarray(flat_idx, dtype=np.int64)
    out = np.empty(idx.shape[0], dtype=np.float64)
    _load().ref_conv_bwd_data_at(ctypes.byref(a._c()), dy, w, idx.shape[0], idx, out)
    return out


def conv_bwd_filters(a: Attrs, x, dy) -> np.ndarray:
    P, Q = out_shape(a)
    x = _f64(x, (a.n, a.c, a.h, a.w)); dy = _f64(dy, (a.n, a.k, P, Q))
    dw = np.empty((a.k, a.c, a.r, a.s), dtype=np.float64)
    _load().ref_conv_bwd_filters(ctypes.byref(a._c()), x, dy, dw)
    return dw


def conv_bwd_filters_at(a: Attrs, x, dy, flat_idx) -> np.ndarray:
    P, Q = out_shape(a)
    x = _f64(x, (a.n, a.c, a.h, a.w)); dy = _f64(dy, (a.n, a.k, P, Q))
    idx = np.ascontiguousarray(flat_idx, dtype=np.int64)
    out = np.empty(idx.shape[0], dtype=np.float64)
    _load().ref_conv_bwd_filters_at(ctypes.byref(a._c()), x, dy, idx.shape[0], idx, out)
    return out


def relu_bwd_mask(g, z) -> np.ndarray:
    """ReLU backprop: g where z > 0, else 0 (z: the ReLU's output, or equally its input)."""
    g = np.ascontiguousarray(g, dtype=np.float64)
    z = np.ascontiguousarray(z, dtype=np.float64)
    assert g.shape == z.shape
    out = np.empty_like(g)
    _load().ref_relu_bwd_mask(g.size, g.reshape(-1), z.reshape(-1), out.reshape(-1))
    return out


def bias_grad(dy) -> np.ndarray:
    """db[k] = sum over n, p, q of dy[n,k,p,q]."""
    dy = np.ascontiguousarray(dy, dtype=np.float64)
    n, k, p, q = dy.shape
    db = np.empty(k, dtype=np.float64)
    _load().ref_bias_grad(n, k, p, q, dy.reshape(-1), db)
    return db


def conv_bwd_data_relu(a: Attrs, dy, w, x_in) -> np.ndarray:
    """ConvolutionBackpropData followed by the backprop of the ReLU that produced the convolution's
    input: dx[i] if x_in[i] > 0 else 0 (the two ops in the order the derivative graph has them)."""
    return relu_bwd_mask(conv_bwd_data(a, dy, w), x_in)


def _elem_bytes(arr: np.ndarray) -> int:
    if arr.dtype.itemsize not in (2, 4):
        raise ValueError("layout permutation is defined for 2- and 4-byte elements")
    return arr.dtype.itemsize


def nchw_to_blocked16(x: np.ndarray) -> np.ndarray:
    """[N,C,H,W] -> [N,ceil(C/16),H,W,16], tail lanes zero bits.  Bit copy."""
    x = np.ascontiguousarray(x)
    n, c, h, w = x.shape
    out = np.empty((n, (c + 15) // 16, h, w, 16), dtype=x.dtype)
    _load().ref_nchw_to_blocked16(n, c, h, w, _elem_bytes(x), x.ctypes.data, out.ctypes.data)
    return out


def blocked16_to_nchw(xb: np.ndarray, c: int) -> np.ndarray:
    xb = np.ascontiguousarray(xb)
    n, cb, h, w, sixteen = xb.shape
    if sixteen != 16 or cb != (c + 15) // 16:
        raise ValueError("not a 16-channel-blocked tensor for this C")
    out = np.empty((n, c, h, w), dtype=xb.dtype)
    _load().ref_blocked16_to_nchw(n, c, h, w, _elem_bytes(xb), xb.ctypes.data, out.ctypes.data)
    return out


def f32_to_bf16_bits_rne(a) -> np.ndarray:
    """fp32 -> bf16 bit patterns, round-to-nearest-even."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    out = np.empty(a.shape, dtype=np.uint16)
    _load().ref_f32_to_bf16_rne_array(a.size, a.ctypes.data, out.ctypes.data)
    return out


def bf16_bits_to_f64(b) -> np.ndarray:
    """Exact widening of bf16 bit patterns."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def max_normalised_error(got, ref) -> float:
    """e = max|got - ref| / max|ref|  (L-inf error over the L-inf norm of the reference)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if got.shape != ref.shape:
        raise ValueError(f"shape mismatch {got.shape} vs {ref.shape}")
    if ref.size == 0:
        return 0.0
    denom = float(np.max(np.abs(ref)))
    diff = np.abs(got - ref)
    if not np.isfinite(diff).all():          # a NaN or an infinity in either tensor never passes a bound
        return float("inf")
    err = float(np.max(diff))
    if denom == 0.0:
        return 0.0 if err == 0.0 else float("inf")
    return err / denom
