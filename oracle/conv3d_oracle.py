"""CPU oracle for Convolution over three spatial axes (N, C, D, H, W) -- TEST INFRASTRUCTURE ONLY.

The paper's IR is rank-general: tensors of any rank, ops defined by inputs and
constant attributes (Sec. 2; Sec. 3 for the derivative ops).  The rank-3 spatial
Convolution is the same definition as the rank-2 one with one more window axis
(cross-correlation, no filter flip, floor output size), written out in fp64 numpy:

    O = floor((D + pbd + pad - dd*(T-1) - 1) / sd) + 1,  P, Q likewise
    y[n,k,o,p,q]   = sum_{c,t,r,s} X(n,c, o*sd - pbd + t*dd, p*sh - pbh + r*dh, q*sw - pbw + s*dw) * w[k,c,t,r,s]
                     X = x inside the volume, 0 outside
    dx             = adjoint of y w.r.t. x applied to dy (0 where no window reaches)
    dw[k,c,t,r,s]  = sum_{n,o,p,q} dy[n,k,o,p,q] * X(n,c, ...same input coordinate...)

Each function is one loop over the window taps (t, r, s); per tap the strided slice of the
explicitly zero-padded input that the tap reads is contracted over channels with numpy's
einsum.  No blocking, no reordering beyond that.  The *_at functions evaluate single
elements by an explicit loop over the window (used on sampled outputs of large tensors).

Pins (tests/test_oracle_pins.py): the rank-2 C oracle on every pair of axes (the third
axis of extent 1), a scalar brute force from the definition on tiny inputs,
scipy.signal.correlate on single-channel volumes, the adjoint identities between the three
ops, closed forms (all-ones overlap counts, off-centre delta filters).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass
class Attrs3:
    """Constant attributes of the three ops: shapes [N,C,D,H,W] and [K,C,T,R,S], window
    movement strides s*, window dilation d*, padding below pb* / above pa* per axis (d, h, w)."""
    n: int
    c: int
    d: int
    h: int
    w: int
    k: int
    t: int
    r: int
    s: int
    sd: int = 1
    sh: int = 1
    sw: int = 1
    dd: int = 1
    dh: int = 1
    dw: int = 1
    pbd: int = 0
    pbh: int = 0
    pbw: int = 0
    pad: int = 0
    pah: int = 0
    paw: int = 0


def _out(extent, below, above, dil, taps, stride):
    return (extent + below + above - dil * (taps - 1) - 1) // stride + 1


def out_shape3(a: Attrs3):
    """(O, P, Q): floor-mode output extents."""
    return (_out(a.d, a.pbd, a.pad, a.dd, a.t, a.sd), _out(a.h, a.pbh, a.pah, a.dh, a.r, a.sh),
            _out(a.w, a.pbw, a.paw, a.dw, a.s, a.sw))


def _f64(v, shape):
    v = np.ascontiguousarray(v, dtype=np.float64)
    if tuple(v.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(v.shape)}")
    return v


def _padded(a: Attrs3, x=None):
    """Zero volume of the padded extents, with x copied into its interior if given."""
    xp = np.zeros((a.n, a.c, a.d + a.pbd + a.pad, a.h + a.pbh + a.pah, a.w + a.pbw + a.paw), dtype=np.float64)
    if x is not None:
        xp[:, :, a.pbd:a.pbd + a.d, a.pbh:a.pbh + a.h, a.pbw:a.pbw + a.w] = x
    return xp


def _tap_slices(a: Attrs3, O, P, Q, t, r, s):
    """Padded-input elements tap (t, r, s) reads for outputs (0..O-1, 0..P-1, 0..Q-1)."""
    return (slice(t * a.dd, t * a.dd + (O - 1) * a.sd + 1, a.sd),
            slice(r * a.dh, r * a.dh + (P - 1) * a.sh + 1, a.sh),
            slice(s * a.dw, s * a.dw + (Q - 1) * a.sw + 1, a.sw))


def conv3d_fwd(a: Attrs3, x, w, bias=None, relu=False) -> np.ndarray:
    O, P, Q = out_shape3(a)
    x = _f64(x, (a.n, a.c, a.d, a.h, a.w)); w = _f64(w, (a.k, a.c, a.t, a.r, a.s))
    xp = _padded(a, x)
    y = np.zeros((a.n, a.k, O, P, Q), dtype=np.float64)
    for t in range(a.t):
        for r in range(a.r):
            for s in range(a.s):
                sd, sh, sw = _tap_slices(a, O, P, Q, t, r, s)
                y += np.einsum("ncopq,kc->nkopq", xp[:, :, sd, sh, sw], w[:, :, t, r, s])
    if bias is not None:
        y += _f64(bias, (a.k,))[None, :, None, None, None]
    if relu:
        y = np.maximum(y, 0.0)
    return y


def conv3d_bwd_data(a: Attrs3, dy, w) -> np.ndarray:
    """Scatter form of the adjoint: every (output element, tap) adds into the input element it read."""
    O, P, Q = out_shape3(a)
    dy = _f64(dy, (a.n, a.k, O, P, Q)); w = _f64(w, (a.k, a.c, a.t, a.r, a.s))
    dxp = _padded(a)
    for t in range(a.t):
        for r in range(a.r):
            for s in range(a.s):
                sd, sh, sw = _tap_slices(a, O, P, Q, t, r, s)
                dxp[:, :, sd, sh, sw] += np.einsum("nkopq,kc->ncopq", dy, w[:, :, t, r, s])
    return np.ascontiguousarray(dxp[:, :, a.pbd:a.pbd + a.d, a.pbh:a.pbh + a.h, a.pbw:a.pbw + a.w])


def conv3d_bwd_filters(a: Attrs3, x, dy) -> np.ndarray:
    O, P, Q = out_shape3(a)
    x = _f64(x, (a.n, a.c, a.d, a.h, a.w)); dy = _f64(dy, (a.n, a.k, O, P, Q))
    xp = _padded(a, x)
    dw = np.zeros((a.k, a.c, a.t, a.r, a.s), dtype=np.float64)
    for t in range(a.t):
        for r in range(a.r):
            for s in range(a.s):
                sd, sh, sw = _tap_slices(a, O, P, Q, t, r, s)
                dw[:, :, t, r, s] = np.einsum("nkopq,ncopq->kc", dy, xp[:, :, sd, sh, sw])
    return dw


def _window(a: Attrs3):
    return [(t, r, s) for t in range(a.t) for r in range(a.r) for s in range(a.s)]


def conv3d_fwd_at(a: Attrs3, x, w, flat_idx, bias=None, relu=False) -> np.ndarray:
    """Forward definition evaluated at flat indices into y[N,K,O,P,Q]."""
    O, P, Q = out_shape3(a)
    x = _f64(x, (a.n, a.c, a.d, a.h, a.w)); w = _f64(w, (a.k, a.c, a.t, a.r, a.s))
    out = np.empty(len(flat_idx), dtype=np.float64)
    for i, f in enumerate(np.asarray(flat_idx, dtype=np.int64)):
        n, k, o, p, q = np.unravel_index(int(f), (a.n, a.k, O, P, Q))
        acc = 0.0
        for t, r, s in _window(a):
            z, yy, xx = o * a.sd - a.pbd + t * a.dd, p * a.sh - a.pbh + r * a.dh, q * a.sw - a.pbw + s * a.dw
            if 0 <= z < a.d and 0 <= yy < a.h and 0 <= xx < a.w:
                acc += float(np.dot(x[n, :, z, yy, xx], w[k, :, t, r, s]))
        if bias is not None:
            acc += float(bias[k])
        out[i] = max(acc, 0.0) if relu else acc
    return out


def conv3d_bwd_data_at(a: Attrs3, dy, w, flat_idx) -> np.ndarray:
    """Gather form of the adjoint at flat indices into dx[N,C,D,H,W]."""
    O, P, Q = out_shape3(a)
    dy = _f64(dy, (a.n, a.k, O, P, Q)); w = _f64(w, (a.k, a.c, a.t, a.r, a.s))
    out = np.empty(len(flat_idx), dtype=np.float64)
    for i, f in enumerate(np.asarray(flat_idx, dtype=np.int64)):
        n, c, z, yy, xx = np.unravel_index(int(f), (a.n, a.c, a.d, a.h, a.w))
        acc = 0.0
        for t, r, s in _window(a):
            no, np_, nq = z + a.pbd - t * a.dd, yy + a.pbh - r * a.dh, xx + a.pbw - s * a.dw
            if no < 0 or np_ < 0 or nq < 0 or no % a.sd or np_ % a.sh or nq % a.sw:
                continue
            o, p, q = no // a.sd, np_ // a.sh, nq // a.sw
            if o < O and p < P and q < Q:
                acc += float(np.dot(dy[n, :, o, p, q], w[:, c, t, r, s]))
        out[i] = acc
    return out


def conv3d_bwd_filters_at(a: Attrs3, x, dy, flat_idx) -> np.ndarray:
    """dw at flat indices into [K,C,T,R,S]."""
    O, P, Q = out_shape3(a)
    x = _f64(x, (a.n, a.c, a.d, a.h, a.w)); dy = _f64(dy, (a.n, a.k, O, P, Q))
    xp = _padded(a, x)
    out = np.empty(len(flat_idx), dtype=np.float64)
    for i, f in enumerate(np.asarray(flat_idx, dtype=np.int64)):
        k, c, t, r, s = np.unravel_index(int(f), (a.k, a.c, a.t, a.r, a.s))
        sd, sh, sw = _tap_slices(a, O, P, Q, t, r, s)
        out[i] = float(np.sum(dy[:, k] * xp[:, c, sd, sh, sw]))
    return out
