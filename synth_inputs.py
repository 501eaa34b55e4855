"""Seeded synthetic input tensors for the Convolution op family.

This module is *data only*: it holds no convolution, layout or epilogue
arithmetic.  It is the single place both the CPU oracle's tests and the HIP
path's tests / benchmark take their inputs from, so that the two sides see the
same bits.

Generator: counter based.  Element ``i`` of tensor ``tensor_id`` under ``seed``
is a pure function of ``(seed, tensor_id, i)`` (a splitmix64-style finaliser of
a 64-bit counter), so results do not depend on numpy's or torch's RNG streams,
on chunking, or on the order tensors are generated in.

* uniform tensors: 53-bit uniform in [0,1) mapped affinely to [lo, hi)
* normal tensors : Box-Muller on two such uniforms (counters 2i and 2i+1)
* values are produced in fp64, cast to fp32, and, for bf16 configurations,
  rounded once to bf16 (round-to-nearest-even) here on the host; the bf16
  bit patterns are what both sides consume.

Workload recipes (shapes / distributions of the five benchmark configurations,
ResNet-shaped layers) live in :func:`config_layers`.
"""
from __future__ import annotations

import math
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import Dict, List, Optional, Tuple

import numpy as np

TENSOR_X, TENSOR_W, TENSOR_BIAS, TENSOR_DY = 0, 1, 2, 3

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 20
_THREADS = max(1, min(16, os.cpu_count() or 1))


def _fill_chunks(n: int, fill) -> None:
    """Run fill(start, count) over [0, n) in chunks; chunks are independent
    (counter-based generator), so they may run on several host threads."""
    starts = range(0, n, _CHUNK)
    if n <= _CHUNK or _THREADS == 1:
        for s in starts:
            fill(s, min(_CHUNK, n - s))
        return
    with ThreadPoolExecutor(_THREADS) as ex:
        list(ex.map(lambda s: fill(s, min(_CHUNK, n - s)), starts))


def _mix64(z: np.ndarray) -> np.ndarray:
    """splitmix64 output function on an array of uint64 (wrapping arithmetic)."""
    z = z.copy()
    z ^= z >> np.uint64(30)
    z *= _M1
    z ^= z >> np.uint64(27)
    z *= _M2
    z ^= z >> np.uint64(31)
    return z


def _stream_key(seed: int, tensor_id: int) -> np.uint64:
    with np.errstate(over="ignore"):
        k = _mix64(np.array([np.uint64(seed & 0xFFFFFFFFFFFFFFFF)]))[0]
        k = _mix64(np.array([k ^ (np.uint64(tensor_id + 1) * _GOLDEN)]))[0]
    return k


def _uniform01(key: np.uint64, start: int, count: int) -> np.ndarray:
    """`count` uniforms in [0,1) for counters start .. start+count-1."""
    with np.errstate(over="ignore"):
        ctr = np.arange(start, start + count, dtype=np.uint64)
        bits = _mix64(key + (ctr + np.uint64(1)) * _GOLDEN)
    return (bits >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def uniform(seed: int, tensor_id: int, shape, lo: float, hi: float) -> np.ndarray:
    """fp32 tensor, elements U[lo, hi)."""
    n = int(np.prod(shape, dtype=np.int64))
    out = np.empty(n, dtype=np.float32)
    key = _stream_key(seed, tensor_id)

    def fill(s, c):
        out[s:s + c] = (lo + (hi - lo) * _uniform01(key, s, c)).astype(np.float32)

    _fill_chunks(n, fill)
    return out.reshape(shape)


def normal(seed: int, tensor_id: int, shape, mean: float, std: float) -> np.ndarray:
    """fp32 tensor, elements N(mean, std^2) by Box-Muller (cosine branch)."""
    n = int(np.prod(shape, dtype=np.int64))
    out = np.empty(n, dtype=np.float32)
    key = _stream_key(seed, tensor_id)

    def fill(s, c):
        u = _uniform01(key, 2 * s, 2 * c)
        u1 = 1.0 - u[0::2]            # (0,1]  -> log is finite
        u2 = u[1::2]
        z = np.sqrt(-2.0 * np.log(u1)) * np.cos((2.0 * math.pi) * u2)
        out[s:s + c] = (mean + std * z).astype(np.float32)

    _fill_chunks(n, fill)
    return out.reshape(shape)


# --------------------------------------------------------------------------
# bf16 containers (bit patterns in uint16).  Data preparation only.
# --------------------------------------------------------------------------

def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 -> bf16, round-to-nearest-even; returns uint16 bit patterns.
    Inputs are finite by construction (no NaN handling needed)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u.astype(np.uint64) + np.uint64(0x7FFF) + lsb.astype(np.uint64)) >> np.uint64(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to fp32 exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# Workload recipes
# --------------------------------------------------------------------------

@dataclass
class ConvLayer:
    """One convolution layer of a benchmark configuration (logical NCHW axes)."""
    name: str
    n: int
    c: int
    h: int
    w: int
    k: int
    r: int
    s: int
    stride: int = 1
    pad: int = 0
    dil: int = 1
    dtype: str = "bf16"             # "f32" | "bf16"
    bias_relu: bool = True          # forward epilogue
    ops: Tuple[str, ...] = ("fwd", "bwd_data", "bwd_filters")
    x_dist: Tuple = ("normal", 0.0, 1.0)
    dy_dist: Tuple = ("normal", 0.0, 0.1)
    w_dist: Tuple = ("he",)
    seed: int = 0
    count: int = 1                  # multiplicity inside the configuration
    # per-axis / per-side attributes where they differ from the scalars above: (h, w) pairs
    strides: Optional[Tuple[int, int]] = None
    dilation: Optional[Tuple[int, int]] = None
    pad_below: Optional[Tuple[int, int]] = None
    pad_above: Optional[Tuple[int, int]] = None

    @property
    def attrs15(self) -> Tuple[int, ...]:
        """(n, c, h, w, k, r, s, sh, sw, dh, dw, pbh, pbw, pah, paw): the constant attributes of the node."""
        sh, sw = self.strides or (self.stride, self.stride)
        dh, dw = self.dilation or (self.dil, self.dil)
        pbh, pbw = self.pad_below or (self.pad, self.pad)
        pah, paw = self.pad_above or (self.pad, self.pad)
        return (self.n, self.c, self.h, self.w, self.k, self.r, self.s, sh, sw, dh, dw, pbh, pbw, pah, paw)

    @property
    def p(self) -> int:
        _, _, h, _, _, r, _, sh, _, dh, _, pbh, _, pah, _ = self.attrs15
        return (h + pbh + pah - dh * (r - 1) - 1) // sh + 1

    @property
    def q(self) -> int:
        _, _, _, w, _, _, s, _, sw, _, dw, _, pbw, _, paw = self.attrs15
        return (w + pbw + paw - dw * (s - 1) - 1) // sw + 1

    @property
    def flop_per_op(self) -> float:
        return 2.0 * self.n * self.k * self.p * self.q * self.c * self.r * self.s


BASE_SEED = 180108058 * 10


def _resnet50_layers(n: int) -> List[ConvLayer]:
    """The 53 convolutions of ResNet-50 (stride 2 on the first 3x3 of stages 2-4,
    projection 1x1 with the stage stride), as unique shapes with multiplicities."""
    layers: List[Tuple[Tuple, int]] = []

    def add(c, k, hw, r, stride, pad):
        key = (c, k, hw, r, stride, pad)
        for i, (kk, cnt) in enumerate(layers):
            if kk == key:
                layers[i] = (kk, cnt + 1)
                return
        layers.append((key, 1))

    add(3, 64, 224, 7, 2, 3)
    hw, cin = 56, 64
    for stage, (width, blocks) in enumerate(((64, 3), (128, 4), (256, 6), (512, 3))):
        for b in range(blocks):
            stride = 2 if (stage > 0 and b == 0) else 1
            add(cin, width, hw, 1, 1, 0)                    # 1x1 a (input resolution)
            add(width, width, hw, 3, stride, 1)             # 3x3
            hw_out = hw // stride
            add(width, 4 * width, hw_out, 1, 1, 0)          # 1x1 c
            if b == 0:
                add(cin, 4 * width, hw, 1, stride, 0)       # projection
            cin, hw = 4 * width, hw_out
    out = []
    for idx, ((c, k, hw_, r, stride, pad), cnt) in enumerate(layers):
        out.append(ConvLayer(
            name=f"c{c}k{k}hw{hw_}r{r}s{stride}", n=n, c=c, h=hw_, w=hw_, k=k, r=r, s=r,
            stride=stride, pad=pad, dtype="bf16", bias_relu=True,
            x_dist=("uniform", 0.0, 1.0) if c == 3 else ("normal", 0.0, 1.0),
            seed=BASE_SEED + 5 + 1000 * idx, count=cnt))
    return out


def _general_attribute_layers(n: int) -> List[ConvLayer]:
    """Layers that exercise the attributes the ResNet stack does not: window dilation, padding that
    differs below / above, rectangular and larger windows, per-axis strides (shapes in the style of
    atrous segmentation heads and of factorised 1x7 / 7x1 and 5x5 inception branches)."""
    mk = lambda i, name, **kw: ConvLayer(name, n, seed=BASE_SEED + 6 + 1000 * i, **kw)
    return [
        mk(0, "g_3x3_dil2_c256", c=256, h=28, w=28, k=256, r=3, s=3, pad=2, dil=2),
        mk(1, "g_3x3_dil4_c128", c=128, h=56, w=56, k=128, r=3, s=3, pad=4, dil=4),
        mk(2, "g_5x5_c64k128", c=64, h=28, w=28, k=128, r=5, s=5, pad=2),
        mk(3, "g_1x7_c128k192", c=128, h=17, w=17, k=192, r=1, s=7, pad_below=(0, 3), pad_above=(0, 3)),
        mk(4, "g_7x1_c128k192", c=128, h=17, w=17, k=192, r=7, s=1, pad_below=(3, 0), pad_above=(3, 0)),
        mk(5, "g_3x3_s2_padabove", c=128, h=56, w=56, k=128, r=3, s=3, stride=2, pad_below=(0, 0), pad_above=(1, 1)),
        mk(6, "g_2x2_s2_c64k128", c=64, h=56, w=56, k=128, r=2, s=2, stride=2),
        mk(7, "g_3x3_s1x2_dil2x1", c=64, h=30, w=40, k=64, r=3, s=3, strides=(1, 2), dilation=(2, 1),
           pad_below=(2, 1), pad_above=(2, 0)),
    ]


def config_layers(cfg: int, batch: int | None = None) -> List[ConvLayer]:
    """Layer list of benchmark configuration `cfg` (1..5; 6 = general-attribute layers, not one of the
    headline configurations).  `batch` overrides N
    (used by tests that want the same recipe at a size the oracle finishes)."""
    if cfg == 1:
        return [ConvLayer("cfg1_f32_3x3", batch or 2, 16, 16, 16, 32, 3, 3, 1, 1, dtype="f32",
                          x_dist=("uniform", -1.0, 1.0), dy_dist=("uniform", -1.0, 1.0),
                          w_dist=("uniform", -1.0, 1.0), seed=BASE_SEED + 1)]
    if cfg == 2:
        return [ConvLayer("cfg2_3x3_c64", batch or 64, 64, 56, 56, 64, 3, 3, 1, 1, seed=BASE_SEED + 2)]
    if cfg == 3:
        return [ConvLayer("cfg3_1x1_c256k64", batch or 64, 256, 56, 56, 64, 1, 1, 1, 0,
                          bias_relu=False, seed=BASE_SEED + 3)]
    if cfg == 4:
        return [ConvLayer("cfg4_stem7x7", batch or 64, 3, 224, 224, 64, 7, 7, 2, 3,
                          ops=("fwd", "bwd_filters"), x_dist=("uniform", 0.0, 1.0),
                          seed=BASE_SEED + 4)]
    if cfg == 5:
        return _resnet50_layers(batch or 128)
    if cfg == 6:
        return _general_attribute_layers(batch or 32)
    raise ValueError(f"unknown configuration {cfg}")


@dataclass
class SoftmaxCase:
    """One softmax workload: a dense [rows, cols] tensor, softmax over cols."""
    name: str
    rows: int
    cols: int
    dtype: str = "bf16"
    seed: int = 0


def softmax_cases(scale: int = 1) -> List[SoftmaxCase]:
    """Softmax workloads: classifier logits, attention-score rows, a vocabulary-sized row (longer than the
    one-pass kernel holds in registers) and an fp32 case.  `scale` divides the row counts (tests)."""
    mk = lambda i, name, rows, cols, dtype="bf16": SoftmaxCase(name, max(1, rows // scale), cols, dtype,
                                                             BASE_SEED + 7 + 1000 * i)
    return [mk(0, "sm_logits_1000", 32768, 1000), mk(1, "sm_attn_512", 262144, 512),
            mk(2, "sm_vocab_32000", 4096, 32000), mk(3, "sm_f32_1024", 65536, 1024, "f32")]


def softmax_tensors(c: SoftmaxCase) -> Dict[str, np.ndarray]:
    """x ~ N(0, 3^2) (logit-like spread), dy ~ N(0, 0.1^2); bf16 cases hold bf16-representable values."""
    x = normal(c.seed, TENSOR_X, (c.rows, c.cols), 0.0, 3.0)
    dy = normal(c.seed, TENSOR_DY, (c.rows, c.cols), 0.0, 0.1)
    if c.dtype == "bf16":
        x, dy = bf16_bits_to_f32(f32_to_bf16_bits(x)), bf16_bits_to_f32(f32_to_bf16_bits(dy))
    return {"x": x, "dy": dy}


def _draw(dist: Tuple, seed: int, tid: int, shape, fan_in: int) -> np.ndarray:
    if dist[0] == "uniform":
        return uniform(seed, tid, shape, dist[1], dist[2])
    if dist[0] == "normal":
        return normal(seed, tid, shape, dist[1], dist[2])
    if dist[0] == "he":
        return normal(seed, tid, shape, 0.0, math.sqrt(2.0 / fan_in))
    raise ValueError(dist)


def layer_tensors(L: ConvLayer, which=("x", "w", "bias", "dy")) -> Dict[str, np.ndarray]:
    """Synthetic tensors of a layer, logical NCHW / KCRS axis order.

    Returns fp32 arrays.  For bf16 layers x, w and dy hold values that are
    exactly representable in bf16 (rounded once here); bias stays fp32."""
    out: Dict[str, np.ndarray] = {}
    fan_in = L.c * L.r * L.s
    if "x" in which:
        out["x"] = _draw(L.x_dist, L.seed, TENSOR_X, (L.n, L.c, L.h, L.w), fan_in)
    if "w" in which:
        out["w"] = _draw(L.w_dist, L.seed, TENSOR_W, (L.k, L.c, L.r, L.s), fan_in)
    if "bias" in which:
        out["bias"] = uniform(L.seed, TENSOR_BIAS, (L.k,), -0.1, 0.1)
    if "dy" in which:
        out["dy"] = _draw(L.dy_dist, L.seed, TENSOR_DY, (L.n, L.k, L.p, L.q), fan_in)
    if L.dtype == "bf16":
        for name in ("x", "w", "dy"):
            if name in out:
                out[name] = bf16_bits_to_f32(f32_to_bf16_bits(out[name]))
    return out


# ---------------------------------------------------------------- convolution over three spatial axes
@dataclass
class Conv3dLayer:
    """One convolution layer over (D, H, W), logical NCDHW axes; per-axis attributes as (d, h, w) triples."""
    name: str
    n: int
    c: int
    d: int
    h: int
    w: int
    k: int
    t: int
    r: int
    s: int
    strides: Tuple[int, int, int] = (1, 1, 1)
    dilation: Tuple[int, int, int] = (1, 1, 1)
    pad_below: Tuple[int, int, int] = (0, 0, 0)
    pad_above: Tuple[int, int, int] = (0, 0, 0)
    dtype: str = "bf16"
    bias_relu: bool = True
    x_dist: Tuple = ("normal", 0.0, 1.0)
    dy_dist: Tuple = ("normal", 0.0, 0.1)
    w_dist: Tuple = ("he",)
    seed: int = 0
    count: int = 1

    @property
    def attrs21(self) -> Tuple[int, ...]:
        """(n, c, d, h, w, k, t, r, s, strides, dilation, pad below, pad above): the constant attributes of the node."""
        return (self.n, self.c, self.d, self.h, self.w, self.k, self.t, self.r, self.s, *self.strides, *self.dilation,
                *self.pad_below, *self.pad_above)

    @property
    def opq(self) -> Tuple[int, int, int]:
        ext, taps = (self.d, self.h, self.w), (self.t, self.r, self.s)
        return tuple((ext[i] + self.pad_below[i] + self.pad_above[i] - self.dilation[i] * (taps[i] - 1) - 1) // self.strides[i] + 1
                     for i in range(3))

    @property
    def flop_per_op(self) -> float:
        o, p, q = self.opq
        return 2.0 * self.n * self.k * o * p * q * self.c * self.t * self.r * self.s


def video_layers(n: int | None = None, scale: int = 1) -> List[Conv3dLayer]:
    """Configuration 7: layers in the shapes of video networks on 16-frame clips (full 3x3x3 windows,
    a strided 3x3x3, the 1x3x3 + 3x1x1 pair of factorised space / time blocks, a 1x1x1 projection) and
    one layer with per-axis strides, dilation and one-sided padding.  `scale` divides the clip length and
    the image sides (tests that want the same recipe at a size the oracle finishes in seconds)."""
    n = n or 8
    f = lambda v: max(v // scale, 3)
    mk = lambda i, name, **kw: Conv3dLayer(name, n, seed=BASE_SEED + 7 + 1000 * i, **kw)
    return [
        mk(0, "v_3x3x3_c64k128", c=64, d=f(16), h=f(56), w=f(56), k=128, t=3, r=3, s=3, pad_below=(1, 1, 1), pad_above=(1, 1, 1)),
        mk(1, "v_3x3x3_c128k256", c=128, d=f(8), h=f(28), w=f(28), k=256, t=3, r=3, s=3, pad_below=(1, 1, 1), pad_above=(1, 1, 1)),
        mk(2, "v_3x3x3_s2_c128", c=128, d=f(8), h=f(28), w=f(28), k=128, t=3, r=3, s=3, strides=(2, 2, 2),
           pad_below=(1, 1, 1), pad_above=(1, 1, 1)),
        mk(3, "v_1x3x3_c64k128", c=64, d=f(16), h=f(56), w=f(56), k=128, t=1, r=3, s=3, pad_below=(0, 1, 1), pad_above=(0, 1, 1)),
        mk(4, "v_3x1x1_c128k64", c=128, d=f(16), h=f(56), w=f(56), k=64, t=3, r=1, s=1, pad_below=(1, 0, 0), pad_above=(1, 0, 0)),
        mk(5, "v_1x1x1_c256k64", c=256, d=f(8), h=f(28), w=f(28), k=64, t=1, r=1, s=1, bias_relu=False),
        mk(6, "v_3x3x3_general", c=64, d=f(8), h=f(20), w=f(24), k=64, t=3, r=3, s=3, strides=(1, 2, 1), dilation=(2, 1, 2),
           pad_below=(2, 0, 1), pad_above=(1, 1, 3)),
    ]


def layer3_tensors(L: Conv3dLayer, which=("x", "w", "bias", "dy")) -> Dict[str, np.ndarray]:
    """Synthetic tensors of a layer, logical NCDHW / KCTRS axis order, fp32 arrays; for bf16 layers x, w and dy
    hold values exactly representable in bf16 (rounded once here)."""
    out: Dict[str, np.ndarray] = {}
    fan_in = L.c * L.t * L.r * L.s
    if "x" in which:
        out["x"] = _draw(L.x_dist, L.seed, TENSOR_X, (L.n, L.c, L.d, L.h, L.w), fan_in)
    if "w" in which:
        out["w"] = _draw(L.w_dist, L.seed, TENSOR_W, (L.k, L.c, L.t, L.r, L.s), fan_in)
    if "bias" in which:
        out["bias"] = uniform(L.seed, TENSOR_BIAS, (L.k,), -0.1, 0.1)
    if "dy" in which:
        out["dy"] = _draw(L.dy_dist, L.seed, TENSOR_DY, (L.n, L.k, *L.opq), fan_in)
    if L.dtype == "bf16":
        for name in ("x", "w", "dy"):
            if name in out:
                out[name] = bf16_bits_to_f32(f32_to_bf16_bits(out[name]))
    return out
