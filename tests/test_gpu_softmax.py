"""GPU parity of ngc_softmax / ngc_softmax_bwd (through the C ABI) against the fp64 oracle.
Tolerances (max normalised error): 1e-5 for fp32, 2e-2 for bf16 (one rounding of a value in (0, 1])."""
import numpy as np
import pytest
import torch

import oracle
import paper_1801_08058_amd as ng
import synth_inputs
from gpu_util import TOL, dev, encode, host, stream

pytestmark = pytest.mark.gpu


def _decode(t, dtype, shape):
    raw = host(t, np.float32 if dtype == "f32" else np.uint16).reshape(shape)
    return raw.astype(np.float64) if dtype == "f32" else oracle.bf16_bits_to_f64(raw)


def _run(x, dy, dtype, offset=0, in_place=False):
    """offset (elements): shifts the tensors inside their allocation, which takes them off the 16-byte grid."""
    rows, cols = x.shape
    code = ng.NGC_F32 if dtype == "f32" else ng.NGC_BF16
    tdt = torch.float32 if dtype == "f32" else torch.int16

    def place(values):
        buf = torch.zeros(rows * cols + offset, dtype=tdt, device="cuda")
        buf[offset:] = dev(encode(values, dtype)).reshape(-1)
        return buf, buf[offset:]

    xb, xd = place(x)
    if in_place:
        yb, yd = xb, xd
    else:
        yb = torch.full((rows * cols + offset,), 0x7FC0 if dtype == "bf16" else -12345.0, dtype=tdt, device="cuda")
        yd = yb[offset:]
    front = yb[:offset].clone()
    print(f"softmax rows={rows} cols={cols} dtype={dtype} offset={offset} in_place={in_place}", flush=True)
    ng.ngc_softmax(code, rows, cols, xd, yd, stream())
    torch.cuda.synchronize()
    y = _decode(yd, dtype, (rows, cols))
    dyb, dyd = place(dy)
    dxb = torch.full((rows * cols + offset,), 0x7FC0 if dtype == "bf16" else -12345.0, dtype=tdt, device="cuda")
    ng.ngc_softmax_bwd(code, rows, cols, yd, dyd, dxb[offset:], stream())
    torch.cuda.synchronize()
    dx = _decode(dxb[offset:], dtype, (rows, cols))
    assert torch.equal(yb[:offset], front)                           # nothing written in front of the tensor
    return y, dx


def _check(x, dy, dtype, **kw):
    y, dx = _run(x, dy, dtype, **kw)
    tol = TOL[dtype]
    ref = oracle.softmax(x)
    assert np.isfinite(y).all()
    e = np.abs(y - ref).max() / ref.max()
    assert e <= tol, f"softmax err {e}"
    # rows sum to one up to the rounding of the stored elements
    assert np.abs(y.sum(axis=-1) - 1.0).max() <= (2e-2 if dtype == "bf16" else 1e-4)
    # backprop is checked on the y the device produced (its own rounded output is its input)
    ref_dx = oracle.softmax_bwd(y, dy)
    e = np.abs(dx - ref_dx).max() / max(np.abs(ref_dx).max(), 1e-30)
    assert e <= tol, f"softmax_bwd err {e}"


def _inputs(rows, cols, dtype, seed):
    x = synth_inputs.normal(seed, 0, (rows, cols), 0.0, 3.0)
    dy = synth_inputs.normal(seed, 3, (rows, cols), 0.0, 0.1)
    if dtype == "bf16":
        rt = lambda t: synth_inputs.bf16_bits_to_f32(synth_inputs.f32_to_bf16_bits(t))
        x, dy = rt(x), rt(dy)
    return x, dy


# row lengths: every vectors-per-lane variant of the wave kernel (ragged last vector row), the
# workgroup-per-row kernel (odd lengths, lengths past the register budget), a single column
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("rows,cols", [(5, 8), (7, 512), (9, 1000), (6, 1032), (5, 2048), (3, 3000), (3, 4096), (2, 8192),
                                       (3, 8200), (4, 1001), (6, 37), (1, 1), (2, 20000), (1030, 64), (2, 32768),
                                       (2, 16384), (3, 33000), (2, 40008)])
def test_softmax_small(dtype, rows, cols):
    x, dy = _inputs(rows, cols, dtype, 100 + rows * 7 + cols)
    e = 8 if dtype == "bf16" else 4
    expect = "softmax_rows_block" if cols % e else "softmax_rows_wave" if cols <= 256 * e else \
        "softmax_rows_wg" if cols <= 4096 * e else "softmax_rows_block"
    assert ng.ngc_softmax_variant(ng.NGC_BF16 if dtype == "bf16" else ng.NGC_F32, cols) == expect
    _check(x, dy, dtype)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_softmax_unaligned_tensors_and_in_place(dtype):
    x, dy = _inputs(6, 512, dtype, 77)
    _check(x, dy, dtype, offset=1)                  # off the 16-byte grid: workgroup-per-row kernel
    _check(x, dy, dtype, in_place=True)
    _check(x, dy, dtype, offset=3, in_place=True)


def test_softmax_large_magnitudes_and_dominant_elements():
    rows, cols = 8, 1024
    x = synth_inputs.normal(5, 0, (rows, cols), 0.0, 1.0).astype(np.float32)
    x[0] += 30000.0                                  # exp overflows without the shift
    x[1] -= 30000.0
    x[2, 17] = 200.0                                 # one element takes all the mass
    x[3] = 0.0                                       # constant row -> 1 / cols
    y, _ = _run(x, np.zeros_like(x), "f32")
    ref = oracle.softmax(x)
    assert np.isfinite(y).all() and np.abs(y - ref).max() <= 1e-5
    assert y[2, 17] == 1.0 and np.allclose(y[3], 1.0 / cols, rtol=1e-6)


@pytest.mark.parametrize("idx", range(4))
def test_softmax_workloads_reduced_rows(idx):
    c = synth_inputs.softmax_cases(scale=256)[idx]
    t = synth_inputs.softmax_tensors(c)
    _check(t["x"], t["dy"], c.dtype)


@pytest.mark.parametrize("idx", range(4))
def test_softmax_workloads_full_size_sampled_rows(idx):
    """The launch configuration bench.py times; the oracle evaluates a sample of whole rows."""
    c = synth_inputs.softmax_cases()[idx]
    t = synth_inputs.softmax_tensors(c)
    code = ng.NGC_F32 if c.dtype == "f32" else ng.NGC_BF16
    xd, dyd = dev(encode(t["x"], c.dtype)), dev(encode(t["dy"], c.dtype))
    yd, dxd = torch.empty_like(xd), torch.empty_like(xd)
    print(f"softmax workload {c.name}", flush=True)
    ng.ngc_softmax(code, c.rows, c.cols, xd, yd, stream())
    ng.ngc_softmax_bwd(code, c.rows, c.cols, yd, dyd, dxd, stream())
    torch.cuda.synchronize()
    y, dx = _decode(yd, c.dtype, (c.rows, c.cols)), _decode(dxd, c.dtype, (c.rows, c.cols))
    assert np.isfinite(y).all() and np.isfinite(dx).all()
    rows = np.random.default_rng(c.seed % 2 ** 32).integers(0, c.rows, 512)
    rows[:2] = (0, c.rows - 1)
    ref = oracle.softmax(t["x"][rows])
    tol = TOL[c.dtype]
    assert np.abs(y[rows] - ref).max() / ref.max() <= tol
    ref_dx = oracle.softmax_bwd(y[rows], t["dy"][rows])
    assert np.abs(dx[rows] - ref_dx).max() / np.abs(ref_dx).max() <= tol
    assert np.abs(y.sum(axis=-1) - 1.0).max() <= (2e-2 if c.dtype == "bf16" else 1e-4)
