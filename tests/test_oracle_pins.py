"""Pins for the CPU oracle (no GPU).  Each test fixes the oracle against something
other than itself: hand-worked values, an independent brute force written in a
different code shape, a library matmul, adjoint / finite-difference identities,
closed forms and construction identities.  A dropped term, wrong sign, wrong
index or transposed operand in oracle/conv_ref.c fails at least one of them."""
import itertools
import json
import os

import numpy as np
import pytest

import oracle
from oracle import Attrs

GOLD = os.path.join(os.path.dirname(__file__), "golden", "hand_examples.json")
rng = np.random.default_rng(20180125)


def _attrs_from(d):
    return Attrs(d["n"], d["c"], d["h"], d["w"], d["k"], d["r"], d["s"],
                 d["stride"], d["stride"], d["dilation"], d["dilation"],
                 d["pad_below"], d["pad_below"], d["pad_above"], d["pad_above"])


# ---------------------------------------------------------------- P1 hand examples
def test_hand_example_1():
    g = json.load(open(GOLD))["example_1"]
    a = _attrs_from(g["attrs"])
    x = np.array(g["x"], float).reshape(1, 1, 3, 3)
    w = np.array(g["w"], float).reshape(1, 1, 2, 2)
    dy = np.array(g["dy"], float).reshape(1, 1, 2, 2)
    y = oracle.conv_fwd(a, x, w)
    assert np.array_equal(y[0, 0], np.array(g["y"], float))
    assert np.array_equal(oracle.conv_fwd(a, x, w, bias=[5.0], relu=True)[0, 0], np.array(g["y_bias5_relu"], float))
    assert np.array_equal(oracle.conv_fwd(a, x, w, bias=[0.0], relu=True)[0, 0], np.array(g["y_bias0_relu"], float))
    dx = oracle.conv_bwd_data(a, dy, w)
    assert np.array_equal(dx[0, 0], np.array(g["dx"], float))
    assert np.array_equal(oracle.conv_bwd_data_gather(a, dy, w), dx)
    dw = oracle.conv_bwd_filters(a, x, dy)
    assert np.array_equal(dw[0, 0], np.array(g["dw"], float))
    ip = g["inner_product"]
    assert (y * dy).sum() == ip and (x * dx).sum() == ip and (w * dw).sum() == ip


def test_hand_example_2_stride_pad():
    g = json.load(open(GOLD))["example_2"]
    a = _attrs_from(g["attrs"])
    assert oracle.out_shape(a) == (2, 2)
    x = np.array(g["x"], float).reshape(1, 1, 3, 3)
    w = np.array(g["w"], float).reshape(1, 1, 3, 3)
    assert np.array_equal(oracle.conv_fwd(a, x, w)[0, 0], np.array(g["y"], float))


# ---------------------------------------------------------------- P2 brute force
def _brute(a: Attrs, x, w, dy):
    """Independent 7-loop scalar routine on an explicitly zero-padded copy of x
    (no bounds tests); returns y, dx, dw.  Written from the definition, different
    code shape from the oracle (padding buffer, flat python loops, dict of terms)."""
    Hp = a.h + a.pbh + a.pah
    Wp = a.w + a.pbw + a.paw
    xp = np.zeros((a.n, a.c, Hp, Wp))
    xp[:, :, a.pbh:a.pbh + a.h, a.pbw:a.pbw + a.w] = x
    P = (Hp - (a.dh * (a.r - 1) + 1)) // a.sh + 1 if Hp >= a.dh * (a.r - 1) + 1 else 0
    Q = (Wp - (a.dw * (a.s - 1) + 1)) // a.sw + 1 if Wp >= a.dw * (a.s - 1) + 1 else 0
    y = np.zeros((a.n, a.k, P, Q))
    dxp = np.zeros_like(xp)
    dw = np.zeros((a.k, a.c, a.r, a.s))
    for n, k, p, q, c, r, s in itertools.product(range(a.n), range(a.k), range(P), range(Q),
                                                 range(a.c), range(a.r), range(a.s)):
        ii = p * a.sh + r * a.dh
        jj = q * a.sw + s * a.dw
        y[n, k, p, q] += xp[n, c, ii, jj] * w[k, c, r, s]
        if dy is not None:
            dxp[n, c, ii, jj] += dy[n, k, p, q] * w[k, c, r, s]
            dw[k, c, r, s] += dy[n, k, p, q] * xp[n, c, ii, jj]
    dx = dxp[:, :, a.pbh:a.pbh + a.h, a.pbw:a.pbw + a.w]
    return y, dx, dw, (P, Q)


def _random_attrs(max_hw=7):
    while True:
        a = Attrs(n=int(rng.integers(1, 4)), c=int(rng.integers(1, 4)), h=int(rng.integers(1, max_hw + 1)),
                  w=int(rng.integers(1, max_hw + 1)), k=int(rng.integers(1, 4)), r=int(rng.integers(1, 4)),
                  s=int(rng.integers(1, 4)), sh=int(rng.integers(1, 4)), sw=int(rng.integers(1, 4)),
                  dh=int(rng.integers(1, 3)), dw=int(rng.integers(1, 3)),
                  pbh=int(rng.integers(0, 3)), pbw=int(rng.integers(0, 3)),
                  pah=int(rng.integers(0, 3)), paw=int(rng.integers(0, 3)))
        P, Q = oracle.out_shape(a)
        if P > 0 and Q > 0:
            return a


def _random_tensors(a):
    P, Q = oracle.out_shape(a)
    return (rng.uniform(-1, 1, (a.n, a.c, a.h, a.w)), rng.uniform(-1, 1, (a.k, a.c, a.r, a.s)),
            rng.uniform(-1, 1, (a.n, a.k, P, Q)))


@pytest.mark.parametrize("trial", range(40))
def test_brute_force_tiny(trial):
    a = _random_attrs()
    x, w, dy = _random_tensors(a)
    y_b, dx_b, dw_b, pq = _brute(a, x, w, dy)
    assert pq == oracle.out_shape(a)
    np.testing.assert_allclose(oracle.conv_fwd(a, x, w), y_b, rtol=0, atol=1e-13)
    np.testing.assert_allclose(oracle.conv_bwd_data(a, dy, w), dx_b, rtol=0, atol=1e-13)
    np.testing.assert_allclose(oracle.conv_bwd_data_gather(a, dy, w), dx_b, rtol=0, atol=1e-13)
    np.testing.assert_allclose(oracle.conv_bwd_filters(a, x, dy), dw_b, rtol=0, atol=1e-13)


def test_sampled_entry_points_match_full():
    for _ in range(5):
        a = _random_attrs(9)
        x, w, dy = _random_tensors(a)
        b = rng.uniform(-1, 1, a.k)
        y = oracle.conv_fwd(a, x, w, bias=b, relu=True)
        dx = oracle.conv_bwd_data(a, dy, w)
        dw = oracle.conv_bwd_filters(a, x, dy)
        for full, fn in ((y, lambda i: oracle.conv_fwd_at(a, x, w, i, bias=b, relu=True)),
                         (dx, lambda i: oracle.conv_bwd_data_at(a, dy, w, i)),
                         (dw, lambda i: oracle.conv_bwd_filters_at(a, x, dy, i))):
            idx = rng.integers(0, full.size, size=min(64, full.size))
            np.testing.assert_allclose(fn(idx), full.reshape(-1)[idx], rtol=0, atol=1e-13)


# ---------------------------------------------------------------- P3 1x1 conv == matmul
def test_1x1_is_matmul():
    a = Attrs(n=3, c=7, h=5, w=6, k=4, r=1, s=1)
    x, w, dy = _random_tensors(a)
    y = oracle.conv_fwd(a, x, w)
    W2 = w.reshape(a.k, a.c)
    for n in range(a.n):
        np.testing.assert_allclose(y[n].reshape(a.k, -1), W2 @ x[n].reshape(a.c, -1), rtol=0, atol=1e-13)
    dx = oracle.conv_bwd_data(a, dy, w)
    for n in range(a.n):
        np.testing.assert_allclose(dx[n].reshape(a.c, -1), W2.T @ dy[n].reshape(a.k, -1), rtol=0, atol=1e-13)
    dw = oracle.conv_bwd_filters(a, x, dy)
    ref = sum(dy[n].reshape(a.k, -1) @ x[n].reshape(a.c, -1).T for n in range(a.n))
    np.testing.assert_allclose(dw.reshape(a.k, a.c), ref, rtol=0, atol=1e-12)


# ---------------------------------------------------------------- P4 adjoint identities
@pytest.mark.parametrize("trial", range(12))
def test_adjoint_identities(trial):
    a = _random_attrs(11)
    if trial == 0:   # stride 2 with a leftover row / column no window reaches
        a = Attrs(n=2, c=3, h=8, w=10, k=4, r=3, s=3, sh=2, sw=2, pbh=0, pbw=1, pah=0, paw=0)
    x, w, dy = _random_tensors(a)
    lhs = float((oracle.conv_fwd(a, x, w) * dy).sum())
    mid = float((x * oracle.conv_bwd_data(a, dy, w)).sum())
    rhs = float((w * oracle.conv_bwd_filters(a, x, dy)).sum())
    scale = max(abs(lhs), 1e-30)
    assert abs(lhs - mid) / scale < 1e-12 and abs(lhs - rhs) / scale < 1e-12


def test_unreached_pixels_get_zero_gradient():
    # 1x1 stride 2: odd rows / columns of dx are never touched
    a = Attrs(n=1, c=2, h=6, w=6, k=3, r=1, s=1, sh=2, sw=2)
    x, w, dy = _random_tensors(a)
    dx = oracle.conv_bwd_data(a, dy, w)
    assert np.all(dx[:, :, 1::2, :] == 0) and np.all(dx[:, :, :, 1::2] == 0)
    assert np.any(dx[:, :, 0::2, 0::2] != 0)


# ---------------------------------------------------------------- P5 finite differences
def test_finite_differences_exact_by_linearity():
    a = Attrs(n=2, c=3, h=7, w=6, k=4, r=3, s=2, sh=2, sw=1, dh=1, dw=2, pbh=1, pbw=0, pah=2, paw=1)
    x, w, dy = _random_tensors(a)
    v = rng.uniform(-1, 1, w.shape)
    u = rng.uniform(-1, 1, x.shape)
    base = (oracle.conv_fwd(a, x, w) * dy).sum()
    dw = oracle.conv_bwd_filters(a, x, dy)
    dx = oracle.conv_bwd_data(a, dy, w)
    for eps in (1.0, 1e-3):
        fd_w = ((oracle.conv_fwd(a, x, w + eps * v) * dy).sum() - base) / eps
        fd_x = ((oracle.conv_fwd(a, x + eps * u, w) * dy).sum() - base) / eps
        assert abs(fd_w - (v * dw).sum()) < 1e-9 / eps * 1e-3 + 1e-10
        assert abs(fd_x - (u * dx).sum()) < 1e-9 / eps * 1e-3 + 1e-10


# ---------------------------------------------------------------- P6 closed forms
def test_all_ones_counts_window_overlap():
    a = Attrs(n=1, c=3, h=6, w=5, k=2, r=3, s=3, sh=2, sw=1, dh=2, dw=1, pbh=2, pbw=1, pah=1, paw=2)
    P, Q = oracle.out_shape(a)
    y = oracle.conv_fwd(a, np.ones((1, 3, 6, 5)), np.ones((2, 3, 3, 3)))
    for p in range(P):
        for q in range(Q):
            ch = sum(1 for r in range(a.r) if 0 <= p * a.sh - a.pbh + r * a.dh < a.h)
            cw = sum(1 for s in range(a.s) if 0 <= q * a.sw - a.pbw + s * a.dw < a.w)
            assert np.all(y[:, :, p, q] == a.c * ch * cw)


def test_delta_filter_is_identity():
    a = Attrs(n=2, c=3, h=5, w=4, k=3, r=3, s=3, pbh=1, pbw=1, pah=1, paw=1)
    x = rng.uniform(-1, 1, (2, 3, 5, 4))
    w = np.zeros((3, 3, 3, 3))
    for k in range(3):
        w[k, k, 1, 1] = 1.0
    assert np.array_equal(oracle.conv_fwd(a, x, w), x)


def test_no_flip_off_centre_delta():
    # tap (r,s)=(0,2) of a 3x3 filter picks x[p-1, q+1] under pad 1: cross-correlation, not flipped
    a = Attrs(n=1, c=1, h=4, w=4, k=1, r=3, s=3, pbh=1, pbw=1, pah=1, paw=1)
    x = rng.uniform(-1, 1, (1, 1, 4, 4))
    w = np.zeros((1, 1, 3, 3)); w[0, 0, 0, 2] = 1.0
    y = oracle.conv_fwd(a, x, w)
    exp = np.zeros_like(x)
    exp[0, 0, 1:, :3] = x[0, 0, :3, 1:]
    assert np.array_equal(y, exp)


# ---------------------------------------------------------------- P7 construction identities
def test_padding_equals_explicit_zero_pad():
    a = Attrs(n=2, c=2, h=5, w=6, k=3, r=3, s=2, sh=1, sw=2, pbh=2, pbw=1, pah=0, paw=3)
    x, w, _ = _random_tensors(a)
    xp = np.zeros((2, 2, 5 + 2, 6 + 4)); xp[:, :, 2:7, 1:7] = x
    b = Attrs(n=2, c=2, h=7, w=10, k=3, r=3, s=2, sh=1, sw=2)
    assert np.array_equal(oracle.conv_fwd(a, x, w), oracle.conv_fwd(b, xp, w))


def test_stride_is_subsample_of_stride1():
    a1 = Attrs(n=1, c=2, h=9, w=8, k=2, r=3, s=3, pbh=1, pbw=1, pah=1, paw=1)
    a2 = Attrs(n=1, c=2, h=9, w=8, k=2, r=3, s=3, sh=2, sw=3, pbh=1, pbw=1, pah=1, paw=1)
    x, w, _ = _random_tensors(a1)
    y1 = oracle.conv_fwd(a1, x, w)
    y2 = oracle.conv_fwd(a2, x, w)
    assert np.array_equal(y2, y1[:, :, ::2, ::3][:, :, :y2.shape[2], :y2.shape[3]])


def test_dilation_equals_zero_stuffed_filter():
    a = Attrs(n=1, c=2, h=9, w=9, k=2, r=3, s=2, dh=2, dw=3, pbh=1, pbw=2, pah=2, paw=1)
    x, w, _ = _random_tensors(a)
    wz = np.zeros((2, 2, 5, 4)); wz[:, :, ::2, ::3] = w
    b = Attrs(n=1, c=2, h=9, w=9, k=2, r=5, s=4, pbh=1, pbw=2, pah=2, paw=1)
    assert oracle.out_shape(a) == oracle.out_shape(b)
    assert np.array_equal(oracle.conv_fwd(a, x, w), oracle.conv_fwd(b, x, wz))


# ---------------------------------------------------------------- P8 linearity
def test_linearity():
    a = Attrs(n=2, c=3, h=6, w=6, k=2, r=3, s=3, pbh=1, pbw=1, pah=1, paw=1)
    x1, w, _ = _random_tensors(a)
    x2 = rng.uniform(-1, 1, x1.shape)
    lhs = oracle.conv_fwd(a, 2.5 * x1 + x2, w)
    rhs = 2.5 * oracle.conv_fwd(a, x1, w) + oracle.conv_fwd(a, x2, w)
    np.testing.assert_allclose(lhs, rhs, rtol=0, atol=1e-12)


# ---------------------------------------------------------------- P9 epilogue
def test_epilogue_bias_then_relu():
    a = Attrs(n=2, c=3, h=6, w=6, k=4, r=3, s=3, pbh=1, pbw=1, pah=1, paw=1)
    x, w, _ = _random_tensors(a)
    b = rng.uniform(-0.5, 0.5, a.k)
    y = oracle.conv_fwd(a, x, w)
    yb = oracle.conv_fwd(a, x, w, bias=b)
    z = oracle.conv_fwd(a, x, w, bias=b, relu=True)
    np.testing.assert_array_equal(yb, y + b[None, :, None, None])
    assert np.all(z >= 0)
    assert np.array_equal(z, np.where(yb > 0, yb, 0.0))
    assert np.array_equal(oracle.conv_fwd(a, x, w, relu=True), np.where(y > 0, y, 0.0))
    assert (yb < 0).any() and (yb > 0).any()


# ---------------------------------------------------------------- P10 layout
@pytest.mark.parametrize("dtype", [np.uint16, np.uint32])
@pytest.mark.parametrize("c", [1, 3, 16, 17, 40])
def test_layout_roundtrip_and_formula(dtype, c):
    n, h, w = 2, 3, 5
    x = rng.integers(1, np.iinfo(dtype).max, size=(n, c, h, w), dtype=dtype)   # never 0
    xb = oracle.nchw_to_blocked16(x)
    cb = (c + 15) // 16
    assert xb.shape == (n, cb, h, w, 16) and xb.dtype == dtype
    # independent statement of the permutation with numpy axis moves
    pad = np.zeros((n, cb * 16, h, w), dtype=dtype); pad[:, :c] = x
    exp = pad.reshape(n, cb, 16, h, w).transpose(0, 1, 3, 4, 2)
    assert np.array_equal(xb, exp)
    assert np.count_nonzero(xb) == x.size                  # tail lanes are zero bits
    assert np.array_equal(oracle.blocked16_to_nchw(xb, c), x)
    assert np.array_equal(np.sort(xb[xb != 0].ravel()), np.sort(x.ravel()))


# ---------------------------------------------------------------- P11 bf16 rounding
def test_bf16_rne_fixed_cases():
    lib = oracle.conv_oracle._load()
    for src, want in json.load(open(GOLD))["bf16_rne"]["cases"]:
        assert lib.ref_f32_bits_to_bf16_rne(int(src, 16)) == int(want, 16), src


def test_bf16_rne_matches_torch_and_generator():
    import torch
    import synth_inputs
    v = rng.standard_normal(1_000_000).astype(np.float32) * np.float32(10.0) ** rng.integers(-20, 20, 1_000_000).astype(np.float32)
    v[:1000] = np.ldexp(1.0 + (2 * rng.integers(0, 128, 1000) + 1) / 256.0, rng.integers(-10, 10, 1000)).astype(np.float32)  # exact ties
    ours = oracle.f32_to_bf16_bits_rne(v)
    t = torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, t)
    assert np.array_equal(ours, synth_inputs.f32_to_bf16_bits(v))
    assert np.array_equal(oracle.bf16_bits_to_f64(ours), torch.from_numpy(t.view(np.int16)).view(torch.bfloat16).double().numpy())


# ---------------------------------------------------------------- P12 backward compounding: ReLU mask, bias gradient
def test_relu_bwd_mask_cases():
    g = np.array([1.5, -2.0, 3.0, 4.0, -5.0, 6.0, 7.0])
    z = np.array([2.0, 1e-30, 0.0, -0.0, -1.0, np.inf, np.nan])
    out = oracle.relu_bwd_mask(g, z)
    # strictly positive z passes the gradient; +0, -0, negative and NaN block it
    np.testing.assert_array_equal(out, np.array([1.5, -2.0, 0.0, 0.0, 0.0, 6.0, 0.0]))
    big = rng.normal(size=(3, 4, 5, 6))
    np.testing.assert_array_equal(oracle.relu_bwd_mask(big, np.abs(big) + 1.0), big)      # identity
    np.testing.assert_array_equal(oracle.relu_bwd_mask(big, -np.abs(big)), np.zeros_like(big))


def test_bias_grad_closed_form_and_brute_force():
    n, k, p, q = 3, 5, 4, 7
    np.testing.assert_allclose(oracle.bias_grad(np.full((n, k, p, q), 0.25)), np.full(k, 0.25 * n * p * q), rtol=1e-15)
    dy = rng.normal(size=(n, k, p, q))
    brute = [sum(dy[nn, kk, i, j] for nn in range(n) for i in range(p) for j in range(q)) for kk in range(k)]
    np.testing.assert_allclose(oracle.bias_grad(dy), brute, rtol=1e-13)
    # only channel kk of dy reaches db[kk]
    e = np.zeros((n, k, p, q)); e[1, 2, 3, 4] = 2.0
    np.testing.assert_array_equal(oracle.bias_grad(e), np.array([0, 0, 2.0, 0, 0]))


def test_bias_grad_is_adjoint_of_bias_broadcast():
    a = Attrs(n=2, c=3, h=7, w=6, k=4, r=3, s=2, sh=2, sw=1, pbh=1, pbw=0, pah=1, paw=1)
    x, w, dy = _random_tensors(a)
    b = rng.uniform(-1, 1, a.k)
    lhs = ((oracle.conv_fwd(a, x, w, bias=b) - oracle.conv_fwd(a, x, w)) * dy).sum()
    assert abs(lhs - (b * oracle.bias_grad(dy)).sum()) < 1e-10


def test_relu_conv_chain_gradient_by_central_differences():
    """L(u) = <dy, conv(relu(u), w)>: dL/du = conv_bwd_data(dy, w) * [u > 0]; convolution is linear, so central
    differences are exact up to rounding as long as no element crosses zero (|u| >= 0.5, step 1e-3)."""
    a = Attrs(n=1, c=2, h=6, w=5, k=3, r=3, s=3, sh=1, sw=2, pbh=1, pbw=1, pah=1, paw=0)
    _, w, dy = _random_tensors(a)
    u = rng.uniform(0.5, 1.5, (a.n, a.c, a.h, a.w)) * rng.choice([-1.0, 1.0], (a.n, a.c, a.h, a.w))
    loss = lambda t: float((oracle.conv_fwd(a, np.maximum(t, 0.0), w) * dy).sum())
    grad = oracle.conv_bwd_data_relu(a, dy, w, np.maximum(u, 0.0))
    assert np.all(grad[u < 0] == 0)
    eps = 1e-3
    for idx in itertools.islice(np.ndindex(u.shape), 0, None, 7):
        up, dn = u.copy(), u.copy()
        up[idx] += eps; dn[idx] -= eps
        fd = (loss(up) - loss(dn)) / (2 * eps)
        assert abs(fd - grad[idx]) < 1e-9, (idx, fd, grad[idx])


# ---------------------------------------------------------------- P13 softmax and its backprop
def test_softmax_closed_forms():
    # constant rows -> 1/n whatever the constant (also where exp would overflow without the shift)
    for n in (1, 2, 7, 1000):
        for c in (0.0, -3.5, 800.0, -800.0):
            np.testing.assert_allclose(oracle.softmax(np.full((2, n), c)), np.full((2, n), 1.0 / n), rtol=1e-15)
    # two elements: the logistic function of the difference
    a, b = rng.normal(size=50) * 5, rng.normal(size=50) * 5
    y = oracle.softmax(np.stack([a, b], axis=-1))
    np.testing.assert_allclose(y[:, 0], 1.0 / (1.0 + np.exp(b - a)), rtol=1e-14)
    np.testing.assert_allclose(y[:, 1], 1.0 / (1.0 + np.exp(a - b)), rtol=1e-14)
    # arithmetic progression x_j = j t: geometric series, y_j = q^j (q - 1) / (q^n - 1), q = e^t
    n, t = 9, 0.37
    q = np.exp(t)
    np.testing.assert_allclose(oracle.softmax(t * np.arange(n)), q ** np.arange(n) * (q - 1) / (q ** n - 1), rtol=1e-13)
    # one dominant element
    x = np.array([0.0, 50.0, -2.0])
    y = oracle.softmax(x)
    assert abs(y[1] - 1.0) < 1e-20 + 2e-16 and abs(y[0] - np.exp(-50.0)) < 1e-30 and y.argmax() == 1


def test_softmax_matches_the_unshifted_definition_and_scipy():
    import scipy.special
    x = rng.normal(size=(6, 4, 33)) * 3
    direct = np.exp(x) / np.exp(x).sum(axis=-1, keepdims=True)           # no overflow at this magnitude
    np.testing.assert_allclose(oracle.softmax(x), direct, rtol=1e-13)
    np.testing.assert_allclose(oracle.softmax(x), scipy.special.softmax(x, axis=-1), rtol=1e-13)
    # the last axis is the one normalised, not another one
    assert not np.allclose(oracle.softmax(x), scipy.special.softmax(x, axis=1))
    big = rng.normal(size=(5, 100)) * 200 + 3000
    np.testing.assert_allclose(oracle.softmax(big), scipy.special.softmax(big, axis=-1), rtol=1e-12)


def test_softmax_invariants():
    x = rng.normal(size=(17, 301)) * 4
    y = oracle.softmax(x)
    np.testing.assert_allclose(y.sum(axis=-1), 1.0, rtol=1e-14)
    assert (y > 0).all() and (y < 1).all()
    np.testing.assert_allclose(oracle.softmax(x + rng.normal(size=(17, 1)) * 100), y, rtol=1e-11)     # shift invariance
    # order preserving, and ratios are exp of differences
    assert np.array_equal(np.argsort(x, axis=-1), np.argsort(y, axis=-1))
    np.testing.assert_allclose(y[:, 5] / y[:, 9], np.exp(x[:, 5] - x[:, 9]), rtol=1e-12)
    # rows are independent
    x2 = x.copy(); x2[3] += rng.normal(size=301)
    y2 = oracle.softmax(x2)
    assert np.array_equal(np.delete(y2, 3, axis=0), np.delete(y, 3, axis=0)) and not np.allclose(y2[3], y[3])


def test_softmax_bwd_is_the_transposed_jacobian_and_matches_central_differences():
    n = 6
    x = rng.normal(size=(3, n))
    y = oracle.softmax(x)
    dy = rng.normal(size=(3, n))
    dx = oracle.softmax_bwd(y, dy)
    for i in range(3):
        jac = np.diag(y[i]) - np.outer(y[i], y[i])                        # d y_j / d x_k
        np.testing.assert_allclose(dx[i], jac.T @ dy[i], rtol=1e-13, atol=1e-16)
    loss = lambda t: float((oracle.softmax(t) * dy).sum())
    eps = 1e-5
    for idx in np.ndindex(x.shape):
        up, dn = x.copy(), x.copy()
        up[idx] += eps; dn[idx] -= eps
        fd = (loss(up) - loss(dn)) / (2 * eps)
        assert abs(fd - dx[idx]) < 1e-9, (idx, fd, dx[idx])
    # a constant delta has no effect (rows of y sum to one), and dx rows sum to zero
    np.testing.assert_allclose(oracle.softmax_bwd(y, np.full_like(y, 2.5)), 0.0, atol=1e-15)
    np.testing.assert_allclose(dx.sum(axis=-1), 0.0, atol=1e-15)
    # hand-worked: y = (1/2, 1/2), dy = (1, 0): s = 1/2, dx = (1/4, -1/4)
    np.testing.assert_allclose(oracle.softmax_bwd(np.array([0.5, 0.5]), np.array([1.0, 0.0])), [0.25, -0.25], rtol=1e-15)


# ---------------------------------------------------------------- P14 convolution over three spatial axes
from oracle import Attrs3  # noqa: E402


def _rand3(a: Attrs3, g):
    O, P, Q = oracle.out_shape3(a)
    x = g.integers(-3, 4, size=(a.n, a.c, a.d, a.h, a.w)).astype(float)
    w = g.integers(-3, 4, size=(a.k, a.c, a.t, a.r, a.s)).astype(float)
    dy = g.integers(-3, 4, size=(a.n, a.k, O, P, Q)).astype(float)
    return x, w, dy


# (extent, taps, stride, dilation, pad below, pad above) of two active axes; the third has extent 1
_PAIR_CASES = [((7, 3, 1, 1, 1, 1), (6, 2, 2, 1, 0, 1)), ((9, 3, 2, 2, 2, 0), (8, 3, 1, 1, 0, 2)),
               ((5, 1, 1, 1, 0, 0), (11, 4, 3, 2, 3, 1))]


@pytest.mark.parametrize("axes", [(0, 1), (0, 2), (1, 2), (1, 0), (2, 0)])
@pytest.mark.parametrize("case", _PAIR_CASES)
def test_conv3d_on_two_axes_is_the_rank2_oracle(axes, case):
    """With one spatial axis of extent 1 (window 1, no padding) the rank-3 ops are the rank-2 ones on the
    other two axes, whichever pair that is and in either order: pins the stride / dilation / padding
    handling of each axis, per side, against the C oracle."""
    g = np.random.default_rng(7 + 10 * axes[0] + axes[1])
    ext, taps, st, dil, pb, pa = ([1] * 3 for _ in range(6))
    st, dil = [1] * 3, [1] * 3
    pb, pa = [0] * 3, [0] * 3
    for ax, (e, t_, s_, d_, b_, a_) in zip(axes, case):
        ext[ax], taps[ax], st[ax], dil[ax], pb[ax], pa[ax] = e, t_, s_, d_, b_, a_
    a3 = Attrs3(2, 3, ext[0], ext[1], ext[2], 4, taps[0], taps[1], taps[2], st[0], st[1], st[2],
                dil[0], dil[1], dil[2], pb[0], pb[1], pb[2], pa[0], pa[1], pa[2])
    (e0, t0, s0, d0, b0, p0), (e1, t1, s1, d1, b1, p1) = case
    a2 = Attrs(2, 3, e0, e1, 4, t0, t1, s0, s1, d0, d1, b0, b1, p0, p1)
    x, w, dy = _rand3(a3, g)
    # move the two active axes (in the order given) to the front of the spatial axes and drop the third
    idle = ({0, 1, 2} - set(axes)).pop()
    perm = [0, 1, 2 + axes[0], 2 + axes[1], 2 + idle]
    to2 = lambda v: np.transpose(v, perm)[..., 0]
    bias = g.integers(-5, 6, size=4).astype(float)
    assert oracle.out_shape3(a3)[axes[0]] == oracle.out_shape(a2)[0] and oracle.out_shape3(a3)[axes[1]] == oracle.out_shape(a2)[1]
    assert np.array_equal(to2(oracle.conv3d_fwd(a3, x, w, bias, True)), oracle.conv_fwd(a2, to2(x), to2(w), bias, True))
    assert np.array_equal(to2(oracle.conv3d_bwd_data(a3, dy, w)), oracle.conv_bwd_data(a2, to2(dy), to2(w)))
    assert np.array_equal(to2(oracle.conv3d_bwd_filters(a3, x, dy)), oracle.conv_bwd_filters(a2, to2(x), to2(dy)))


def _brute3(a: Attrs3, x, w, dy):
    """Scalar loops from the definition, with bounds tests instead of a padded copy."""
    O, P, Q = oracle.out_shape3(a)
    y = np.zeros((a.n, a.k, O, P, Q)); dx = np.zeros_like(x); dw = np.zeros_like(w)
    for n, k, o, p, q, c, t, r, s in itertools.product(range(a.n), range(a.k), range(O), range(P), range(Q),
                                                       range(a.c), range(a.t), range(a.r), range(a.s)):
        z, i, j = o * a.sd - a.pbd + t * a.dd, p * a.sh - a.pbh + r * a.dh, q * a.sw - a.pbw + s * a.dw
        if not (0 <= z < a.d and 0 <= i < a.h and 0 <= j < a.w):
            continue
        y[n, k, o, p, q] += x[n, c, z, i, j] * w[k, c, t, r, s]
        dx[n, c, z, i, j] += dy[n, k, o, p, q] * w[k, c, t, r, s]
        dw[k, c, t, r, s] += dy[n, k, o, p, q] * x[n, c, z, i, j]
    return y, dx, dw


_TINY3 = [Attrs3(1, 2, 4, 5, 3, 2, 2, 3, 2, 1, 2, 1, 2, 1, 1, 1, 0, 1, 0, 2, 0),
          Attrs3(2, 1, 5, 4, 6, 2, 3, 2, 3, 2, 1, 2, 1, 1, 2, 2, 1, 3, 1, 0, 2),
          Attrs3(1, 2, 3, 3, 3, 1, 3, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1)]


@pytest.mark.parametrize("a", _TINY3)
def test_conv3d_brute_force_tiny(a):
    g = np.random.default_rng(a.d * 100 + a.h * 10 + a.w)
    x, w, dy = _rand3(a, g)
    y, dx, dw = _brute3(a, x, w, dy)
    assert np.array_equal(oracle.conv3d_fwd(a, x, w), y)
    assert np.array_equal(oracle.conv3d_bwd_data(a, dy, w), dx)
    assert np.array_equal(oracle.conv3d_bwd_filters(a, x, dy), dw)
    O, P, Q = oracle.out_shape3(a)
    assert np.array_equal(oracle.conv3d_fwd_at(a, x, w, np.arange(y.size)), y.reshape(-1))
    assert np.array_equal(oracle.conv3d_bwd_data_at(a, dy, w, np.arange(dx.size)), dx.reshape(-1))
    assert np.array_equal(oracle.conv3d_bwd_filters_at(a, x, dy, np.arange(dw.size)), dw.reshape(-1))


def test_conv3d_single_channel_is_scipy_correlate():
    from scipy.signal import correlate
    g = np.random.default_rng(5)
    a = Attrs3(1, 1, 6, 7, 8, 1, 3, 2, 4)
    x, w, _ = _rand3(a, g)
    assert np.array_equal(oracle.conv3d_fwd(a, x, w)[0, 0], correlate(x[0, 0], w[0, 0], mode="valid", method="direct"))
    # full zero padding on both sides of every axis = scipy's "full" mode
    af = Attrs3(1, 1, 6, 7, 8, 1, 3, 2, 4, 1, 1, 1, 1, 1, 1, 2, 1, 3, 2, 1, 3)
    assert np.array_equal(oracle.conv3d_fwd(af, x, w)[0, 0], correlate(x[0, 0], w[0, 0], mode="full", method="direct"))


@pytest.mark.parametrize("a", [Attrs3(2, 3, 6, 5, 7, 4, 3, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1),
                               Attrs3(2, 3, 7, 6, 5, 4, 3, 2, 3, 2, 1, 2, 1, 2, 1, 1, 0, 2, 2, 1, 0)])
def test_conv3d_adjoint_identities(a):
    g = np.random.default_rng(11)
    x, w, dy = _rand3(a, g)
    ip = (oracle.conv3d_fwd(a, x, w) * dy).sum()
    assert ip == (x * oracle.conv3d_bwd_data(a, dy, w)).sum() == (w * oracle.conv3d_bwd_filters(a, x, dy)).sum()


def test_conv3d_closed_forms():
    # all ones, stride 1, one voxel of padding all round: y = C * (taps inside the volume)
    a = Attrs3(1, 2, 4, 4, 4, 1, 3, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1)
    y = oracle.conv3d_fwd(a, np.ones((1, 2, 4, 4, 4)), np.ones((1, 2, 3, 3, 3)))[0, 0]
    side = np.array([2, 3, 3, 2])
    assert np.array_equal(y, 2.0 * side[:, None, None] * side[None, :, None] * side[None, None, :])
    # an off-centre delta filter is a shift: no flip on any axis
    w = np.zeros((1, 1, 3, 3, 3)); w[0, 0, 2, 0, 1] = 1.0
    x = np.arange(4 * 4 * 4, dtype=float).reshape(1, 1, 4, 4, 4)
    a1 = Attrs3(1, 1, 4, 4, 4, 1, 3, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1)
    y = oracle.conv3d_fwd(a1, x, w)[0, 0]
    want = np.zeros((4, 4, 4)); want[:3, 1:, :] = x[0, 0, 1:, :3, :]
    assert np.array_equal(y, want)


# ------------------------------------------------------------------ P15: the error metric every parity assert goes through
def test_max_normalised_error_hand_vectors(oracle_mod):
    """e = max|got - ref| / max|ref| on vectors worked by hand; the gate itself must not let a broken result through."""
    o = oracle_mod
    # largest difference 0.5 (third element), largest |ref| 4 (the negative one): 0.5 / 4
    assert o.max_normalised_error([1.0, 2.0, 3.5, -4.0], [1.0, 2.0, 3.0, -4.0]) == 0.125
    # normalised by the reference's norm, not element by element: an error of 1 on the element 0 is 1 / 10
    assert o.max_normalised_error([1.0, 10.0], [0.0, 10.0]) == 0.1
    # not by the result's norm either
    assert o.max_normalised_error([100.0, 1.0], [0.0, 1.0]) == 100.0
    assert o.max_normalised_error(np.full((2, 3), 7.0), np.full((2, 3), 7.0)) == 0.0
    # sign matters: -x against x is an error of 2
    assert o.max_normalised_error([-3.0], [3.0]) == 2.0
    # tensors of any rank, compared element by element in place (a transposed result is an error)
    a = np.arange(6.0).reshape(2, 3)
    assert o.max_normalised_error(a, a) == 0.0
    assert o.max_normalised_error(np.ascontiguousarray(a.T).reshape(2, 3), a) == 2.0 / 5.0


def test_max_normalised_error_rejects_broken_results(oracle_mod):
    o = oracle_mod
    ref = np.array([1.0, -2.0, 0.5])
    for bad in (np.nan, np.inf, -np.inf):
        got = ref.copy()
        got[1] = bad
        e = o.max_normalised_error(got, ref)
        assert e == float("inf") and not (e <= 2e-2)
    # a non-finite reference is no licence either
    assert o.max_normalised_error(ref, np.array([1.0, np.nan, 0.5])) == float("inf")
    # zero reference: exact zeros pass, anything else is infinitely wrong
    assert o.max_normalised_error(np.zeros(4), np.zeros(4)) == 0.0
    assert o.max_normalised_error(np.array([0.0, 1e-30]), np.zeros(2)) == float("inf")
    # shapes must agree: no broadcasting of a short result against the reference
    with pytest.raises(ValueError):
        o.max_normalised_error(np.zeros(3), np.zeros((3, 1)))
    with pytest.raises(ValueError):
        o.max_normalised_error(np.zeros(1), np.zeros(4))
    assert o.max_normalised_error(np.zeros((0,)), np.zeros((0,))) == 0.0
