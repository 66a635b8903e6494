"""Pins for the CPU oracle: closed forms, brute force written differently,
adjoint identities, finite differences, library routines (numpy matmul,
numpy float16).  None of these retypes the oracle's own loops."""
import math
import os

import numpy as np
import pytest

import oracle as O
from oracle import resnet50 as R

RNG = np.random.default_rng(1234)


def golden():
    out = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "closed_forms.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = line.split("=")
                out[k.strip()] = float(v)
    return out


# ------------------------------------------------------------------ fp16 rounding
def test_round_binary16_matches_numpy_float16():
    a = np.concatenate([
        RNG.standard_normal(20000) * 10.0 ** RNG.uniform(-9, 5, 20000),
        np.array([0.0, -0.0, 65504.0, 65519.9, 65520.0, 70000.0, -65520.0, 2.0 ** -24, 2.0 ** -25,
                  1.5 * 2.0 ** -25, 2.0 ** -14, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, np.inf, -np.inf])])
    with np.errstate(over="ignore"):
        want = a.astype(np.float16).astype(np.float64)
    got = O.round_binary16(a)
    assert np.array_equal(got, want)
    a32 = a.astype(np.float32)
    with np.errstate(over="ignore"):
        want32 = a32.astype(np.float16).astype(np.float32)
    assert np.array_equal(O.round_binary16(a32), want32)


# ------------------------------------------------------------------ conv fwd
def im2col_conv(x, w, stride, pad):
    """Independent structure: explicit patch matrix times filter matrix."""
    n, h, wd, c = x.shape
    k, r, s, _ = w.shape
    xp = np.zeros((n, h + 2 * pad, wd + 2 * pad, c), x.dtype)
    xp[:, pad:pad + h, pad:pad + wd] = x
    p, q = (h + 2 * pad - r) // stride + 1, (wd + 2 * pad - s) // stride + 1
    cols = np.empty((n, p, q, r, s, c), x.dtype)
    for i in range(p):
        for j in range(q):
            cols[:, i, j] = xp[:, i * stride:i * stride + r, j * stride:j * stride + s]
    return (cols.reshape(n * p * q, r * s * c) @ w.reshape(k, r * s * c).T).reshape(n, p, q, k)


CONV_CASES = [  # n,h,w,c,k,r,stride,pad
    (2, 7, 6, 3, 4, 3, 1, 1), (1, 9, 9, 2, 3, 3, 2, 1), (2, 8, 8, 5, 4, 1, 1, 0), (2, 8, 8, 5, 4, 1, 2, 0),
    (1, 15, 13, 3, 2, 7, 2, 3), (1, 5, 5, 2, 2, 3, 2, 1), (1, 6, 7, 1, 1, 3, 1, 0)]


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_fwd_vs_im2col(case):
    n, h, w, c, k, r, stride, pad = case
    x = RNG.standard_normal((n, h, w, c))
    f = RNG.standard_normal((k, r, r, c))
    assert np.allclose(O.conv_fwd(x, f, stride, pad), im2col_conv(x, f, stride, pad), rtol=1e-12, atol=1e-12)
    y32 = O.conv_fwd(x.astype(np.float32), f.astype(np.float32), stride, pad)
    assert y32.dtype == np.float32
    assert np.allclose(y32, im2col_conv(x, f, stride, pad), rtol=1e-5, atol=1e-5)


def test_conv_fwd_hand_example():
    # 1 channel 3x3 image, 2x2 filter, no padding: worked by hand.
    x = np.arange(1.0, 10.0).reshape(1, 3, 3, 1)
    f = np.array([1.0, 10.0, 100.0, 1000.0]).reshape(1, 2, 2, 1)
    y = O.conv_fwd(x, f, 1, 0)
    assert y.reshape(-1).tolist() == [5421.0, 6532.0, 8754.0, 9865.0]
    # pad 1, stride 2 -> taps hitting only x[0,0], x[0,2], x[2,0], x[2,2] via the last filter tap
    y2 = O.conv_fwd(x, f, 2, 1)
    assert y2.reshape(-1).tolist() == [1000.0, 100 * 2 + 1000 * 3, 10 * 4 + 1000 * 7, 1 * 5 + 10 * 6 + 100 * 8 + 1000 * 9]


def test_conv_fwd_special_cases():
    x = RNG.standard_normal((2, 6, 5, 4))
    # 1x1 stride 1 is a plain matmul
    f = RNG.standard_normal((7, 1, 1, 4))
    assert np.allclose(O.conv_fwd(x, f, 1, 0), (x.reshape(-1, 4) @ f.reshape(7, 4).T).reshape(2, 6, 5, 7))
    # delta filter reproduces the input
    d = np.zeros((4, 3, 3, 4))
    for c in range(4):
        d[c, 1, 1, c] = 1.0
    assert np.array_equal(O.conv_fwd(x, d, 1, 1), x)
    # shifted delta (tap r=0,s=2) reads x[h-1, w+1]
    d2 = np.zeros((4, 3, 3, 4))
    for c in range(4):
        d2[c, 0, 2, c] = 1.0
    y = O.conv_fwd(x, d2, 1, 1)
    assert np.array_equal(y[:, 1:, :-1], x[:, :-1, 1:]) and np.all(y[:, 0] == 0) and np.all(y[:, :, -1] == 0)
    # filter as large as the image, no padding: one dot product
    f2 = RNG.standard_normal((3, 6, 5, 4))
    x1 = x[:1]
    yy = O.conv_fwd(x1, f2, 1, 0)
    assert yy.shape == (1, 1, 1, 3)
    assert np.allclose(yy.reshape(-1), f2.reshape(3, -1) @ x1.reshape(-1))
    # linearity in x and in w
    xb = RNG.standard_normal(x.shape)
    fa, fb = RNG.standard_normal((5, 3, 3, 4)), RNG.standard_normal((5, 3, 3, 4))
    assert np.allclose(O.conv_fwd(2 * x - 3 * xb, fa, 2, 1), 2 * O.conv_fwd(x, fa, 2, 1) - 3 * O.conv_fwd(xb, fa, 2, 1))
    assert np.allclose(O.conv_fwd(x, fa + 0.5 * fb, 1, 1), O.conv_fwd(x, fa, 1, 1) + 0.5 * O.conv_fwd(x, fb, 1, 1))


# ------------------------------------------------------------------ dgrad / wgrad
def resnet50_unique_conv_shapes():
    net = R.Net(1, (224, 224))
    seen, out = set(), []
    hw = {"stem": 224}
    h = 56
    for b in net.block_list:
        n = b["name"]
        hw[n + "c1"] = h; hw[n + "c2"] = h; hw[n + "p"] = h
        h //= b["stride"]
        hw[n + "c3"] = h
    for name, cv in net.convs.items():
        key = (cv["cin"], cv["cout"], cv["r"], cv["stride"], cv["pad"], hw[name])
        if key not in seen:
            seen.add(key)
            out.append(key)
    return out


def test_resnet50_has_23_unique_conv_shapes_and_53_convs():
    assert len(R.Net(1, (224, 224)).convs) == 53
    assert len(resnet50_unique_conv_shapes()) == 23


@pytest.mark.parametrize("shape", resnet50_unique_conv_shapes())
def test_adjoint_identities_all_resnet_shapes(shape):
    """<conv(x,w),dy> = <x,dgrad(dy,w)> = <w,wgrad(x,dy)> with real channel counts, small images."""
    cin, cout, r, stride, pad, _ = shape
    h, w = (9, 8) if r > 1 else (4, 5)
    if cin * cout > 600000:
        h, w = 3, 2 if r == 1 else 3
    x = RNG.standard_normal((1, h, w, cin))
    f = RNG.standard_normal((cout, r, r, cin))
    y = O.conv_fwd(x, f, stride, pad)
    dy = RNG.standard_normal(y.shape)
    a = float(np.sum(y * dy))
    b = float(np.sum(x * O.conv_dgrad(dy, f, x.shape, stride, pad)))
    c = float(np.sum(f * O.conv_wgrad(x, dy, f.shape, stride, pad)))
    assert abs(a - b) <= 1e-10 * max(1.0, abs(a)) and abs(a - c) <= 1e-10 * max(1.0, abs(a))


@pytest.mark.parametrize("case", CONV_CASES)
def test_dgrad_wgrad_finite_differences(case):
    n, h, w, c, k, r, stride, pad = case
    x = RNG.standard_normal((n, h, w, c))
    f = RNG.standard_normal((k, r, r, c))
    dy = RNG.standard_normal(O.conv_fwd(x, f, stride, pad).shape)
    dx = O.conv_dgrad(dy, f, x.shape, stride, pad)
    dw = O.conv_wgrad(x, dy, f.shape, stride, pad)
    L = lambda xx, ff: float(np.sum(im2col_conv(xx, ff, stride, pad) * dy))   # noqa: E731
    for _ in range(6):
        i = tuple(RNG.integers(0, s) for s in x.shape)
        e = np.zeros_like(x); e[i] = 1e-4
        assert abs((L(x + e, f) - L(x - e, f)) / 2e-4 - dx[i]) < 1e-6
        j = tuple(RNG.integers(0, s) for s in f.shape)
        e = np.zeros_like(f); e[j] = 1e-4
        assert abs((L(x, f + e) - L(x, f - e)) / 2e-4 - dw[j]) < 1e-6


def test_dgrad_hand_example_stride2():
    # 1x1 stride-2 filter: dx is dy*w on the sampled pixels and exactly zero elsewhere
    dy = RNG.standard_normal((1, 2, 2, 3))
    f = RNG.standard_normal((3, 1, 1, 2))
    dx = O.conv_dgrad(dy, f, (1, 4, 4, 2), 2, 0)
    assert np.allclose(dx[:, ::2, ::2], dy @ f.reshape(3, 2))
    mask = np.ones((4, 4), bool); mask[::2, ::2] = False
    assert np.all(dx[0][mask] == 0)


# ------------------------------------------------------------------ batch norm
def test_bn_fwd_properties():
    m, c = 500, 6
    x = RNG.standard_normal((m, c)) * RNG.uniform(0.5, 3, c) + RNG.uniform(-2, 2, c)
    gamma, beta = RNG.uniform(0.5, 2, c), RNG.uniform(-1, 1, c)
    eps = 1e-5
    y, mean, invstd, sqmean = O.bn_relu_fwd(x, gamma, beta, eps, relu=False)
    assert np.allclose(mean, x.mean(0)) and np.allclose(sqmean, (x * x).mean(0))
    var = x.var(0)                                         # biased (ddof = 0)
    assert np.allclose(sqmean - mean ** 2, var) and np.all(sqmean - mean ** 2 >= 0)
    assert np.allclose(invstd, 1 / np.sqrt(var + eps))
    assert np.allclose(y.mean(0), beta) and np.allclose(y.var(0), gamma ** 2 * var / (var + eps))
    # constant input -> beta ; positive rescale leaves y unchanged up to eps
    yc, *_ = O.bn_relu_fwd(np.full((m, c), 3.25), gamma, beta, eps, relu=False)
    assert np.allclose(yc, beta)
    ys, *_ = O.bn_relu_fwd(7.0 * x, gamma, beta, eps, relu=False)
    assert np.allclose(ys, y, atol=1e-4)
    # residual and relu
    res = RNG.standard_normal((m, c))
    yr, *_ = O.bn_relu_fwd(x, gamma, beta, eps, relu=True, residual=res)
    assert np.allclose(yr, np.maximum(y + res, 0))
    # a channel whose mean is 100 sigma: two-pass variance stays exact
    xb = x.copy(); xb[:, 0] = 100.0 + RNG.standard_normal(m)
    _, mb, ib, _ = O.bn_relu_fwd(xb.astype(np.float32), gamma.astype(np.float32), beta.astype(np.float32), eps, False)
    assert abs(ib[0] - 1 / math.sqrt(xb[:, 0].astype(np.float32).astype(np.float64).var() + eps)) < 1e-5 * ib[0]


def bn_numpy(x, gamma, beta, eps, relu, res):
    mu, var = x.mean(0), x.var(0)
    y = gamma * (x - mu) / np.sqrt(var + eps) + beta
    if res is not None:
        y = y + res
    return np.maximum(y, 0) if relu else y


@pytest.mark.parametrize("relu,with_res", [(False, False), (True, False), (True, True)])
def test_bn_bwd_invariants_and_finite_differences(relu, with_res):
    m, c = 40, 3
    x = RNG.standard_normal((m, c)) + 0.3
    gamma, beta = RNG.uniform(0.5, 2, c), RNG.uniform(-0.5, 0.5, c)
    res = RNG.standard_normal((m, c)) if with_res else None
    eps = 1e-5
    y, mean, invstd, _ = O.bn_relu_fwd(x, gamma, beta, eps, relu, res)
    dy = RNG.standard_normal((m, c))
    dx, dres, dgamma, dbeta = O.bn_relu_bwd(dy, x, y, gamma, mean, invstd, relu, with_res)
    xhat = (x - mean) * invstd
    g = dy * (y > 0) if relu else dy
    assert np.allclose(dx.sum(0), 0, atol=1e-12)
    # sum dx*xhat vanishes up to the eps in invstd: it equals gamma*invstd*dgamma*(1 - mean(xhat^2))
    resid = gamma * invstd * (g * xhat).sum(0) * (1.0 - (xhat ** 2).mean(0))
    assert np.allclose((dx * xhat).sum(0), resid, atol=1e-12) and np.all(np.abs(resid) < 1e-3)
    assert np.allclose(dbeta, g.sum(0)) and np.allclose(dgamma, (g * xhat).sum(0))
    if with_res:
        assert np.array_equal(dres, g)
    L = lambda xx, gg, bb, rr: float(np.sum(bn_numpy(xx, gg, bb, eps, relu, rr) * dy))   # noqa: E731
    h = 1e-6
    for _ in range(8):
        i = (RNG.integers(0, m), RNG.integers(0, c))
        e = np.zeros_like(x); e[i] = h
        assert abs((L(x + e, gamma, beta, res) - L(x - e, gamma, beta, res)) / (2 * h) - dx[i]) < 1e-5
        if with_res:
            assert abs((L(x, gamma, beta, res + e) - L(x, gamma, beta, res - e)) / (2 * h) - dres[i]) < 1e-5
    for j in range(c):
        e = np.zeros(c); e[j] = h
        assert abs((L(x, gamma + e, beta, res) - L(x, gamma - e, beta, res)) / (2 * h) - dgamma[j]) < 1e-5
        assert abs((L(x, gamma, beta + e, res) - L(x, gamma, beta - e, res)) / (2 * h) - dbeta[j]) < 1e-5


# ------------------------------------------------------------------ pooling / FC
def test_maxpool_bruteforce_and_first_max_rule():
    x = RNG.standard_normal((2, 7, 6, 3))
    y = O.maxpool_fwd(x, 3, 2, 1)
    xp = np.full((2, 9, 8, 3), -np.inf); xp[:, 1:8, 1:7] = x
    want = np.stack([np.stack([xp[:, 2 * p:2 * p + 3, 2 * q:2 * q + 3].max(axis=(1, 2)) for q in range(3)], 1)
                     for p in range(4)], 1)
    assert np.array_equal(y, want)
    dy = RNG.standard_normal(y.shape)
    dx = O.maxpool_bwd(x, dy, 3, 2, 1)
    assert np.isclose(dx.sum(), dy.sum())
    assert np.all((dx != 0) <= np.isin(x, y))              # gradient only lands on window maxima
    # ties: all-equal input -> first in-bounds tap of each window (row-major) gets the gradient
    xt = np.zeros((1, 4, 4, 1)); dyt = np.arange(1.0, 5.0).reshape(1, 2, 2, 1)
    dxt = O.maxpool_bwd(xt, dyt, 3, 2, 1)[0, :, :, 0]
    want_t = np.zeros((4, 4)); want_t[0, 0] = 1; want_t[0, 1] = 2; want_t[1, 0] = 3; want_t[1, 1] = 4
    assert np.array_equal(dxt, want_t)
    # overlapping windows accumulate on a shared maximum
    xo = np.zeros((1, 4, 4, 1)); xo[0, 1, 1, 0] = 5.0
    dxo = O.maxpool_bwd(xo, np.ones((1, 2, 2, 1)), 3, 2, 1)[0, :, :, 0]
    assert dxo[1, 1] == 4.0 and dxo.sum() == 4.0


def test_avgpool_and_fc():
    x = RNG.standard_normal((3, 7, 7, 5))
    a = O.avgpool_fwd(x)
    assert np.allclose(a, x.mean(axis=(1, 2)))
    da = RNG.standard_normal((3, 5))
    dx = O.avgpool_bwd(da, (7, 7))
    assert np.allclose(dx, np.broadcast_to(da[:, None, None, :] / 49.0, x.shape))
    w, b = RNG.standard_normal((11, 5)), RNG.standard_normal(11)
    z = O.fc_fwd(a, w, b)
    assert np.allclose(z, a @ w.T + b)
    dz = RNG.standard_normal(z.shape)
    dw, db, da2 = O.fc_bwd(a, w, dz)
    assert np.allclose(dw, dz.T @ a) and np.allclose(db, dz.sum(0)) and np.allclose(da2, dz @ w)


# ------------------------------------------------------------------ loss
def test_ls_xent_closed_forms():
    gold = golden()
    k = 1000
    for eps in (0.0, 0.1, 0.3):
        loss, per, dz = O.ls_xent_fwd_bwd(np.full((4, k), 0.37), np.array([0, 5, 999, 17]), eps)
        assert abs(loss - gold["ln_1000"]) < 1e-12 and np.allclose(per, math.log(k))
    z = RNG.standard_normal((6, k)) * 3
    lab = RNG.integers(0, k, 6)
    # eps = 0 is ordinary cross-entropy
    p = np.exp(z - z.max(1, keepdims=True)); p /= p.sum(1, keepdims=True)
    loss0, per0, dz0 = O.ls_xent_fwd_bwd(z, lab, 0.0)
    assert np.allclose(per0, -np.log(p[np.arange(6), lab]))
    # smoothed targets recovered from the gradient: q = p - dz
    loss, per, dz = O.ls_xent_fwd_bwd(z, lab, 0.1)
    q = p - dz
    assert np.allclose(q.sum(1), 1.0)
    assert np.allclose(q[np.arange(6), lab], gold["q_true_eps0.1_K1000"])
    mask = np.ones_like(q, bool); mask[np.arange(6), lab] = False
    assert np.allclose(q[mask], gold["q_false_eps0.1_K1000"])
    assert np.allclose(per, -(q * np.log(p)).sum(1)) and abs(loss - per.mean()) < 1e-12
    assert np.allclose(dz.sum(1), 0, atol=1e-12)
    # shift invariance and grad_scale
    loss_s, _, dz_s = O.ls_xent_fwd_bwd(z + 123.0, lab, 0.1, grad_scale=0.25)
    assert abs(loss_s - loss) < 1e-10 and np.allclose(dz_s, 0.25 * dz)
    # large logits do not overflow
    lossb, _, _ = O.ls_xent_fwd_bwd((z * 1e3).astype(np.float32), lab, 0.1)
    assert np.isfinite(lossb)


def test_ls_xent_finite_differences():
    k = 12
    z = RNG.standard_normal((3, k))
    lab = np.array([1, 7, 11])
    _, per, dz = O.ls_xent_fwd_bwd(z, lab, 0.1)
    for i in range(3):
        for j in range(k):
            e = np.zeros_like(z); e[i, j] = 1e-6
            lp = O.ls_xent_fwd_bwd(z + e, lab, 0.1)[1].sum()
            lm = O.ls_xent_fwd_bwd(z - e, lab, 0.1)[1].sum()
            assert abs((lp - lm) / 2e-6 - dz[i, j]) < 1e-8


def test_bn_split_at_the_exchange_points_equals_whole_batch_bn():
    """Two "GPUs" with different local batches: averaging their (mean, mean of squares) weighted by rows and
    applying from those moments must reproduce batch norm over the union; adding their backward sums must
    reproduce its backward pass (both already pinned above)."""
    c = 16
    xa, xb = RNG.standard_normal((3, 5, 4, c)) * 2 + 1, RNG.standard_normal((2, 5, 4, c)) - 0.5
    gamma, beta = RNG.standard_normal(c), RNG.standard_normal(c)
    res = RNG.standard_normal((5, 5, 4, c))
    x = np.concatenate([xa, xb])
    y, mean, invstd, sqmean = O.bn_relu_fwd(x, gamma, beta, 1e-5, True, res)
    ma, qa = O.bn_moments(xa)
    mb, qb = O.bn_moments(xb)
    na, nb = xa.size // c, xb.size // c
    m_all, q_all = (ma * na + mb * nb) / (na + nb), (qa * na + qb * nb) / (na + nb)
    assert np.allclose(m_all, mean, rtol=1e-12, atol=1e-14) and np.allclose(q_all, sqmean, rtol=1e-12)
    ya, inv_a = O.bn_relu_fwd_from_moments(xa, gamma, beta, m_all, q_all, 1e-5, True, res[:3])
    yb, _ = O.bn_relu_fwd_from_moments(xb, gamma, beta, m_all, q_all, 1e-5, True, res[3:])
    assert np.allclose(np.concatenate([ya, yb]), y, rtol=1e-10, atol=1e-12) and np.allclose(inv_a, invstd, rtol=1e-10)
    dy = RNG.standard_normal(x.shape)
    dx, dres, dgamma, dbeta = O.bn_relu_bwd(dy, x, y, gamma, mean, invstd, True, True)
    sa = O.bn_bwd_sums(dy[:3], xa, y[:3], mean, invstd, True)
    sb = O.bn_bwd_sums(dy[3:], xb, y[3:], mean, invstd, True)
    sg, sgx = sa[0] + sb[0], sa[1] + sb[1]
    assert np.allclose(sg, dbeta, rtol=1e-10, atol=1e-12) and np.allclose(sgx, dgamma, rtol=1e-10, atol=1e-12)
    dxa, dra = O.bn_relu_bwd_from_sums(dy[:3], xa, y[:3], gamma, mean, invstd, sg, sgx, na + nb, True, True)
    dxb, drb = O.bn_relu_bwd_from_sums(dy[3:], xb, y[3:], gamma, mean, invstd, sg, sgx, na + nb, True, True)
    assert np.allclose(np.concatenate([dxa, dxb]), dx, rtol=1e-9, atol=1e-11)
    assert np.array_equal(np.concatenate([dra, drb]), dres)
    # without ReLU and residual
    y2, mean2, invstd2, _ = O.bn_relu_fwd(x, gamma, beta, 1e-5, False)
    ya2, _ = O.bn_relu_fwd_from_moments(xa, gamma, beta, m_all, q_all, 1e-5, False)
    assert np.allclose(ya2, y2[:3], rtol=1e-10, atol=1e-12)
    dx2 = O.bn_relu_bwd(dy, x, y2, gamma, mean2, invstd2, False)[0]
    s2 = O.bn_bwd_sums(dy, x, y2, mean2, invstd2, False)
    assert np.allclose(O.bn_relu_bwd_from_sums(dy, x, y2, gamma, mean2, invstd2, s2[0], s2[1], na + nb, False)[0], dx2, rtol=1e-9, atol=1e-11)


# ------------------------------------------------------------------ update
def test_sgd_closed_forms():
    n = 1000
    g, w0 = RNG.standard_normal(n), RNG.standard_normal(n)
    lr, mu, wd, s = 0.1, 0.9, 1e-4, 1 / 128.0
    w, v = w0.copy(), np.zeros(n)
    low = O.sgd_momentum_flat(g, w, v, lr, mu, wd, s)
    assert np.allclose(w, w0 - lr * (g * s + wd * w0), rtol=1e-14) and np.allclose(v, g * s + wd * w0, rtol=1e-14)
    assert np.array_equal(low, w.astype(np.float16).astype(np.float64))
    # wd = 0, constant g: geometric closed form after t steps
    w, v = w0.copy(), np.zeros(n)
    t = 25
    for _ in range(t):
        O.sgd_momentum_flat(g, w, v, lr, mu, 0.0, 1.0, want_lowp=False)
    assert np.allclose(v, g * (1 - mu ** t) / (1 - mu), rtol=1e-12)
    assert np.allclose(w, w0 - lr * g * (t / (1 - mu) - mu * (1 - mu ** t) / (1 - mu) ** 2), rtol=1e-11, atol=1e-12)
    # mu = 0 is plain SGD
    w, v = w0.copy(), RNG.standard_normal(n)
    O.sgd_momentum_flat(g, w, v, lr, 0.0, 0.0, 1.0, want_lowp=False)
    assert np.allclose(w, w0 - lr * g, rtol=1e-14)
    # fp32 instantiation agrees with fp64 to fp32 rounding
    w32, v32 = w0.astype(np.float32), np.zeros(n, np.float32)
    O.sgd_momentum_flat(g.astype(np.float32), w32, v32, lr, mu, wd, s)
    assert np.allclose(w32, w0 - lr * (g * s + wd * w0), rtol=1e-6, atol=1e-7)


def test_lars_worked_example_and_invariants():
    """LARS with momentum (Sec. 3.2, training configurations: coefficient 0.01, eps 1e-6, FP32)."""
    # worked by hand: w = (3,4) so ||w|| = 5, g = (1,0) so ||g|| = 1, wd = 0.2, eta = 0.01, eps = 0:
    #   rate = 0.01*5 / (1 + 0.2*5) = 0.025; g + wd*w = (1.6, 0.8); lr = 2, mu = 0.5, v0 = (1,1)
    #   v = 0.5*(1,1) + 2*0.025*(1.6,0.8) = (0.58, 0.54); w = (3,4) - v = (2.42, 3.46)
    w, v = np.array([3.0, 4.0]), np.array([1.0, 1.0])
    _, rate = O.lars_momentum_flat(np.array([1.0, 0.0]), w, v, [(0, 2, True)], 2.0, 0.5, 0.2, 0.01, 0.0)
    assert abs(rate[0] - 0.025) < 1e-15
    assert np.allclose(v, [0.58, 0.54], rtol=0, atol=1e-15) and np.allclose(w, [2.42, 3.46], rtol=0, atol=1e-15)
    # a gradient parallel to the weights: rate*(g + wd*w) = eta*||w||*g/||g||, whatever wd is
    for wd in (0.0, 0.1, 0.7):
        w, v = np.array([3.0, 4.0]), np.zeros(2)
        O.lars_momentum_flat(np.array([0.6, 0.8]), w, v, [(0, 2, True)], 2.0, 0.9, wd, 0.01, 0.0)
        assert np.allclose(v, 2.0 * 0.01 * 5.0 * np.array([0.6, 0.8]), rtol=1e-14)
    n = 4096
    g, w0 = RNG.standard_normal(n), RNG.standard_normal(n)
    segs = [(0, 1000, True), (1000, 24, False), (1024, 3072, True)]
    lr, mu, eta = 0.3, 0.9, 0.01
    # wd = 0, eps = 0, v = 0: the step of a LARS segment has length lr*eta*||w|| and does not depend on the
    # scale of the gradient; a plain segment takes lr*g (the momentum-SGD oracle with wd = 0 on its first step)
    ref = None
    for c in (1.0, 1e-3, 512.0):
        w, v = w0.copy(), np.zeros(n)
        O.lars_momentum_flat(g * c, w, v, segs, lr, mu, 0.0, eta, 0.0, want_lowp=False)
        for o, cnt, use in segs:
            if use:
                assert abs(np.linalg.norm(w[o:o + cnt] - w0[o:o + cnt]) / (lr * eta * np.linalg.norm(w0[o:o + cnt])) - 1) < 1e-12
        lars_part = np.concatenate([w[:1000], w[1024:]])
        ref = lars_part if ref is None else ref
        assert np.allclose(lars_part, ref, rtol=1e-11, atol=1e-13)
        ws, vs = w0[1000:1024].copy(), np.zeros(24)
        O.sgd_momentum_flat(g[1000:1024] * c, ws, vs, lr, mu, 0.0, 1.0, want_lowp=False)
        assert np.allclose(w[1000:1024], ws, rtol=1e-14)
    # grad_scale multiplies the gradient before anything else: same result as a pre-scaled gradient
    w1, v1, w2, v2 = w0.copy(), np.zeros(n), w0.copy(), np.zeros(n)
    O.lars_momentum_flat(g, w1, v1, segs, lr, mu, 1e-4, eta, 1e-6, grad_scale=1 / 64.0, want_lowp=False)
    O.lars_momentum_flat(g / 64.0, w2, v2, segs, lr, mu, 1e-4, eta, 1e-6, want_lowp=False)
    assert np.allclose(w1, w2, rtol=1e-13) and np.allclose(v1, v2, rtol=1e-13)
    # segments are independent of each other and of their order; elements outside every segment stay untouched
    w3, v3 = w0.copy(), np.zeros(n)
    low, rate = O.lars_momentum_flat(g / 64.0, w3, v3, [segs[2], segs[0]], lr, mu, 1e-4, eta, 1e-6)
    assert np.array_equal(w3[:1000], w2[:1000]) and np.array_equal(w3[1024:], w2[1024:])
    assert np.array_equal(w3[1000:1024], w0[1000:1024]) and np.all(v3[1000:1024] == 0)
    touched = np.r_[0:1000, 1024:n]
    assert np.array_equal(low[touched], w3[touched].astype(np.float16).astype(np.float64))
    # eps only matters when the norms are tiny: rate = eta*||w|| / (||g|| + wd*||w|| + eps)
    wt, vt = np.full(4, 1e-7), np.zeros(4)
    _, r = O.lars_momentum_flat(np.full(4, 2e-7), wt, vt, [(0, 4, True)], 1.0, 0.0, 0.0, 0.01, 1e-6)
    assert abs(r[0] - 0.01 * 2e-7 / (4e-7 + 1e-6)) < 1e-15
    # a zero gradient or zero weights switch the layer-wise scaling off (rate 1) instead of dividing by zero
    wz, vz = np.zeros(8), np.zeros(8)
    _, r = O.lars_momentum_flat(np.ones(8), wz, vz, [(0, 8, True)], 0.5, 0.0, 0.0, 0.01, 0.0)
    assert r[0] == 1.0 and np.allclose(wz, -0.5)
    wz, vz = np.ones(8), np.full(8, 2.0)
    _, r = O.lars_momentum_flat(np.zeros(8), wz, vz, [(0, 8, True)], 0.5, 0.5, 0.0, 0.01, 0.0)
    assert r[0] == 1.0 and np.allclose(vz, 1.0) and np.allclose(wz, 0.0)
    # fp32 instantiation agrees with fp64 to fp32 rounding
    w32, v32 = w0.astype(np.float32), np.zeros(n, np.float32)
    O.lars_momentum_flat((g / 64.0).astype(np.float32), w32, v32, segs, lr, mu, 1e-4, eta, 1e-6, want_lowp=False)
    assert np.allclose(w32, w2, rtol=2e-6, atol=1e-7)


def test_schedule_config_b_and_table3():
    """Values worked by hand from the printed formulas of configuration B and read off Table 3."""
    from oracle import schedule as S
    assert S.lr_b(0) == 0.2 and abs(S.lr_b(2.5) - 14.6) < 1e-12            # 0.2 + 28.8/2
    assert abs(S.lr_b(5) - 29 * (85 / 90) ** 2) < 1e-12                     # the warm-up ends just below 29
    assert abs(S.lr_b(5 - 1e-9) - 29.0) < 1e-6                              # ... which the warm-up reaches
    assert abs(S.lr_b(29.999999) - 29 * 4 / 9) < 1e-5 and abs(S.lr_b(30) - 50 * 4 / 9) < 1e-12   # base LR 29 -> 50 at epoch 30
    assert abs(S.lr_b(45) - 12.5) < 1e-12 and S.lr_b(90) == 0.0            # 50 * (1/2)^2
    assert abs(S.noise_scale_b(45) - 12.5 * 327680) < 1e-6                 # 32*1024/0.1 = 327680
    # the learning rate cancels: Momentum = 1 - 0.1*B/32768; B = 32K reproduces the 0.9 the noise scale is built on
    for e in (0.0, 3.0, 17.0, 60.0):
        assert abs(S.momentum_b(e, 32 * 1024) - 0.9) < 1e-12
        assert abs(S.momentum_b(e, 54 * 1024) - 0.83125) < 1e-12
        assert abs(S.momentum_b(e, 64 * 1024) - 0.8) < 1e-12
    assert S.batch(0, 10) == (32, 32768) and S.batch(0, 89) == (32, 32768)
    assert S.batch(1, 29.9) == (16, 34816) and S.batch(1, 30) == (32, 69632)
    assert S.batch(2, 0) == (16, 55296) and S.batch(2, 60) == (32, 55296)
    assert S.batch(3, 29) == (16, 55296) and S.batch(3, 31) == (32, 65536)
    assert [S.batch(4, e) for e in (0, 30, 44.9, 45, 74.9, 75, 90)] == [
        (16, 34816), (16, 69632), (16, 69632), (32, 87040), (32, 87040), (32, 121856), (32, 121856)]
    # 3456 workers x 16 = 54K, 2176 x 16 = 34K (the #GPUs column of the same table)
    assert 3456 * 16 == S.batch(2, 0)[1] and 2176 * 16 == S.batch(1, 0)[1] and 2176 * 32 == S.batch(1, 40)[1]


# ------------------------------------------------------------------ layout + whole step
def test_flat_layout_counts():
    gold = golden()
    net = R.Net(32, (224, 224))
    assert net.param_count == gold["resnet50_param_count"]
    by = lambda kinds: sum(s.count for s in net.segments if s.kind in kinds)   # noqa: E731
    assert by((R.KIND_CONV,)) == gold["resnet50_conv_params"]
    assert by((R.KIND_GAMMA, R.KIND_BETA)) == gold["resnet50_bn_params"]
    assert by((R.KIND_FCW, R.KIND_FCB)) == gold["resnet50_fc_params"]
    assert all(s.offset % 8 == 0 for s in net.segments) and net.segments[-1].kind == R.KIND_FCB
    off = 0
    for s in net.segments:
        assert s.offset == off
        off += s.count
    assert abs((556522 / 1024) / (2565 / 4) - gold["table6_eff_1024"]) < 5e-5


def tiny_net_and_inputs(has_stem):
    from paper_1811_05233_amd import synth
    if has_stem:
        net = R.Net(2, (16, 16), True, (1, 1), base_width=8, classes=10)
        x = synth.normal_f16(1, (2, 16, 16, 3)).astype(np.float64)
    else:
        net = R.Net(2, (6, 6), False, (1,), base_width=8, classes=10)
        x = synth.normal_f16(1, (2, 6, 6, 8)).astype(np.float64)
    w = synth.flat_params(3, [(s.kind, s.offset, s.count, s.fan_in) for s in net.segments]).astype(np.float64)
    # make BN affine and FC bias non-trivial so their gradients are exercised
    r = np.random.default_rng(5)
    for s in net.segments:
        if s.kind in (R.KIND_GAMMA, R.KIND_BETA, R.KIND_FCB):
            w[s.offset:s.offset + s.count] += 0.2 * r.standard_normal(s.count)
    lab = synth.labels(2, 2, 10)
    return net, x, lab, w


@pytest.mark.parametrize("has_stem", [False, True])
def test_step_ref_gradient_finite_differences(has_stem):
    net, x, lab, w = tiny_net_and_inputs(has_stem)
    v = np.zeros_like(w)
    kw = dict(lr=0.1, mu=0.9, wd=1e-4, lowp=False, dtype=np.float64)
    out = R.step_ref(net, x, lab, w, v, **kw)
    r = np.random.default_rng(11)
    idx = [int(s.offset + r.integers(0, s.count)) for s in net.segments]
    h = 1e-5
    worst = 0.0
    for i in idx:
        e = np.zeros_like(w); e[i] = h
        lp = R.step_ref(net, x, lab, w + e, v, update=False, **kw)["loss"]
        lm = R.step_ref(net, x, lab, w - e, v, update=False, **kw)["loss"]
        fd = (lp - lm) / (2 * h)
        worst = max(worst, abs(fd - out["grad"][i]) / max(1e-3, abs(fd)))
    assert worst < 2e-4, worst
    # determinism and update formula
    out2 = R.step_ref(net, x, lab, w, v, **kw)
    assert out2["loss"] == out["loss"] and np.array_equal(out2["grad"], out["grad"])
    assert np.allclose(out["w"], w - 0.1 * (out["grad"] + 1e-4 * w), rtol=1e-13)
    # a small step on the same batch lowers the loss
    small = R.step_ref(net, x, lab, w, v, lr=0.01, mu=0.9, wd=0.0, lowp=False, dtype=np.float64)
    again = R.step_ref(net, x, lab, small["w"], v, update=False, **kw)
    assert again["loss"] < out["loss"]


def test_step_ref_lowp_close_to_exact_and_loss_scale_consistent():
    net, x, lab, w = tiny_net_and_inputs(True)
    v = np.zeros_like(w)
    ex = R.step_ref(net, x, lab, w, v, 0.1, 0.9, 1e-4, lowp=False)
    lo = R.step_ref(net, x, lab, w, v, 0.1, 0.9, 1e-4, lowp=True, loss_scale=128.0)
    assert abs(lo["loss"] - ex["loss"]) < 2e-2 * ex["loss"]
    gl, ge = lo["grad"] / 128.0, ex["grad"]
    assert np.linalg.norm(gl - ge) < 5e-2 * np.linalg.norm(ge)
    lo32 = R.step_ref(net, x.astype(np.float32), lab, w.astype(np.float32), v.astype(np.float32), 0.1, 0.9, 1e-4,
                      lowp=True, loss_scale=128.0, dtype=np.float32)
    assert abs(lo32["loss"] - lo["loss"]) < 1e-3
