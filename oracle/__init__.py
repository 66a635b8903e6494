"""CPU oracle for the per-GPU ResNet-50 SGD iteration -- TEST INFRASTRUCTURE ONLY.

numpy-facing wrappers around the plain-C definitions in rn50_oracle.c.  Each
wrapper works on float32 or float64 arrays (the dtype of its first array
argument selects the instantiation) and returns freshly allocated outputs.
Only tests, the smoke check and the benchmark's cpu_baseline leg import this
package; the HIP product path never does, and this package imports nothing
from the product.

Layouts: activations NHWC, filters KRSC, C-contiguous.
Paper passages followed: Sec. 2 (one training iteration per GPU), Sec. 2.1
(label smoothing), Sec. 3.2 (ResNet-50; FP16 forward/backward, FP32 optimizer,
batch normalisation from batch mean and batch squared mean, no moving average).
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None


def lib():
    global _LIB
    if _LIB is None:
        path = _build.build(force=False)
        _LIB = ctypes.CDLL(path)
        _LIB.oracle_round_binary16.restype = ctypes.c_double
        _LIB.oracle_round_binary16.argtypes = [ctypes.c_double]
        _LIB.oracle_max_threads.restype = ctypes.c_int
        _LIB.oracle_set_threads.argtypes = [ctypes.c_int]
        _LIB.oracle_set_threads.restype = None
    return _LIB


def max_threads():
    return int(lib().oracle_max_threads())


def set_threads(n):
    """OpenMP threads the oracle uses from now on (timing only; results do not depend on it)."""
    lib().oracle_set_threads(int(n))


def _sfx(a):
    if a.dtype == np.float32:
        return "_f32"
    if a.dtype == np.float64:
        return "_f64"
    raise TypeError("oracle works on float32 or float64 arrays, got %s" % a.dtype)


def _p(a):
    if a is None:
        return ctypes.c_void_p(0)
    assert a.flags["C_CONTIGUOUS"]
    return ctypes.c_void_p(a.ctypes.data)


def _c(a, dt):
    return np.ascontiguousarray(a, dtype=dt)


def _real(dt, v):
    return ctypes.c_float(v) if dt == np.float32 else ctypes.c_double(v)


def out_hw(h, w, r, s, stride, pad):
    return (h + 2 * pad - r) // stride + 1, (w + 2 * pad - s) // stride + 1


def conv_fwd(x, w, stride, pad):
    dt = x.dtype
    x = _c(x, dt); w = _c(w, dt)
    n, h, wd, c = x.shape
    k, r, s, c2 = w.shape
    assert c == c2
    p, q = out_hw(h, wd, r, s, stride, pad)
    y = np.empty((n, p, q, k), dt)
    getattr(lib(), "conv_fwd" + _sfx(x))(n, h, wd, c, k, r, s, stride, pad, _p(x), _p(w), _p(y))
    return y


def conv_dgrad(dy, w, x_shape, stride, pad):
    dt = dy.dtype
    dy = _c(dy, dt); w = _c(w, dt)
    n, h, wd, c = x_shape
    k, r, s, c2 = w.shape
    assert c == c2 and dy.shape == (n,) + out_hw(h, wd, r, s, stride, pad) + (k,)
    dx = np.empty((n, h, wd, c), dt)
    getattr(lib(), "conv_dgrad" + _sfx(dy))(n, h, wd, c, k, r, s, stride, pad, _p(dy), _p(w), _p(dx))
    return dx


def conv_wgrad(x, dy, w_shape, stride, pad):
    dt = x.dtype
    x = _c(x, dt); dy = _c(dy, dt)
    n, h, wd, c = x.shape
    k, r, s, c2 = w_shape
    assert c == c2 and dy.shape == (n,) + out_hw(h, wd, r, s, stride, pad) + (k,)
    dw = np.empty((k, r, s, c), dt)
    getattr(lib(), "conv_wgrad" + _sfx(x))(n, h, wd, c, k, r, s, stride, pad, _p(x), _p(dy), _p(dw))
    return dw


def bn_relu_fwd(x, gamma, beta, eps=1e-5, relu=True, residual=None):
    """x: [..., C].  Returns y, mean, invstd, sqmean."""
    dt = x.dtype
    x = _c(x, dt); gamma = _c(gamma, dt); beta = _c(beta, dt)
    if residual is not None:
        residual = _c(residual, dt)
        assert residual.shape == x.shape
    c = x.shape[-1]
    m = x.size // c
    y = np.empty_like(x)
    mean = np.empty(c, dt); invstd = np.empty(c, dt); sqmean = np.empty(c, dt)
    getattr(lib(), "bn_relu_fwd" + _sfx(x))(
        ctypes.c_long(m), c, ctypes.c_double(eps), int(bool(relu)),
        _p(x), _p(gamma), _p(beta), _p(residual), _p(y), _p(mean), _p(invstd), _p(sqmean))
    return y, mean, invstd, sqmean


def bn_relu_bwd(dy, x, y, gamma, mean, invstd, relu=True, want_dresidual=False):
    """Returns dx, dresidual (or None), dgamma, dbeta."""
    dt = dy.dtype
    dy = _c(dy, dt); x = _c(x, dt); y = _c(y, dt)
    gamma = _c(gamma, dt); mean = _c(mean, dt); invstd = _c(invstd, dt)
    c = x.shape[-1]
    m = x.size // c
    dx = np.empty_like(x)
    dres = np.empty_like(x) if want_dresidual else None
    dgamma = np.empty(c, dt); dbeta = np.empty(c, dt)
    getattr(lib(), "bn_relu_bwd" + _sfx(dy))(
        ctypes.c_long(m), c, int(bool(relu)), _p(dy), _p(x), _p(y), _p(gamma), _p(mean), _p(invstd),
        _p(dx), _p(dres), _p(dgamma), _p(dbeta))
    return dx, dres, dgamma, dbeta


# ---- batch normalisation split at the points where GPUs would exchange statistics (Sec. 3.2: "the communication
# to synchronize batch mean and batch squared mean was also conducted in FP32").  Plain numpy, double inside.
def bn_moments(x):
    """Per-channel (mean, mean of squares) over all rows of x [..., C]."""
    x2 = np.asarray(x, np.float64).reshape(-1, x.shape[-1])
    return x2.mean(axis=0).astype(x.dtype), (x2 * x2).mean(axis=0).astype(x.dtype)


def bn_relu_fwd_from_moments(x, gamma, beta, mean, sqmean, eps=1e-5, relu=True, residual=None):
    """y = gamma*(x-mean)*invstd + beta (+residual)(ReLU) with var = max(sqmean - mean^2, 0).  Returns y, invstd."""
    f = np.float64
    mean64, sq64 = np.asarray(mean, f), np.asarray(sqmean, f)
    invstd = 1.0 / np.sqrt(np.maximum(sq64 - mean64 * mean64, 0.0) + eps)
    y = np.asarray(gamma, f) * ((np.asarray(x, f) - mean64) * invstd) + np.asarray(beta, f)
    if residual is not None:
        y = y + np.asarray(residual, f)
    if relu:
        y = np.maximum(y, 0.0)
    return y.astype(x.dtype), invstd.astype(x.dtype)


def bn_bwd_sums(dy, x, y, mean, invstd, relu=True):
    """Per-channel (sum g, sum g*xhat) with g = dy*[y>0] if relu else dy."""
    f = np.float64
    c = x.shape[-1]
    g = np.asarray(dy, f).reshape(-1, c)
    if relu:
        g = g * (np.asarray(y).reshape(-1, c) > 0)
    xh = (np.asarray(x, f).reshape(-1, c) - np.asarray(mean, f)) * np.asarray(invstd, f)
    return g.sum(axis=0).astype(x.dtype), (g * xh).sum(axis=0).astype(x.dtype)


def bn_relu_bwd_from_sums(dy, x, y, gamma, mean, invstd, sum_g, sum_gxhat, total_rows, relu=True, want_dresidual=False):
    """dx = gamma*invstd*(g - sum_g/M - xhat*sum_gxhat/M) with M = total_rows (rows of ALL participants)."""
    f = np.float64
    g = np.asarray(dy, f)
    if relu:
        g = g * (np.asarray(y) > 0)
    xh = (np.asarray(x, f) - np.asarray(mean, f)) * np.asarray(invstd, f)
    dx = np.asarray(gamma, f) * np.asarray(invstd, f) * (g - np.asarray(sum_g, f) / total_rows - xh * np.asarray(sum_gxhat, f) / total_rows)
    return dx.astype(x.dtype), (g.astype(x.dtype) if want_dresidual else None)


def maxpool_fwd(x, r=3, stride=2, pad=1):
    dt = x.dtype
    x = _c(x, dt)
    n, h, w, c = x.shape
    p, q = out_hw(h, w, r, r, stride, pad)
    y = np.empty((n, p, q, c), dt)
    getattr(lib(), "maxpool_fwd" + _sfx(x))(n, h, w, c, r, stride, pad, _p(x), _p(y))
    return y


def maxpool_bwd(x, dy, r=3, stride=2, pad=1):
    dt = x.dtype
    x = _c(x, dt); dy = _c(dy, dt)
    n, h, w, c = x.shape
    assert dy.shape == (n,) + out_hw(h, w, r, r, stride, pad) + (c,)
    dx = np.empty_like(x)
    getattr(lib(), "maxpool_bwd" + _sfx(x))(n, h, w, c, r, stride, pad, _p(x), _p(dy), _p(dx))
    return dx


def avgpool_fwd(x):
    dt = x.dtype
    x = _c(x, dt)
    n, h, w, c = x.shape
    y = np.empty((n, c), dt)
    getattr(lib(), "avgpool_fwd" + _sfx(x))(n, h * w, c, _p(x), _p(y))
    return y


def avgpool_bwd(dy, hw):
    dt = dy.dtype
    dy = _c(dy, dt)
    n, c = dy.shape
    h, w = hw
    dx = np.empty((n, h, w, c), dt)
    getattr(lib(), "avgpool_bwd" + _sfx(dy))(n, h * w, c, _p(dy), _p(dx))
    return dx


def fc_fwd(a, wt, b):
    dt = a.dtype
    a = _c(a, dt); wt = _c(wt, dt); b = _c(b, dt)
    bsz, cin = a.shape
    cout = wt.shape[0]
    assert wt.shape == (cout, cin) and b.shape == (cout,)
    z = np.empty((bsz, cout), dt)
    getattr(lib(), "fc_fwd" + _sfx(a))(bsz, cin, cout, _p(a), _p(wt), _p(b), _p(z))
    return z


def fc_bwd(a, wt, dz):
    """Returns dWt, db, da."""
    dt = a.dtype
    a = _c(a, dt); wt = _c(wt, dt); dz = _c(dz, dt)
    bsz, cin = a.shape
    cout = wt.shape[0]
    dwt = np.empty((cout, cin), dt); db = np.empty(cout, dt); da = np.empty((bsz, cin), dt)
    getattr(lib(), "fc_bwd" + _sfx(a))(bsz, cin, cout, _p(a), _p(wt), _p(dz), _p(dwt), _p(db), _p(da))
    return dwt, db, da


def ls_xent_fwd_bwd(z, labels, eps=0.1, grad_scale=1.0):
    """Returns loss_mean (python float), loss_per_sample, dz."""
    dt = z.dtype
    z = _c(z, dt)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    b, k = z.shape
    assert labels.shape == (b,) and labels.min() >= 0 and labels.max() < k
    loss = np.empty(1, dt); per = np.empty(b, dt); dz = np.empty((b, k), dt)
    getattr(lib(), "ls_xent_fwd_bwd" + _sfx(z))(
        b, k, _p(z), _p(labels), ctypes.c_double(eps), ctypes.c_double(grad_scale), _p(loss), _p(per), _p(dz))
    return float(loss[0]), per, dz


def sgd_momentum_flat(g, w, v, lr, mu, wd, grad_scale=1.0, want_lowp=True):
    """Updates w and v IN PLACE.  Returns w rounded to binary16 (as w.dtype) or None."""
    dt = w.dtype
    assert g.dtype == dt and v.dtype == dt and w.flags["C_CONTIGUOUS"] and v.flags["C_CONTIGUOUS"]
    g = _c(g, dt)
    n = w.size
    lowp = np.empty(n, dt) if want_lowp else None
    getattr(lib(), "sgd_momentum_flat" + _sfx(w))(
        ctypes.c_size_t(n), _p(g), _real(dt, grad_scale), _p(w), _p(v), _p(lowp),
        _real(dt, lr), _real(dt, mu), _real(dt, wd))
    return lowp


def lars_momentum_flat(g, w, v, segments, lr, mu, wd, eta, eps, grad_scale=1.0, want_lowp=True):
    """LARS with momentum; segments = [(offset, count, use_lars), ...].  Updates w and v IN PLACE.
    Returns (w rounded to binary16 or None, per-segment rate)."""
    dt = w.dtype
    assert g.dtype == dt and v.dtype == dt and w.flags["C_CONTIGUOUS"] and v.flags["C_CONTIGUOUS"]
    g = _c(g, dt)
    nseg = len(segments)
    off = np.array([s[0] for s in segments], dtype=np.uint64)
    cnt = np.array([s[1] for s in segments], dtype=np.uint64)
    use = np.array([1 if s[2] else 0 for s in segments], dtype=np.int32)
    assert all(int(o) + int(c) <= w.size for o, c in zip(off, cnt))
    lowp = np.array(w, copy=True) if want_lowp else None
    rate = np.empty(nseg, dt)
    getattr(lib(), "lars_momentum_flat" + _sfx(w))(
        ctypes.c_size_t(nseg), _p(off), _p(cnt), _p(use), _p(g), _real(dt, grad_scale), _p(w), _p(v), _p(lowp),
        _real(dt, lr), _real(dt, mu), _real(dt, wd), _real(dt, eta), _real(dt, eps), _p(rate))
    return lowp, rate


def round_binary16(a):
    """Copy of a with every element rounded to the nearest binary16 value (ties to even)."""
    out = np.array(a, copy=True, order="C")
    getattr(lib(), "round_binary16" + _sfx(out))(ctypes.c_size_t(out.size), _p(out))
    return out
