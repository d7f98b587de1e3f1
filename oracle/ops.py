"""numpy-facing wrappers of the C oracle (fp64, logical NCHW / KCRS).

Test infrastructure only: imported by tests/, the smoke check and the cpu_baseline
leg of the benchmark.  Inputs of any float dtype are promoted exactly to float64.
"""
import ctypes as C

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.build())
        _lib.orc_softmax_ce.restype = C.c_double
        for f in ("orc_alpha_sgd", "orc_alpha_sgd_transition", "orc_alpha_rmsprop", "orc_lr_base", "orc_lr_slow_start"):
            getattr(_lib, f).restype = C.c_double
    return _lib


def _d(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def num_threads():
    return int(lib().orc_num_threads())


def out_size(h, r, stride, pad):
    return (h + 2 * pad - r) // stride + 1


def conv2d_fwd(x, w, stride, pad):
    x, w = _d(x), _d(w)
    n, c, h, ww = x.shape
    k, c2, r, s = w.shape
    assert c == c2
    y = np.empty((n, k, out_size(h, r, stride, pad), out_size(ww, s, stride, pad)))
    lib().orc_conv2d_fwd(n, c, h, ww, k, r, s, stride, pad, _p(x), _p(w), _p(y))
    return y


def conv2d_bwd_data(dy, w, stride, pad, h, ww):
    dy, w = _d(dy), _d(w)
    n, k = dy.shape[:2]
    k2, c, r, s = w.shape
    assert k == k2 and dy.shape[2] == out_size(h, r, stride, pad) and dy.shape[3] == out_size(ww, s, stride, pad)
    dx = np.empty((n, c, h, ww))
    lib().orc_conv2d_bwd_data(n, c, h, ww, k, r, s, stride, pad, _p(dy), _p(w), _p(dx))
    return dx


def conv2d_bwd_weight(x, dy, r, s, stride, pad):
    x, dy = _d(x), _d(dy)
    n, c, h, ww = x.shape
    k = dy.shape[1]
    assert dy.shape == (n, k, out_size(h, r, stride, pad), out_size(ww, s, stride, pad))
    dw = np.empty((k, c, r, s))
    lib().orc_conv2d_bwd_weight(n, c, h, ww, k, r, s, stride, pad, _p(x), _p(dy), _p(dw))
    return dw


def bn_fwd(x, gamma, beta, eps, residual=None, relu=False):
    x, gamma, beta = _d(x), _d(gamma), _d(beta)
    residual = _d(residual) if residual is not None else None
    n, c, h, w = x.shape
    y = np.empty_like(x)
    mean, invstd = np.empty(c), np.empty(c)
    lib().orc_bn_fwd(n, c, h, w, _p(x), _p(gamma), _p(beta), C.c_double(eps), _p(residual), int(relu),
                     _p(y), _p(mean), _p(invstd))
    return y, mean, invstd


def bn_bwd(x, dy, y, gamma, mean, invstd, relu=False, want_dresidual=False):
    x, dy, gamma, mean, invstd = _d(x), _d(dy), _d(gamma), _d(mean), _d(invstd)
    y = _d(y) if y is not None else None
    assert not relu or y is not None
    n, c, h, w = x.shape
    dx = np.empty_like(x)
    dres = np.empty_like(x) if want_dresidual else None
    dgamma, dbeta = np.empty(c), np.empty(c)
    lib().orc_bn_bwd(n, c, h, w, _p(x), _p(dy), _p(y), _p(gamma), _p(mean), _p(invstd), int(relu),
                     _p(dx), _p(dres), _p(dgamma), _p(dbeta))
    return dx, dres, dgamma, dbeta


def bn_inference(x, gamma, beta, mean, invstd, residual=None, relu=False):
    """BN forward with GIVEN statistics (validation side, Section 2: the last minibatch's statistics, averaged over the
    workers, are used instead of moving averages): y = gamma*(x - mean)*invstd + beta [+ residual] [ReLU].
    x: N x C x H x W; the per-channel vectors have C entries."""
    x = _d(x)
    bc = lambda v: _d(v)[None, :, None, None]
    y = bc(gamma) * (x - bc(mean)) * bc(invstd) + bc(beta)
    if residual is not None:
        y = y + _d(residual)
    return np.maximum(y, 0.0) if relu else y


def bn_stats_average(means, invstds, eps):
    """Average over the workers of the last minibatch's per-channel mean and variance (Section 2; the all-reduce before
    validation).  means, invstds: n_sets x C, with invstd = 1/sqrt(var + eps) as the training forward saves it.
    Returns (mean, invstd) of the averaged mean and the averaged (biased) variance."""
    means, invstds = _d(means), _d(invstds)
    var = 1.0 / (invstds * invstds) - eps
    return means.mean(axis=0), 1.0 / np.sqrt(var.mean(axis=0) + eps)


def maxpool_fwd(x, r=3, stride=2, pad=1):
    x = _d(x)
    n, c, h, w = x.shape
    p, q = out_size(h, r, stride, pad), out_size(w, r, stride, pad)
    y = np.empty((n, c, p, q))
    arg = np.empty((n, c, p, q), dtype=np.int32)
    lib().orc_maxpool_fwd(n, c, h, w, r, stride, pad, _p(x), _p(y), _p(arg))
    return y, arg


def maxpool_bwd(dy, arg, h, w, r=3, stride=2, pad=1):
    dy = _d(dy)
    arg = np.ascontiguousarray(arg, dtype=np.int32)
    n, c = dy.shape[:2]
    dx = np.empty((n, c, h, w))
    lib().orc_maxpool_bwd(n, c, h, w, r, stride, pad, _p(dy), _p(arg), _p(dx))
    return dx


def avgpool_fwd(x):
    x = _d(x)
    n, c, h, w = x.shape
    y = np.empty((n, c))
    lib().orc_avgpool_fwd(n, c, h, w, _p(x), _p(y))
    return y


def avgpool_bwd(dy, h, w):
    dy = _d(dy)
    n, c = dy.shape
    dx = np.empty((n, c, h, w))
    lib().orc_avgpool_bwd(n, c, h, w, _p(dy), _p(dx))
    return dx


def fc_fwd(f, w, b):
    f, w, b = _d(f), _d(w), _d(b)
    n, j = f.shape
    k = w.shape[0]
    y = np.empty((n, k))
    lib().orc_fc_fwd(n, j, k, _p(f), _p(w), _p(b), _p(y))
    return y


def fc_bwd(f, w, dy):
    f, w, dy = _d(f), _d(w), _d(dy)
    n, j = f.shape
    k = w.shape[0]
    df, dw, db = np.empty((n, j)), np.empty((k, j)), np.empty(k)
    lib().orc_fc_bwd(n, j, k, _p(f), _p(w), _p(dy), _p(df), _p(dw), _p(db))
    return df, dw, db


def softmax_ce(logits, labels, want_grad=True):
    logits = _d(logits)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    n, k = logits.shape
    assert labels.shape == (n,) and labels.min() >= 0 and labels.max() < k
    dl = np.empty_like(logits) if want_grad else None
    loss = lib().orc_softmax_ce(n, k, _p(logits), _p(labels), _p(dl))
    return loss, dl


def grad_pack_fp16(g):
    g = np.ascontiguousarray(g, dtype=np.float32)
    out = np.empty(g.shape, dtype=np.uint16)
    lib().orc_grad_pack_fp16(C.c_size_t(g.size), _p(g), _p(out))
    return out


def grad_unpack_fp16(h16, scale):
    h16 = np.ascontiguousarray(h16, dtype=np.uint16)
    g = np.empty(h16.shape, dtype=np.float64)
    lib().orc_grad_unpack_fp16(C.c_size_t(h16.size), _p(h16), C.c_double(scale), _p(g))
    return g


def opt_update(theta, delta, m, g, eta, mu1, mu2, eps, a_sgd, a_rms, wd=0.0, decay=None):
    """Returns new (theta, delta, m) as float64 arrays; inputs are not modified."""
    theta, delta, m = _d(theta).copy(), _d(delta).copy(), _d(m).copy()
    g = _d(g)
    if decay is not None:
        decay = np.ascontiguousarray(decay, dtype=np.uint8)
        assert decay.size == theta.size
    lib().orc_opt_update(C.c_size_t(theta.size), _p(theta), _p(delta), _p(m), _p(g), _p(decay),
                         C.c_double(eta), C.c_double(mu1), C.c_double(mu2), C.c_double(eps),
                         C.c_double(a_sgd), C.c_double(a_rms), C.c_double(wd))
    return theta, delta, m


def alpha_sgd(epoch, center=10.0, period=5.0, as_printed=False):
    return lib().orc_alpha_sgd(C.c_double(epoch), C.c_double(center), C.c_double(period), int(as_printed))


def alpha_sgd_transition(epoch, kind, center=10.0, period=5.0):
    """Appendix A.1's rejected transition functions (1 linear, 2 sigmoid, 3 sudden switch; 0 = the paper's own)."""
    return lib().orc_alpha_sgd_transition(C.c_double(epoch), C.c_double(center), C.c_double(period), int(kind))


def alpha_rmsprop(a_sgd, eta_rmsprop=3e-4, eta_sgd=6.4):
    return lib().orc_alpha_rmsprop(C.c_double(a_sgd), C.c_double(eta_rmsprop), C.c_double(eta_sgd))


def lr_base(n_workers, b_local):
    return lib().orc_lr_base(int(n_workers), int(b_local))


def lr_slow_start(epoch, n_workers=1024, b_local=32):
    return lib().orc_lr_slow_start(C.c_double(epoch), int(n_workers), int(b_local))
