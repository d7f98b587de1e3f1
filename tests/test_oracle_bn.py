"""Pins of the oracle's batch normalization (current-minibatch statistics only)."""
import numpy as np
import pytest

from oracle import ops


def _data(seed, shape=(4, 5, 6, 7)):
    g = np.random.default_rng(seed)
    x = g.standard_normal(shape) * g.uniform(0.5, 3.0, size=(1, shape[1], 1, 1)) + g.uniform(-5, 5, size=(1, shape[1], 1, 1))
    gamma, beta = g.uniform(0.5, 1.5, shape[1]), g.standard_normal(shape[1])
    return g, x, gamma, beta


def test_statistics_and_invariants():
    g, x, gamma, beta = _data(0)
    eps = 2e-5
    y, mean, invstd = ops.bn_fwd(x, np.ones(5), np.zeros(5), eps)
    np.testing.assert_allclose(mean, x.mean(axis=(0, 2, 3)), atol=1e-13)
    var = x.var(axis=(0, 2, 3))  # numpy's default is the biased (divide by M) variance
    np.testing.assert_allclose(invstd, 1 / np.sqrt(var + eps), rtol=1e-13)
    # before the affine step: mean 0, variance var/(var+eps)
    np.testing.assert_allclose(y.mean(axis=(0, 2, 3)), 0, atol=1e-13)
    np.testing.assert_allclose(y.var(axis=(0, 2, 3)), var / (var + eps), rtol=1e-12)
    # affine step
    y2, _, _ = ops.bn_fwd(x, gamma, beta, eps)
    np.testing.assert_allclose(y2, y * gamma[None, :, None, None] + beta[None, :, None, None], atol=1e-13)
    # BN(a*x+b) = BN(x) for a > 0 when eps = 0
    y3, _, _ = ops.bn_fwd(3.0 * x - 7.0, gamma, beta, 0.0)
    y4, _, _ = ops.bn_fwd(x, gamma, beta, 0.0)
    np.testing.assert_allclose(y3, y4, atol=1e-11)


def test_residual_and_relu_composition():
    g, x, gamma, beta = _data(1)
    res = g.standard_normal(x.shape)
    plain, _, _ = ops.bn_fwd(x, gamma, beta, 1e-5)
    y, _, _ = ops.bn_fwd(x, gamma, beta, 1e-5, residual=res, relu=True)
    np.testing.assert_array_equal(y, np.maximum(plain + res, 0.0))
    y, _, _ = ops.bn_fwd(x, gamma, beta, 1e-5, relu=True)
    np.testing.assert_array_equal(y, np.maximum(plain, 0.0))
    y, _, _ = ops.bn_fwd(x, gamma, beta, 1e-5, residual=res)
    np.testing.assert_array_equal(y, plain + res)


@pytest.mark.parametrize("relu,use_res", [(False, False), (True, False), (True, True), (False, True)])
def test_backward_finite_differences(relu, use_res):
    g, x, gamma, beta = _data(2, (3, 4, 3, 5))
    eps = 1e-3
    res = g.standard_normal(x.shape) if use_res else None
    dy = g.standard_normal(x.shape)

    def loss(x_, gamma_, beta_, res_):
        y_, _, _ = ops.bn_fwd(x_, gamma_, beta_, eps, residual=res_, relu=relu)
        return np.sum(y_ * dy)

    y, mean, invstd = ops.bn_fwd(x, gamma, beta, eps, residual=res, relu=relu)
    dx, dres, dgamma, dbeta = ops.bn_bwd(x, dy, y, gamma, mean, invstd, relu=relu, want_dresidual=use_res)
    h = 1e-6
    for _ in range(12):
        i = tuple(g.integers(0, s) for s in x.shape)
        xp, xm = x.copy(), x.copy()
        xp[i] += h
        xm[i] -= h
        assert abs((loss(xp, gamma, beta, res) - loss(xm, gamma, beta, res)) / (2 * h) - dx[i]) < 1e-6
        if use_res:
            rp, rm = res.copy(), res.copy()
            rp[i] += h
            rm[i] -= h
            assert abs((loss(x, gamma, beta, rp) - loss(x, gamma, beta, rm)) / (2 * h) - dres[i]) < 1e-6
    for c in range(x.shape[1]):
        e = np.zeros(x.shape[1])
        e[c] = h
        assert abs((loss(x, gamma + e, beta, res) - loss(x, gamma - e, beta, res)) / (2 * h) - dgamma[c]) < 1e-6
        assert abs((loss(x, gamma, beta + e, res) - loss(x, gamma, beta - e, res)) / (2 * h) - dbeta[c]) < 1e-6


def test_backward_invariants():
    g, x, gamma, beta = _data(3)
    eps = 2e-5
    y, mean, invstd = ops.bn_fwd(x, gamma, beta, eps, relu=True)
    dy = g.standard_normal(x.shape)
    dx, _, dgamma, dbeta = ops.bn_bwd(x, dy, y, gamma, mean, invstd, relu=True)
    dz = dy * (y > 0)
    xhat = (x - mean[None, :, None, None]) * invstd[None, :, None, None]
    np.testing.assert_allclose(dbeta, dz.sum(axis=(0, 2, 3)), atol=1e-12)
    np.testing.assert_allclose(dgamma, (dz * xhat).sum(axis=(0, 2, 3)), atol=1e-12)
    # dx is orthogonal to the constant and to xhat within each channel
    np.testing.assert_allclose(dx.sum(axis=(0, 2, 3)), 0, atol=1e-11)
    # sum dx*xhat = gamma*invstd*dgamma*(1 - mean(xhat^2)) which is gamma*invstd*dgamma*eps*invstd^2
    np.testing.assert_allclose((dx * xhat).sum(axis=(0, 2, 3)), gamma * invstd * dgamma * eps * invstd**2, atol=1e-10)


def test_inference_mode_with_given_statistics():
    """Validation-side BN (Section 2: the last minibatch's statistics replace moving averages)."""
    # hand-worked: x = 1,2,3 with mean 2, variance 1 (invstd 1), gamma 2, beta 1 -> -1, 1, 3
    x = np.array([1.0, 2.0, 3.0]).reshape(3, 1, 1, 1)
    y = ops.bn_inference(x, [2.0], [1.0], [2.0], [1.0])
    np.testing.assert_array_equal(y.ravel(), [-1.0, 1.0, 3.0])
    np.testing.assert_array_equal(ops.bn_inference(x, [2.0], [1.0], [2.0], [1.0], residual=-x, relu=True).ravel(), [0.0, 0.0, 0.0])
    # with the batch's own statistics it is the training-mode forward
    g, x, gamma, beta = _data(5)
    res = g.standard_normal(x.shape)
    for residual, relu in ((None, False), (res, True)):
        y, mean, invstd = ops.bn_fwd(x, gamma, beta, 2e-5, residual=residual, relu=relu)
        np.testing.assert_allclose(ops.bn_inference(x, gamma, beta, mean, invstd, residual=residual, relu=relu), y, atol=1e-12)
    # other statistics: a per-channel affine map of the input, nothing else
    mean2, inv2 = g.standard_normal(5), g.uniform(0.5, 2.0, 5)
    y = ops.bn_inference(x, gamma, beta, mean2, inv2)
    c = 3
    np.testing.assert_allclose(y[:, c], gamma[c] * inv2[c] * x[:, c] + (beta[c] - gamma[c] * inv2[c] * mean2[c]), atol=1e-12)


def test_statistics_average_over_workers():
    g = np.random.default_rng(6)
    eps = 2e-5
    means, var = g.standard_normal((4, 7)), g.uniform(0.1, 3.0, (4, 7))
    inv = 1 / np.sqrt(var + eps)
    m, i = ops.bn_stats_average(means[:1], inv[:1], eps)          # one worker: unchanged
    np.testing.assert_allclose(m, means[0], atol=1e-15)
    np.testing.assert_allclose(i, inv[0], rtol=1e-12)
    m, i = ops.bn_stats_average(means, inv, eps)                  # arithmetic means of mean and of variance
    np.testing.assert_allclose(m, means.sum(axis=0) / 4, atol=1e-15)
    np.testing.assert_allclose(1 / (i * i) - eps, var.sum(axis=0) / 4, rtol=1e-11)
    # workers that saw the same statistics: the average is that statistic
    m, i = ops.bn_stats_average(np.repeat(means[:1], 3, axis=0), np.repeat(inv[:1], 3, axis=0), eps)
    np.testing.assert_allclose(i, inv[0], rtol=1e-12)
