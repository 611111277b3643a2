"""Pins of the training-mode BatchNorm oracle (oracle/bn_oracle.py) against what the mathematics fixes."""
import numpy as np
import pytest

from oracle import bn_oracle as bno


def rnd(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_statistics_of_arithmetic_progressions_closed_form():
    """Channel c holds a + d*i, i = 0..N-1 (in any order): mean = a + d(N-1)/2, biased variance = d^2 (N^2-1)/12."""
    B, C, T = 3, 4, 10
    n = B * T
    z = np.empty((B, C, T))
    a, d = np.array([0.0, 1.5, -2.0, 7.0]), np.array([1.0, 0.25, -3.0, 0.5])
    perm = np.random.default_rng(0).permutation(n)
    for c in range(C):
        z[:, c, :] = (a[c] + d[c] * perm).reshape(B, T)
    y, mean, invstd = bno.bn_train_fwd(z, np.ones(C), np.zeros(C), 0.0)
    np.testing.assert_allclose(mean, a + d * (n - 1) / 2, rtol=1e-13)
    np.testing.assert_allclose(1.0 / invstd ** 2, d * d * (n * n - 1) / 12.0, rtol=1e-12)
    # the normalised progression is the same for every channel up to the sign of d
    np.testing.assert_allclose(y[:, 0, :], np.sign(d[2]) * y[:, 2, :], atol=1e-12)


def test_normalised_values_have_zero_mean_and_known_variance():
    z = 3.0 * rnd((4, 5, 33), 1) + 2.0
    eps = 1e-3
    y, mean, invstd = bno.bn_train_fwd(z, np.ones(5), np.zeros(5), eps)
    var = z.var(axis=(0, 2))
    np.testing.assert_allclose(y.mean(axis=(0, 2)), 0.0, atol=1e-13)
    np.testing.assert_allclose(y.var(axis=(0, 2)), var / (var + eps), rtol=1e-12)
    np.testing.assert_allclose(mean, z.mean(axis=(0, 2)), rtol=1e-13)
    # gamma, beta, residual enter linearly after the normalisation
    g, b, r = rnd(5, 2), rnd(5, 3), rnd(z.shape, 4)
    y2, _, _ = bno.bn_train_fwd(z, g, b, eps, residual=r)
    np.testing.assert_allclose(y2, g[None, :, None] * y + b[None, :, None] + r, rtol=1e-13, atol=1e-13)
    y3, _, _ = bno.bn_train_fwd(z, g, b, eps, residual=r, relu=True)
    np.testing.assert_array_equal(y3, np.maximum(y2, 0.0))


def test_affine_invariance_without_eps():
    """z -> a*z + b per channel (a > 0) does not change the normalised values when eps = 0."""
    z = rnd((2, 3, 17), 5)
    a, b = np.array([0.5, 2.0, 7.0]), np.array([1.0, -3.0, 0.25])
    y0, _, _ = bno.bn_train_fwd(z, np.ones(3), np.zeros(3), 0.0)
    y1, _, _ = bno.bn_train_fwd(a[None, :, None] * z + b[None, :, None], np.ones(3), np.zeros(3), 0.0)
    np.testing.assert_allclose(y1, y0, rtol=1e-11, atol=1e-12)


def loss_and_grads(z, gamma, beta, eps, res, relu, G):
    y, mean, invstd = bno.bn_train_fwd(z, gamma, beta, eps, res, relu)
    dz, dres, dgamma, dbeta = bno.bn_train_bwd(G, z, y, gamma, mean, invstd, relu)
    return float((G * y).sum()), dz, dres, dgamma, dbeta


@pytest.mark.parametrize("relu", [False, True])
def test_finite_differences_through_the_statistics(relu):
    B, C, T = 2, 3, 7
    z, gamma, beta = rnd((B, C, T), 6), 1.0 + 0.3 * rnd(C, 7), 0.2 * rnd(C, 8)
    res, G = rnd((B, C, T), 9), rnd((B, C, T), 10)
    eps = 1e-2
    y, _, _ = bno.bn_train_fwd(z, gamma, beta, eps, res, False)
    assert np.abs(y).min() > 1e-3  # no point next to the ReLU kink (fixed seeds)
    L0, dz, dres, dgamma, dbeta = loss_and_grads(z, gamma, beta, eps, res, relu, G)
    h = 1e-6

    def fd(arr, idx):
        ap, am = arr.copy(), arr.copy()
        ap[idx] += h
        am[idx] -= h
        return ap, am

    for idx in [(0, 0, 0), (1, 2, 6), (0, 1, 3), (1, 0, 5)]:
        zp, zm = fd(z, idx)
        num = (loss_and_grads(zp, gamma, beta, eps, res, relu, G)[0] - loss_and_grads(zm, gamma, beta, eps, res, relu, G)[0]) / (2 * h)
        assert abs(num - dz[idx]) <= 1e-6 * (1 + abs(num)), (idx, num, dz[idx])
        rp, rm = fd(res, idx)
        num = (loss_and_grads(z, gamma, beta, eps, rp, relu, G)[0] - loss_and_grads(z, gamma, beta, eps, rm, relu, G)[0]) / (2 * h)
        assert abs(num - dres[idx]) <= 1e-6 * (1 + abs(num))
    for c in range(C):
        gp, gm = fd(gamma, (c,))
        num = (loss_and_grads(z, gp, beta, eps, res, relu, G)[0] - loss_and_grads(z, gm, beta, eps, res, relu, G)[0]) / (2 * h)
        assert abs(num - dgamma[c]) <= 1e-6 * (1 + abs(num))
        bp, bm = fd(beta, (c,))
        num = (loss_and_grads(z, gamma, bp, eps, res, relu, G)[0] - loss_and_grads(z, gamma, bm, eps, res, relu, G)[0]) / (2 * h)
        assert abs(num - dbeta[c]) <= 1e-6 * (1 + abs(num))


def test_backward_orthogonality_identities():
    """dz carries no component along the constant and along zhat in any channel."""
    z, G = rnd((3, 4, 21), 11), rnd((3, 4, 21), 12)
    gamma, beta = 1.0 + 0.2 * rnd(4, 13), rnd(4, 14)
    eps = 0.0
    y, mean, invstd = bno.bn_train_fwd(z, gamma, beta, eps, None, True)
    dz, dres, dgamma, dbeta = bno.bn_train_bwd(G, z, y, gamma, mean, invstd, True)
    zhat = (z - mean[None, :, None]) * invstd[None, :, None]
    np.testing.assert_allclose(dz.sum(axis=(0, 2)), 0.0, atol=1e-12)
    np.testing.assert_allclose((dz * zhat).sum(axis=(0, 2)), 0.0, atol=1e-11)
    np.testing.assert_array_equal(dres, np.where(y > 0, G, 0.0))


def test_against_torch_float64_batch_norm_with_autograd():
    import torch
    import torch.nn.functional as F
    B, C, T = 3, 5, 19
    z, res, G = rnd((B, C, T), 15), rnd((B, C, T), 16), rnd((B, C, T), 17)
    gamma, beta, eps = 1.0 + 0.3 * rnd(C, 18), 0.1 * rnd(C, 19), 1e-3
    zt = torch.tensor(z, requires_grad=True)
    gt, bt = torch.tensor(gamma, requires_grad=True), torch.tensor(beta, requires_grad=True)
    rt = torch.tensor(res, requires_grad=True)
    yt = torch.relu(F.batch_norm(zt, None, None, gt, bt, training=True, momentum=0.0, eps=eps) + rt)
    yt.backward(torch.tensor(G))
    y, mean, invstd = bno.bn_train_fwd(z, gamma, beta, eps, res, True)
    dz, dres, dgamma, dbeta = bno.bn_train_bwd(G, z, y, gamma, mean, invstd, True)
    np.testing.assert_allclose(y, yt.detach().numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dz, zt.grad.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(dres, rt.grad.numpy(), rtol=1e-12, atol=0)
    np.testing.assert_allclose(dgamma, gt.grad.numpy(), rtol=1e-10)
    np.testing.assert_allclose(dbeta, bt.grad.numpy(), rtol=1e-10)
