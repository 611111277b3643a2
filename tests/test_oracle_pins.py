"""Pins of the CPU oracle against things other than itself (CPU only).

The paper prints no worked numeric example for its convolutional encoder (Section 4.1.1
shows module wiring only; Section 3 leaves forward/backward to the backend), so every
pin is a closed form, an invariant, a brute-force enumeration or a library special case.
Each is chosen so that one plausible mistake in the oracle (a dropped term, a flipped
kernel, a wrong pad/dilation/stride index, a transposed operand, a wrong epilogue order)
fails at least one of them.
"""
import itertools

import numpy as np
import pytest

from oracle import conv1d_oracle as orc

RNG = np.random.default_rng(1234)


def rand(*shape):
    return RNG.standard_normal(shape)


GEOMS = [  # (B, Cin, Cout, T, K, stride, dilation, pad)
    (2, 3, 4, 16, 3, 1, 1, 1),
    (1, 5, 2, 17, 5, 1, 2, 4),
    (2, 4, 3, 19, 4, 2, 1, 2),
    (1, 2, 5, 23, 3, 3, 3, 0),
    (2, 3, 3, 12, 1, 1, 1, 0),
    (1, 3, 2, 14, 5, 2, 2, 6),
    (1, 2, 2, 9, 2, 1, 1, 3),   # even K, pad larger than needed
]


# ---- I5: brute-force index set ---------------------------------------------------------
def brute_force_conv(x, w, stride, dilation, pad):
    """Materialise the zero-padded signal and the zero-stuffed (dilated) kernel and slide."""
    B, Cin, T = x.shape
    Cout, _, K = w.shape
    xp = np.zeros((B, Cin, T + 2 * pad))
    xp[:, :, pad:pad + T] = x
    Kd = dilation * (K - 1) + 1
    wd = np.zeros((Cout, Cin, Kd))
    wd[:, :, ::dilation] = w
    n_pos = T + 2 * pad - Kd + 1          # stride-1 window positions
    if n_pos <= 0:
        return None
    starts = list(range(0, n_pos, stride))
    z = np.zeros((B, Cout, len(starts)))
    for j, s in enumerate(starts):
        window = xp[:, :, s:s + Kd]                       # [B, Cin, Kd]
        z[:, :, j] = np.einsum("bck,ock->bo", window, wd)
    return z


def test_out_len_and_index_set_brute_force():
    for T, K, s, d, pad in itertools.product(range(1, 13), range(1, 6), range(1, 4), range(1, 4), range(0, 7)):
        Kd = d * (K - 1) + 1
        n_pos = T + 2 * pad - Kd + 1
        expect = len(range(0, n_pos, s)) if n_pos > 0 else -1
        assert orc.out_len(T, K, s, d, pad) == expect, (T, K, s, d, pad)


@pytest.mark.parametrize("geom", GEOMS)
def test_forward_matches_brute_force_padding_and_dilation(geom):
    B, Cin, Cout, T, K, s, d, pad = geom
    x, w = rand(B, Cin, T), rand(Cout, Cin, K)
    z = orc.block_fwd(x, w, stride=s, dilation=d, pad=pad)
    ref = brute_force_conv(x, w, s, d, pad)
    assert z.shape == ref.shape
    np.testing.assert_allclose(z, ref, rtol=1e-12, atol=1e-12)


# ---- I1: K = 1 is a matrix product --------------------------------------------------------
def test_k1_is_matmul():
    B, Cin, Cout, T = 3, 7, 5, 11
    x, w = rand(B, Cin, T), rand(Cout, Cin, 1)
    z = orc.block_fwd(x, w)
    for b in range(B):
        np.testing.assert_allclose(z[b], np.matmul(w[:, :, 0], x[b]), rtol=1e-12, atol=1e-12)
    # a transposed operand would give a shape error or different numbers:
    g = rand(B, Cout, T)
    dx = orc.bwd_data(g, w, T)
    dw = orc.bwd_weight(x, g, 1)
    for b in range(B):
        np.testing.assert_allclose(dx[b], np.matmul(w[:, :, 0].T, g[b]), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dw[:, :, 0], sum(np.matmul(g[b], x[b].T) for b in range(B)),
                               rtol=1e-12, atol=1e-12)


# ---- I2: (bi)linearity -----------------------------------------------------------------------
def test_bilinearity():
    B, Cin, Cout, T, K, s, d, pad = 2, 3, 4, 15, 3, 2, 2, 2
    x1, x2, w1, w2 = rand(B, Cin, T), rand(B, Cin, T), rand(Cout, Cin, K), rand(Cout, Cin, K)
    f = lambda x, w: orc.block_fwd(x, w, stride=s, dilation=d, pad=pad)
    a, b = 0.7, -1.9
    np.testing.assert_allclose(f(a * x1 + b * x2, w1), a * f(x1, w1) + b * f(x2, w1), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(f(x1, a * w1 + b * w2), a * f(x1, w1) + b * f(x1, w2), rtol=1e-11, atol=1e-12)


# ---- I3: an impulse recovers every weight (orientation, dilation, completeness) --------------
@pytest.mark.parametrize("geom", GEOMS)
def test_impulse_recovers_weights(geom):
    B, Cin, Cout, T, K, s, d, pad = geom
    w = rand(Cout, Cin, K)
    To = orc.out_len(T, K, s, d, pad)
    for ci0 in range(Cin):
        for t0 in sorted({0, 1, T // 2, T - 2, T - 1} & set(range(T))):
            x = np.zeros((B, Cin, T))
            b0 = B - 1
            x[b0, ci0, t0] = 1.0
            z = orc.block_fwd(x, w, stride=s, dilation=d, pad=pad)
            expect = np.zeros((B, Cout, To))
            for t in range(To):
                for k in range(K):
                    if t * s - pad + k * d == t0:
                        expect[b0, :, t] = w[:, ci0, k]   # exactly, no sum: at most one k per t
            np.testing.assert_array_equal(z, expect)


# ---- I4: all-ones closed-form counts (padding edges) ----------------------------------------
@pytest.mark.parametrize("geom", GEOMS)
def test_all_ones_counts(geom):
    B, Cin, Cout, T, K, s, d, pad = geom
    z = orc.block_fwd(np.ones((B, Cin, T)), np.ones((Cout, Cin, K)), stride=s, dilation=d, pad=pad)
    To = orc.out_len(T, K, s, d, pad)
    for t in range(To):
        # number of taps whose sample lies inside [0, T): closed form by counting k in a range
        lo = t * s - pad                       # sample read by tap 0
        k_min = max(0, -(lo // d)) if lo < 0 else 0      # ceil(-lo/d)
        k_max = min(K - 1, (T - 1 - lo) // d) if T - 1 - lo >= 0 else -1
        count = max(0, k_max - k_min + 1)
        assert np.all(z[:, :, t] == Cin * count), (geom, t)
    if s == 1 and d == 1 and To > 2 * K:
        assert z[0, 0, To // 2] == Cin * K


# ---- I6 / I7 / I8 ---------------------------------------------------------------------------
def test_stride_is_subsampling():
    B, Cin, Cout, T, K, d, pad = 2, 3, 2, 21, 5, 2, 3
    x, w = rand(B, Cin, T), rand(Cout, Cin, K)
    z1 = orc.block_fwd(x, w, stride=1, dilation=d, pad=pad)
    for s in (2, 3, 4):
        zs = orc.block_fwd(x, w, stride=s, dilation=d, pad=pad)
        np.testing.assert_array_equal(zs, z1[:, :, ::s][:, :, :zs.shape[2]])
        assert zs.shape[2] == len(range(0, z1.shape[2], s))


def test_dilation_is_zero_stuffed_kernel():
    B, Cin, Cout, T, K, pad = 1, 3, 2, 25, 4, 5
    x, w = rand(B, Cin, T), rand(Cout, Cin, K)
    for d in (2, 3):
        wd = np.zeros((Cout, Cin, d * (K - 1) + 1))
        wd[:, :, ::d] = w
        np.testing.assert_allclose(orc.block_fwd(x, w, dilation=d, pad=pad),
                                   orc.block_fwd(x, wd, dilation=1, pad=pad), rtol=1e-12, atol=1e-13)


def test_shift_equivariance():
    B, Cin, Cout, T, K, pad = 1, 2, 3, 40, 5, 2
    x, w = np.zeros((B, Cin, T)), rand(Cout, Cin, K)
    x[:, :, 10:25] = rand(B, Cin, 15)
    xs = np.roll(x, 6, axis=2)
    z, zs = orc.block_fwd(x, w, pad=pad), orc.block_fwd(xs, w, pad=pad)
    np.testing.assert_allclose(np.roll(z, 6, axis=2), zs, rtol=1e-12, atol=1e-13)


# ---- I9: adjoint identities (no step size, exact up to rounding) -----------------------------
@pytest.mark.parametrize("geom", GEOMS)
def test_adjoint_identities(geom):
    B, Cin, Cout, T, K, s, d, pad = geom
    x, w = rand(B, Cin, T), rand(Cout, Cin, K)
    To = orc.out_len(T, K, s, d, pad)
    g = rand(B, Cout, To)
    z = orc.block_fwd(x, w, stride=s, dilation=d, pad=pad)
    dx = orc.bwd_data(g, w, T, stride=s, dilation=d, pad=pad)
    dw = orc.bwd_weight(x, g, K, stride=s, dilation=d, pad=pad)
    lhs = np.sum(g * z)
    assert abs(lhs - np.sum(dx * x)) <= 1e-11 * (abs(lhs) + 1)
    assert abs(lhs - np.sum(dw * w)) <= 1e-11 * (abs(lhs) + 1)


# ---- I10: finite differences of the whole block ----------------------------------------------
@pytest.mark.parametrize("geom", GEOMS[:6])
def test_finite_differences_whole_block(geom):
    B, Cin, Cout, T, K, s, d, pad = geom
    To = orc.out_len(T, K, s, d, pad)
    x, w = rand(B, Cin, T), rand(Cout, Cin, K)
    scale, shift = RNG.uniform(0.5, 1.5, Cout), 0.1 * rand(Cout)
    res, g = rand(B, Cout, To), rand(B, Cout, To)
    kw = dict(stride=s, dilation=d, pad=pad)

    def loss(x_, w_, r_):
        return np.sum(g * orc.block_fwd(x_, w_, scale, shift, r_, True, **kw))

    y, z = orc.block_fwd(x, w, scale, shift, res, True, return_z=True, **kw)
    v = scale[None, :, None] * z + shift[None, :, None] + res
    assert np.min(np.abs(v)) > 1e-4, "redraw: a pre-activation sits on the ReLU kink"
    dz, dres = orc.epilogue_bwd(g, y, scale, relu=True)
    dx = orc.bwd_data(dz, w, T, **kw)
    dw = orc.bwd_weight(x, dz, K, **kw)
    h = 1e-6
    for arr, grad, which in ((x, dx, 0), (w, dw, 1), (res, dres, 2)):
        flat = arr.reshape(-1)
        for i in RNG.choice(flat.size, size=min(25, flat.size), replace=False):
            old = flat[i]
            args = [x, w, res]
            flat[i] = old + h
            lp = loss(*args)
            flat[i] = old - h
            lm = loss(*args)
            flat[i] = old
            fd = (lp - lm) / (2 * h)
            assert abs(fd - grad.reshape(-1)[i]) <= 1e-6 * (1 + abs(fd)), (which, i, fd, grad.reshape(-1)[i])


# ---- I11: epilogue closed forms ---------------------------------------------------------------
def test_epilogue_closed_forms():
    B, Cin, Cout, T, K, pad = 2, 3, 4, 13, 3, 1
    x, w = rand(B, Cin, T), rand(Cout, Cin, K)
    z = orc.block_fwd(x, w, pad=pad)
    scale, shift, res = RNG.uniform(0.5, 1.5, Cout), rand(Cout), rand(B, Cout, T)
    s3, h3 = scale[None, :, None], shift[None, :, None]
    np.testing.assert_array_equal(orc.block_fwd(x, w, np.ones(Cout), np.zeros(Cout), pad=pad), z)
    np.testing.assert_allclose(orc.block_fwd(x, w, residual=res, pad=pad), z + res, rtol=1e-15)
    np.testing.assert_allclose(orc.block_fwd(x, w, scale, shift, pad=pad), s3 * z + h3, rtol=1e-15)
    # order: affine, then residual, then ReLU (the residual is inside the activation)
    y = orc.block_fwd(x, w, scale, shift, res, True, pad=pad)
    np.testing.assert_allclose(y, np.maximum(s3 * z + h3 + res, 0.0), rtol=1e-15)
    assert (y >= 0).all() and (y == 0).any() and (y > 0).any()
    g = rand(B, Cout, T)
    dz, dres = orc.epilogue_bwd(g, y, scale, relu=True)
    np.testing.assert_array_equal(dres, g * (y > 0))
    np.testing.assert_allclose(dz, g * (y > 0) * s3, rtol=1e-15)
    dz2, dres2 = orc.epilogue_bwd(g, None, None, relu=False)
    np.testing.assert_array_equal(dz2, g)
    np.testing.assert_array_equal(dres2, g)
    # derivative at exactly zero output is zero
    dz3, _ = orc.epilogue_bwd(np.ones((1, 1, 3)), np.array([[[0.0, -0.0, 1e-300]]]), None, relu=True)
    np.testing.assert_array_equal(dz3, [[[0.0, 0.0, 1.0]]])


# ---- I12: library special case ----------------------------------------------------------------
@pytest.mark.parametrize("geom", GEOMS + [(2, 16, 24, 64, 11, 1, 1, 5), (2, 8, 8, 50, 7, 2, 2, 6)])
def test_library_conv1d_float64(geom):
    torch = pytest.importorskip("torch")
    B, Cin, Cout, T, K, s, d, pad = geom
    x, w = rand(B, Cin, T), rand(Cout, Cin, K)
    To = orc.out_len(T, K, s, d, pad)
    g = rand(B, Cout, To)
    xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    wt = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    zt = torch.nn.functional.conv1d(xt, wt, stride=s, padding=pad, dilation=d)
    zt.backward(torch.tensor(g))
    np.testing.assert_allclose(orc.block_fwd(x, w, stride=s, dilation=d, pad=pad), zt.detach().numpy(),
                               rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(orc.bwd_data(g, w, T, stride=s, dilation=d, pad=pad), xt.grad.numpy(),
                               rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(orc.bwd_weight(x, g, K, stride=s, dilation=d, pad=pad), wt.grad.numpy(),
                               rtol=1e-11, atol=1e-12)


# ---- sampled evaluators are the full ones at the sampled positions ------------------------------
@pytest.mark.parametrize("geom", GEOMS + [(2, 8, 8, 50, 7, 2, 2, 6)])
def test_sampled_evaluators_match_full(geom):
    B, Cin, Cout, T, K, s, d, pad = geom
    To = orc.out_len(T, K, s, d, pad)
    x, w = rand(B, Cin, T), rand(Cout, Cin, K)
    scale, shift, res, g = RNG.uniform(0.5, 1.5, Cout), rand(Cout), rand(B, Cout, To), rand(B, Cout, To)
    kw = dict(stride=s, dilation=d, pad=pad)
    y = orc.block_fwd(x, w, scale, shift, res, True, **kw)
    idx = np.arange(y.size)
    np.testing.assert_array_equal(orc.block_fwd_at(x, w, idx, scale, shift, res, True, **kw), y.reshape(-1))
    dx = orc.bwd_data(g, w, T, **kw)                 # scatter form
    np.testing.assert_allclose(orc.bwd_data_at(g, w, T, np.arange(dx.size), **kw), dx.reshape(-1),
                               rtol=1e-12, atol=1e-13)   # gather form: different summation order
    dw = orc.bwd_weight(x, g, K, **kw)
    np.testing.assert_array_equal(orc.bwd_weight_at(x, g, K, np.arange(dw.size), **kw), dw.reshape(-1))


def test_degenerate_geometries():
    assert orc.out_len(4, 5, 1, 1, 0) == -1          # kernel longer than the padded signal
    assert orc.out_len(4, 5, 1, 1, 1) == 2
    assert orc.out_len(1, 1, 1, 1, 0) == 1
    assert orc.out_len(0, 1, 1, 1, 0) == -1
    z = orc.block_fwd(np.ones((1, 1, 1)), np.full((1, 1, 1), 3.0))
    assert z.shape == (1, 1, 1) and z[0, 0, 0] == 3.0


# ---- per-sample lengths ------------------------------------------------------------------------
def test_masking_ignores_whatever_lies_in_the_padding():
    rng = np.random.default_rng(41)
    B, Cin, Cout, T, K = 3, 5, 4, 23, 5
    x, w = rng.standard_normal((B, Cin, T)), rng.standard_normal((Cout, Cin, K))
    lengths = np.array([23, 9, 1])
    ref = orc.block_fwd_masked(x, w, lengths, pad=2)
    junk = x.copy()
    for b, n in enumerate(lengths):
        junk[b, :, n:] = 1e30 * rng.standard_normal((Cin, T - n))
    np.testing.assert_array_equal(orc.block_fwd_masked(junk, w, lengths, pad=2), ref)
    dz = rng.standard_normal((B, Cout, T))
    np.testing.assert_array_equal(orc.bwd_weight_masked(junk, dz, K, lengths, pad=2), orc.bwd_weight_masked(x, dz, K, lengths, pad=2))
    # full lengths: nothing changes
    full = np.full(B, T)
    np.testing.assert_array_equal(orc.block_fwd_masked(x, w, full, pad=2), orc.block_fwd(x, w, pad=2))


def test_masked_forward_equals_the_convolution_of_the_cut_sample():
    # Behind a cut-off sample the block sees zeros, exactly like the zero padding of the convolution itself:
    # outputs whose taps all lie inside [0, len) equal those of the sample convolved on its own.
    rng = np.random.default_rng(42)
    Cin, Cout, T, K, pad, n = 3, 2, 30, 7, 3, 17
    x, w = rng.standard_normal((1, Cin, T)), rng.standard_normal((Cout, Cin, K))
    masked = orc.block_fwd_masked(x, w, [n], pad=pad)
    alone = orc.block_fwd(x[:, :, :n], w, pad=pad)               # T_out = n
    np.testing.assert_allclose(masked[:, :, :n], alone, rtol=1e-13, atol=1e-13)
    # beyond n + (K-1) - pad the output depends on nothing but zeros
    assert np.all(masked[:, :, n + K - 1 - pad:] == 0)
    assert list(orc.out_lengths([n, 0, 5], K, 1, 1, pad)) == [n, 0, 5]
    assert list(orc.out_lengths([20, 21], 11, 2, 1, 5)) == [10, 11]


def test_masked_gradients_are_the_derivatives_of_the_masked_forward():
    rng = np.random.default_rng(43)
    B, Cin, Cout, T, K, pad = 2, 3, 2, 12, 3, 1
    x, w = rng.standard_normal((B, Cin, T)), rng.standard_normal((Cout, Cin, K))
    lengths = np.array([12, 7])
    dz = rng.standard_normal((B, Cout, T))
    loss = lambda xx, ww: float(np.sum(orc.block_fwd_masked(xx, ww, lengths, pad=pad) * dz))
    dx, dw = orc.bwd_data_masked(dz, w, T, lengths, pad=pad), orc.bwd_weight_masked(x, dz, K, lengths, pad=pad)
    eps = 1e-6
    for idx in [(0, 1, 11), (1, 2, 6), (1, 0, 7), (1, 1, 11)]:      # the last two lie in the padding: derivative 0
        xp, xm = x.copy(), x.copy()
        xp[idx] += eps
        xm[idx] -= eps
        np.testing.assert_allclose((loss(xp, w) - loss(xm, w)) / (2 * eps), dx[idx], rtol=1e-6, atol=1e-8)
    assert dx[1, 0, 7] == 0 and dx[1, 1, 11] == 0
    for idx in [(0, 0, 0), (1, 2, 2)]:
        wp, wm = w.copy(), w.copy()
        wp[idx] += eps
        wm[idx] -= eps
        np.testing.assert_allclose((loss(x, wp) - loss(x, wm)) / (2 * eps), dw[idx], rtol=1e-6, atol=1e-8)
