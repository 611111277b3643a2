"""Pins of the decoder-tail oracle (oracle/decoder_oracle.py) to things other than itself: closed
forms, invariants of a log-softmax, scipy's routine, and the convolution oracle (a K=1 block) for
the logits."""
import numpy as np
from scipy.special import log_softmax, logsumexp

from oracle import conv1d_oracle as corc
from oracle import decoder_oracle as dorc


def rnd(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def test_two_classes_closed_form():
    # one input channel, weights +1 / -1, no bias: z = (x, -x) and logp = -log(1 + exp(-+2x))
    x = np.array([[[0.0, 1.0, -2.5, 30.0]]])
    w = np.array([[1.0], [-1.0]])
    got = dorc.decoder_logsoftmax(x, w)
    xs = x[0, 0]
    np.testing.assert_allclose(got[0, 0], -np.log1p(np.exp(-2 * xs)), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(got[0, 1], -2 * xs - np.log1p(np.exp(-2 * xs)), rtol=1e-13, atol=1e-13)


def test_uniform_logits_give_minus_log_n():
    x = rnd(0, 2, 5, 7)
    w = np.zeros((29, 5))
    np.testing.assert_allclose(dorc.decoder_logsoftmax(x, w, np.full(29, 3.25)), -np.log(29.0), rtol=1e-14)


def test_probabilities_sum_to_one_and_order_is_kept():
    x, w, b = rnd(1, 3, 16, 11), rnd(2, 29, 16), rnd(3, 29)
    logp = dorc.decoder_logsoftmax(x, w, b)
    np.testing.assert_allclose(np.exp(logp).sum(axis=1), 1.0, rtol=1e-13)
    assert (logp <= 0).all()
    z = dorc.decoder_logits(x, w, b)
    assert np.array_equal(np.argsort(z, axis=1), np.argsort(logp, axis=1))
    # differences of log-probabilities are differences of logits
    np.testing.assert_allclose(logp[:, 1:] - logp[:, :-1], z[:, 1:] - z[:, :-1], rtol=1e-10, atol=1e-12)


def test_invariant_to_a_common_bias_shift_and_safe_for_large_logits():
    x, w, b = rnd(4, 2, 8, 5), rnd(5, 6, 8), rnd(6, 6)
    base = dorc.decoder_logsoftmax(x, w, b)
    np.testing.assert_allclose(dorc.decoder_logsoftmax(x, w, b + 1234.5), base, rtol=1e-9, atol=1e-9)
    big = dorc.log_softmax_over_classes(np.array([[[1000.0], [999.0], [-1000.0]]]))
    assert np.isfinite(big).all()
    np.testing.assert_allclose(big[0, :2, 0], [-np.log1p(np.exp(-1.0)), -1.0 - np.log1p(np.exp(-1.0))], rtol=1e-12)


def test_against_scipy_and_the_convolution_oracle():
    # logits from the K=1 convolution oracle with the bias as its shift; log-softmax from scipy
    x, w, b = rnd(7, 2, 24, 13), rnd(8, 29, 24), rnd(9, 29)
    z = corc.block_fwd(x, w[:, :, None], np.ones(29), b, None, False)
    np.testing.assert_allclose(dorc.decoder_logits(x, w, b), z, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dorc.decoder_logsoftmax(x, w, b), log_softmax(z, axis=1), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dorc.decoder_logsoftmax(x, w, b), z - logsumexp(z, axis=1, keepdims=True), rtol=1e-12,
                               atol=1e-12)


def test_a_planted_mistake_is_caught():
    # softmax over the wrong axis, a dropped bias, a transposed weight: each fails one of the pins above
    x, w, b = rnd(10, 2, 6, 6), rnd(11, 6, 6), rnd(12, 6)
    good = dorc.decoder_logsoftmax(x, w, b)
    wrong_axis = dorc.decoder_logits(x, w, b)
    wrong_axis = wrong_axis - logsumexp(wrong_axis, axis=2, keepdims=True)
    assert not np.allclose(np.exp(wrong_axis).sum(axis=1), 1.0)
    assert not np.allclose(dorc.decoder_logsoftmax(x, w), good)
    assert not np.allclose(dorc.decoder_logsoftmax(x, w.T.copy(), b), good)
