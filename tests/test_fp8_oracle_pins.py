"""Pins of the 8-bit (E4M3) oracle: the codec and the scaled quantisation rule are checked against what
the published format fixes and against routines that share no code with it (torch's CPU float8_e4m3fn
casts, a brute-force nearest-neighbour search over the table of finite values)."""
import numpy as np
import pytest

from oracle import conv1d_oracle as orc
from oracle import fp8_oracle as f8

ALL = np.arange(256, dtype=np.uint8)
FINITE = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)


def test_values_the_format_fixes():
    """1-4-3 layout, bias 7: smallest subnormal 2^-9, largest subnormal 7*2^-9, smallest normal 2^-6,
    one = 0x38, two = 0x40, largest finite 448 = 0x7E, no infinities, S.1111.111 is NaN, signed zero."""
    d = f8.e4m3_decode(ALL)
    assert d[0x00] == 0.0 and d[0x80] == 0.0 and np.signbit(d[0x80])
    assert d[0x01] == 2.0 ** -9
    assert d[0x07] == 7 * 2.0 ** -9
    assert d[0x08] == 2.0 ** -6
    assert d[0x38] == 1.0 and d[0x40] == 2.0 and d[0x3C] == 1.5
    assert d[0x7E] == 448.0 and d[0xFE] == -448.0
    assert d[0x78] == 256.0  # exponent field 15 is an ordinary binade except for its last code
    assert np.isnan(d[0x7F]) and np.isnan(d[0xFF])
    assert np.isfinite(d[FINITE]).all() and np.abs(d[FINITE]).max() == 448.0


def test_decode_matches_torch_for_every_code():
    torch = pytest.importorskip("torch")
    ref = torch.from_numpy(ALL.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    got = f8.e4m3_decode(ALL)
    assert np.array_equal(np.isnan(ref), np.isnan(got))
    ok = ~np.isnan(ref)
    assert np.array_equal(ref[ok], got[ok])
    assert np.array_equal(np.signbit(ref[ok]), np.signbit(got[ok]))


def test_round_trip_and_monotone():
    d = f8.e4m3_decode(FINITE)
    assert np.array_equal(f8.e4m3_encode(d.astype(np.float32)), FINITE)
    v = np.sort(np.random.default_rng(0).uniform(-500, 500, 20000).astype(np.float32))
    q = f8.e4m3_decode(f8.e4m3_encode(v))
    assert (np.diff(q) >= 0).all()


def brute_force_encode(v):
    """Nearest finite table value; of two equally near ones the code with the even mantissa; the sign of v."""
    pos = np.array([c for c in range(0x7F)], dtype=np.uint8)
    table = f8.e4m3_decode(pos)
    out = np.empty(v.shape, dtype=np.uint8)
    for i, val in enumerate(v.astype(np.float64)):
        a = min(abs(val), 448.0)
        dist = np.abs(table - a)
        best = np.flatnonzero(dist == dist.min())
        c = best[0] if len(best) == 1 else [b for b in best if pos[b] % 2 == 0][0]
        out[i] = pos[c] | (0x80 if np.signbit(val) else 0)
    return out


def test_encode_against_brute_force_and_ties():
    rng = np.random.default_rng(1)
    pos = f8.e4m3_decode(np.arange(0x7F, dtype=np.uint8))
    mid = (pos[:-1] + pos[1:]) / 2                      # every tie point (exact in float32)
    v = np.concatenate([rng.normal(0, 1, 3000), rng.uniform(-460, 460, 3000), rng.normal(0, 0.01, 2000),
                        mid, -mid, np.nextafter(mid.astype(np.float32), np.float32(0)),
                        np.nextafter(mid.astype(np.float32), np.float32(1e9)), [0.0, -0.0, 448.0, 449.0, 1e30, -1e30]])
    v = v.astype(np.float32)
    assert np.array_equal(f8.e4m3_encode(v), brute_force_encode(v))
    # ties go to the even mantissa: the midpoint of codes c and c+1 takes whichever of them is even
    enc_mid = f8.e4m3_encode(mid.astype(np.float32))
    assert (enc_mid % 2 == 0).all()
    assert np.array_equal(enc_mid, np.arange(0x7E, dtype=np.uint8) + (np.arange(0x7E) % 2))
    assert f8.e4m3_encode(np.float32(np.nan)) == 0x7F


def test_encode_matches_torch_in_range():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(2)
    v = np.concatenate([rng.normal(0, 1, 20000), rng.uniform(-464, 464, 20000), rng.normal(0, 0.004, 20000)]).astype(np.float32)
    ref = torch.from_numpy(v).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(f8.e4m3_encode(v), ref)


def test_scales_and_quantisation_rule():
    rng = np.random.default_rng(3)
    x = rng.normal(0, 1, (4, 64)).astype(np.float32)
    x[2] = 0
    s = f8.row_scales(x, 4)
    assert s.dtype == np.float32 and s[2] == 1.0
    assert np.array_equal(s[[0, 1, 3]], (np.abs(x).max(axis=1) / np.float32(448))[[0, 1, 3]])
    q = f8.quantize_rows(x, s)
    # the largest magnitude of every row lands on +-448 and nothing saturates beyond it
    d = f8.e4m3_decode(q)
    assert np.array_equal(np.abs(d).max(axis=1)[[0, 1, 3]], [448.0] * 3) and (d[2] == 0).all()
    # the values the codes stand for are within half a spacing of x: relative error at most 2^-4 for normals
    back = d * s[:, None].astype(np.float64)
    big = np.abs(x) > s[:, None] * 2.0 ** -6
    assert (np.abs(back - x)[big] <= np.abs(x)[big] * 2.0 ** -4 * 1.0001).all()
    # power-of-two scale: quantisation commutes with it exactly
    assert np.array_equal(f8.quantize_rows(x * 4, s * 4), q)


def test_block_is_the_plain_block_on_the_decoded_values():
    """K=1: the block is a matrix product of the decoded codes times the scales (textbook form)."""
    rng = np.random.default_rng(4)
    B, Cin, Cout, T = 2, 16, 8, 12
    x = rng.normal(0, 1, (B, Cin, T)).astype(np.float32)
    w = rng.normal(0, 0.25, (Cout, Cin, 1)).astype(np.float32)
    sx = f8.row_scales(x, 1)
    sw = f8.row_scales(w, Cout)
    xq, wq = f8.quantize_rows(x, sx), f8.quantize_rows(w, sw)
    scale = rng.uniform(0.5, 1.5, Cout).astype(np.float32)
    shift = rng.normal(0, 0.1, Cout).astype(np.float32)
    y = f8.block_fwd_fp8(orc.block_fwd, xq, sx[0], wq, sw, scale, shift, None, True,
                         stride=1, dilation=1, pad=0)
    xd = f8.e4m3_decode(xq) * float(sx[0])
    wd = f8.e4m3_decode(wq)[:, :, 0] * sw.astype(np.float64)[:, None]
    ref = np.maximum(np.einsum("oc,bct->bot", wd, xd) * scale.astype(np.float64)[None, :, None]
                     + shift.astype(np.float64)[None, :, None], 0)
    np.testing.assert_allclose(y, ref, rtol=1e-12, atol=1e-12)
    # and it approximates the unquantised block to the accuracy of two 3-bit mantissas
    exact = orc.block_fwd(x.astype(np.float64), w.astype(np.float64), scale, shift, None, True, stride=1, dilation=1, pad=0)
    assert np.sqrt(np.mean((y - exact) ** 2)) / np.sqrt(np.mean(exact ** 2)) < 0.08


def test_input_gradient_on_codes_is_the_textbook_product_for_k1_and_the_adjoint_of_the_forward():
    rng = np.random.default_rng(5)
    B, Cin, Cout, T, K = 2, 12, 8, 20, 1
    w = rng.normal(0, 0.3, (Cout, Cin, K)).astype(np.float32)
    scale = rng.uniform(0.5, 1.5, Cout).astype(np.float32)
    dy = rng.normal(0, 1, (B, Cout, T)).astype(np.float32)
    y = rng.normal(0, 1, (B, Cout, T))
    g = f8.masked_gradient(dy, y, True)
    assert np.array_equal(g, dy * (y > 0))
    sg = f8.row_scales(g, 1)
    gq = f8.quantize_rows(g, sg)
    wt = f8.dgrad_weights(w, scale)
    assert wt.shape == (Cin, Cout, K) and np.array_equal(wt[3, 5, 0], np.float32(w[5, 3, 0] * scale[5]))
    swt = f8.dgrad_weight_scales(w, scale)
    assert np.array_equal(swt, np.abs(wt).reshape(Cin, -1).max(axis=1) / np.float32(448))
    wtq = f8.quantize_rows(wt, swt)
    dx = f8.bwd_data_fp8(orc.bwd_data, gq, sg[0], wtq, swt, T, stride=1, dilation=1, pad=0)
    gd = f8.e4m3_decode(gq) * float(sg[0])
    wd = f8.e4m3_decode(wtq)[:, :, 0] * swt.astype(np.float64)[:, None]          # [ci][co]
    np.testing.assert_allclose(dx, np.einsum("io,bot->bit", wd, gd), rtol=1e-12, atol=1e-12)
    # K > 1: <conv(x, W), dz> == <x, dgrad(dz, W)> for the weights the codes stand for
    K, pad = 5, 2
    w = rng.normal(0, 0.3, (Cout, Cin, K)).astype(np.float32)
    swt = f8.dgrad_weight_scales(w, None)
    wtq = f8.quantize_rows(f8.dgrad_weights(w, None), swt)
    w_eff = np.transpose(f8.e4m3_decode(wtq) * swt.astype(np.float64)[:, None, None], (1, 0, 2))
    x = rng.normal(0, 1, (B, Cin, T))
    z = orc.block_fwd(x, w_eff, None, None, None, False, stride=1, dilation=1, pad=pad)
    dx = f8.bwd_data_fp8(orc.bwd_data, gq, sg[0], wtq, swt, T, stride=1, dilation=1, pad=pad)
    np.testing.assert_allclose(np.sum(z * gd), np.sum(x * dx), rtol=1e-10)


def test_weight_gradient_on_codes_is_the_textbook_product_for_k1_and_matches_finite_differences():
    rng = np.random.default_rng(6)
    B, Cin, Cout, T = 2, 10, 6, 24
    x = rng.normal(0, 1, (B, Cin, T)).astype(np.float32)
    g = rng.normal(0, 1, (B, Cout, T)).astype(np.float32)
    scale = rng.uniform(0.5, 1.5, Cout).astype(np.float32)
    sx, sg = f8.row_scales(x, 1), f8.row_scales(g, 1)
    xq, gq = f8.quantize_rows(x, sx), f8.quantize_rows(g, sg)
    dw = f8.bwd_weight_fp8(orc.bwd_weight, xq, sx[0], gq, sg[0], scale, 1, stride=1, dilation=1, pad=0)
    xd, gd = f8.e4m3_decode(xq) * float(sx[0]), f8.e4m3_decode(gq) * float(sg[0])
    ref = np.einsum("bot,bit->oi", gd, xd) * scale.astype(np.float64)[:, None]
    np.testing.assert_allclose(dw[:, :, 0], ref, rtol=1e-12, atol=1e-12)
    # K = 5: dw is the derivative of <conv(xd, w) * scale, gd> with respect to w (linear in w: one difference is exact)
    K, pad = 5, 2
    dw = f8.bwd_weight_fp8(orc.bwd_weight, xq, sx[0], gq, sg[0], scale, K, stride=1, dilation=1, pad=pad)
    w0 = rng.normal(0, 1, (Cout, Cin, K))

    def loss(w):
        return np.sum(orc.block_fwd(xd, w, scale, None, None, False, stride=1, dilation=1, pad=pad) * gd)
    for (co, ci, k) in [(0, 0, 0), (5, 9, 4), (2, 3, 2)]:
        e = np.zeros_like(w0)
        e[co, ci, k] = 1.0
        np.testing.assert_allclose(loss(w0 + e) - loss(w0), dw[co, ci, k], rtol=1e-9, atol=1e-9)
