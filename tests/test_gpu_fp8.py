"""GPU parity of the 8-bit floating-point (E4M3) variant against the oracle (oracle/fp8_oracle.py +
conv1d_oracle).

Scales and codes are integer-like results of a float32 rule that both sides state the same way (float32
division and multiplication, round to nearest even, saturation): they are compared bit for bit.  The
block output is compared with the oracle's block on the values the oracle's own codes stand for -- the
inputs, scales and quantisation rule are shared, no GPU result feeds the oracle -- at the gate of the bf16
block: products of two E4M3 values are exact in float32, so the GPU result differs from the fp64 one by
float32 accumulation (about 1e-6 relative to the rms) and the final rounding to bf16 (unit roundoff 2^-8).
"""
import numpy as np
import pytest

import _util as U
from oracle import conv1d_oracle as orc
from oracle import fp8_oracle as f8
from paper_1909_09577_amd import binding as nm
from paper_1909_09577_amd import inputs as syn
from paper_1909_09577_amd.inputs import LayerCfg

pytestmark = pytest.mark.gpu
DT = "bf16"


def L(name, B, Cin, Cout, T, K, dilation=1, pad=None, affine=True, relu=True, residual=False, seed=51):
    pad = dilation * (K - 1) // 2 if pad is None else pad
    return LayerCfg(name, B, Cin, Cout, T, K, 1, dilation, pad, affine, relu, residual, seed,
                    T_out=orc.out_len(T, K, 1, dilation, pad))


def bf16_dev(a):
    """device bf16 tensor holding float32 array a rounded to bf16, and the rounded values as float32"""
    import torch
    bits = syn.f32_to_bf16_bits(np.ascontiguousarray(a, dtype=np.float32))
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16), syn.bf16_bits_to_f32(bits)


@pytest.mark.parametrize("shape,rows", [((3, 1000), 3), ((1, 77777), 1), ((64, 64, 17), 64), ((5, 8191), 5), ((2, 4, 333), 1)])
def test_scales_and_codes_are_bit_exact(shape, rows):
    rng = np.random.default_rng(7)
    a = rng.normal(0, 1, shape).astype(np.float32)
    a.reshape(rows, -1)[0, :5] = [0.0, -0.0, 1e-30, -3e-5, 2.5]           # zeros, underflow to zero, subnormal codes
    if rows > 2:
        a.reshape(rows, -1)[1] = 0.0                                      # an all-zero slice: scale 1
        a.reshape(rows, -1)[2] *= 1e-3
    d, a16 = bf16_dev(a)
    s_gpu = nm.nm_fp8_row_scales(d, rows)
    s_ref = f8.row_scales(a16, rows)
    assert np.array_equal(s_gpu.cpu().numpy().view(np.uint32), s_ref.view(np.uint32))
    q_gpu = nm.nm_fp8_quantize_rows(d, s_gpu).cpu().numpy()
    q_ref = f8.quantize_rows(a16, s_ref)
    assert np.array_equal(q_gpu, q_ref)
    # a scale that is too small for the data: saturation at +-448 on both sides
    import torch
    tiny = (s_ref / np.float32(37.0)).astype(np.float32)
    q_gpu = nm.nm_fp8_quantize_rows(d, torch.from_numpy(tiny).cuda()).cpu().numpy()
    assert np.array_equal(q_gpu, f8.quantize_rows(a16, tiny))
    assert (q_gpu & 0x7F).max() == 0x7E


def test_every_tie_and_every_code_boundary():
    """All 16-bit patterns of bf16 that are finite, quantised with scale 1: covers every tie point of E4M3
    that bf16 can express, both signs, the subnormal range and the saturation boundary."""
    import torch
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = syn.bf16_bits_to_f32(bits)
    keep = np.isfinite(vals)
    d = torch.from_numpy(bits[keep].view(np.int16)).cuda().view(torch.bfloat16)
    one = torch.ones(1, dtype=torch.float32, device="cuda")
    q = nm.nm_fp8_quantize_rows(d, one).cpu().numpy()
    assert np.array_equal(q, f8.quantize_rows(vals[keep], np.ones(1, np.float32)))


CASES = [
    L("f8_two_tiles", 2, 64, 64, 200, 17, residual=True),                 # ragged second time tile
    L("f8_nine_pairs", 3, 128, 192, 333, 21, residual=True),              # (b, tile) pairs not a multiple of 4, odd length
    L("f8_k25", 2, 192, 128, 160, 25, relu=False),
    L("f8_k29_d2", 2, 128, 64, 248, 29, dilation=2),
    L("f8_short_pad", 2, 64, 128, 180, 17, pad=3, affine=False),          # T_out < T
    L("f8_long_pad", 2, 64, 64, 100, 17, pad=16, residual=True),          # T_out > T
    L("f8_one_frame_tile", 1, 64, 64, 161, 17),                           # a time tile with a single valid frame
    L("f8_many_tiles", 32, 64, 256, 1600, 17, residual=True),             # 1280 tiles: every wavefront runs a second tile
    # few tiles and at least four chunks: every tile is shared by the four wavefronts of a workgroup
    L("f8_shared_8", 2, 256, 128, 200, 17, residual=True),
    L("f8_shared_uneven_chunks", 3, 320, 64, 333, 21, residual=True),     # 5 chunks over 4 wavefronts, empty tile ids, odd length
    L("f8_shared_k25", 2, 512, 192, 320, 25, relu=False),
    # more tiles than wavefronts with a small remainder: private rounds followed by a shared one
    L("f8_private_then_shared", 33, 256, 256, 1280, 17, residual=True),   # 33*8*4 = 1056 tiles = 1024 + 32
]


def run_case(cfg):
    inp = syn.make_inputs(cfg, DT)
    kw = U.geom_kw(cfg)
    sx = f8.row_scales(inp["x"], 1)
    sw = f8.row_scales(inp["w"], cfg.Cout)
    xq, wq = f8.quantize_rows(inp["x"], sx), f8.quantize_rows(inp["w"], sw)
    scale = inp["scale"] if cfg.affine else None
    shift = inp["shift"] if cfg.affine else None
    res = inp["residual"] if cfg.residual else None
    ref = f8.block_fwd_fp8(orc.block_fwd, xq, sx[0], wq, sw, scale, shift, res, cfg.relu, **kw)

    xd, wd = U.to_dev(inp, "x", DT), U.to_dev(inp, "w", DT)
    sxd = nm.nm_fp8_row_scales(xd, 1)
    swd = nm.nm_fp8_row_scales(wd, cfg.Cout)
    assert np.array_equal(sxd.cpu().numpy(), sx) and np.array_equal(swd.cpu().numpy(), sw)
    y = nm.nm_conv1d_block_fwd_fp8(
        xd, sxd, wd, swd, U.to_dev(inp, "scale", DT) if cfg.affine else None,
        U.to_dev(inp, "shift", DT) if cfg.affine else None, U.to_dev(inp, "residual", DT) if cfg.residual else None,
        relu=cfg.relu, **kw)
    assert tuple(y.shape) == (cfg.B, cfg.Cout, cfg.T_out)
    return U.to_host_f64(y), ref, inp


@pytest.mark.parametrize("cfg", CASES, ids=lambda c: c.name)
def test_block_fwd_fp8(cfg):
    assert nm.nm_conv1d_fp8_supported(cfg.B, cfg.Cin, cfg.Cout, cfg.T, cfg.K, 1, cfg.dilation, cfg.pad)
    got, ref, _ = run_case(cfg)
    U.assert_close(got, ref, DT, f"{cfg.name} y")


@pytest.mark.parametrize("cfg", [
    L("f8_b3_512_k17", 32, 512, 512, 800, 17, residual=True, seed=2),
    L("f8_768_k25", 32, 768, 768, 800, 25, residual=True, seed=6),
], ids=lambda c: c.name)
def test_block_fwd_fp8_full_size_full_tensor(cfg):
    got, ref, inp = run_case(cfg)
    U.assert_close(got, ref, DT, f"{cfg.name} y")
    # how far the 8-bit block is from the unquantised one (reported, loosely bounded: two 3-bit mantissas)
    exact = U.oracle_fwd(cfg, inp)
    rel = np.sqrt(np.mean((ref - exact) ** 2)) / np.sqrt(np.mean(exact ** 2))
    print(f"{cfg.name}: relative rms distance of the E4M3 block from the fp64 block on unquantised inputs: {rel:.4f}")
    assert rel < 0.06


def test_impulse_recovers_the_quantised_weights():
    """x = one unit sample in one channel: y[co, t] = decode(wq[co, ci, k]) * sw[co] * decode(xq) * sx at
    t = t0 + pad - k, so every (chunk, lane half, byte) position of both operands is exercised on its own."""
    import torch
    B, Cin, Cout, T, K, pad = 1, 128, 64, 160, 17, 8
    rng = np.random.default_rng(9)
    w = syn.bf16_bits_to_f32(syn.f32_to_bf16_bits(rng.normal(0, 0.05, (Cout, Cin, K)).astype(np.float32)))
    wd, _ = bf16_dev(w)
    sw = f8.row_scales(w, Cout)
    wq = f8.e4m3_decode(f8.quantize_rows(w, sw)) * sw.astype(np.float64)[:, None, None]
    swd = torch.from_numpy(sw).cuda()
    sxd = torch.ones(1, dtype=torch.float32, device="cuda")
    t0 = 70
    for ci in (0, 31, 32, 63, 64, 100, 127):
        x = np.zeros((B, Cin, T), dtype=np.float32)
        x[0, ci, t0] = 1.0
        xd, _ = bf16_dev(x)
        y = U.to_host_f64(nm.nm_conv1d_block_fwd_fp8(xd, sxd, wd, swd, stride=1, dilation=1, pad=pad))
        expect = np.zeros((Cout, T))
        for k in range(K):
            expect[:, t0 + pad - k] = wq[:, ci, k]
        got = y[0]
        assert np.array_equal(got != 0, expect != 0), f"channel {ci}: support of the response"
        np.testing.assert_allclose(got, expect, rtol=2.0 ** -8, atol=0)


# ---- input gradient on E4M3 operands ------------------------------------------------------------------
DGRAD_CASES = [
    L("f8d_two_tiles", 2, 64, 64, 200, 17, residual=True),
    L("f8d_nine_pairs", 3, 192, 128, 333, 21, residual=True),             # odd length: element-wise passes
    L("f8d_k25_no_relu", 2, 128, 192, 160, 25, relu=False, affine=False),
    L("f8d_k29_d2", 2, 64, 128, 248, 29, dilation=2),
    L("f8d_short_pad", 2, 128, 64, 180, 17, pad=3),                        # T_out < T: left padding of g is 13
    L("f8d_long_pad", 2, 64, 64, 104, 17, pad=16),                         # T_out > T
    L("f8d_shared", 2, 128, 256, 200, 17, residual=True),                 # reduction over 256 output channels: shared tiles
    L("f8d_private_then_shared", 33, 256, 256, 1280, 17),                 # 1056 tiles = 1024 + 32
]


def run_dgrad_case(cfg):
    import torch
    inp = syn.make_inputs(cfg, DT)
    kw = U.geom_kw(cfg)
    scale = inp["scale"] if cfg.affine else None
    y_saved = inp["y_saved"]
    g = f8.masked_gradient(inp["dy"], y_saved, cfg.relu)
    sg = f8.row_scales(inp["dy"], 1)                      # the scale of dy bounds g
    gq = f8.quantize_rows(g, sg)
    swt = f8.dgrad_weight_scales(inp["w"], scale)
    wtq = f8.quantize_rows(f8.dgrad_weights(inp["w"], scale), swt)
    dx_ref = f8.bwd_data_fp8(orc.bwd_data, gq, sg[0], wtq, swt, cfg.T, **kw)

    dyd, wd = U.to_dev(inp, "dy", DT), U.to_dev(inp, "w", DT)
    yd = U.to_dev(inp, "y_saved", DT) if cfg.relu else None
    scd = U.to_dev(inp, "scale", DT) if cfg.affine else None
    sgd = nm.nm_fp8_row_scales(dyd, 1)
    swtd = nm.nm_fp8_dgrad_weight_scales(wd, scd)
    assert np.array_equal(sgd.cpu().numpy(), sg)
    assert np.array_equal(swtd.cpu().numpy().view(np.uint32), swt.view(np.uint32)), "per-input-channel weight scales"
    dx, dres = nm.nm_conv1d_bwd_data_fp8(dyd, sgd, wd, swtd, cfg.T, y=yd, scale=scd, relu=cfg.relu, want_dres=True, **kw)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(U.to_host_f64(dres), g.astype(np.float64))   # dres = g, bit for bit
    return U.to_host_f64(dx), dx_ref


@pytest.mark.parametrize("cfg", DGRAD_CASES, ids=lambda c: c.name)
def test_bwd_data_fp8(cfg):
    got, ref = run_dgrad_case(cfg)
    assert got.shape == (cfg.B, cfg.Cin, cfg.T)
    U.assert_close(got, ref, DT, f"{cfg.name} dx")


def test_bwd_data_fp8_full_size_full_tensor():
    cfg = L("f8d_b3_512_k17", 32, 512, 512, 800, 17, residual=True, seed=2)
    got, ref = run_dgrad_case(cfg)
    U.assert_close(got, ref, DT, f"{cfg.name} dx")


# ---- weight gradient on E4M3 operands -----------------------------------------------------------------
# The products of two E4M3 values are exact, but the matrix core does not add the 64 products of one instruction as
# 64 float32 additions: it sums them in a wider fixed-point tree aligned to the largest product and rounds once into
# the float32 accumulator, dropping low bits of much smaller products.  Observed against the fp64 oracle: relative rms
# 1e-5, largest scaled error 2.3e-4 (elements whose sum nearly cancels).  Gates an order of magnitude below the bf16
# gate and far below the 3-bit mantissa of the operands themselves.
WGRAD_TOL = 1e-3
WGRAD_RMS = 1e-4


def run_wgrad_case(cfg, accumulate=False):
    import torch
    inp = syn.make_inputs(cfg, DT)
    kw = U.geom_kw(cfg)
    scale = inp["scale"] if cfg.affine else None
    g = f8.masked_gradient(inp["dy"], inp["y_saved"], cfg.relu)
    sg, sx = f8.row_scales(inp["dy"], 1), f8.row_scales(inp["x"], 1)
    gq, xq = f8.quantize_rows(g, sg), f8.quantize_rows(inp["x"], sx)
    dw_ref = f8.bwd_weight_fp8(orc.bwd_weight, xq, sx[0], gq, sg[0], scale, cfg.K, **kw)
    xd, dyd = U.to_dev(inp, "x", DT), U.to_dev(inp, "dy", DT)
    yd = U.to_dev(inp, "y_saved", DT) if cfg.relu else None
    scd = U.to_dev(inp, "scale", DT) if cfg.affine else None
    sxd, sgd = nm.nm_fp8_row_scales(xd, 1), nm.nm_fp8_row_scales(dyd, 1)
    dw = nm.nm_conv1d_bwd_weight_fp8(xd, sxd, dyd, sgd, cfg.K, y=yd, scale=scd, relu=cfg.relu, **kw)
    if accumulate:
        dw2 = nm.nm_conv1d_bwd_weight_fp8(xd, sxd, dyd, sgd, cfg.K, y=yd, scale=scd, dw=dw.clone(), relu=cfg.relu,
                                          accumulate=True, **kw)
        np.testing.assert_allclose(dw2.cpu().numpy(), 2 * dw.cpu().numpy(), rtol=1e-6)
        again = nm.nm_conv1d_bwd_weight_fp8(xd, sxd, dyd, sgd, cfg.K, y=yd, scale=scd, relu=cfg.relu, **kw)
        assert torch.equal(again, dw), "the weight gradient must be deterministic"
    return dw.cpu().numpy().astype(np.float64), dw_ref


@pytest.mark.parametrize("cfg", [
    L("f8w_one_unit", 1, 64, 64, 64, 17),
    L("f8w_ragged_units", 3, 128, 64, 200, 17, residual=True),            # 200 = 3 units + 8 steps; several batch items
    L("f8w_odd_length", 2, 64, 128, 333, 21, relu=False),                 # element-wise quantisation passes
    L("f8w_k25", 2, 192, 128, 160, 25),
    L("f8w_k29_d2", 2, 128, 64, 248, 29, dilation=2),
    L("f8w_short_pad", 2, 64, 64, 180, 17, pad=3, affine=False),
    L("f8w_long_pad", 2, 64, 64, 104, 17, pad=16),
    L("f8w_many_tiles", 4, 512, 256, 320, 17),                            # 64 tiles, four workgroups per tile
], ids=lambda c: c.name)
def test_bwd_weight_fp8(cfg):
    got, ref = run_wgrad_case(cfg, accumulate=cfg.name == "f8w_ragged_units")
    mx, rr = U.err_metrics(got, ref)
    assert mx <= WGRAD_TOL and rr <= WGRAD_RMS, f"{cfg.name} dw: max scaled error {mx:.3e}, rel rms {rr:.3e}"


def test_bwd_weight_fp8_full_size_full_tensor():
    cfg = L("f8w_b3_512_k17", 32, 512, 512, 800, 17, residual=True, seed=2)
    got, ref = run_wgrad_case(cfg)
    mx, rr = U.err_metrics(got, ref)
    assert mx <= WGRAD_TOL and rr <= WGRAD_RMS, f"{cfg.name} dw: max scaled error {mx:.3e}, rel rms {rr:.3e}"


def random_fp8_layers(n, seed):
    """Seeded random geometries inside the served set (stride 1, channels in multiples of 64, the encoder's taps)."""
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        K, dil = [(17, 1), (21, 1), (25, 1), (29, 2)][int(rng.integers(0, 4))]
        Cin, Cout = 64 * int(rng.integers(1, 6)), 64 * int(rng.integers(1, 5))
        B, T = int(rng.integers(1, 5)), int(rng.integers((K - 1) * dil + 1, 420))
        pad = int(rng.integers(0, (K - 1) * dil + 1))
        out.append(L(f"f8r{i}_b{B}_{Cin}to{Cout}_t{T}_k{K}d{dil}p{pad}", B, Cin, Cout, T, K, dilation=dil, pad=pad,
                     affine=bool(rng.integers(0, 2)), relu=bool(rng.integers(0, 2)), residual=bool(rng.integers(0, 2)),
                     seed=100 + i))
    return out


@pytest.mark.parametrize("cfg", random_fp8_layers(12, 2024), ids=lambda c: c.name)
def test_random_geometries_all_three_passes(cfg):
    got, ref, _ = run_case(cfg)
    U.assert_close(got, ref, DT, f"{cfg.name} y")
    got, ref = run_dgrad_case(cfg)
    U.assert_close(got, ref, DT, f"{cfg.name} dx")
    got, ref = run_wgrad_case(cfg)
    mx, rr = U.err_metrics(got, ref)
    assert mx <= WGRAD_TOL and rr <= WGRAD_RMS, f"{cfg.name} dw: max scaled error {mx:.3e}, rel rms {rr:.3e}"


@pytest.mark.parametrize("cfg", [
    L("f8b_ragged", 3, 128, 64, 200, 17, residual=True),
    L("f8b_odd_length", 2, 64, 128, 333, 21),
    L("f8b_k25_no_relu", 2, 192, 128, 160, 25, relu=False, affine=False),
    L("f8b_k29_d2", 2, 128, 64, 248, 29, dilation=2),
    L("f8b_short_pad", 2, 64, 64, 180, 17, pad=3),
    L("f8b_long_pad", 2, 64, 64, 104, 17, pad=16),
    L("f8b_b3_512_k17", 32, 512, 512, 800, 17, residual=True, seed=2),
], ids=lambda c: c.name)
def test_fused_backward_fp8_is_bit_identical_to_the_two_calls(cfg):
    import torch
    inp = syn.make_inputs(cfg, DT)
    kw = U.geom_kw(cfg)
    xd, dyd, wd = U.to_dev(inp, "x", DT), U.to_dev(inp, "dy", DT), U.to_dev(inp, "w", DT)
    yd = U.to_dev(inp, "y_saved", DT) if cfg.relu else None
    scd = U.to_dev(inp, "scale", DT) if cfg.affine else None
    sxd, sgd = nm.nm_fp8_row_scales(xd, 1), nm.nm_fp8_row_scales(dyd, 1)
    swtd = nm.nm_fp8_dgrad_weight_scales(wd, scd)
    dx, dres = nm.nm_conv1d_bwd_data_fp8(dyd, sgd, wd, swtd, cfg.T, y=yd, scale=scd, relu=cfg.relu, want_dres=True, **kw)
    dw = nm.nm_conv1d_bwd_weight_fp8(xd, sxd, dyd, sgd, cfg.K, y=yd, scale=scd, relu=cfg.relu, **kw)
    dx1, dres1, dw1 = nm.nm_conv1d_bwd_fp8(xd, sxd, dyd, sgd, wd, swtd, y=yd, scale=scd, relu=cfg.relu, want_dres=True, **kw)
    assert torch.equal(dx1, dx) and torch.equal(dres1, dres) and torch.equal(dw1, dw)
    dx2, dres2, dw2 = nm.nm_conv1d_bwd_fp8(xd, sxd, dyd, sgd, wd, swtd, y=yd, scale=scd, relu=cfg.relu, **kw)
    assert dres2 is None and torch.equal(dx2, dx) and torch.equal(dw2, dw)
