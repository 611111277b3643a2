"""GPU parity of the three passes on padded batches (per-sample lengths) against the oracle.

The padding of x is filled with huge values and NaNs: a kernel that multiplies it by zero instead of
not reading it would produce NaNs.  Gates as in test_gpu_parity.py."""
import numpy as np
import pytest

import _util as U
from oracle import conv1d_oracle as orc
from paper_1909_09577_amd import binding as nm
from paper_1909_09577_amd import inputs as syn
from paper_1909_09577_amd.inputs import LayerCfg

pytestmark = pytest.mark.gpu


def L(name, B, Cin, Cout, T, K, stride=1, dilation=1, pad=0, affine=True, relu=True, residual=False, seed=31):
    return LayerCfg(name, B, Cin, Cout, T, K, stride, dilation, pad, affine, relu, residual, seed,
                    T_out=orc.out_len(T, K, stride, dilation, pad))


CASES = [
    (L("k_small", 3, 8, 8, 40, 3, pad=1, residual=True), [40, 17, 1]),
    (L("k_ragged", 3, 72, 100, 336, 11, pad=5, residual=True), [336, 200, 37]),
    (L("k_two_tiles", 2, 128, 192, 320, 17, pad=8), [163, 320]),
    (L("k_k1", 2, 256, 160, 400, 1, affine=False, relu=False), [400, 123]),
    (L("k_k1_bigtile", 2, 136, 1000, 200, 1, residual=True), [200, 77]),   # K=1 kernel, 512 x 128 tile (forward)
    (L("k_k1_bigtile_t", 2, 1000, 136, 200, 1), [131, 200]),               # the same tile in the input gradient
    (L("k_stride2", 2, 64, 96, 400, 11, stride=2, pad=5), [399, 201]),
    (L("k_dil2", 2, 96, 80, 248, 9, dilation=2, pad=8), [248, 100]),
    (L("k_zero_len", 2, 16, 16, 64, 5, pad=2), [0, 64]),
    (L("k_odd_len", 2, 40, 48, 333, 7, pad=3, residual=True), [333, 150]),
    # the weight-gradient kernel with shared staging (8 x 32 = 256 output tiles) and the K=1 kernel at full width
    (L("k_shared_wgrad", 2, 1024, 512, 160, 17, pad=8, affine=False, relu=False), [160, 77]),
    (L("k_shared_wgrad_k13", 3, 1024, 512, 240, 13, pad=6, affine=False, relu=False), [1, 239, 100]),
    # the same kernel walks only the units that reach below the valid length: empty items at both ends, fewer live
    # units than workgroups per tile, a batch with nothing in it (dw = 0, dx = 0)
    (L("k_shared_wgrad_gaps", 4, 1024, 512, 160, 17, pad=8, affine=False, relu=False), [0, 160, 0, 9]),
    (L("k_shared_wgrad_one_unit", 3, 1024, 512, 240, 13, pad=6, residual=True), [0, 0, 50]),
    (L("k_shared_wgrad_empty", 2, 1024, 512, 160, 17, pad=8, affine=False, relu=False), [0, 0]),
]


@pytest.mark.parametrize("force_direct", [False, True], ids=["auto", "direct"])
@pytest.mark.parametrize("case", CASES, ids=lambda c: c[0].name)
def test_masked_passes(case, force_direct):
    check_case(case[0], case[1], force_direct)


def test_masked_passes_full_size_full_tensor():
    """The headline block (B=32, 512 -> 512, K=17, T=800) on a ragged batch: lengths drawn uniformly from
    [T/2, T] with one full-length item, every output element of all three passes compared."""
    cfg = syn.shrink(syn.HEADLINE, B=syn.HEADLINE.B)
    rng = np.random.default_rng(77)
    lengths = rng.integers(cfg.T // 2, cfg.T + 1, cfg.B)
    lengths[5] = cfg.T
    lengths[11] = 437          # not a multiple of 8
    check_case(cfg, [int(n) for n in lengths], False)


def check_case(cfg, lengths, force_direct):
    import torch
    dtype = "bf16"
    inp = syn.make_inputs(cfg, dtype)
    lens = np.asarray(lengths, dtype=np.int32)
    kw = U.geom_kw(cfg)
    scale = inp["scale"] if cfg.affine else None
    shift = inp["shift"] if cfg.affine else None
    res = inp["residual"] if cfg.residual else None
    # poison the padding of the x that goes to the GPU
    x_bits = inp["x_bits"].copy()
    for b, n in enumerate(lens):
        x_bits[b, :, n:] = np.where(np.arange(cfg.T - n) % 2 == 0, 0x7FC0, 0x7F00).astype(np.uint16)  # NaN, 1.7e38
    xd = torch.from_numpy(x_bits.view(np.int16)).cuda().view(torch.bfloat16)
    ld = torch.from_numpy(lens).cuda()
    wd = U.to_dev(inp, "w", dtype)
    sc = U.to_dev(inp, "scale", dtype) if cfg.affine else None
    sh = U.to_dev(inp, "shift", dtype) if cfg.affine else None
    rd = U.to_dev(inp, "residual", dtype) if cfg.residual else None

    y = nm.nm_conv1d_block_fwd(xd, wd, sc, sh, rd, relu=cfg.relu, force_direct=force_direct, lengths=ld, **kw)
    y_ref = orc.block_fwd_masked(inp["x"], inp["w"], lens, scale, shift, res, cfg.relu, **kw)
    U.assert_close(U.to_host_f64(y), y_ref, dtype, f"{cfg.name} y")

    y_saved = U.round_to_storage(y_ref, dtype)
    ysv = U.arr_to_dev(y_saved, dtype) if cfg.relu else None
    dyd = U.to_dev(inp, "dy", dtype)
    dx, dres = nm.nm_conv1d_bwd_data(dyd, wd, cfg.T, y=ysv, scale=sc, relu=cfg.relu, want_dres=True,
                                     force_direct=force_direct, lengths=ld, **kw)
    dw = nm.nm_conv1d_bwd_weight(xd, dyd, cfg.K, y=ysv, scale=sc, relu=cfg.relu, force_direct=force_direct, lengths=ld, **kw)
    dz, dres_ref = orc.epilogue_bwd(inp["dy"], y_saved.astype(np.float64) if cfg.relu else None, scale, cfg.relu)
    dx_ref = orc.bwd_data_masked(dz, inp["w"], cfg.T, lens, **kw)
    dw_ref = orc.bwd_weight_masked(inp["x"], dz, cfg.K, lens, **kw)
    dxh = U.to_host_f64(dx)
    for b, n in enumerate(lens):
        assert np.all(dxh[b, :, n:] == 0), "the input gradient on the padding must be exactly zero"
    # the gate is applied to the valid part: the exact zeros of the padding would only shrink rms(o)
    valid = np.concatenate([dxh[b, :, :n].reshape(-1) for b, n in enumerate(lens)])
    valid_ref = np.concatenate([dx_ref[b, :, :n].reshape(-1) for b, n in enumerate(lens)])
    if valid.size:
        U.assert_close(valid, valid_ref, dtype, f"{cfg.name} dx")
        U.assert_close(U.to_host_f64(dw), dw_ref, dtype, f"{cfg.name} dw", rms_bound=U.RMS_DW_BF16)
    else:  # a batch with nothing in it: every x reads as zero, so the weight gradient is exactly zero
        assert not np.any(dw_ref) and not np.any(U.to_host_f64(dw)), f"{cfg.name}: dw of an empty batch"
    # both gradients from one call: bit-identical to the two calls
    dx1, dres1, dw1 = nm.nm_conv1d_bwd(xd, dyd, wd, y=ysv, scale=sc, relu=cfg.relu, want_dres=True, force_direct=force_direct,
                                       lengths=ld, **kw)
    assert torch.equal(dx1, dx) and torch.equal(dres1, dres) and torch.equal(dw1, dw), f"{cfg.name}: fused masked backward"
    np.testing.assert_array_equal(U.to_host_f64(dres), dres_ref)
