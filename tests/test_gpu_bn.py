"""GPU parity of the block with training-mode BatchNorm (nm_conv1d_bn_fwd / nm_conv1d_bn_bwd) against the
oracle: conv1d_oracle for the convolution and its gradients, bn_oracle for the normalisation.

Forward: z is compared with the oracle's convolution; the statistics and y are computed by the library
from the stored z, so they are compared with the oracle's BatchNorm applied to the z the GPU stored (for
float32 storage that is the oracle's own z to 1e-5).  Backward: the saved tensors and statistics come from
the oracle (rounded to storage on the host), never from the GPU.  Gates as in test_gpu_parity.py; the
per-channel float32 outputs (mean, invstd, dgamma, dbeta) are held to the float32 gate.
"""
import numpy as np
import pytest

import _util as U
from oracle import bn_oracle as bno
from oracle import conv1d_oracle as orc
from paper_1909_09577_amd import binding as nm
from paper_1909_09577_amd import inputs as syn
from paper_1909_09577_amd.inputs import LayerCfg

pytestmark = pytest.mark.gpu
EPS = 1e-3


def L(name, B, Cin, Cout, T, K, stride=1, dilation=1, pad=0, relu=True, residual=False, seed=41):
    return LayerCfg(name, B, Cin, Cout, T, K, stride, dilation, pad, True, relu, residual, seed,
                    T_out=orc.out_len(T, K, stride, dilation, pad))


CASES = [
    L("bn_small", 2, 8, 8, 40, 3, pad=1, residual=True),
    L("bn_odd_len", 3, 12, 20, 37, 5, pad=2),                      # T % 8 != 0: element-wise passes, plain kernels
    L("bn_ragged", 3, 72, 100, 336, 11, pad=5, residual=True),
    L("bn_k17", 4, 128, 192, 320, 17, pad=8, residual=True),
    L("bn_k1_proj", 2, 256, 384, 320, 1, relu=False),
    L("bn_stride2", 2, 64, 96, 400, 11, stride=2, pad=5),
    L("bn_b9", 9, 32, 64, 160, 7, pad=3, residual=True),            # more batch items than reduction groups
    # statistics written by the convolution kernel's epilogue (unrolled engine): tiles ragged in rows and time
    L("bn_k11_ragged_tiles", 3, 128, 200, 328, 11, pad=5, residual=True),
    L("bn_k25_ragged_tiles", 2, 256, 72, 168, 25, pad=12),
]


def chan(a):
    return np.asarray(a, dtype=np.float64)


@pytest.mark.parametrize("mode", ["bf16-auto", "bf16-direct", "f32-direct"])
@pytest.mark.parametrize("cfg", CASES, ids=lambda c: c.name)
def test_bn_block_forward_and_backward(cfg, mode):
    import torch
    dtype, fd = mode.split("-")[0], mode.endswith("direct")
    inp = syn.make_inputs(cfg, dtype)
    kw = U.geom_kw(cfg)
    # gamma, beta: the recipe's scale ~ U(0.5, 1.5) and shift ~ N(0, 0.1)
    gamma, beta = inp["scale"], inp["shift"]
    res = inp["residual"] if cfg.residual else None
    x, w = U.to_dev(inp, "x", dtype), U.to_dev(inp, "w", dtype)
    gd, bd = U.to_dev(inp, "scale", dtype), U.to_dev(inp, "shift", dtype)
    rd = U.to_dev(inp, "residual", dtype) if cfg.residual else None

    z, y, mean, invstd = nm.nm_conv1d_bn_fwd(x, w, gd, bd, rd, eps=EPS, relu=cfg.relu, force_direct=fd, **kw)
    z_ref = orc.block_fwd(inp["x"], inp["w"], None, None, None, False, **kw)
    zg = U.to_host_f64(z)
    U.assert_close(zg, z_ref, dtype, f"{cfg.name} z")
    y_ref, mean_ref, invstd_ref = bno.bn_train_fwd(zg, gamma, beta, EPS, res, cfg.relu)
    # mean is compared on the scale of the channel's spread (it is close to zero itself)
    std_ref = 1.0 / invstd_ref
    assert np.max(np.abs(chan(mean.cpu().numpy()) - mean_ref) / std_ref) <= 1e-5
    U.assert_close(chan(invstd.cpu().numpy()), invstd_ref, "f32", f"{cfg.name} invstd")
    U.assert_close(U.to_host_f64(y), y_ref, dtype, f"{cfg.name} y")

    # backward from saved tensors of the oracle's own forward, rounded to storage on the host
    z_saved = U.round_to_storage(z_ref, dtype)
    y_o, mean_o, invstd_o = bno.bn_train_fwd(z_saved.astype(np.float64), gamma, beta, EPS, res, cfg.relu)
    y_saved = U.round_to_storage(y_o, dtype)
    mean32, invstd32 = mean_o.astype(np.float32), invstd_o.astype(np.float32)
    dz_ref, dres_ref, dgamma_ref, dbeta_ref = bno.bn_train_bwd(inp["dy"], z_saved, y_saved, gamma, mean32, invstd32, cfg.relu)
    dx_ref = orc.bwd_data(dz_ref, inp["w"], cfg.T, **kw)
    dw_ref = orc.bwd_weight(inp["x"], dz_ref, cfg.K, **kw)
    dx, dres, dw, dgamma, dbeta = nm.nm_conv1d_bn_bwd(
        x, w, gd, U.arr_to_dev(z_saved, dtype), U.arr_to_dev(y_saved, dtype) if cfg.relu else None,
        torch.from_numpy(mean32).cuda(), torch.from_numpy(invstd32).cuda(), U.to_dev(inp, "dy", dtype),
        relu=cfg.relu, want_dres=True, force_direct=fd, **kw)
    np.testing.assert_array_equal(U.to_host_f64(dres), dres_ref)
    U.assert_close(chan(dgamma.cpu().numpy()), dgamma_ref, "f32", f"{cfg.name} dgamma")
    U.assert_close(chan(dbeta.cpu().numpy()), dbeta_ref, "f32", f"{cfg.name} dbeta")
    U.assert_close(U.to_host_f64(dx), dx_ref, dtype, f"{cfg.name} dx")
    U.assert_close(U.to_host_f64(dw), dw_ref, dtype, f"{cfg.name} dw", rms_bound=U.RMS_DW_BF16)


def test_bn_forward_statistics_from_private_and_shared_tiles():
    """1280 tiles on 256 CUs: every wavefront finishes a tile of its own and every workgroup one more with a split
    reduction; both epilogues write their parts of the statistics.  Forward only, whole tensors."""
    cfg = L("bn_1280_tiles", 20, 128, 512, 1280, 13, pad=6, residual=True)
    dtype = "bf16"
    inp = syn.make_inputs(cfg, dtype)
    kw = U.geom_kw(cfg)
    x, w, gd, bd, rd = (U.to_dev(inp, n, dtype) for n in ("x", "w", "scale", "shift", "residual"))
    z, y, mean, invstd = nm.nm_conv1d_bn_fwd(x, w, gd, bd, rd, eps=EPS, relu=True, **kw)
    zg = U.to_host_f64(z)
    U.assert_close(zg, orc.block_fwd(inp["x"], inp["w"], None, None, None, False, **kw), dtype, "z")
    y_ref, mean_ref, invstd_ref = bno.bn_train_fwd(zg, inp["scale"], inp["shift"], EPS, inp["residual"], True)
    assert np.max(np.abs(chan(mean.cpu().numpy()) - mean_ref) * invstd_ref) <= 1e-5
    U.assert_close(chan(invstd.cpu().numpy()), invstd_ref, "f32", "invstd")
    U.assert_close(U.to_host_f64(y), y_ref, dtype, "y")


def test_bn_backward_accumulates_and_is_deterministic():
    import torch
    cfg = CASES[2]
    dtype = "bf16"
    inp = syn.make_inputs(cfg, dtype)
    kw = U.geom_kw(cfg)
    x, w, gd, bd = (U.to_dev(inp, n, dtype) for n in ("x", "w", "scale", "shift"))
    rd, dy = U.to_dev(inp, "residual", dtype), U.to_dev(inp, "dy", dtype)
    z, y, mean, invstd = nm.nm_conv1d_bn_fwd(x, w, gd, bd, rd, eps=EPS, relu=True, **kw)
    z2, y2, mean2, invstd2 = nm.nm_conv1d_bn_fwd(x, w, gd, bd, rd, eps=EPS, relu=True, **kw)
    assert torch.equal(y, y2) and torch.equal(mean, mean2) and torch.equal(invstd, invstd2)
    a = nm.nm_conv1d_bn_bwd(x, w, gd, z, y, mean, invstd, dy, relu=True, want_dres=True, **kw)
    b = nm.nm_conv1d_bn_bwd(x, w, gd, z, y, mean, invstd, dy, relu=True, want_dres=True, **kw)
    for u, v in zip(a, b):
        assert torch.equal(u, v)
    dx, dres, dw, dgamma, dbeta = (t.clone() for t in a)
    nm.nm_conv1d_bn_bwd(x, w, gd, z, y, mean, invstd, dy, relu=True, accumulate=True, dw=dw, dgamma=dgamma, dbeta=dbeta, **kw)
    np.testing.assert_allclose(dw.cpu().numpy(), 2 * a[2].cpu().numpy(), rtol=1e-6)
    np.testing.assert_allclose(dgamma.cpu().numpy(), 2 * a[3].cpu().numpy(), rtol=1e-6)
    np.testing.assert_allclose(dbeta.cpu().numpy(), 2 * a[4].cpu().numpy(), rtol=1e-6)
