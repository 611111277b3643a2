"""Helpers shared by the GPU parity tests: the error metric, host<->device transfers of
seeded inputs, and one-call runners for the GPU path and the oracle."""
from __future__ import annotations

import numpy as np

from oracle import conv1d_oracle as orc
from paper_1909_09577_amd import inputs as syn

# Tolerances of the parity gate: max_i |g_i - o_i| / (|o_i| + rms(o)).
TOL_BF16 = 1e-2     # bf16 storage, float32 accumulation
TOL_F32 = 1e-5      # float32 storage
RMS_BF16 = 3e-3     # relative RMS error bound for a bf16-rounded output (expected ~1.1e-3)
RMS_DW_BF16 = 3e-3  # dw is float32 but is built from a bf16-rounded dz


def err_metrics(got: np.ndarray, ref: np.ndarray, rms_ref: float | None = None):
    """(max scaled error, relative RMS error); ``rms_ref`` overrides rms(ref) for samples."""
    got = np.asarray(got, dtype=np.float64).reshape(-1)
    ref = np.asarray(ref, dtype=np.float64).reshape(-1)
    assert got.shape == ref.shape
    assert np.isfinite(got).all(), "non-finite values in the GPU result"
    rms = float(np.sqrt(np.mean(ref * ref))) if rms_ref is None else float(rms_ref)
    if rms == 0.0:
        return (0.0 if np.array_equal(got, ref) else np.inf), 0.0
    diff = np.abs(got - ref)
    return float(np.max(diff / (np.abs(ref) + rms))), float(np.sqrt(np.mean(diff * diff)) / rms)


def assert_close(got, ref, dtype: str, what: str, rms_bound: float | None = None):
    tol = TOL_BF16 if dtype == "bf16" else TOL_F32
    mx, rr = err_metrics(got, ref)
    assert mx <= tol, f"{what}: max scaled error {mx:.3e} > {tol:g} (rel rms {rr:.3e})"
    if dtype == "bf16":
        bound = RMS_BF16 if rms_bound is None else rms_bound
        assert rr <= bound, f"{what}: relative rms error {rr:.3e} > {bound:g}"
    return mx, rr


# ---- host <-> device ---------------------------------------------------------------------
def to_dev(inp: dict, name: str, dtype: str):
    """Device tensor holding exactly the bits of inp[name] in the storage dtype."""
    import torch
    if name in ("scale", "shift") or dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(inp[name], dtype=np.float32)).cuda()
    bits = inp[name + "_bits"]
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def arr_to_dev(a: np.ndarray, dtype: str):
    """Device tensor of a float array; for bf16 the values must already be representable."""
    import torch
    if dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    bits = syn.f32_to_bf16_bits(np.ascontiguousarray(a, dtype=np.float32))
    assert np.array_equal(syn.bf16_bits_to_f32(bits), np.asarray(a, dtype=np.float32)), "not bf16-representable"
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def to_host_f64(t) -> np.ndarray:
    import torch
    torch.cuda.synchronize()
    if t.dtype == torch.bfloat16:
        bits = t.view(torch.int16).cpu().numpy().view(np.uint16)
        return syn.bf16_bits_to_f64(bits)
    return t.cpu().numpy().astype(np.float64)


def round_to_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    """float64 -> the float32 value the storage dtype would hold (host side, for inputs only)."""
    a32 = np.asarray(a, dtype=np.float32)
    if dtype == "f32":
        return a32
    return syn.bf16_bits_to_f32(syn.f32_to_bf16_bits(a32))


# ---- oracle on a LayerCfg --------------------------------------------------------------------
def geom_kw(cfg):
    return dict(stride=cfg.stride, dilation=cfg.dilation, pad=cfg.pad)


def oracle_fwd(cfg, inp):
    return orc.block_fwd(inp["x"], inp["w"], inp["scale"] if cfg.affine else None,
                         inp["shift"] if cfg.affine else None, inp["residual"] if cfg.residual else None,
                         cfg.relu, **geom_kw(cfg))


def oracle_bwd(cfg, inp, y_saved):
    """(dx, dw, dres) of the oracle for upstream gradient inp['dy'] and saved output y_saved."""
    dz, dres = orc.epilogue_bwd(inp["dy"], y_saved if cfg.relu else None, inp["scale"] if cfg.affine else None,
                                cfg.relu)
    dx = orc.bwd_data(dz, inp["w"], cfg.T, **geom_kw(cfg))
    dw = orc.bwd_weight(inp["x"], dz, cfg.K, **geom_kw(cfg))
    return dx, dw, dres
