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


# ---- host <-> device (shared with the benchmark: paper_1909_09577_amd/device_inputs.py) ---------
from paper_1909_09577_amd.device_inputs import arr_to_dev, geom_kw, to_dev, to_host_f64  # noqa: E402,F401


def round_to_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    """float64 -> the float32 value the storage dtype would hold (host side, for inputs only)."""
    a32 = np.asarray(a, dtype=np.float32)
    if dtype == "f32":
        return a32
    return syn.bf16_bits_to_f32(syn.f32_to_bf16_bits(a32))


# ---- oracle on a LayerCfg --------------------------------------------------------------------
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
