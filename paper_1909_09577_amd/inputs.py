"""Seeded synthetic inputs for the conv1d sub-block, shared by tests and the benchmark.

This module holds no arithmetic of the method: only the layer geometries of the
Jasper-shaped workloads, the random draws, and the bf16 <-> float bit conversions
needed to hand identical bits to every consumer.  It depends on numpy only.

Recipe.  With ``rng = numpy.random.default_rng(seed)`` the tensors are drawn in
float32 in this fixed order: x ~ N(0,1) [B,Cin,T]; w ~ N(0, variance 1/(Cin*K))
[Cout,Cin,K]; scale ~ U(0.5,1.5) [Cout]; shift ~ N(0, std 0.1) [Cout];
residual ~ N(0,1) [B,Cout,T_out]; dy ~ N(0,1) [B,Cout,T_out]; and last a stand-in for
a saved forward output, y_saved = max(N(0,1), 0) [B,Cout,T_out] (about half zeros, like
a post-ReLU activation), used by backward-only checks.  All seven are always drawn (so
the stream does not depend on which are used).  For the bf16 workloads x,
w, residual and dy are then rounded to bf16 (round to nearest even) and it is those
rounded values that every consumer sees; scale and shift stay float32.  The
activations stand in for the spectrogram-derived feature maps of the paper's
Jasper encoder (Section 4.1.1); no dataset is involved.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Optional

import numpy as np


@dataclass(frozen=True)
class LayerCfg:
    """Geometry and epilogue of one conv1d sub-block."""
    name: str
    B: int
    Cin: int
    Cout: int
    T: int
    K: int
    stride: int = 1
    dilation: int = 1
    pad: int = 0
    affine: bool = True
    relu: bool = True
    residual: bool = False
    seed: int = 0
    # Length of the layer's output rows.  It is part of the workload's shape and is given as data by
    # whoever builds the workload (the named ones below state it; tests take it from the oracle, the
    # benchmark from the library): this module shapes random draws with it and computes nothing.
    T_out: int = -1

    def __post_init__(self):
        if self.T_out < 1:
            raise ValueError(f"{self.name}: T_out (the output length of the layer) must be given")

    @property
    def flops_per_pass(self) -> int:
        """Nominal 2*B*Cout*T_out*Cin*K (padded taps counted)."""
        return 2 * self.B * self.Cout * self.T_out * self.Cin * self.K

    def dims(self):
        return (self.B, self.Cin, self.Cout, self.T, self.K, self.stride, self.dilation, self.pad)


# The single-layer workloads.
TINY = LayerCfg("tiny_64to256_k11", B=2, Cin=64, Cout=256, T=200, K=11, pad=5, residual=False, seed=0, T_out=200)
JASPER_B1 = LayerCfg("b1_256_k11", B=32, Cin=256, Cout=256, T=800, K=11, pad=5, residual=True, seed=1, T_out=800)
JASPER_B3 = LayerCfg("b3_512_k17", B=32, Cin=512, Cout=512, T=800, K=17, pad=8, residual=True, seed=2, T_out=800)
EPILOG_A = LayerCfg("epilog_768to896_k29_d2", B=32, Cin=768, Cout=896, T=800, K=29, dilation=2,
                    pad=28, seed=3, T_out=800)
EPILOG_B = LayerCfg("epilog_896to1024_k1", B=32, Cin=896, Cout=1024, T=800, K=1, seed=4, T_out=800)
EPILOG_C = LayerCfg("epilog_1024to29_k1", B=32, Cin=1024, Cout=29, T=800, K=1, affine=False,
                    relu=False, seed=5, T_out=800)

SINGLE_LAYER_CFGS = [TINY, JASPER_B1, JASPER_B3, EPILOG_A, EPILOG_B, EPILOG_C]
HEADLINE = JASPER_B3


def jasper_10x5_layers(B: int = 32, T_in: int = 1600, seed: int = 4) -> List[dict]:
    """Layer list of the 10x5-shaped encoder stack.

    Each entry is ``{"cfg": LayerCfg, "role": ..., "block": i}`` with role one of
    "prolog", "sub" (sub-block j of a block; the 5th takes the block's residual),
    "proj" (the block's K=1 residual projection: affine, no ReLU), "epilog".
    Padding is "same": dilation*(K-1)/2.
    """
    layers: List[dict] = []
    n = 0

    def add(role, block, **kw):
        nonlocal n
        cfg = LayerCfg(name=f"L{n:02d}_{role}", B=B, seed=seed * 1000 + n, **kw)
        layers.append({"cfg": cfg, "role": role, "block": block})
        n += 1
        return cfg

    if T_in % 2:
        raise ValueError("T_in must be even (the stride-2 prolog halves it)")
    T = T_in // 2  # K=11, stride 2, pad 5 on an even length; every later layer keeps the length ("same" padding)
    add("prolog", -1, Cin=64, Cout=256, T=T_in, K=11, stride=2, pad=5, T_out=T)
    cin = 256
    spec = [(256, 11), (256, 11), (384, 13), (384, 13), (512, 17), (512, 17), (640, 21), (640, 21),
            (768, 25), (768, 25)]
    for bi, (ch, k) in enumerate(spec):
        add("proj", bi, Cin=cin, Cout=ch, T=T, K=1, pad=0, relu=False, T_out=T)
        c_in = cin
        for j in range(5):
            add("sub", bi, Cin=c_in, Cout=ch, T=T, K=k, pad=(k - 1) // 2, residual=(j == 4), T_out=T)
            c_in = ch
        cin = ch
    add("epilog", 10, Cin=cin, Cout=896, T=T, K=29, dilation=2, pad=28, T_out=T)
    add("epilog", 10, Cin=896, Cout=1024, T=T, K=1, T_out=T)
    add("epilog", 10, Cin=1024, Cout=29, T=T, K=1, affine=False, relu=False, T_out=T)
    return layers


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns.
    Inputs here are finite, so NaN handling is not needed."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(bits).astype(np.float64)


def make_inputs(cfg: LayerCfg, dtype: str = "bf16", seed: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Draw the six tensors of one layer.

    Returns float32 arrays under "x","w","scale","shift","residual","dy","y_saved" holding the
    values every consumer must use (already bf16-representable when dtype == "bf16"),
    plus, for bf16, the uint16 bit patterns under "x_bits", "w_bits", "residual_bits",
    "dy_bits", "y_saved_bits".  Tensors a layer does not use are still returned; the caller drops them.
    """
    if dtype not in ("bf16", "f32"):
        raise ValueError("dtype must be 'bf16' or 'f32'")
    rng = np.random.default_rng(cfg.seed if seed is None else seed)
    To = cfg.T_out
    out: Dict[str, np.ndarray] = {}
    out["x"] = rng.standard_normal((cfg.B, cfg.Cin, cfg.T), dtype=np.float32)
    std_w = np.float32(1.0 / np.sqrt(cfg.Cin * cfg.K))
    out["w"] = rng.standard_normal((cfg.Cout, cfg.Cin, cfg.K), dtype=np.float32) * std_w
    out["scale"] = rng.uniform(0.5, 1.5, size=cfg.Cout).astype(np.float32)
    out["shift"] = (rng.standard_normal(cfg.Cout, dtype=np.float32) * np.float32(0.1))
    out["residual"] = rng.standard_normal((cfg.B, cfg.Cout, To), dtype=np.float32)
    out["dy"] = rng.standard_normal((cfg.B, cfg.Cout, To), dtype=np.float32)
    out["y_saved"] = np.maximum(rng.standard_normal((cfg.B, cfg.Cout, To), dtype=np.float32), np.float32(0))
    if dtype == "bf16":
        for name in ("x", "w", "residual", "dy", "y_saved"):
            bits = f32_to_bf16_bits(out[name])
            out[name + "_bits"] = bits
            out[name] = bf16_bits_to_f32(bits)
    return out


def shrink(cfg: LayerCfg, **kw) -> LayerCfg:
    """A copy of a workload with some fields replaced (e.g. a smaller batch)."""
    return replace(cfg, **kw)
