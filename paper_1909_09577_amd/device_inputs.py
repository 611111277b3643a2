"""Host <-> device transfer of the seeded synthetic inputs (bit-exact for bf16 storage).

No arithmetic of the method lives here: a tensor goes to the device holding exactly the bits the
input recipe produced, and comes back widened exactly to float64.  torch is used for the device
memory only.
"""
from __future__ import annotations

import numpy as np

from . import inputs as syn


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


def geom_kw(cfg):
    return dict(stride=cfg.stride, dilation=cfg.dilation, pad=cfg.pad)
