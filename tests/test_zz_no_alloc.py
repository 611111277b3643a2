"""The forward entry point that allocates nothing (scratch in a fixed array inside the library),
called through the C ABI, against nm_conv1d_block_fwd on the same inputs: bit-identical outputs, on
two calls in a row, the second with a smaller geometry (the array keeps the first call's contents).
"""
import numpy as np
import pytest

import _util as U
from oracle import conv1d_oracle as orc
from paper_1909_09577_amd import binding as nm
from paper_1909_09577_amd import inputs as syn
from paper_1909_09577_amd.inputs import LayerCfg

pytestmark = pytest.mark.gpu


def L(name, B, Cin, Cout, T, K, stride=1, dilation=1, pad=0, affine=True, relu=True, residual=False, seed=21):
    return LayerCfg(name, B, Cin, Cout, T, K, stride, dilation, pad, affine, relu, residual, seed,
                    T_out=orc.out_len(T, K, stride, dilation, pad))


# first a layer that fills several tiles (packed weights: 2.4 MB of the 32 MiB array), then a smaller one
# with another tap count, then one on the plain kernels (odd length: no scratch at all)
CASES = [
    L("na_big", 4, 256, 256, 480, 17, pad=8, residual=True),
    L("na_small", 2, 72, 100, 176, 11, pad=5, residual=True),
    L("na_plain", 2, 40, 48, 333, 7, pad=3),
]


def test_forward_without_allocation_matches_the_workspace_entry_point():
    import torch
    dtype = "bf16"
    for cfg in CASES:
        inp = syn.make_inputs(cfg, dtype)
        x, w = U.to_dev(inp, "x", dtype), U.to_dev(inp, "w", dtype)
        scale, shift = U.to_dev(inp, "scale", dtype), U.to_dev(inp, "shift", dtype)
        res = U.to_dev(inp, "residual", dtype) if cfg.residual else None
        kw = U.geom_kw(cfg)
        y_ref = nm.nm_conv1d_block_fwd(x, w, scale, shift, res, relu=cfg.relu, **kw)
        y = torch.full_like(y_ref, float("nan"))
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        nm.nm_conv1d_block_fwd_static(x, w, scale, shift, res, y=y, relu=cfg.relu, **kw)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(y.view(torch.int16), y_ref.view(torch.int16)), cfg.name
        # and the result is the oracle's
        U.assert_close(U.to_host_f64(y), U.oracle_fwd(cfg, inp), dtype, f"{cfg.name} y")


def test_scratch_limit_is_reported():
    import torch
    # 768 -> 896 channels, 29 taps: 41 MB of packed weights, more than the fixed array holds
    x = torch.zeros(1, 768, 160, dtype=torch.bfloat16, device="cuda")
    w = torch.zeros(896, 768, 29, dtype=torch.bfloat16, device="cuda")
    y = torch.zeros(1, 896, 160, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(nm.NmError) as e:
        nm.nm_conv1d_block_fwd_static(x, w, y=y, dilation=2, pad=28)
    assert e.value.status == nm.NM_ERR_SCRATCH_LIMIT
