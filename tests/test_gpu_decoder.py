"""GPU parity of the decoder tail (nm_decoder_logsoftmax_fwd) against oracle/decoder_oracle.py.

Gate: max |g - o| / (|o| + rms(o)) <= 5e-5.  The logits are float32 sums of exact bf16 x bf16
products (<= 1024 terms: error about 2e-6 of their size), exp/log are float32 library functions, the
output is float32 and log-probabilities have an rms of a few units, so errors stay below 1e-5 of
that; the float32-storage path sums in float32 blocks and meets the same gate."""
import numpy as np
import pytest

import _util as U
from oracle import decoder_oracle as dorc
from paper_1909_09577_amd import binding as nm
from paper_1909_09577_amd import inputs as syn

pytestmark = pytest.mark.gpu
TOL = 5e-5


def make(B, Cin, Ncls, T, seed, dtype):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((B, Cin, T), dtype=np.float32)
    w = rng.standard_normal((Ncls, Cin), dtype=np.float32) / np.float32(np.sqrt(Cin))
    bias = (rng.standard_normal(Ncls, dtype=np.float32) * np.float32(0.5))
    if dtype == "bf16":
        x = syn.bf16_bits_to_f32(syn.f32_to_bf16_bits(x))
        w = syn.bf16_bits_to_f32(syn.f32_to_bf16_bits(w))
    return x, w, bias


def run(x, w, bias, dtype, force_direct):
    import torch
    xd, wd = U.arr_to_dev(x, dtype), U.arr_to_dev(w, dtype)
    bd = torch.from_numpy(bias).cuda() if bias is not None else None
    return nm.nm_decoder_logsoftmax_fwd(xd, wd, bd, force_direct=force_direct).cpu().numpy().astype(np.float64)


CASES = [  # B, Cin, Ncls, T
    (2, 64, 29, 96), (3, 1024, 29, 200), (1, 48, 5, 40), (2, 32, 32, 264), (1, 16, 1, 8),
    (2, 40, 29, 64),      # Cin % 16 != 0: plain kernel
    (2, 64, 29, 50),      # T % 8 != 0: plain kernel
    (1, 64, 70, 64),      # more than 32 classes: plain kernel
]


@pytest.mark.parametrize("force_direct", [False, True], ids=["auto", "direct"])
@pytest.mark.parametrize("case", CASES, ids=lambda c: "x".join(map(str, c)))
def test_decoder_tail_full_tensor(case, force_direct):
    B, Cin, Ncls, T = case
    x, w, bias = make(B, Cin, Ncls, T, 3, "bf16")
    got = run(x, w, bias, "bf16", force_direct)
    ref = dorc.decoder_logsoftmax(x, w, bias)
    mx, _ = U.err_metrics(got, ref)
    assert mx <= TOL, f"max scaled error {mx:.3e}"
    np.testing.assert_allclose(np.exp(got).sum(axis=1), 1.0, rtol=1e-5)
    # without a bias
    got0 = run(x, w, None, "bf16", force_direct)
    mx, _ = U.err_metrics(got0, dorc.decoder_logsoftmax(x, w))
    assert mx <= TOL


def test_decoder_tail_float32_storage():
    x, w, bias = make(2, 96, 29, 120, 5, "f32")
    got = run(x, w, bias, "f32", False)
    mx, _ = U.err_metrics(got, dorc.decoder_logsoftmax(x, w, bias))
    assert mx <= TOL


def test_decoder_tail_full_size_and_large_logits():
    # the encoder's output size: B=32, 1024 channels, 800 frames, 29 classes
    x, w, bias = make(32, 1024, 29, 800, 7, "bf16")
    got = run(x, w, bias, "bf16", False)
    ref = dorc.decoder_logsoftmax(x, w, bias)
    mx, _ = U.err_metrics(got, ref)
    assert mx <= TOL, f"max scaled error {mx:.3e}"
    # logits of size 100: exponentials must not overflow
    got = run(x[:1] * 64, w * 2, bias, "bf16", False)
    assert np.isfinite(got).all()
    mx, _ = U.err_metrics(got, dorc.decoder_logsoftmax(x[:1] * 64, w * 2, bias))
    assert mx <= TOL
