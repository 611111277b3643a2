"""CPU oracle of the decoder tail: per-frame class log-probabilities.

TEST INFRASTRUCTURE ONLY: imported by ``tests/`` and by the benchmark's CPU-baseline leg.  The GPU
product path never imports this module and this module never imports the GPU package.

The ASR example of the paper (Section 4.1.1) feeds the encoder output to a CTC decoder module whose
output is named log_probs and goes to the CTC loss; the paper gives no formula.  The textbook
definition is used: a 1x1 convolution from the encoder channels to the vocabulary (one logit per
class and frame) followed by a log-softmax over the classes of each frame,

    z[b,c,t]    = sum_ci w[c,ci] * x[b,ci,t] + bias[c]
    logp[b,c,t] = z[b,c,t] - log( sum_c' exp(z[b,c',t]) ),

all in float64 on numpy arrays ([B][Cin][T] activations, [Ncls][Cin] weights, [Ncls] bias).
"""
from __future__ import annotations

from typing import Optional

import numpy as np


def decoder_logits(x: np.ndarray, w: np.ndarray, bias: Optional[np.ndarray] = None) -> np.ndarray:
    """z[b,c,t] = sum_ci w[c,ci] x[b,ci,t] + bias[c]."""
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    B, Cin, T = x.shape
    Ncls, Cin_w = w.shape
    if Cin_w != Cin:
        raise ValueError("channel counts of x and w differ")
    z = np.empty((B, Ncls, T), dtype=np.float64)
    for b in range(B):
        z[b] = w @ x[b]
    if bias is not None:
        z += np.asarray(bias, dtype=np.float64).reshape(1, Ncls, 1)
    return z


def log_softmax_over_classes(z: np.ndarray) -> np.ndarray:
    """logp = z - log(sum_c exp(z)) along axis 1; the largest logit of a frame is taken out of the
    exponentials first so that none of them overflows (the result does not depend on it)."""
    z = np.asarray(z, dtype=np.float64)
    m = z.max(axis=1, keepdims=True)
    return z - m - np.log(np.exp(z - m).sum(axis=1, keepdims=True))


def decoder_logsoftmax(x: np.ndarray, w: np.ndarray, bias: Optional[np.ndarray] = None) -> np.ndarray:
    """logp[b,c,t] of the decoder tail."""
    return log_softmax_over_classes(decoder_logits(x, w, bias))
