"""ctypes front end of the CPU oracle (``conv1d_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's CPU-baseline leg.  The GPU product path never imports this module and
this module never imports the GPU package.

Every function takes and returns ``numpy`` float64 arrays in the layouts the C file
documents ([B][C][T] activations, [Cout][Cin][K] weights).  The mathematics is the
plain definition of the Jasper sub-block (paper Section 4.1.1 names the encoder;
Section 3 leaves forward/backward to the backend, so the definition is the textbook
one and is written out in the C file's header).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv1d_oracle.c")
_LIB = os.path.join(_HERE, "libconv1d_oracle.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall", "-Wextra",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


_D = ctypes.POINTER(ctypes.c_double)
_I64 = ctypes.POINTER(ctypes.c_int64)


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i = ctypes.c_int
        dims = [i] * 8
        lib.oracle_conv1d_out_len.argtypes = [i] * 5
        lib.oracle_conv1d_out_len.restype = i
        lib.oracle_num_threads.argtypes = []
        lib.oracle_num_threads.restype = i
        lib.oracle_conv1d_block_fwd.argtypes = dims + [_D, _D, _D, _D, _D, i, _D, _D]
        lib.oracle_conv1d_block_fwd.restype = None
        lib.oracle_conv1d_block_fwd_at.argtypes = dims + [_D, _D, _D, _D, _D, i, ctypes.c_long, _I64, _D]
        lib.oracle_conv1d_block_fwd_at.restype = None
        lib.oracle_conv1d_epilogue_bwd.argtypes = [i, i, i, _D, _D, _D, i, _D, _D]
        lib.oracle_conv1d_epilogue_bwd.restype = None
        lib.oracle_conv1d_bwd_data.argtypes = dims + [_D, _D, _D]
        lib.oracle_conv1d_bwd_data.restype = None
        lib.oracle_conv1d_bwd_data_at.argtypes = dims + [_D, _D, ctypes.c_long, _I64, _D]
        lib.oracle_conv1d_bwd_data_at.restype = None
        lib.oracle_conv1d_bwd_weight.argtypes = dims + [_D, _D, _D]
        lib.oracle_conv1d_bwd_weight.restype = None
        lib.oracle_conv1d_bwd_weight_at.argtypes = dims + [_D, _D, ctypes.c_long, _I64, _D]
        lib.oracle_conv1d_bwd_weight_at.restype = None
        _lib = lib
    return _lib


def _f64(a, shape) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float64)
    if a.shape != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {a.shape}")
    return a


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(_D)


def _opt(a, shape):
    return None if a is None else _f64(a, shape)


def out_len(T: int, K: int, stride: int, dilation: int, pad: int) -> int:
    """T_out of the convolution, or -1 when the arguments admit no output."""
    return int(_load().oracle_conv1d_out_len(T, K, stride, dilation, pad))


def _dims(x_shape, w_shape, stride, dilation, pad):
    B, Cin, T = x_shape
    Cout, Cin2, K = w_shape
    if Cin2 != Cin:
        raise ValueError("channel mismatch between x and w")
    To = out_len(T, K, stride, dilation, pad)
    if To <= 0:
        raise ValueError("no output positions")
    return B, Cin, Cout, T, K, To


def block_fwd(x, w, scale=None, shift=None, residual=None, relu=False, *, stride=1, dilation=1,
              pad=0, return_z=False):
    """y = [relu](scale*conv(x,w)+shift [+ residual]) in float64.  Optionally also z."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    w = np.ascontiguousarray(w, dtype=np.float64)
    B, Cin, Cout, T, K, To = _dims(x.shape, w.shape, stride, dilation, pad)
    scale = _opt(scale, (Cout,))
    shift = _opt(shift, (Cout,))
    residual = _opt(residual, (B, Cout, To))
    y = np.empty((B, Cout, To), dtype=np.float64)
    z = np.empty_like(y) if return_z else None
    _load().oracle_conv1d_block_fwd(B, Cin, Cout, T, K, stride, dilation, pad, _p(x), _p(w),
                                    _p(scale), _p(shift), _p(residual), int(bool(relu)), _p(y), _p(z))
    return (y, z) if return_z else y


def block_fwd_at(x, w, index, scale=None, shift=None, residual=None, relu=False, *, stride=1,
                 dilation=1, pad=0):
    """block_fwd evaluated only at the flat output indices ``index``."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    w = np.ascontiguousarray(w, dtype=np.float64)
    B, Cin, Cout, T, K, To = _dims(x.shape, w.shape, stride, dilation, pad)
    scale = _opt(scale, (Cout,))
    shift = _opt(shift, (Cout,))
    residual = _opt(residual, (B, Cout, To))
    index = np.ascontiguousarray(index, dtype=np.int64)
    if index.size and (index.min() < 0 or index.max() >= B * Cout * To):
        raise ValueError("index out of range")
    y = np.empty(index.shape, dtype=np.float64)
    _load().oracle_conv1d_block_fwd_at(B, Cin, Cout, T, K, stride, dilation, pad, _p(x), _p(w),
                                       _p(scale), _p(shift), _p(residual), int(bool(relu)),
                                       index.size, index.ctypes.data_as(_I64), _p(y))
    return y


def epilogue_bwd(dy, y_saved=None, scale=None, relu=False):
    """(dz, dres) from the upstream gradient of the block output."""
    dy = np.ascontiguousarray(dy, dtype=np.float64)
    B, Cout, To = dy.shape
    if relu and y_saved is None:
        raise ValueError("relu backward needs the saved output")
    y_saved = _opt(y_saved, dy.shape)
    scale = _opt(scale, (Cout,))
    dz = np.empty_like(dy)
    dres = np.empty_like(dy)
    _load().oracle_conv1d_epilogue_bwd(B, Cout, To, _p(dy), _p(y_saved), _p(scale),
                                       int(bool(relu)), _p(dz), _p(dres))
    return dz, dres


def bwd_data(dz, w, T, *, stride=1, dilation=1, pad=0):
    """dx [B][Cin][T] from dz [B][Cout][T_out] (scatter form)."""
    dz = np.ascontiguousarray(dz, dtype=np.float64)
    w = np.ascontiguousarray(w, dtype=np.float64)
    Cout, Cin, K = w.shape
    B = dz.shape[0]
    To = out_len(T, K, stride, dilation, pad)
    if dz.shape != (B, Cout, To):
        raise ValueError("dz shape does not match the convolution geometry")
    dx = np.empty((B, Cin, T), dtype=np.float64)
    _load().oracle_conv1d_bwd_data(B, Cin, Cout, T, K, stride, dilation, pad, _p(dz), _p(w), _p(dx))
    return dx


def bwd_data_at(dz, w, T, index, *, stride=1, dilation=1, pad=0):
    """dx at flat indices of [B][Cin][T] (gather form)."""
    dz = np.ascontiguousarray(dz, dtype=np.float64)
    w = np.ascontiguousarray(w, dtype=np.float64)
    Cout, Cin, K = w.shape
    B = dz.shape[0]
    To = out_len(T, K, stride, dilation, pad)
    if dz.shape != (B, Cout, To):
        raise ValueError("dz shape does not match the convolution geometry")
    index = np.ascontiguousarray(index, dtype=np.int64)
    if index.size and (index.min() < 0 or index.max() >= B * Cin * T):
        raise ValueError("index out of range")
    dx = np.empty(index.shape, dtype=np.float64)
    _load().oracle_conv1d_bwd_data_at(B, Cin, Cout, T, K, stride, dilation, pad, _p(dz), _p(w),
                                      index.size, index.ctypes.data_as(_I64), _p(dx))
    return dx


def bwd_weight(x, dz, K, *, stride=1, dilation=1, pad=0):
    """dw [Cout][Cin][K] from x [B][Cin][T] and dz [B][Cout][T_out]."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    dz = np.ascontiguousarray(dz, dtype=np.float64)
    B, Cin, T = x.shape
    Cout = dz.shape[1]
    To = out_len(T, K, stride, dilation, pad)
    if dz.shape != (B, Cout, To):
        raise ValueError("dz shape does not match the convolution geometry")
    dw = np.empty((Cout, Cin, K), dtype=np.float64)
    _load().oracle_conv1d_bwd_weight(B, Cin, Cout, T, K, stride, dilation, pad, _p(x), _p(dz), _p(dw))
    return dw


def bwd_weight_at(x, dz, K, index, *, stride=1, dilation=1, pad=0):
    """dw at flat indices of [Cout][Cin][K]."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    dz = np.ascontiguousarray(dz, dtype=np.float64)
    B, Cin, T = x.shape
    Cout = dz.shape[1]
    To = out_len(T, K, stride, dilation, pad)
    if dz.shape != (B, Cout, To):
        raise ValueError("dz shape does not match the convolution geometry")
    index = np.ascontiguousarray(index, dtype=np.int64)
    if index.size and (index.min() < 0 or index.max() >= Cout * Cin * K):
        raise ValueError("index out of range")
    dw = np.empty(index.shape, dtype=np.float64)
    _load().oracle_conv1d_bwd_weight_at(B, Cin, Cout, T, K, stride, dilation, pad, _p(x), _p(dz),
                                        index.size, index.ctypes.data_as(_I64), _p(dw))
    return dw


# ---- per-sample lengths ----------------------------------------------------------------------
# The encoder of the paper's ASR example takes the length of every utterance besides the padded
# batch and returns encoded lengths (Section 4.1.1: encoded, encoded_len = jasper_encoder(audio_signal,
# length)); the paper gives no formula.  Reading used here: samples at t >= length[b] are padding and
# count as zero for every block that reads them; a block's own output is not masked (the next block
# masks what it reads); the gradient with respect to padding is zero; the valid length behind a block
# is the convolution's output length applied to length[b].
def mask_time(x, lengths):
    """Copy of x [B][C][T] with x[b, :, t >= lengths[b]] set to zero (lengths are clipped to [0, T])."""
    x = np.array(x, dtype=np.float64, copy=True)
    for b, n in enumerate(np.asarray(lengths).reshape(-1)):
        x[b, :, max(0, min(int(n), x.shape[2])):] = 0.0
    return x


def out_lengths(lengths, K: int, stride: int, dilation: int, pad: int):
    """Valid length behind the block for every sample (0 where no output position exists)."""
    return np.array([max(0, out_len(int(n), K, stride, dilation, pad)) if n > 0 else 0 for n in np.asarray(lengths).reshape(-1)],
                    dtype=np.int64)


def block_fwd_masked(x, w, lengths, scale=None, shift=None, residual=None, relu=False, *, stride=1, dilation=1, pad=0):
    """Block forward on the batch with its padding zeroed."""
    return block_fwd(mask_time(x, lengths), w, scale, shift, residual, relu, stride=stride, dilation=dilation, pad=pad)


def bwd_data_masked(dz, w, T, lengths, *, stride=1, dilation=1, pad=0):
    """Input gradient; zero on the padding."""
    return mask_time(bwd_data(dz, w, T, stride=stride, dilation=dilation, pad=pad), lengths)


def bwd_weight_masked(x, dz, K, lengths, *, stride=1, dilation=1, pad=0):
    """Weight gradient from the batch with its padding zeroed."""
    return bwd_weight(mask_time(x, lengths), dz, K, stride=stride, dilation=dilation, pad=pad)


def num_threads() -> int:
    """Threads the OpenMP runtime uses for the loops of the C file."""
    return int(_load().oracle_num_threads())
