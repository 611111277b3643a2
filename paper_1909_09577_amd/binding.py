"""Thin ctypes binding of libnmconv1d.so (C ABI: include/nm_conv1d.h).

Only argument marshalling happens here: tensors are torch device tensors whose
``data_ptr()`` is handed to the library, the stream is torch's current HIP stream,
and outputs / workspace are ``torch.empty`` buffers when the caller passes none.
Every arithmetic step runs inside the library's kernels.  If the library has not
been built, loading raises: there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libnmconv1d.so")

NM_OK, NM_ERR_BAD_ARG, NM_ERR_UNSUPPORTED, NM_ERR_WORKSPACE, NM_ERR_DEVICE, NM_ERR_SCRATCH_LIMIT = 0, -1, -2, -3, -4, -5
NM_STATIC_SCRATCH_BYTES = 32 << 20
NM_BF16, NM_F32 = 0, 1
NM_RELU, NM_ACCUM_DW, NM_FORCE_DIRECT, NM_ACCUM_DX = 1, 2, 4, 8
NM_OP_FWD, NM_OP_BWD_DATA, NM_OP_BWD_WEIGHT, NM_OP_BWD, NM_OP_BN_FWD, NM_OP_BN_BWD = 0, 1, 2, 3, 4, 5

EXPORTS = ("nm_conv1d_out_len", "nm_conv1d_workspace_bytes", "nm_strerror", "nm_conv1d_block_fwd",
           "nm_conv1d_bwd_data", "nm_conv1d_bwd_weight", "nm_conv1d_bwd", "nm_conv1d_block_fwd_masked", "nm_conv1d_bwd_data_masked",
           "nm_conv1d_bwd_weight_masked", "nm_decoder_logsoftmax_fwd", "nm_conv1d_block_fwd_static", "nm_conv1d_time_next_kernel_of", "nm_conv1d_bn_fwd", "nm_conv1d_bn_bwd", "nm_conv1d_bwd_masked", "nm_conv1d_time_next_main_kernel",
           "nm_fp8_row_scales", "nm_fp8_quantize_rows", "nm_conv1d_fp8_supported", "nm_conv1d_fp8_workspace_bytes",
           "nm_conv1d_block_fwd_fp8", "nm_conv1d_bwd_data_fp8", "nm_conv1d_fp8_bwd_data_workspace_bytes",
           "nm_fp8_dgrad_weight_scales", "nm_conv1d_bwd_weight_fp8", "nm_conv1d_fp8_bwd_weight_workspace_bytes",
           "nm_conv1d_bwd_fp8", "nm_conv1d_fp8_bwd_workspace_bytes")

_lib = None


class NmError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({strerror(status)})")


def lib() -> ctypes.CDLL:
    """Load the HIP library (raises FileNotFoundError if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
        L = ctypes.CDLL(LIB_PATH)
        i, u, vp, sz = ctypes.c_int, ctypes.c_uint, ctypes.c_void_p, ctypes.c_size_t
        L.nm_conv1d_out_len.argtypes = [i] * 5
        L.nm_conv1d_out_len.restype = i
        L.nm_conv1d_workspace_bytes.argtypes = [i] * 9 + [i, u]
        L.nm_conv1d_workspace_bytes.restype = sz
        L.nm_strerror.argtypes = [i]
        L.nm_strerror.restype = ctypes.c_char_p
        L.nm_conv1d_block_fwd.argtypes = [i] * 8 + [vp] * 6 + [u, i, vp, sz, vp]
        L.nm_conv1d_block_fwd.restype = i
        L.nm_conv1d_block_fwd_static.argtypes = [i] * 8 + [vp] * 6 + [u, i, vp]
        L.nm_conv1d_block_fwd_static.restype = i
        L.nm_conv1d_bwd_data.argtypes = [i] * 8 + [vp] * 6 + [u, i, vp, sz, vp]
        L.nm_conv1d_bwd_data.restype = i
        L.nm_conv1d_bwd_weight.argtypes = [i] * 8 + [vp] * 5 + [u, i, vp, sz, vp]
        L.nm_conv1d_bwd_weight.restype = i
        L.nm_conv1d_block_fwd_masked.argtypes = [i] * 8 + [vp] * 7 + [u, i, vp, sz, vp]
        L.nm_conv1d_block_fwd_masked.restype = i
        L.nm_conv1d_bwd_data_masked.argtypes = [i] * 8 + [vp] * 7 + [u, i, vp, sz, vp]
        L.nm_conv1d_bwd_data_masked.restype = i
        L.nm_conv1d_bwd_weight_masked.argtypes = [i] * 8 + [vp] * 6 + [u, i, vp, sz, vp]
        L.nm_conv1d_bwd_weight_masked.restype = i
        L.nm_conv1d_bwd.argtypes = [i] * 8 + [vp] * 8 + [u, i, vp, sz, vp]
        L.nm_conv1d_bwd.restype = i
        L.nm_conv1d_bwd_masked.argtypes = [i] * 8 + [vp] * 9 + [u, i, vp, sz, vp]
        L.nm_conv1d_bwd_masked.restype = i
        L.nm_conv1d_bn_fwd.argtypes = [i] * 8 + [vp] * 4 + [ctypes.c_float] + [vp] * 5 + [u, i, vp, sz, vp]
        L.nm_conv1d_bn_fwd.restype = i
        L.nm_conv1d_bn_bwd.argtypes = [i] * 8 + [vp] * 13 + [u, i, vp, sz, vp]
        L.nm_conv1d_bn_bwd.restype = i
        L.nm_decoder_logsoftmax_fwd.argtypes = [i] * 4 + [vp] * 4 + [u, i, vp]
        L.nm_decoder_logsoftmax_fwd.restype = i
        L.nm_conv1d_time_next_main_kernel.argtypes = [vp, vp]
        L.nm_conv1d_time_next_main_kernel.restype = i
        L.nm_conv1d_time_next_kernel_of.argtypes = [vp, vp, i]
        L.nm_conv1d_time_next_kernel_of.restype = i
        L.nm_fp8_row_scales.argtypes = [vp, i, sz, vp, vp]
        L.nm_fp8_row_scales.restype = i
        L.nm_fp8_quantize_rows.argtypes = [vp, i, sz, vp, vp, vp]
        L.nm_fp8_quantize_rows.restype = i
        L.nm_conv1d_fp8_supported.argtypes = [i] * 8
        L.nm_conv1d_fp8_supported.restype = i
        L.nm_conv1d_fp8_workspace_bytes.argtypes = [i] * 8
        L.nm_conv1d_fp8_workspace_bytes.restype = sz
        L.nm_conv1d_block_fwd_fp8.argtypes = [i] * 8 + [vp] * 8 + [u, vp, sz, vp]
        L.nm_conv1d_block_fwd_fp8.restype = i
        L.nm_conv1d_bwd_data_fp8.argtypes = [i] * 8 + [vp] * 8 + [u, vp, sz, vp]
        L.nm_conv1d_bwd_data_fp8.restype = i
        L.nm_conv1d_fp8_bwd_data_workspace_bytes.argtypes = [i] * 8
        L.nm_conv1d_fp8_bwd_data_workspace_bytes.restype = sz
        L.nm_fp8_dgrad_weight_scales.argtypes = [i] * 3 + [vp] * 4
        L.nm_fp8_dgrad_weight_scales.restype = i
        L.nm_conv1d_bwd_weight_fp8.argtypes = [i] * 8 + [vp] * 7 + [u, vp, sz, vp]
        L.nm_conv1d_bwd_weight_fp8.restype = i
        L.nm_conv1d_fp8_bwd_weight_workspace_bytes.argtypes = [i] * 8
        L.nm_conv1d_fp8_bwd_weight_workspace_bytes.restype = sz
        L.nm_conv1d_bwd_fp8.argtypes = [i] * 8 + [vp] * 11 + [u, vp, sz, vp]
        L.nm_conv1d_bwd_fp8.restype = i
        L.nm_conv1d_fp8_bwd_workspace_bytes.argtypes = [i] * 8
        L.nm_conv1d_fp8_bwd_workspace_bytes.restype = sz
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().nm_strerror(int(status)).decode()


def nm_conv1d_out_len(T: int, K: int, stride: int = 1, dilation: int = 1, pad: int = 0) -> int:
    return int(lib().nm_conv1d_out_len(T, K, stride, dilation, pad))


def nm_conv1d_workspace_bytes(op: int, B, Cin, Cout, T, K, stride=1, dilation=1, pad=0, dtype=NM_BF16,
                              flags=0) -> int:
    return int(lib().nm_conv1d_workspace_bytes(op, B, Cin, Cout, T, K, stride, dilation, pad, dtype, flags))


def nm_conv1d_time_next_main_kernel(start_event, stop_event) -> None:
    """Arm the one-shot timer with two torch.cuda.Event(enable_timing=True) objects that have
    been recorded at least once (torch creates the underlying handle lazily), or None to disarm."""
    if start_event is None or stop_event is None:
        lib().nm_conv1d_time_next_main_kernel(None, None)
        return
    lib().nm_conv1d_time_next_main_kernel(ctypes.c_void_p(start_event.cuda_event), ctypes.c_void_p(stop_event.cuda_event))


def nm_conv1d_time_next_kernel_of(start_event, stop_event, op: int) -> None:
    """Like nm_conv1d_time_next_main_kernel for the main kernel of pass `op` (NM_OP_FWD / _BWD_DATA / _BWD_WEIGHT)."""
    st = lib().nm_conv1d_time_next_kernel_of(ctypes.c_void_p(start_event.cuda_event), ctypes.c_void_p(stop_event.cuda_event),
                                             int(op))
    if st != NM_OK:
        raise NmError(st, "nm_conv1d_time_next_kernel_of")


# ---- tensor marshalling -----------------------------------------------------------------
def _torch():
    import torch
    return torch


def _dtype_code(t) -> int:
    torch = _torch()
    if t.dtype == torch.bfloat16:
        return NM_BF16
    if t.dtype == torch.float32:
        return NM_F32
    raise TypeError(f"unsupported storage dtype {t.dtype}")


def _ptr(t, dtype=None, shape=None, name="tensor"):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must have dtype {dtype}, got {t.dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    torch = _torch()
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _workspace(op, dims, dtype_code, flags, workspace, device):
    torch = _torch()
    need = nm_conv1d_workspace_bytes(op, *dims, dtype_code, flags)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=device)
    return workspace, ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size()


def nm_conv1d_block_fwd(x, w, scale=None, shift=None, residual=None, y=None, *, stride=1, dilation=1,
                        pad=0, relu=False, force_direct=False, workspace=None, stream=None, lengths=None):
    """y = relu?(scale*conv1d(x,w)+shift+residual); returns y (allocated if not given).
    lengths (int32 [B], optional): valid length of every sample, the rest of x reads as zero."""
    torch = _torch()
    B, Cin, T = x.shape
    Cout, _, K = w.shape
    To = nm_conv1d_out_len(T, K, stride, dilation, pad)
    if To <= 0:
        raise NmError(NM_ERR_BAD_ARG, "nm_conv1d_block_fwd")
    code = _dtype_code(x)
    if y is None:
        y = torch.empty((B, Cout, To), dtype=x.dtype, device=x.device)
    flags = (NM_RELU if relu else 0) | (NM_FORCE_DIRECT if force_direct else 0)
    dims = (B, Cin, Cout, T, K, stride, dilation, pad)
    ws, ws_ptr, ws_bytes = _workspace(NM_OP_FWD, dims, code, flags, workspace, x.device)
    fn, extra = (lib().nm_conv1d_block_fwd, ()) if lengths is None else (
        lib().nm_conv1d_block_fwd_masked, (_ptr(lengths, torch.int32, (B,), "lengths"),))
    st = fn(
        *dims, *extra, _ptr(x, name="x"), _ptr(w, x.dtype, (Cout, Cin, K), "w"),
        _ptr(scale, torch.float32, (Cout,), "scale"), _ptr(shift, torch.float32, (Cout,), "shift"),
        _ptr(residual, x.dtype, (B, Cout, To), "residual"), _ptr(y, x.dtype, (B, Cout, To), "y"),
        flags, code, ws_ptr, ws_bytes, _stream(stream))
    if st != NM_OK:
        raise NmError(st, "nm_conv1d_block_fwd")
    return y


def nm_conv1d_block_fwd_static(x, w, scale=None, shift=None, residual=None, *, y, stride=1, dilation=1, pad=0,
                               relu=False, force_direct=False, stream=None):
    """nm_conv1d_block_fwd without a workspace: scratch is the library's fixed array.  The caller passes
    the output tensor y (this wrapper allocates nothing either); returns y."""
    torch = _torch()
    B, Cin, T = x.shape
    Cout, _, K = w.shape
    To = y.shape[2]
    flags = (NM_RELU if relu else 0) | (NM_FORCE_DIRECT if force_direct else 0)
    st = lib().nm_conv1d_block_fwd_static(
        B, Cin, Cout, T, K, stride, dilation, pad, _ptr(x, name="x"), _ptr(w, x.dtype, (Cout, Cin, K), "w"),
        _ptr(scale, torch.float32, (Cout,), "scale"), _ptr(shift, torch.float32, (Cout,), "shift"),
        _ptr(residual, x.dtype, (B, Cout, To), "residual"), _ptr(y, x.dtype, (B, Cout, To), "y"),
        flags, _dtype_code(x), _stream(stream))
    if st != NM_OK:
        raise NmError(st, "nm_conv1d_block_fwd_static")
    return y


def nm_conv1d_bwd_data(dy, w, T, y=None, scale=None, dx=None, dres=None, *, stride=1, dilation=1, pad=0,
                       relu=False, want_dres=False, force_direct=False, workspace=None, stream=None, lengths=None,
                       accumulate_dx=False):
    """dx (and optionally dres) from the upstream gradient dy; returns (dx, dres).
    lengths (int32 [B], optional): valid input length of every sample; dx is zero beyond it."""
    torch = _torch()
    B, Cout, To = dy.shape
    _, Cin, K = w.shape
    code = _dtype_code(dy)
    if dx is None:
        if accumulate_dx:
            raise ValueError("accumulate_dx needs an existing dx")
        dx = torch.empty((B, Cin, T), dtype=dy.dtype, device=dy.device)
    if dres is None and want_dres:
        dres = torch.empty_like(dy)
    flags = (NM_RELU if relu else 0) | (NM_FORCE_DIRECT if force_direct else 0) | (NM_ACCUM_DX if accumulate_dx else 0)
    dims = (B, Cin, Cout, T, K, stride, dilation, pad)
    ws, ws_ptr, ws_bytes = _workspace(NM_OP_BWD_DATA, dims, code, flags, workspace, dy.device)
    fn, extra = (lib().nm_conv1d_bwd_data, ()) if lengths is None else (
        lib().nm_conv1d_bwd_data_masked, (_ptr(lengths, torch.int32, (B,), "lengths"),))
    st = fn(
        *dims, *extra, _ptr(dy, name="dy"), _ptr(y, dy.dtype, (B, Cout, To), "y"),
        _ptr(scale, torch.float32, (Cout,), "scale"), _ptr(w, dy.dtype, (Cout, Cin, K), "w"),
        _ptr(dx, dy.dtype, (B, Cin, T), "dx"), _ptr(dres, dy.dtype, (B, Cout, To), "dres"),
        flags, code, ws_ptr, ws_bytes, _stream(stream))
    if st != NM_OK:
        raise NmError(st, "nm_conv1d_bwd_data")
    return dx, dres


def nm_conv1d_bwd_weight(x, dy, K, y=None, scale=None, dw=None, *, stride=1, dilation=1, pad=0,
                         relu=False, accumulate=False, force_direct=False, workspace=None, stream=None, lengths=None):
    """dw [Cout,Cin,K] float32 from x and the upstream gradient dy; returns dw.
    lengths (int32 [B], optional): valid length of every sample, the rest of x reads as zero."""
    torch = _torch()
    B, Cin, T = x.shape
    _, Cout, To = dy.shape
    code = _dtype_code(x)
    if dw is None:
        if accumulate:
            raise ValueError("accumulate needs an existing dw")
        dw = torch.empty((Cout, Cin, K), dtype=torch.float32, device=x.device)
    flags = (NM_RELU if relu else 0) | (NM_ACCUM_DW if accumulate else 0) | (NM_FORCE_DIRECT if force_direct else 0)
    dims = (B, Cin, Cout, T, K, stride, dilation, pad)
    ws, ws_ptr, ws_bytes = _workspace(NM_OP_BWD_WEIGHT, dims, code, flags, workspace, x.device)
    fn, extra = (lib().nm_conv1d_bwd_weight, ()) if lengths is None else (
        lib().nm_conv1d_bwd_weight_masked, (_ptr(lengths, torch.int32, (B,), "lengths"),))
    st = fn(
        *dims, *extra, _ptr(x, name="x"), _ptr(dy, x.dtype, (B, Cout, To), "dy"), _ptr(y, x.dtype, (B, Cout, To), "y"),
        _ptr(scale, torch.float32, (Cout,), "scale"), _ptr(dw, torch.float32, (Cout, Cin, K), "dw"),
        flags, code, ws_ptr, ws_bytes, _stream(stream))
    if st != NM_OK:
        raise NmError(st, "nm_conv1d_bwd_weight")
    return dw


def nm_conv1d_bwd(x, dy, w, y=None, scale=None, dx=None, dres=None, dw=None, *, stride=1, dilation=1, pad=0,
                  relu=False, want_dres=False, accumulate=False, force_direct=False, workspace=None, stream=None,
                  accumulate_dx=False, lengths=None):
    """Both gradients in one call; returns (dx, dres, dw).  lengths (int32 [B], optional): padded batch."""
    torch = _torch()
    B, Cin, T = x.shape
    Cout, _, K = w.shape
    To = dy.shape[2]
    code = _dtype_code(x)
    if dx is None:
        if accumulate_dx:
            raise ValueError("accumulate_dx needs an existing dx")
        dx = torch.empty((B, Cin, T), dtype=x.dtype, device=x.device)
    if dres is None and want_dres:
        dres = torch.empty_like(dy)
    if dw is None:
        if accumulate:
            raise ValueError("accumulate needs an existing dw")
        dw = torch.empty((Cout, Cin, K), dtype=torch.float32, device=x.device)
    flags = (NM_RELU if relu else 0) | (NM_ACCUM_DW if accumulate else 0) | (NM_FORCE_DIRECT if force_direct else 0) | \
        (NM_ACCUM_DX if accumulate_dx else 0)
    dims = (B, Cin, Cout, T, K, stride, dilation, pad)
    ws, ws_ptr, ws_bytes = _workspace(NM_OP_BWD, dims, code, flags, workspace, x.device)
    fn, extra = (lib().nm_conv1d_bwd, ()) if lengths is None else (
        lib().nm_conv1d_bwd_masked, (_ptr(lengths, torch.int32, (B,), "lengths"),))
    st = fn(
        *dims, *extra, _ptr(x, name="x"), _ptr(dy, x.dtype, (B, Cout, To), "dy"), _ptr(y, x.dtype, (B, Cout, To), "y"),
        _ptr(scale, torch.float32, (Cout,), "scale"), _ptr(w, x.dtype, (Cout, Cin, K), "w"),
        _ptr(dx, x.dtype, (B, Cin, T), "dx"), _ptr(dres, x.dtype, (B, Cout, To), "dres"),
        _ptr(dw, torch.float32, (Cout, Cin, K), "dw"), flags, code, ws_ptr, ws_bytes, _stream(stream))
    if st != NM_OK:
        raise NmError(st, "nm_conv1d_bwd")
    return dx, dres, dw


def nm_conv1d_bn_fwd(x, w, gamma=None, beta=None, residual=None, *, eps=1e-3, stride=1, dilation=1, pad=0, relu=False,
                     force_direct=False, z=None, y=None, mean=None, invstd=None, workspace=None, stream=None):
    """Block forward with training-mode BatchNorm; returns (z, y, mean, invstd)."""
    torch = _torch()
    B, Cin, T = x.shape
    Cout, _, K = w.shape
    To = nm_conv1d_out_len(T, K, stride, dilation, pad)
    if To <= 0:
        raise NmError(NM_ERR_BAD_ARG, "nm_conv1d_bn_fwd")
    code = _dtype_code(x)
    z = torch.empty((B, Cout, To), dtype=x.dtype, device=x.device) if z is None else z
    y = torch.empty((B, Cout, To), dtype=x.dtype, device=x.device) if y is None else y
    mean = torch.empty((Cout,), dtype=torch.float32, device=x.device) if mean is None else mean
    invstd = torch.empty((Cout,), dtype=torch.float32, device=x.device) if invstd is None else invstd
    flags = (NM_RELU if relu else 0) | (NM_FORCE_DIRECT if force_direct else 0)
    dims = (B, Cin, Cout, T, K, stride, dilation, pad)
    ws, ws_ptr, ws_bytes = _workspace(NM_OP_BN_FWD, dims, code, flags, workspace, x.device)
    st = lib().nm_conv1d_bn_fwd(
        *dims, _ptr(x, name="x"), _ptr(w, x.dtype, (Cout, Cin, K), "w"), _ptr(gamma, torch.float32, (Cout,), "gamma"),
        _ptr(beta, torch.float32, (Cout,), "beta"), float(eps), _ptr(residual, x.dtype, (B, Cout, To), "residual"),
        _ptr(z, x.dtype, (B, Cout, To), "z"), _ptr(y, x.dtype, (B, Cout, To), "y"), _ptr(mean, torch.float32, (Cout,), "mean"),
        _ptr(invstd, torch.float32, (Cout,), "invstd"), flags, code, ws_ptr, ws_bytes, _stream(stream))
    if st != NM_OK:
        raise NmError(st, "nm_conv1d_bn_fwd")
    return z, y, mean, invstd


def nm_conv1d_bn_bwd(x, w, gamma, z, y, mean, invstd, dy, *, stride=1, dilation=1, pad=0, relu=False, want_dres=False,
                     force_direct=False, accumulate=False, accumulate_dx=False, dx=None, dres=None, dw=None, dgamma=None,
                     dbeta=None, workspace=None, stream=None):
    """Backward of nm_conv1d_bn_fwd; returns (dx, dres, dw, dgamma, dbeta)."""
    torch = _torch()
    B, Cin, T = x.shape
    Cout, _, K = w.shape
    To = dy.shape[2]
    code = _dtype_code(x)
    if (accumulate and (dw is None or dgamma is None or dbeta is None)) or (accumulate_dx and dx is None):
        raise ValueError("accumulation needs existing output tensors")
    dx = torch.empty((B, Cin, T), dtype=x.dtype, device=x.device) if dx is None else dx
    if dres is None and want_dres:
        dres = torch.empty_like(dy)
    dw = torch.empty((Cout, Cin, K), dtype=torch.float32, device=x.device) if dw is None else dw
    dgamma = torch.empty((Cout,), dtype=torch.float32, device=x.device) if dgamma is None else dgamma
    dbeta = torch.empty((Cout,), dtype=torch.float32, device=x.device) if dbeta is None else dbeta
    flags = (NM_RELU if relu else 0) | (NM_ACCUM_DW if accumulate else 0) | (NM_FORCE_DIRECT if force_direct else 0) | \
        (NM_ACCUM_DX if accumulate_dx else 0)
    dims = (B, Cin, Cout, T, K, stride, dilation, pad)
    ws, ws_ptr, ws_bytes = _workspace(NM_OP_BN_BWD, dims, code, flags, workspace, x.device)
    act = (B, Cout, To)
    st = lib().nm_conv1d_bn_bwd(
        *dims, _ptr(x, name="x"), _ptr(w, x.dtype, (Cout, Cin, K), "w"), _ptr(gamma, torch.float32, (Cout,), "gamma"),
        _ptr(z, x.dtype, act, "z"), _ptr(y, x.dtype, act, "y"), _ptr(mean, torch.float32, (Cout,), "mean"),
        _ptr(invstd, torch.float32, (Cout,), "invstd"), _ptr(dy, x.dtype, act, "dy"), _ptr(dx, x.dtype, (B, Cin, T), "dx"),
        _ptr(dres, x.dtype, act, "dres"), _ptr(dw, torch.float32, (Cout, Cin, K), "dw"),
        _ptr(dgamma, torch.float32, (Cout,), "dgamma"), _ptr(dbeta, torch.float32, (Cout,), "dbeta"),
        flags, code, ws_ptr, ws_bytes, _stream(stream))
    if st != NM_OK:
        raise NmError(st, "nm_conv1d_bn_bwd")
    return dx, dres, dw, dgamma, dbeta


def nm_decoder_logsoftmax_fwd(x, w, bias=None, logp=None, *, force_direct=False, stream=None):
    """logp [B,Ncls,T] float32 = log_softmax over classes of (w @ x + bias); w is [Ncls,Cin]."""
    torch = _torch()
    B, Cin, T = x.shape
    Ncls = w.shape[0]
    code = _dtype_code(x)
    if logp is None:
        logp = torch.empty((B, Ncls, T), dtype=torch.float32, device=x.device)
    st = lib().nm_decoder_logsoftmax_fwd(
        B, Cin, Ncls, T, _ptr(x, name="x"), _ptr(w, x.dtype, (Ncls, Cin), "w"), _ptr(bias, torch.float32, (Ncls,), "bias"),
        _ptr(logp, torch.float32, (B, Ncls, T), "logp"), NM_FORCE_DIRECT if force_direct else 0, code, _stream(stream))
    if st != NM_OK:
        raise NmError(st, "nm_decoder_logsoftmax_fwd")
    return logp


# ---- 8-bit floating-point (E4M3) variant of the block forward (include/nm_conv1d_fp8.h) ------------------
def nm_fp8_row_scales(x, rows: int, *, stream=None):
    """float32 [rows]: amax/448 of each of `rows` equal slices of the bfloat16 tensor x (1 for an all-zero slice)."""
    torch = _torch()
    if x.dtype != torch.bfloat16:
        raise TypeError("x must be bfloat16")
    n = x.numel()
    if rows <= 0 or n % rows:
        raise ValueError("rows must divide the number of elements")
    scales = torch.empty(rows, dtype=torch.float32, device=x.device)
    st = lib().nm_fp8_row_scales(_ptr(x, name="x"), rows, n // rows, _ptr(scales), _stream(stream))
    if st != NM_OK:
        raise NmError(st, "nm_fp8_row_scales")
    return scales


def nm_fp8_quantize_rows(x, scales, *, stream=None):
    """uint8 tensor shaped like x: the E4M3 codes of x with slice r divided by scales[r]."""
    torch = _torch()
    if x.dtype != torch.bfloat16:
        raise TypeError("x must be bfloat16")
    rows = scales.numel()
    n = x.numel()
    if rows <= 0 or n % rows:
        raise ValueError("len(scales) must divide the number of elements")
    codes = torch.empty(x.shape, dtype=torch.uint8, device=x.device)
    st = lib().nm_fp8_quantize_rows(_ptr(x, name="x"), rows, n // rows, _ptr(scales, torch.float32, (rows,), "scales"),
                                    _ptr(codes), _stream(stream))
    if st != NM_OK:
        raise NmError(st, "nm_fp8_quantize_rows")
    return codes


def nm_conv1d_fp8_supported(B, Cin, Cout, T, K, stride=1, dilation=1, pad=0) -> bool:
    return bool(lib().nm_conv1d_fp8_supported(B, Cin, Cout, T, K, stride, dilation, pad))


def nm_conv1d_fp8_workspace_bytes(B, Cin, Cout, T, K, stride=1, dilation=1, pad=0) -> int:
    return int(lib().nm_conv1d_fp8_workspace_bytes(B, Cin, Cout, T, K, stride, dilation, pad))


def nm_conv1d_block_fwd_fp8(x, x_scale, w, w_scales, scale=None, shift=None, residual=None, y=None, *, stride=1,
                            dilation=1, pad=0, relu=False, workspace=None, stream=None):
    """Block forward on E4M3 operands: x and w (bfloat16) are quantised inside the call with x_scale [1] and
    w_scales [Cout] (float32 device tensors); returns y (bfloat16, allocated if not given)."""
    torch = _torch()
    B, Cin, T = x.shape
    Cout, _, K = w.shape
    To = nm_conv1d_out_len(T, K, stride, dilation, pad)
    if To <= 0:
        raise NmError(NM_ERR_BAD_ARG, "nm_conv1d_block_fwd_fp8")
    if y is None:
        y = torch.empty((B, Cout, To), dtype=torch.bfloat16, device=x.device)
    dims = (B, Cin, Cout, T, K, stride, dilation, pad)
    if workspace is None:
        workspace = torch.empty(max(nm_conv1d_fp8_workspace_bytes(*dims), 256), dtype=torch.uint8, device=x.device)
    st = lib().nm_conv1d_block_fwd_fp8(
        *dims, _ptr(x, torch.bfloat16, name="x"), _ptr(x_scale, torch.float32, (1,), "x_scale"),
        _ptr(w, torch.bfloat16, (Cout, Cin, K), "w"), _ptr(w_scales, torch.float32, (Cout,), "w_scales"),
        _ptr(scale, torch.float32, (Cout,), "scale"), _ptr(shift, torch.float32, (Cout,), "shift"),
        _ptr(residual, torch.bfloat16, (B, Cout, To), "residual"), _ptr(y, torch.bfloat16, (B, Cout, To), "y"),
        NM_RELU if relu else 0, ctypes.c_void_p(workspace.data_ptr()), workspace.numel(), _stream(stream))
    if st != NM_OK:
        raise NmError(st, "nm_conv1d_block_fwd_fp8")
    return y


def nm_fp8_dgrad_weight_scales(w, scale=None, *, stream=None):
    """float32 [Cin]: per-input-channel scales of the input gradient's weight operand w[co,ci,k]*scale[co]."""
    torch = _torch()
    Cout, Cin, K = w.shape
    out = torch.empty(Cin, dtype=torch.float32, device=w.device)
    st = lib().nm_fp8_dgrad_weight_scales(Cin, Cout, K, _ptr(w, torch.bfloat16, name="w"),
                                          _ptr(scale, torch.float32, (Cout,), "scale"), _ptr(out), _stream(stream))
    if st != NM_OK:
        raise NmError(st, "nm_fp8_dgrad_weight_scales")
    return out


def nm_conv1d_fp8_bwd_data_workspace_bytes(B, Cin, Cout, T, K, stride=1, dilation=1, pad=0) -> int:
    return int(lib().nm_conv1d_fp8_bwd_data_workspace_bytes(B, Cin, Cout, T, K, stride, dilation, pad))


def nm_conv1d_bwd_data_fp8(dy, g_scale, w, wt_scales, T, y=None, scale=None, dx=None, dres=None, *, stride=1, dilation=1,
                           pad=0, relu=False, want_dres=False, workspace=None, stream=None):
    """Input gradient on E4M3 operands; returns (dx, dres)."""
    torch = _torch()
    B, Cout, To = dy.shape
    _, Cin, K = w.shape
    if dx is None:
        dx = torch.empty((B, Cin, T), dtype=torch.bfloat16, device=dy.device)
    if dres is None and want_dres:
        dres = torch.empty_like(dy)
    dims = (B, Cin, Cout, T, K, stride, dilation, pad)
    if workspace is None:
        workspace = torch.empty(max(nm_conv1d_fp8_bwd_data_workspace_bytes(*dims), 256), dtype=torch.uint8, device=dy.device)
    st = lib().nm_conv1d_bwd_data_fp8(
        *dims, _ptr(dy, torch.bfloat16, name="dy"), _ptr(y, torch.bfloat16, (B, Cout, To), "y"),
        _ptr(g_scale, torch.float32, (1,), "g_scale"), _ptr(w, torch.bfloat16, (Cout, Cin, K), "w"),
        _ptr(scale, torch.float32, (Cout,), "scale"), _ptr(wt_scales, torch.float32, (Cin,), "wt_scales"),
        _ptr(dx, torch.bfloat16, (B, Cin, T), "dx"), _ptr(dres, torch.bfloat16, (B, Cout, To), "dres"),
        NM_RELU if relu else 0, ctypes.c_void_p(workspace.data_ptr()), workspace.numel(), _stream(stream))
    if st != NM_OK:
        raise NmError(st, "nm_conv1d_bwd_data_fp8")
    return dx, dres


def nm_conv1d_fp8_bwd_weight_workspace_bytes(B, Cin, Cout, T, K, stride=1, dilation=1, pad=0) -> int:
    return int(lib().nm_conv1d_fp8_bwd_weight_workspace_bytes(B, Cin, Cout, T, K, stride, dilation, pad))


def nm_conv1d_bwd_weight_fp8(x, x_scale, dy, g_scale, K, y=None, scale=None, dw=None, *, stride=1, dilation=1, pad=0,
                             relu=False, accumulate=False, workspace=None, stream=None):
    """Weight gradient on E4M3 operands; returns dw [Cout, Cin, K] float32."""
    torch = _torch()
    B, Cin, T = x.shape
    _, Cout, To = dy.shape
    if dw is None:
        if accumulate:
            raise ValueError("accumulate needs an existing dw")
        dw = torch.empty((Cout, Cin, K), dtype=torch.float32, device=x.device)
    dims = (B, Cin, Cout, T, K, stride, dilation, pad)
    if workspace is None:
        workspace = torch.empty(max(nm_conv1d_fp8_bwd_weight_workspace_bytes(*dims), 256), dtype=torch.uint8, device=x.device)
    flags = (NM_RELU if relu else 0) | (NM_ACCUM_DW if accumulate else 0)
    st = lib().nm_conv1d_bwd_weight_fp8(
        *dims, _ptr(x, torch.bfloat16, name="x"), _ptr(x_scale, torch.float32, (1,), "x_scale"),
        _ptr(dy, torch.bfloat16, name="dy"), _ptr(y, torch.bfloat16, (B, Cout, To), "y"),
        _ptr(g_scale, torch.float32, (1,), "g_scale"), _ptr(scale, torch.float32, (Cout,), "scale"),
        _ptr(dw, torch.float32, (Cout, Cin, K), "dw"), flags, ctypes.c_void_p(workspace.data_ptr()), workspace.numel(),
        _stream(stream))
    if st != NM_OK:
        raise NmError(st, "nm_conv1d_bwd_weight_fp8")
    return dw


def nm_conv1d_fp8_bwd_workspace_bytes(B, Cin, Cout, T, K, stride=1, dilation=1, pad=0) -> int:
    return int(lib().nm_conv1d_fp8_bwd_workspace_bytes(B, Cin, Cout, T, K, stride, dilation, pad))


def nm_conv1d_bwd_fp8(x, x_scale, dy, g_scale, w, wt_scales, y=None, scale=None, dx=None, dres=None, dw=None, *, stride=1,
                      dilation=1, pad=0, relu=False, want_dres=False, accumulate=False, workspace=None, stream=None):
    """Both gradients on E4M3 operands from one call; returns (dx, dres, dw)."""
    torch = _torch()
    B, Cin, T = x.shape
    _, Cout, To = dy.shape
    K = w.shape[2]
    if dx is None:
        dx = torch.empty_like(x)
    if dres is None and want_dres:
        dres = torch.empty_like(dy)
    if dw is None:
        if accumulate:
            raise ValueError("accumulate needs an existing dw")
        dw = torch.empty((Cout, Cin, K), dtype=torch.float32, device=x.device)
    dims = (B, Cin, Cout, T, K, stride, dilation, pad)
    if workspace is None:
        workspace = torch.empty(max(nm_conv1d_fp8_bwd_workspace_bytes(*dims), 256), dtype=torch.uint8, device=x.device)
    flags = (NM_RELU if relu else 0) | (NM_ACCUM_DW if accumulate else 0)
    st = lib().nm_conv1d_bwd_fp8(
        *dims, _ptr(x, torch.bfloat16, name="x"), _ptr(x_scale, torch.float32, (1,), "x_scale"),
        _ptr(dy, torch.bfloat16, name="dy"), _ptr(y, torch.bfloat16, (B, Cout, To), "y"),
        _ptr(g_scale, torch.float32, (1,), "g_scale"), _ptr(w, torch.bfloat16, (Cout, Cin, K), "w"),
        _ptr(scale, torch.float32, (Cout,), "scale"), _ptr(wt_scales, torch.float32, (Cin,), "wt_scales"),
        _ptr(dx, torch.bfloat16, (B, Cin, T), "dx"), _ptr(dres, torch.bfloat16, (B, Cout, To), "dres"),
        _ptr(dw, torch.float32, (Cout, Cin, K), "dw"), flags, ctypes.c_void_p(workspace.data_ptr()), workspace.numel(),
        _stream(stream))
    if st != NM_OK:
        raise NmError(st, "nm_conv1d_bwd_fp8")
    return dx, dres, dw
