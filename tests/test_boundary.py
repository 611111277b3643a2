"""CPU-only tests of the C boundary: the library loads, exports what the header declares,
and reports every argument error before touching the device (no compute call is made)."""
import ctypes
import itertools
import os
import re

import pytest

from oracle import conv1d_oracle as orc
from paper_1909_09577_amd import binding as nm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = ctypes.c_void_p(0x1000)        # never dereferenced: every call below fails validation first
FAKE2 = ctypes.c_void_p(0x7F0000000000)
FAKE3 = ctypes.c_void_p(0x7E0000000000)
FAKE4 = ctypes.c_void_p(0x7D0000000000)
FAKE5 = ctypes.c_void_p(0x7C0000000000)


def declared_functions():
    names = set()
    for fn in os.listdir(os.path.join(ROOT, "include")):
        if fn.endswith(".h"):
            text = open(os.path.join(ROOT, "include", fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names |= set(re.findall(r"\b(nm_[a-z0-9_]+)\s*\(", text))
    return names


def test_library_exports_every_declared_symbol():
    L = nm.lib()
    names = declared_functions()
    assert set(nm.EXPORTS) <= names and len(names) >= 6
    for name in names:
        assert hasattr(L, name), name


def test_strerror():
    msgs = {nm.strerror(s) for s in (0, -1, -2, -3, -4)}
    assert len(msgs) == 5 and nm.strerror(-99) == "unknown status"


def test_out_len_matches_oracle_brute_force_range():
    for T, K, s, d, pad in itertools.product(range(0, 14), range(0, 6), range(0, 4), range(0, 4), range(-1, 7)):
        got = nm.nm_conv1d_out_len(T, K, s, d, pad)
        if T <= 0 or K <= 0 or s <= 0 or d <= 0 or pad < 0:
            assert got < 0
        else:
            exp = orc.out_len(T, K, s, d, pad)
            assert got == exp or (exp < 0 and got < 0), (T, K, s, d, pad, got, exp)
    assert nm.nm_conv1d_out_len(1600, 11, 2, 1, 5) == 800
    assert nm.nm_conv1d_out_len(800, 29, 1, 2, 28) == 800


GOOD = dict(B=2, Cin=4, Cout=4, T=16, K=3, stride=1, dilation=1, pad=1)


def fwd(dims=None, x=FAKE2, w=FAKE3, y=FAKE4, flags=0, dtype=0, ws=None, ws_bytes=0, res=None):
    d = dict(GOOD, **(dims or {}))
    return nm.lib().nm_conv1d_block_fwd(d["B"], d["Cin"], d["Cout"], d["T"], d["K"], d["stride"], d["dilation"],
                                        d["pad"], x, w, None, None, res, y, flags, dtype, ws, ws_bytes, None)


def bwd_data(dims=None, dy=FAKE2, yv=None, w=FAKE3, dx=FAKE4, flags=0, dtype=0):
    d = dict(GOOD, **(dims or {}))
    return nm.lib().nm_conv1d_bwd_data(d["B"], d["Cin"], d["Cout"], d["T"], d["K"], d["stride"], d["dilation"],
                                       d["pad"], dy, yv, None, w, dx, None, flags, dtype, None, 0, None)


def bwd_weight(dims=None, x=FAKE2, dy=FAKE3, yv=None, dw=FAKE4, flags=0, dtype=0):
    d = dict(GOOD, **(dims or {}))
    return nm.lib().nm_conv1d_bwd_weight(d["B"], d["Cin"], d["Cout"], d["T"], d["K"], d["stride"], d["dilation"],
                                         d["pad"], x, dy, yv, None, dw, flags, dtype, None, 0, None)


def bwd(dims=None, x=FAKE, dy=FAKE2, yv=None, w=FAKE3, dx=FAKE4, dw=FAKE5, flags=0, dtype=0):
    d = dict(GOOD, **(dims or {}))
    return nm.lib().nm_conv1d_bwd(d["B"], d["Cin"], d["Cout"], d["T"], d["K"], d["stride"], d["dilation"], d["pad"],
                                  x, dy, yv, None, w, dx, None, dw, flags, dtype, None, 0, None)


@pytest.mark.parametrize("call", [fwd, bwd_data, bwd_weight, bwd])
def test_bad_geometry_is_rejected(call):
    for bad in (dict(B=0), dict(Cin=0), dict(Cout=-1), dict(T=0), dict(K=0), dict(stride=0), dict(dilation=0),
                dict(pad=-1), dict(T=2, K=5, pad=0)):
        assert call(bad) == nm.NM_ERR_BAD_ARG, bad
    assert call(dtype=7) == nm.NM_ERR_BAD_ARG
    assert call(flags=1 << 9) == nm.NM_ERR_BAD_ARG
    assert call(dict(B=60000, Cin=60000, T=60000)) == nm.NM_ERR_UNSUPPORTED
    assert call(dict(B=70000, T=4)) == nm.NM_ERR_UNSUPPORTED


def test_null_pointers_are_rejected():
    assert fwd(x=None) == nm.NM_ERR_BAD_ARG
    assert fwd(w=None) == nm.NM_ERR_BAD_ARG
    assert fwd(y=None) == nm.NM_ERR_BAD_ARG
    assert bwd_data(dy=None) == nm.NM_ERR_BAD_ARG
    assert bwd_data(w=None) == nm.NM_ERR_BAD_ARG
    assert bwd_data(dx=None) == nm.NM_ERR_BAD_ARG
    assert bwd_data(flags=nm.NM_RELU, yv=None) == nm.NM_ERR_BAD_ARG      # ReLU mask needs y
    assert bwd_weight(x=None) == nm.NM_ERR_BAD_ARG
    assert bwd_weight(dy=None) == nm.NM_ERR_BAD_ARG
    assert bwd_weight(dw=None) == nm.NM_ERR_BAD_ARG
    assert bwd_weight(flags=nm.NM_RELU, yv=None) == nm.NM_ERR_BAD_ARG
    for missing in ("x", "dy", "w", "dx", "dw"):
        assert bwd(**{missing: None}) == nm.NM_ERR_BAD_ARG, missing
    assert bwd(flags=nm.NM_RELU, yv=None) == nm.NM_ERR_BAD_ARG
    assert fwd(flags=nm.NM_ACCUM_DW) == nm.NM_ERR_BAD_ARG                # flag of another entry point
    assert bwd_data(flags=nm.NM_ACCUM_DW) == nm.NM_ERR_BAD_ARG


def test_aliasing_is_rejected():
    assert fwd(x=FAKE2, y=FAKE2) == nm.NM_ERR_BAD_ARG
    assert fwd(w=FAKE3, y=FAKE3) == nm.NM_ERR_BAD_ARG
    assert fwd(res=FAKE4, y=FAKE4) == nm.NM_ERR_BAD_ARG
    assert bwd_data(dy=FAKE2, dx=FAKE2) == nm.NM_ERR_BAD_ARG
    assert bwd_weight(x=FAKE2, dw=ctypes.c_void_p(FAKE2.value + 8)) == nm.NM_ERR_BAD_ARG


def test_workspace_is_checked_before_any_launch():
    # backward with a ReLU mask on the plain path needs room for dz
    need = nm.nm_conv1d_workspace_bytes(nm.NM_OP_BWD_DATA, 2, 4, 4, 16, 3, 1, 1, 1, nm.NM_BF16, nm.NM_RELU | nm.NM_FORCE_DIRECT)
    assert need >= 2 * 4 * 16 * 2 and need % 256 == 0
    assert bwd_data(flags=nm.NM_RELU | nm.NM_FORCE_DIRECT, yv=FAKE) == nm.NM_ERR_WORKSPACE
    assert bwd_weight(flags=nm.NM_RELU | nm.NM_FORCE_DIRECT, yv=FAKE) == nm.NM_ERR_WORKSPACE
    assert nm.nm_conv1d_workspace_bytes(99, 2, 4, 4, 16, 3) == 0
    assert nm.nm_conv1d_workspace_bytes(nm.NM_OP_FWD, 0, 4, 4, 16, 3) == 0
    for op in (nm.NM_OP_FWD, nm.NM_OP_BWD_DATA, nm.NM_OP_BWD_WEIGHT):
        for dims in ((32, 512, 512, 800, 17, 1, 1, 8), (32, 768, 896, 800, 29, 1, 2, 28), (2, 64, 256, 200, 11, 1, 1, 5)):
            n = nm.nm_conv1d_workspace_bytes(op, *dims, nm.NM_BF16, 0)
            assert n % 256 == 0 and n < (1 << 31)
            # a misaligned or short workspace is refused (when one is needed at all)
            if n:
                d = dict(zip(("B", "Cin", "Cout", "T", "K", "stride", "dilation", "pad"), dims))
                if op == nm.NM_OP_FWD:
                    assert fwd(d, ws=ctypes.c_void_p(0x10000100), ws_bytes=n - 1) == nm.NM_ERR_WORKSPACE
                    assert fwd(d, ws=ctypes.c_void_p(0x10000104), ws_bytes=n) == nm.NM_ERR_WORKSPACE


def test_decoder_tail_arguments_are_checked():
    f = nm.lib().nm_decoder_logsoftmax_fwd
    assert f(2, 64, 29, 16, FAKE, FAKE2, None, None, 0, 0, None) == nm.NM_ERR_BAD_ARG       # no output
    assert f(2, 64, 29, 16, None, FAKE2, None, FAKE3, 0, 0, None) == nm.NM_ERR_BAD_ARG
    assert f(2, 64, 29, 16, FAKE, None, None, FAKE3, 0, 0, None) == nm.NM_ERR_BAD_ARG
    for bad in ((0, 64, 29, 16), (2, 0, 29, 16), (2, 64, 0, 16), (2, 64, 29, 0)):
        assert f(*bad, FAKE, FAKE2, None, FAKE3, 0, 0, None) == nm.NM_ERR_BAD_ARG
    assert f(2, 64, 29, 16, FAKE, FAKE2, None, FAKE3, 0, 9, None) == nm.NM_ERR_BAD_ARG      # dtype
    assert f(2, 64, 29, 16, FAKE, FAKE2, None, FAKE3, nm.NM_RELU, 0, None) == nm.NM_ERR_BAD_ARG  # foreign flag
    assert f(60000, 60000, 29, 60000, FAKE, FAKE2, None, FAKE3, 0, 0, None) == nm.NM_ERR_UNSUPPORTED


def test_masked_entry_points_check_their_arguments():
    L = nm.lib()
    d = GOOD
    dims = (d["B"], d["Cin"], d["Cout"], d["T"], d["K"], d["stride"], d["dilation"], d["pad"])
    # no lengths
    assert L.nm_conv1d_block_fwd_masked(*dims, None, FAKE2, FAKE3, None, None, None, FAKE4, 0, 0, None, 0, None) == nm.NM_ERR_BAD_ARG
    assert L.nm_conv1d_bwd_data_masked(*dims, None, FAKE2, None, None, FAKE3, FAKE4, None, 0, 0, None, 0, None) == nm.NM_ERR_BAD_ARG
    assert L.nm_conv1d_bwd_weight_masked(*dims, None, FAKE2, FAKE3, None, None, FAKE4, 0, 0, None, 0, None) == nm.NM_ERR_BAD_ARG
    # the other checks are those of the unmasked calls
    assert L.nm_conv1d_block_fwd_masked(*dims, FAKE, None, FAKE3, None, None, None, FAKE4, 0, 0, None, 0, None) == nm.NM_ERR_BAD_ARG
    bad = (0,) + dims[1:]
    assert L.nm_conv1d_bwd_weight_masked(*bad, FAKE, FAKE2, FAKE3, None, None, FAKE4, 0, 0, None, 0, None) == nm.NM_ERR_BAD_ARG
    assert L.nm_conv1d_bwd_data_masked(*dims, FAKE, FAKE2, None, None, FAKE3, FAKE4, None, nm.NM_RELU, 0, None, 0, None) == nm.NM_ERR_BAD_ARG


# ---- the forward entry point without a workspace ---------------------------------------------------
def fwd_static(dims=None, x=FAKE2, w=FAKE3, y=FAKE4, flags=0, dtype=0):
    d = dict(GOOD, **(dims or {}))
    return nm.lib().nm_conv1d_block_fwd_static(d["B"], d["Cin"], d["Cout"], d["T"], d["K"], d["stride"], d["dilation"],
                                               d["pad"], x, w, None, None, None, y, flags, dtype, None)


def test_static_forward_reports_argument_errors_and_its_scratch_limit_before_any_device_call():
    assert fwd_static(x=None) == nm.NM_ERR_BAD_ARG
    assert fwd_static(dims=dict(T=0)) == nm.NM_ERR_BAD_ARG
    assert fwd_static(flags=1 << 9) == nm.NM_ERR_BAD_ARG
    assert fwd_static(dtype=7) == nm.NM_ERR_BAD_ARG
    # 768 -> 896 channels with 29 taps: 41 MB of packed weights against a 32 MiB array
    big = dict(B=1, Cin=768, Cout=896, T=160, K=29, stride=1, dilation=2, pad=28)
    assert nm.nm_conv1d_workspace_bytes(nm.NM_OP_FWD, *big.values()) > nm.NM_STATIC_SCRATCH_BYTES
    assert fwd_static(dims=big) == nm.NM_ERR_SCRATCH_LIMIT
    assert "scratch" in nm.strerror(nm.NM_ERR_SCRATCH_LIMIT)
    text = open(os.path.join(ROOT, "include", "nm_conv1d.h")).read()
    m = re.search(r"#define NM_STATIC_SCRATCH_BYTES \(\(size_t\)(\d+) << (\d+)\)", text)
    assert m and int(m.group(1)) << int(m.group(2)) == nm.NM_STATIC_SCRATCH_BYTES


def test_declared_output_lengths_of_the_workloads_are_the_oracles():
    from paper_1909_09577_amd import inputs as syn
    cfgs = list(syn.SINGLE_LAYER_CFGS) + [e["cfg"] for e in syn.jasper_10x5_layers()] + \
        [e["cfg"] for e in syn.jasper_10x5_layers(B=1, T_in=320)]
    for c in cfgs:
        assert c.T_out == orc.out_len(c.T, c.K, c.stride, c.dilation, c.pad), c.name
        assert c.T_out == nm.nm_conv1d_out_len(c.T, c.K, c.stride, c.dilation, c.pad), c.name


# ---- the block with training-mode BatchNorm -----------------------------------------------------------
def test_bn_entry_points_report_argument_errors_before_any_device_call():
    L_ = nm.lib()
    d = dict(GOOD)
    dims = (d["B"], d["Cin"], d["Cout"], d["T"], d["K"], d["stride"], d["dilation"], d["pad"])
    eps = ctypes.c_float(1e-3)

    def bn_fwd(x=FAKE2, z=FAKE3, y=FAKE4, mean=FAKE5, dims=dims, flags=0, eps=eps, ws=None, ws_bytes=0):
        return L_.nm_conv1d_bn_fwd(*dims, x, FAKE, None, None, eps, None, z, y, mean, FAKE, flags, 0, ws, ws_bytes, None)

    assert bn_fwd(x=None) == nm.NM_ERR_BAD_ARG
    assert bn_fwd(mean=None) == nm.NM_ERR_BAD_ARG
    assert bn_fwd(eps=ctypes.c_float(-1.0)) == nm.NM_ERR_BAD_ARG
    assert bn_fwd(flags=nm.NM_ACCUM_DW) == nm.NM_ERR_BAD_ARG
    assert bn_fwd(dims=(0,) + dims[1:]) == nm.NM_ERR_BAD_ARG
    assert bn_fwd() == nm.NM_ERR_WORKSPACE  # it always needs scratch for the statistics
    need = nm.nm_conv1d_workspace_bytes(nm.NM_OP_BN_FWD, *dims)
    assert need >= 3 * 8 * d["B"] * d["Cout"] and need % 256 == 0
    assert nm.nm_conv1d_workspace_bytes(nm.NM_OP_BN_BWD, *dims) > nm.nm_conv1d_workspace_bytes(nm.NM_OP_BWD, *dims)

    def bn_bwd(x=FAKE2, y=FAKE3, dy=FAKE4, dx=FAKE5, flags=nm.NM_RELU):
        return L_.nm_conv1d_bn_bwd(*dims, x, FAKE, None, FAKE, y, FAKE, FAKE, dy, dx, None, FAKE, None, None, flags, 0,
                                   None, 0, None)

    assert bn_bwd(x=None) == nm.NM_ERR_BAD_ARG
    assert bn_bwd(y=None) == nm.NM_ERR_BAD_ARG      # NM_RELU needs the saved output
    assert bn_bwd(dx=None) == nm.NM_ERR_BAD_ARG
    assert bn_bwd() == nm.NM_ERR_WORKSPACE


def test_fp8_entry_points_report_argument_errors_before_any_device_call():
    L = nm.lib()
    ok = dict(B=2, Cin=64, Cout=128, T=200, K=17, stride=1, dilation=1, pad=8)

    def sup(**kw):
        d = dict(ok, **kw)
        return nm.nm_conv1d_fp8_supported(d["B"], d["Cin"], d["Cout"], d["T"], d["K"], d["stride"], d["dilation"], d["pad"])

    assert sup() and sup(K=21, pad=10) and sup(K=25, pad=12) and sup(K=29, dilation=2, pad=28) and sup(pad=0) and sup(pad=16)
    assert not sup(K=11, pad=5) and not sup(K=3, pad=1) and not sup(stride=2) and not sup(dilation=2)
    assert not sup(Cin=96) and not sup(Cout=100) and not sup(pad=17) and not sup(B=0) and not sup(T=10, pad=0)
    need = nm.nm_conv1d_fp8_workspace_bytes(**ok)
    # codes of x: 2 items x 1 chunk x (2*160 + 16) rows x 64 B; of w: 2 tiles x 1 chunk x 17 taps x 4 KiB; slack each
    assert need >= 2 * 336 * 64 + 2 * 17 * 4096 and need % 256 == 0
    assert nm.nm_conv1d_fp8_workspace_bytes(**dict(ok, K=5, pad=2)) == 0

    def call(x=FAKE2, xs=FAKE, w=FAKE3, ws=FAKE, y=FAKE4, flags=0, wsp=FAKE5, wsb=None, res=None, **kw):
        d = dict(ok, **kw)
        return L.nm_conv1d_block_fwd_fp8(d["B"], d["Cin"], d["Cout"], d["T"], d["K"], d["stride"], d["dilation"], d["pad"],
                                         x, xs, w, ws, None, None, res, y, flags, wsp, need if wsb is None else wsb, None)

    assert call(K=11, pad=5) == nm.NM_ERR_UNSUPPORTED and call(Cin=96) == nm.NM_ERR_UNSUPPORTED
    assert call(B=0) == nm.NM_ERR_BAD_ARG and call(pad=-1) == nm.NM_ERR_BAD_ARG
    for missing in ("x", "xs", "w", "ws", "y"):
        assert call(**{missing: None}) == nm.NM_ERR_BAD_ARG, missing
    assert call(flags=nm.NM_ACCUM_DW) == nm.NM_ERR_BAD_ARG
    assert call(wsp=None) == nm.NM_ERR_WORKSPACE and call(wsb=need - 1) == nm.NM_ERR_WORKSPACE
    assert call(wsp=ctypes.c_void_p(0x7C0000000010)) == nm.NM_ERR_WORKSPACE
    assert call(y=FAKE2) == nm.NM_ERR_BAD_ARG and call(res=FAKE4) == nm.NM_ERR_BAD_ARG   # y aliases x / the residual
    assert call(w=ctypes.c_void_p(0x7E0000000008)) == nm.NM_ERR_BAD_ARG                    # w not 16-byte aligned
    assert L.nm_fp8_row_scales(None, 1, 8, FAKE, None) == nm.NM_ERR_BAD_ARG
    assert L.nm_fp8_row_scales(FAKE2, 0, 8, FAKE, None) == nm.NM_ERR_BAD_ARG
    assert L.nm_fp8_row_scales(FAKE2, 1 << 20, 1 << 20, FAKE, None) == nm.NM_ERR_UNSUPPORTED
    assert L.nm_fp8_quantize_rows(FAKE2, 1, 0, FAKE, FAKE3, None) == nm.NM_ERR_BAD_ARG
    assert L.nm_fp8_quantize_rows(FAKE2, 2, 8, FAKE, FAKE2, None) == nm.NM_ERR_BAD_ARG       # codes alias x


def test_fp8_input_gradient_reports_argument_errors_before_any_device_call():
    L = nm.lib()
    ok = dict(B=2, Cin=64, Cout=128, T=200, K=17, stride=1, dilation=1, pad=8)
    need = nm.nm_conv1d_fp8_bwd_data_workspace_bytes(**ok)
    # codes of g: 2 items x 2 chunks x (2*160 + 16) rows x 64 B; of the weights: 1 tile x 2 chunks x 17 taps x 4 KiB
    assert need >= 2 * 2 * 336 * 64 + 2 * 17 * 4096 and need % 256 == 0
    assert nm.nm_conv1d_fp8_bwd_data_workspace_bytes(**dict(ok, K=5, pad=2)) == 0

    def call(dy=FAKE2, yv=None, gs=FAKE, w=FAKE3, wts=FAKE, dx=FAKE4, dres=None, flags=0, wsp=FAKE5, wsb=None, **kw):
        d = dict(ok, **kw)
        return L.nm_conv1d_bwd_data_fp8(d["B"], d["Cin"], d["Cout"], d["T"], d["K"], d["stride"], d["dilation"], d["pad"],
                                        dy, yv, gs, w, None, wts, dx, dres, flags, wsp, need if wsb is None else wsb, None)

    assert call(K=11, pad=5) == nm.NM_ERR_UNSUPPORTED and call(Cout=100) == nm.NM_ERR_UNSUPPORTED
    assert call(T=0) == nm.NM_ERR_BAD_ARG
    for missing in ("dy", "gs", "w", "wts", "dx"):
        assert call(**{missing: None}) == nm.NM_ERR_BAD_ARG, missing
    assert call(flags=nm.NM_RELU) == nm.NM_ERR_BAD_ARG                                  # the mask needs y
    assert call(flags=nm.NM_ACCUM_DX) == nm.NM_ERR_BAD_ARG
    assert call(wsp=None) == nm.NM_ERR_WORKSPACE and call(wsb=need - 1) == nm.NM_ERR_WORKSPACE
    assert call(dx=FAKE2) == nm.NM_ERR_BAD_ARG and call(dres=FAKE2) == nm.NM_ERR_BAD_ARG   # dx / dres alias dy
    assert L.nm_fp8_dgrad_weight_scales(64, 64, 17, None, None, FAKE, None) == nm.NM_ERR_BAD_ARG
    assert L.nm_fp8_dgrad_weight_scales(0, 64, 17, FAKE2, None, FAKE, None) == nm.NM_ERR_BAD_ARG


def test_fp8_weight_gradient_reports_argument_errors_before_any_device_call():
    L = nm.lib()
    ok = dict(B=2, Cin=64, Cout=128, T=200, K=17, stride=1, dilation=1, pad=8)
    need = nm.nm_conv1d_fp8_bwd_weight_workspace_bytes(**ok)
    assert need > 0 and need % 256 == 0
    assert nm.nm_conv1d_fp8_bwd_weight_workspace_bytes(**dict(ok, stride=2)) == 0

    def call(x=FAKE2, xs=FAKE, dy=FAKE3, yv=None, gs=FAKE, dw=FAKE4, flags=0, wsp=FAKE5, wsb=None, **kw):
        d = dict(ok, **kw)
        return L.nm_conv1d_bwd_weight_fp8(d["B"], d["Cin"], d["Cout"], d["T"], d["K"], d["stride"], d["dilation"], d["pad"],
                                          x, xs, dy, yv, gs, None, dw, flags, wsp, need if wsb is None else wsb, None)

    assert call(K=13, pad=6) == nm.NM_ERR_UNSUPPORTED and call(Cin=32) == nm.NM_ERR_UNSUPPORTED
    assert call(K=0) == nm.NM_ERR_BAD_ARG
    for missing in ("x", "xs", "dy", "gs", "dw"):
        assert call(**{missing: None}) == nm.NM_ERR_BAD_ARG, missing
    assert call(flags=nm.NM_RELU) == nm.NM_ERR_BAD_ARG                # the mask needs y
    assert call(flags=nm.NM_ACCUM_DX) == nm.NM_ERR_BAD_ARG
    assert call(wsp=None) == nm.NM_ERR_WORKSPACE and call(wsb=need - 1) == nm.NM_ERR_WORKSPACE
    assert call(dw=FAKE2) == nm.NM_ERR_BAD_ARG                          # dw aliases x
