"""CPU oracle of the 8-bit floating-point variant of the conv1d block forward.

TEST INFRASTRUCTURE ONLY: imported by ``tests/`` (and the smoke check / CPU-baseline legs); the GPU
product path never imports this module and this module never imports the GPU package.

The paper trains in mixed precision (Section 3.3): convolutions run on low-precision operands while
sums and master state stay in float32.  It names float16; this variant applies the same contract
with the 8-bit E4M3 format of the published OCP 8-bit floating-point specification (1 sign, 4 exponent
bits with bias 7, 3 mantissa bits; no infinities; S.1111.111 is NaN; largest finite value 448;
subnormals are multiples of 2^-9).  The paper gives no quantisation rule, so the usual scaled one is
taken:

    scale of a tensor (or of one output channel of the weights)   s = amax / 448   (1 if amax == 0)
    code                                                         q = E4M3( v * (1/s) )
    value it stands for                                           s * decode(q)

with amax the largest magnitude, every operation in float32 (s = float32 division, 1/s = float32
division, v*(1/s) = one float32 multiplication), the conversion to E4M3 rounding to nearest with
ties to the even mantissa and saturating at +-448.  The block is then the plain definition on the
values the codes stand for, in float64:

    z[b,co,t] = sum_ci sum_k  decode(wq[co,ci,k]) * decode(xq[b,ci,tau(t,k)])
    y         = relu?( scale[co] * (sx*sw[co]) * z + shift[co] + residual[b,co,t] )

The convolution itself is conv1d_oracle's (this module only supplies the codec and the scales).
Pins: tests/test_fp8_oracle_pins.py (values the format specification fixes, torch's CPU float8_e4m3fn
casts for every code and for random and tie values, brute-force nearest-neighbour rounding over the
table of the 254 finite values, monotonicity, round trip).
"""
from __future__ import annotations

import numpy as np

E4M3_MAX = 448.0


def e4m3_decode(codes) -> np.ndarray:
    """float64 value of each E4M3 code (uint8).  NaN codes (0x7F, 0xFF) decode to NaN."""
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where(c & 0x80, -1.0, 1.0)
    e = (c >> 3) & 0xF
    m = (c & 0x7).astype(np.float64)
    normal = np.ldexp(1.0 + m / 8.0, (e - 7).astype(np.int64))
    subnormal = np.ldexp(m / 8.0, -6)
    v = np.where(e == 0, subnormal, normal)
    v = np.where((e == 15) & ((c & 7) == 7), np.nan, v)
    return sign * v


def e4m3_encode(v) -> np.ndarray:
    """E4M3 code (uint8) of each float32 value: round to nearest, ties to the even mantissa, magnitudes
    above 448 saturate to +-448, NaN gives 0x7F."""
    v = np.asarray(v, dtype=np.float32).astype(np.float64)
    a = np.minimum(np.abs(np.where(np.isnan(v), 0.0, v)), E4M3_MAX)
    # spacing of the representable values around a: 2^(e-3) with e = floor(log2 a), at least 2^-9
    with np.errstate(divide="ignore", invalid="ignore"):
        e = np.floor(np.log2(np.where(a > 0, a, 1.0)))
    e = np.maximum(e, -6.0)
    step = np.ldexp(1.0, (e - 3).astype(np.int64))
    n = np.rint(a / step)                      # numpy rounds halves to even; a/step is exact (power of two)
    q = n * step                               # the rounded magnitude (may have moved up to the next binade)
    # back to fields
    with np.errstate(divide="ignore", invalid="ignore"):
        e2 = np.floor(np.log2(np.where(q > 0, q, 1.0)))
    sub = q < 2.0 ** -6
    e2 = np.where(sub, -6.0, e2)
    mant = np.where(sub, q / 2.0 ** -9, (q / np.ldexp(1.0, e2.astype(np.int64)) - 1.0) * 8.0)
    field_e = np.where(sub, 0, e2 + 7).astype(np.int64)
    code = (field_e << 3) | np.rint(mant).astype(np.int64)
    code = np.where(np.signbit(v), code | 0x80, code)
    code = np.where(np.isnan(v), 0x7F, code)
    return code.astype(np.uint8)


def row_scales(x, rows: int) -> np.ndarray:
    """float32 scale of each of `rows` equal slices of x (flattened): amax/448, or 1 where amax is 0."""
    a = np.abs(np.asarray(x, dtype=np.float32).reshape(rows, -1)).max(axis=1)
    s = (a / np.float32(E4M3_MAX)).astype(np.float32)
    return np.where(a == 0, np.float32(1.0), s).astype(np.float32)


def quantize_rows(x, scales) -> np.ndarray:
    """codes of x (same shape) where slice r of x (flattened into len(scales) equal rows) is divided by
    scales[r] as described above."""
    x32 = np.asarray(x, dtype=np.float32)
    s = np.asarray(scales, dtype=np.float32).reshape(-1)
    inv = (np.float32(1.0) / s).astype(np.float32)
    t = (x32.reshape(s.size, -1) * inv[:, None]).astype(np.float32)
    return e4m3_encode(t).reshape(x32.shape)


def block_fwd_fp8(conv_block_fwd, xq, sx, wq, sw, scale, shift, residual, relu, **geom) -> np.ndarray:
    """y of the block on the values the codes stand for.  `conv_block_fwd` is conv1d_oracle.block_fwd
    (passed in so that this module stays free of imports); xq [B][Cin][T], wq [Cout][Cin][K] codes, sx the
    scale of x, sw [Cout] the scales of the weights, scale/shift/residual as for the bf16 block."""
    x = e4m3_decode(xq)
    w = e4m3_decode(wq)
    sw = np.asarray(sw, dtype=np.float64)
    eff = float(np.float64(np.float32(sx))) * sw
    if scale is not None:
        eff = eff * np.asarray(scale, dtype=np.float64)
    return conv_block_fwd(x, w, eff, shift, residual, relu, **geom)


# ---- input gradient on E4M3 operands ------------------------------------------------------------
# dx[b,ci,s] = sum over (co,t,k) with tau(t,k) = s of (w[co,ci,k]*scale[co]) * g[b,co,t],  g = dy*[y>0].
# The contraction runs over co and k, so the weight operand is quantised per INPUT channel ci (the row of
# the contraction's left operand): the affine factor is multiplied in first (one float32 multiplication),
# then the slice {w[co,ci,k]*scale[co] : co, k} gets its scale amax/448 and is quantised like any other
# slice.  g is exact in bfloat16 (a value of dy or zero) and is quantised with one scale for the tensor.
def dgrad_weights(w, scale):
    """float32 [Cin][Cout][K]: w[co,ci,k]*scale[co] (one float32 multiplication), input channel first."""
    w32 = np.asarray(w, dtype=np.float32)
    if scale is not None:
        w32 = (w32 * np.asarray(scale, dtype=np.float32)[:, None, None]).astype(np.float32)
    return np.ascontiguousarray(np.transpose(w32, (1, 0, 2)))


def dgrad_weight_scales(w, scale) -> np.ndarray:
    """float32 [Cin]: scale of each input channel's slice of the scaled weights."""
    wt = dgrad_weights(w, scale)
    return row_scales(wt, wt.shape[0])


def masked_gradient(dy, y_saved, relu):
    """g = dy*[y>0] (dy without a ReLU), float32, exact for bfloat16 inputs."""
    dy32 = np.asarray(dy, dtype=np.float32)
    if not relu:
        return dy32
    return np.where(np.asarray(y_saved, dtype=np.float64) > 0, dy32, np.float32(0.0)).astype(np.float32)


def bwd_data_fp8(conv_bwd_data, gq, sg, wtq, swt, T, **geom) -> np.ndarray:
    """dx of the block on the values the codes stand for.  `conv_bwd_data` is conv1d_oracle.bwd_data;
    gq [B][Cout][T_out] codes of g with scale sg; wtq [Cin][Cout][K] codes of the scaled weights with the
    per-input-channel scales swt."""
    dz = e4m3_decode(gq) * float(np.float64(np.float32(sg)))
    w_eff = e4m3_decode(wtq) * np.asarray(swt, dtype=np.float64)[:, None, None]   # [ci][co][k]
    return conv_bwd_data(dz, np.ascontiguousarray(np.transpose(w_eff, (1, 0, 2))), T, **geom)


# ---- weight gradient on E4M3 operands -----------------------------------------------------------
# dw[co,ci,k] = scale[co] * sum_b sum_t g[b,co,t] * x[b,ci,tau(t,k)] on the values the codes of g and x stand
# for (one scale per tensor each); the affine factor multiplies the sums, as in the bfloat16 path.
def bwd_weight_fp8(conv_bwd_weight, xq, sx, gq, sg, scale, K, **geom) -> np.ndarray:
    """dw [Cout][Cin][K] float64.  `conv_bwd_weight` is conv1d_oracle.bwd_weight; xq [B][Cin][T] codes with
    scale sx, gq [B][Cout][T_out] codes with scale sg, scale [Cout] or None."""
    x = e4m3_decode(xq) * float(np.float64(np.float32(sx)))
    dz = e4m3_decode(gq) * float(np.float64(np.float32(sg)))
    if scale is not None:
        dz = dz * np.asarray(scale, dtype=np.float64)[None, :, None]
    return conv_bwd_weight(x, dz, K, **geom)
