/*
 * nm_conv1d_fp8.h -- C ABI of the 8-bit floating-point variant of the conv1d block: forward, input gradient
 * and weight gradient (gfx950).
 *
 * The paper's mixed-precision contract (Section 3.3) runs the convolutions on low-precision operands
 * and keeps sums in float32; it names float16.  This variant applies the same contract with the E4M3
 * format of the OCP 8-bit floating-point specification (1 sign, 4 exponent bits, bias 7, 3 mantissa
 * bits, no infinities, largest finite value 448), which the gfx950 matrix cores multiply at twice the
 * bfloat16 rate.  The paper gives no quantisation rule; the usual scaled one is used:
 *
 *   scale of a slice         s    = amax / 448            (1 when the slice is all zero), float32 division
 *   code of an element       q    = E4M3( v * (1/s) )     1/s and the product in float32; round to nearest,
 *                                                          ties to the even mantissa, saturating at +-448
 *   block                    z    = sum_ci sum_k decode(wq[co,ci,k]) * decode(xq[b,ci,tau(t,k)])   (float32 sums)
 *                            y    = relu?( scale[co]*sx*sw[co]*z + shift[co] + residual[b,co,t] )
 *
 * with one scale sx for the activation tensor and one scale sw[co] per output channel of the weights.
 * The scales are inputs of the block (device memory), so a training loop may reuse those of an earlier
 * step; nm_fp8_row_scales computes them from a tensor.
 *
 * Conventions (pointers, ownership, stream, status codes, determinism, argument checks before any device
 * call) are those of nm_conv1d.h.  All tensors here are bfloat16 except where stated.
 */
#ifndef NM_CONV1D_FP8_H
#define NM_CONV1D_FP8_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* scales[r] = max |x[r*row_len .. (r+1)*row_len)| / 448 (1 if that maximum is 0), r < rows.
 *   x       [rows][row_len] bfloat16, device, in
 *   scales  [rows] float, device, out
 * rows >= 1, row_len >= 1, rows*row_len < 2^31.  Needs no workspace. */
int nm_fp8_row_scales(const void *x, int rows, size_t row_len, float *scales, void *hip_stream);

/* codes[i] = E4M3( x[i] * (1/scales[i / row_len]) ), same element order as x.
 *   x       [rows][row_len] bfloat16, device, in
 *   scales  [rows] float, device, in (positive, finite)
 *   codes   [rows][row_len] bytes, device, out */
int nm_fp8_quantize_rows(const void *x, int rows, size_t row_len, const float *scales, unsigned char *codes,
                         void *hip_stream);

/* 1 if nm_conv1d_block_fwd_fp8 serves this geometry, 0 if it returns NM_ERR_UNSUPPORTED (or the
 * arguments are invalid).  Served: stride 1, Cin and Cout multiples of 64, and (K, dilation) one of
 * (17,1) (21,1) (25,1) (29,2) -- the tap counts of the encoder's 512- to 896-channel blocks.  Host only. */
int nm_conv1d_fp8_supported(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad);

/* Bytes of device workspace of nm_conv1d_block_fwd_fp8 (0 for an unsupported or invalid geometry).  Host only. */
size_t nm_conv1d_fp8_workspace_bytes(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad);

/* Block forward on E4M3 operands.
 *   x         [B][Cin][T]        bfloat16, in: quantised inside the call with x_scale
 *   x_scale   [1] float          device, in
 *   w         [Cout][Cin][K]     bfloat16, in: quantised inside the call, output channel co with w_scales[co]
 *   w_scales  [Cout] float       device, in
 *   scale, shift [Cout] float    in, NULL means 1 / 0
 *   residual  [B][Cout][T_out]   bfloat16, in, or NULL
 *   y         [B][Cout][T_out]   bfloat16, out (float32 result rounded to nearest even)
 * flags: 0 or NM_RELU.  workspace: nm_conv1d_fp8_workspace_bytes(...) bytes, 256-byte aligned; it holds the
 * codes of x (time-major in 64-channel groups, zero rows for the padding) and of w (matrix-core fragment
 * order) and is scratch.  Returns NM_ERR_UNSUPPORTED for geometries outside nm_conv1d_fp8_supported. */
int nm_conv1d_block_fwd_fp8(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad,
                            const void *x, const float *x_scale, const void *w, const float *w_scales,
                            const float *scale, const float *shift, const void *residual, void *y,
                            unsigned flags, void *workspace, size_t workspace_bytes, void *hip_stream);

/* Input gradient of the block on E4M3 operands (paper Section 3: a trainable module computes its gradient flows;
 * Section 3.3: in low precision with float32 sums).
 *   g = dy*[y>0] (dy without NM_RELU), exact in bfloat16;  dres = g;
 *   gq = E4M3(g * (1/g_scale)), one scale for the tensor;
 *   the weight operand is w[co,ci,k]*scale[co] (one float32 multiplication), quantised per INPUT channel:
 *   wq[ci,co,k] = E4M3( (w[co,ci,k]*scale[co]) * (1/wt_scales[ci]) );
 *   dx[b,ci,s] = g_scale*wt_scales[ci] * sum over (co,t,k) with tau(t,k)==s of decode(wq[ci,co,k])*decode(gq[b,co,t]),
 *   float32 sums, rounded to bfloat16.
 *   dy, y     [B][Cout][T_out]  bfloat16, in (y required iff NM_RELU)
 *   g_scale   [1] float         device, in (e.g. nm_fp8_row_scales of dy: |g| <= |dy|)
 *   w         [Cout][Cin][K]    bfloat16, in;  scale [Cout] float, in, NULL means 1
 *   wt_scales [Cin] float       device, in (nm_fp8_dgrad_weight_scales)
 *   dx        [B][Cin][T]       bfloat16, out;  dres [B][Cout][T_out] bfloat16, out, or NULL
 * Served geometries: those of nm_conv1d_fp8_supported.  Workspace: nm_conv1d_fp8_bwd_data_workspace_bytes(...). */
int nm_conv1d_bwd_data_fp8(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad,
                           const void *dy, const void *y, const float *g_scale, const void *w, const float *scale,
                           const float *wt_scales, void *dx, void *dres, unsigned flags, void *workspace,
                           size_t workspace_bytes, void *hip_stream);
size_t nm_conv1d_fp8_bwd_data_workspace_bytes(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad);

/* scales[ci] = max over (co,k) of |w[co,ci,k]*scale[co]| / 448 (1 if that maximum is 0): the per-input-channel
 * scales of the input gradient's weight operand.  w [Cout][Cin][K] bfloat16; scale [Cout] float or NULL;
 * scales [Cin] float, device, out. */
int nm_fp8_dgrad_weight_scales(int Cin, int Cout, int K, const void *w, const float *scale, float *scales,
                               void *hip_stream);

/* Weight gradient of the block on E4M3 operands (same passages as the input gradient).
 *   g = dy*[y>0] quantised with g_scale, x quantised with x_scale (one scale per tensor each, as in the forward);
 *   dw[co,ci,k] = scale[co]*g_scale*x_scale * sum_b sum_t decode(gq[b,co,t])*decode(xq[b,ci,tau(t,k)]),
 *   float32 sums; the factor multiplies the sums in the final deterministic reduction.
 *   x   [B][Cin][T] bfloat16, in;  dy, y [B][Cout][T_out] bfloat16, in (y required iff NM_RELU)
 *   x_scale, g_scale [1] float, device, in;  scale [Cout] float, in, NULL means 1
 *   dw  [Cout][Cin][K] float, out (in/out with NM_ACCUM_DW)
 * flags: NM_RELU, NM_ACCUM_DW.  Served geometries: those of nm_conv1d_fp8_supported.
 * Workspace: nm_conv1d_fp8_bwd_weight_workspace_bytes(...). */
int nm_conv1d_bwd_weight_fp8(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad, const void *x,
                             const float *x_scale, const void *dy, const void *y, const float *g_scale,
                             const float *scale, float *dw, unsigned flags, void *workspace, size_t workspace_bytes,
                             void *hip_stream);
size_t nm_conv1d_fp8_bwd_weight_workspace_bytes(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad);

/* Both gradients on E4M3 operands in one call: the results of nm_conv1d_bwd_data_fp8 and nm_conv1d_bwd_weight_fp8
 * on the same arguments, bit for bit; the pass over dy and y that masks and quantises g runs once and feeds both.
 * Arguments as for those two calls (dres may be NULL); flags: NM_RELU, NM_ACCUM_DW.
 * Workspace: nm_conv1d_fp8_bwd_workspace_bytes(...). */
int nm_conv1d_bwd_fp8(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad, const void *x,
                      const float *x_scale, const void *dy, const void *y, const float *g_scale, const void *w,
                      const float *scale, const float *wt_scales, void *dx, void *dres, float *dw, unsigned flags,
                      void *workspace, size_t workspace_bytes, void *hip_stream);
size_t nm_conv1d_fp8_bwd_workspace_bytes(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad);

#ifdef __cplusplus
}
#endif
#endif /* NM_CONV1D_FP8_H */
