/*
 * nm_conv1d.h -- C ABI of the MI355X (gfx950) conv1d sub-block library.
 *
 * The operation is the 1D time-convolution sub-block of the Jasper-style acoustic
 * encoder that the paper's ASR collection trains (Section 4.1.1: JasperEncoder
 * consumes a [batch, feature, time] spectrogram), in the three passes a training
 * step needs (Section 3: a trainable module computes its outputs and its gradient
 * flows).  Operands are low precision and accumulation is float32, following the
 * paper's mixed-precision contract (Section 3.3).  The paper prints no formula; the
 * definition used is the standard one:
 *
 *   T_out      = floor((T + 2*pad - dilation*(K-1) - 1)/stride) + 1
 *   tau(t,k)   = t*stride - pad + k*dilation              (cross-correlation, no flip)
 *   z[b,co,t]  = sum_ci sum_k w[co,ci,k] * x[b,ci,tau(t,k)],   x == 0 outside [0,T)
 *   y          = relu?( scale[co]*z + shift[co] + residual[b,co,t] )
 *   m = [y>0] (1 without ReLU);  dres = dy*m;  dz = dy*m*scale[co]
 *   dx[b,ci,s] = sum over (co,t,k) with tau(t,k)==s of w[co,ci,k]*dz[b,co,t]
 *   dw[co,ci,k]= sum_b sum_t dz[b,co,t] * x[b,ci,tau(t,k)]
 *
 * Conventions common to every entry point
 *  - Tensor pointers are DEVICE pointers to dense row-major buffers with the last
 *    listed dimension innermost: activations [B][C][T], weights [Cout][Cin][K].
 *    The caller owns them; the library never allocates, frees or keeps them.
 *  - `dtype` selects the storage type of x, w, residual, y, dy, dx, dres
 *    (NM_BF16: bfloat16, NM_F32: float).  scale, shift and dw are always float.
 *    Accumulation is float32 in both modes.
 *  - `workspace` is caller-provided device memory of at least
 *    nm_conv1d_workspace_bytes(op, ...) bytes, 256-byte aligned (may be NULL when
 *    that size is 0).  Its contents are scratch: undefined before and after a call.
 *  - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls only enqueue work on that stream; they never synchronise the host.
 *  - Return value: an nm_status.  Argument errors are detected before any device
 *    call, so they are reported identically on a host without a GPU.  No exception,
 *    abort or message crosses the boundary.
 *  - Outputs must not overlap inputs or the workspace.  Results are deterministic:
 *    identical inputs give bit-identical outputs.
 *  - Each tensor must hold fewer than 2^31 elements.
 */
#ifndef NM_CONV1D_H
#define NM_CONV1D_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    NM_OK = 0,
    NM_ERR_BAD_ARG = -1,     /* NULL required pointer, non-positive size, unknown flag/dtype, T_out <= 0 */
    NM_ERR_UNSUPPORTED = -2, /* valid request this build cannot serve (e.g. a tensor of 2^31 elements or more) */
    NM_ERR_WORKSPACE = -3,   /* workspace NULL, misaligned or smaller than required */
    NM_ERR_DEVICE = -4,      /* the HIP runtime refused a launch */
    NM_ERR_SCRATCH_LIMIT = -5 /* nm_conv1d_block_fwd_static only: the geometry needs more scratch than
                                 NM_STATIC_SCRATCH_BYTES */
} nm_status;

typedef enum { NM_BF16 = 0, NM_F32 = 1 } nm_dtype;

/* flags */
enum {
    NM_RELU = 1u,        /* forward: apply max(.,0); backward: mask with [y > 0] (y required) */
    NM_ACCUM_DW = 2u,    /* bwd_weight: dw += result instead of dw = result (gradient
                            accumulation over several batches, paper Section 3.3) */
    NM_FORCE_DIRECT = 4u, /* use the plain one-thread-per-output kernels instead of the
                            matrix-core kernels (always used for NM_F32) */
    NM_ACCUM_DX = 8u     /* bwd_data / bwd: dx = round(dx + gradient), one rounding, instead of dx = gradient:
                            sums the two gradients that meet at the input of a residual block (the first
                            sub-block's and the residual projection's) without a pass of its own */
};

enum { NM_OP_FWD = 0, NM_OP_BWD_DATA = 1, NM_OP_BWD_WEIGHT = 2, NM_OP_BWD = 3, NM_OP_BN_FWD = 4, NM_OP_BN_BWD = 5 };

/* T_out of the convolution (formula above), or NM_ERR_BAD_ARG (<0) if any argument is
 * out of range or no output position exists.  Host only. */
int nm_conv1d_out_len(int T, int K, int stride, int dilation, int pad);

/* Bytes of device workspace that operation `op` (NM_OP_*) needs for this geometry,
 * dtype and flags.  Returns 0 for invalid arguments (the operation itself then
 * reports NM_ERR_BAD_ARG).  Host only. */
size_t nm_conv1d_workspace_bytes(int op, int B, int Cin, int Cout, int T, int K, int stride,
                                 int dilation, int pad, int dtype, unsigned flags);

/* Static, NUL-terminated description of a status code. */
const char *nm_strerror(int status);

/* Block forward (conv + folded-BatchNorm affine + optional residual + optional ReLU).
 *   x        [B][Cin][T]        in,  dtype
 *   w        [Cout][Cin][K]     in,  dtype
 *   scale    [Cout] float       in,  NULL means 1
 *   shift    [Cout] float       in,  NULL means 0
 *   residual [B][Cout][T_out]   in,  dtype, NULL means none; added before the ReLU
 *   y        [B][Cout][T_out]   out, dtype (float32 result rounded to nearest even)
 */
int nm_conv1d_block_fwd(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad,
                        const void *x, const void *w, const float *scale, const float *shift,
                        const void *residual, void *y, unsigned flags, int dtype,
                        void *workspace, size_t workspace_bytes, void *hip_stream);

/* Input gradient of the block.
 *   dy    [B][Cout][T_out]  in,  dtype: gradient with respect to the block output y
 *   y     [B][Cout][T_out]  in,  dtype: saved forward output; required iff NM_RELU
 *   scale [Cout] float      in,  NULL means 1
 *   w     [Cout][Cin][K]    in,  dtype
 *   dx    [B][Cin][T]       out, dtype
 *   dres  [B][Cout][T_out]  out, dtype, or NULL: gradient with respect to the residual
 * In NM_BF16 mode the matrix-core kernels contract g = dy*m (exact in bfloat16) with the weights
 * bf16(w[co,ci,k]*scale[co]): the affine factor is folded into the weight operand, rounded once per weight.
 * The weight gradient contracts the same g and multiplies its float32 sums by scale[co].  The plain
 * kernels (NM_FORCE_DIRECT, NM_F32) form dz = g*scale in the storage type instead.
 * With lengths and NM_ACCUM_DX, positions at or beyond a sample's length keep their old value.
 */
int nm_conv1d_bwd_data(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad,
                       const void *dy, const void *y, const float *scale, const void *w,
                       void *dx, void *dres, unsigned flags, int dtype,
                       void *workspace, size_t workspace_bytes, void *hip_stream);

/* Weight gradient of the block.
 *   x     [B][Cin][T]       in,  dtype
 *   dy, y, scale            as for nm_conv1d_bwd_data
 *   dw    [Cout][Cin][K]    out, float (in/out with NM_ACCUM_DW)
 */
int nm_conv1d_bwd_weight(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad,
                         const void *x, const void *dy, const void *y, const float *scale,
                         float *dw, unsigned flags, int dtype,
                         void *workspace, size_t workspace_bytes, void *hip_stream);

/* Both gradients of the block in one call (paper Section 3.3: the backward pass of a module).
 * Same results as nm_conv1d_bwd_data followed by nm_conv1d_bwd_weight on the same arguments,
 * bit for bit; where the matrix-core kernels apply, the mask-and-scale pass over dy and y that
 * forms dz runs once and feeds both gradients.  Arguments as for those two calls; dres may be
 * NULL; workspace of nm_conv1d_workspace_bytes(NM_OP_BWD, ...) bytes. */
int nm_conv1d_bwd(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad,
                  const void *x, const void *dy, const void *y, const float *scale, const void *w,
                  void *dx, void *dres, float *dw, unsigned flags, int dtype,
                  void *workspace, size_t workspace_bytes, void *hip_stream);

/* The block with training-mode BatchNorm (paper Section 4.1.1 trains the encoder with the `train` action;
 * Section 3: a trainable module computes its outputs and its gradient flows).  Instead of a given affine the
 * normalisation uses the statistics of the batch, taken per output channel over batch and time
 * (N = B*T_out elements):
 *   z = conv(x, w), stored in `dtype`;  mean[c] = (1/N) sum z;  var[c] = (1/N) sum (z-mean)^2 (biased);
 *   invstd[c] = 1/sqrt(var[c]+eps);  zhat = (z-mean)*invstd;  y = relu?( gamma[c]*zhat + beta[c] + residual ).
 * The statistics and y are computed from the stored z (in NM_BF16 mode: the rounded values).
 *   nm_conv1d_bn_fwd:  x, w, residual (or NULL) in; gamma, beta [Cout] float in (NULL: 1 / 0);
 *                      z, y [B][Cout][T_out] out (dtype); mean, invstd [Cout] float out (saved for backward).
 *   nm_conv1d_bn_bwd:  x, w, gamma, the saved z, y (y required iff NM_RELU), mean, invstd and dy in;
 *                      g = dy*[y>0];  dres = g (or NULL);  dbeta[c] = sum g;  dgamma[c] = sum g*zhat (NULL: not wanted);
 *                      dz = gamma*invstd*( g - dbeta/N - zhat*dgamma/N ), rounded to dtype, is then contracted:
 *                      dx [B][Cin][T] and dw [Cout][Cin][K] float as by nm_conv1d_bwd on dz.
 *                      NM_ACCUM_DW adds into dw, dgamma and dbeta; NM_ACCUM_DX into dx.
 * Workspace: nm_conv1d_workspace_bytes(NM_OP_BN_FWD / NM_OP_BN_BWD, ...).  Sums are deterministic.  Other
 * conventions and errors as for the calls above. */
int nm_conv1d_bn_fwd(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad, const void *x,
                     const void *w, const float *gamma, const float *beta, float eps, const void *residual, void *z,
                     void *y, float *mean, float *invstd, unsigned flags, int dtype, void *workspace,
                     size_t workspace_bytes, void *hip_stream);
int nm_conv1d_bn_bwd(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad, const void *x,
                     const void *w, const float *gamma, const void *z, const void *y, const float *mean,
                     const float *invstd, const void *dy, void *dx, void *dres, float *dw, float *dgamma, float *dbeta,
                     unsigned flags, int dtype, void *workspace, size_t workspace_bytes, void *hip_stream);

/* The three passes on a padded batch (paper Section 4.1.1: the encoder takes the length of every
 * utterance next to the padded batch).  lengths [B] int32 (device): samples of batch item b at
 * t >= lengths[b] are padding; values are clipped to [0, T].
 *   block_fwd_masked:   padding of x reads as zero (whatever the buffer holds there, NaN included);
 *                       y is written for all T_out positions (the block does not mask its output;
 *                       the valid length behind it is nm_conv1d_out_len(lengths[b], ...)).
 *   bwd_weight_masked:  dw from x with its padding read as zero.
 *   bwd_data_masked:    dx is zero on the padding.
 *   bwd_masked:         both of these in one call.
 * All other arguments, the workspace size and the error behaviour are those of the unmasked calls;
 * lengths == NULL is NM_ERR_BAD_ARG. */
int nm_conv1d_block_fwd_masked(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad,
                               const int *lengths, const void *x, const void *w, const float *scale,
                               const float *shift, const void *residual, void *y, unsigned flags,
                               int dtype, void *workspace, size_t workspace_bytes, void *hip_stream);
int nm_conv1d_bwd_data_masked(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad,
                              const int *lengths, const void *dy, const void *y, const float *scale,
                              const void *w, void *dx, void *dres, unsigned flags, int dtype,
                              void *workspace, size_t workspace_bytes, void *hip_stream);
int nm_conv1d_bwd_weight_masked(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad,
                                const int *lengths, const void *x, const void *dy, const void *y,
                                const float *scale, float *dw, unsigned flags, int dtype,
                                void *workspace, size_t workspace_bytes, void *hip_stream);
/* nm_conv1d_bwd on a padded batch: the results of bwd_data_masked and bwd_weight_masked, bit for bit, from one call. */
int nm_conv1d_bwd_masked(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad, const int *lengths,
                         const void *x, const void *dy, const void *y, const float *scale, const void *w, void *dx,
                         void *dres, float *dw, unsigned flags, int dtype, void *workspace, size_t workspace_bytes,
                         void *hip_stream);

/* Decoder tail (paper Section 4.1.1: the CTC decoder module turns the encoder output into per-frame
 * log-probabilities over the vocabulary): a 1x1 convolution to Ncls classes followed by a log-softmax
 * over the classes of every frame,
 *   z[b,c,t] = sum_ci w[c,ci]*x[b,ci,t] + bias[c],   logp[b,c,t] = z[b,c,t] - log(sum_c' exp(z[b,c',t])).
 *   x    [B][Cin][T]    in,  dtype
 *   w    [Ncls][Cin]    in,  dtype
 *   bias [Ncls] float   in,  NULL means 0
 *   logp [B][Ncls][T]   out, float
 * flags: 0 or NM_FORCE_DIRECT.  Needs no workspace.  Device pointers owned by the caller; the call
 * only enqueues on hip_stream.  Errors as for the other entry points. */
int nm_decoder_logsoftmax_fwd(int B, int Cin, int Ncls, int T, const void *x, const void *w,
                              const float *bias, float *logp, unsigned flags, int dtype,
                              void *hip_stream);

/* Block forward for callers that cannot allocate device memory or size a workspace: code running under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation, arguments,
 * results (bit for bit) and error behaviour as nm_conv1d_block_fwd, without the workspace arguments: the
 * scratch its kernels need (the weights in matrix-core fragment order) lives in a fixed array of
 * NM_STATIC_SCRATCH_BYTES inside the library, one copy per GPU, held until the process ends.  The call
 * allocates and frees nothing.  A geometry whose nm_conv1d_workspace_bytes(NM_OP_FWD, ...) exceeds
 * NM_STATIC_SCRATCH_BYTES returns NM_ERR_SCRATCH_LIMIT before anything is launched.  Every call on a GPU
 * uses that GPU's one array: calls that overlap in time on one GPU (different streams or threads) race on
 * it and must be serialised by the caller.  Nothing in the array has to survive between calls. */
#define NM_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
int nm_conv1d_block_fwd_static(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad,
                               const void *x, const void *w, const float *scale, const float *shift,
                               const void *residual, void *y, unsigned flags, int dtype, void *hip_stream);

/* Measurement aid (no effect on results; the only state the library keeps besides the array above, and
 * it is per thread).  Arms a one-shot timer for the calling thread: the next entry-point call made by this
 * thread records `start_event` immediately before and `stop_event` immediately after a main convolution
 * kernel of that call, on the call's stream (helper kernels -- weight packing, the mask pass, the final dw
 * reduction -- stay outside the pair).  Which kernel: the first main kernel the call launches
 * (nm_conv1d_time_next_main_kernel: the input-gradient kernel of an nm_conv1d_bwd call), or the main
 * kernel of pass `op` (nm_conv1d_time_next_kernel_of: NM_OP_FWD, NM_OP_BWD_DATA or NM_OP_BWD_WEIGHT; other
 * values return NM_ERR_BAD_ARG), which reaches the weight-gradient kernel inside nm_conv1d_bwd.  Both
 * arguments are hipEvent_t handles created by the caller with timing enabled; passing NULL for either
 * disarms.  The pair is consumed by that call whether it succeeds, runs such a kernel, or not.
 * Returns NM_OK. */
int nm_conv1d_time_next_main_kernel(void *start_event, void *stop_event);
int nm_conv1d_time_next_kernel_of(void *start_event, void *stop_event, int op);

#ifdef __cplusplus
}
#endif
#endif /* NM_CONV1D_H */
