// Internal declarations shared by the translation units of the conv1d library.
// Nothing here is part of the public C ABI (that is include/nm_conv1d.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace nm {

// Geometry of one conv1d sub-block; To is T_out.
struct Geom {
    int B, Cin, Cout, T, K, stride, dil, pad, To;
    // valid input length of every batch item (device pointer, [B]) or NULL: samples at t >= len[b] are
    // padding -- read as zero by the forward pass and the weight gradient, given a zero input gradient
    const int *len;
};
// length of batch item b clipped to [0, T] (T without lengths)
__device__ __forceinline__ int valid_len(const Geom &g, int b)
{
    if (!g.len) return g.T;
    const int n = g.len[b];
    return n < 0 ? 0 : (n > g.T ? g.T : n);
}

typedef uint16_t bf16_t;  // raw bfloat16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// float -> bfloat16, round to nearest, ties to even (finite inputs; NaN stays NaN).
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

__device__ __forceinline__ float load_as_f32(const float *p, size_t i) { return p[i]; }
__device__ __forceinline__ float load_as_f32(const bf16_t *p, size_t i) { return bf16_to_f32(p[i]); }
__device__ __forceinline__ void store_from_f32(float *p, size_t i, float v) { p[i] = v; }
// Interleave two registers of packed 16-bit values: (lo halves of a, b) and (hi halves of a, b), each
// with a's half in the low 16 bits -- one byte-permute instruction apiece.
__device__ __forceinline__ uint32_t zip_lo16(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x05040100u); }
__device__ __forceinline__ uint32_t zip_hi16(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }

// Two floats to a packed bf16 pair (lo in the low half) with the hardware conversion: round to
// nearest even like f32_to_bf16, a NaN stays a NaN.
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ void store_from_f32(bf16_t *p, size_t i, float v) { p[i] = f32_to_bf16(v); }
// Value a stored element will read back as (identity for float, bf16 rounding otherwise).
__device__ __forceinline__ float round_to_storage(float v, const float *) { return v; }
__device__ __forceinline__ float round_to_storage(float v, const bf16_t *) { return bf16_to_f32(f32_to_bf16(v)); }

// Eight consecutive elements (one 16-byte group, index i) of the epilogue backward for bf16 tensors
// whose rows are 16-byte aligned: g = dy * [y > 0]; dres = g; dz = bf16(g * scale[co]).
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void epilogue_bwd_vec8_item(size_t i, int Cout, int To8, const u32x4_t *__restrict__ dy,
                                                       const u32x4_t *__restrict__ y, const float *__restrict__ scale,
                                                       int relu, u32x4_t *__restrict__ dz, u32x4_t *__restrict__ dres)
{
    u32x4_t g = dy[i];
    if (relu) {
        const u32x4_t yv = y[i];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            // y > 0 on the bf16 bits: 0x0001..0x7f80 (positive, not zero, not NaN)
            const uint32_t lo = yv[j] & 0xffffu, hi = yv[j] >> 16;
            const uint32_t keep_lo = (lo - 1u < 0x7f80u) ? 0x0000ffffu : 0u;
            const uint32_t keep_hi = (hi - 1u < 0x7f80u) ? 0xffff0000u : 0u;
            g[j] &= keep_lo | keep_hi;
        }
    }
    if (dres) dres[i] = g;
    if (dz) {
        u32x4_t r = g;
        if (scale) {
            const float sc = scale[(int)((i / (size_t)To8) % (size_t)Cout)];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float g0 = __uint_as_float(g[j] << 16) * sc, g1 = __uint_as_float(g[j] & 0xffff0000u) * sc;
                r[j] = pack_bf16x2(g0, g1);
            }
        }
        dz[i] = r;
    }
}

// g = dy * [y > 0] for one 16-byte group (8 bf16): the mask works on the bits, so g is exact.
__device__ __forceinline__ u32x4_t masked_grad8(u32x4_t g, const u32x4_t yv)
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t lo = yv[j] & 0xffffu, hi = yv[j] >> 16;  // y > 0 on bf16 bits: 0x0001..0x7f80
        g[j] &= ((lo - 1u < 0x7f80u) ? 0x0000ffffu : 0u) | ((hi - 1u < 0x7f80u) ? 0xffff0000u : 0u);
    }
    return g;
}

// One wavefront's share of the pass that forms g = dy*[y>0] for the weight-gradient kernels: 32 channels
// (block cm) x 64 time steps (four 16-step fragments from st4*4 on) of batch item b.  Reads are whole
// 128-byte lines (lane = 8 rows x 8 groups of 8 steps, four times); g goes out in MFMA A-fragment order
// [B][ncm][nst][64 lanes][8] (lane l of a fragment: channel l%32, steps 8*(l/32) .. +7; zeros outside the
// tensor), again in whole lines, and, when gplain is given, also in the layout of dy.
__device__ __forceinline__ void mask_pack_wave(int lane, int b, int cm, int st4, int Cout, int To, int ncm, int nst,
                                               const bf16_t *__restrict__ dy, const bf16_t *__restrict__ y, int relu,
                                               u32x4_t *__restrict__ gplain, u32x4_t *__restrict__ gf)
{
    const int tg = lane & 7, st = st4 * 4 + (tg >> 1);
    const int t = 64 * st4 + 8 * tg;
    u32x4_t g[4];
    size_t idx[4];
    bool ok[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int co = cm * 32 + 8 * i + (lane >> 3);
        ok[i] = co < Cout && t + 8 <= To;
        idx[i] = (((size_t)b * Cout + co) * To + t) / 8;  // 16-byte group index
        g[i] = u32x4_t{0u, 0u, 0u, 0u};
        if (ok[i]) g[i] = reinterpret_cast<const u32x4_t *>(dy)[idx[i]];
    }
    if (relu) {
        u32x4_t yv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (ok[i]) yv[i] = reinterpret_cast<const u32x4_t *>(y)[idx[i]];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (ok[i]) g[i] = masked_grad8(g[i], yv[i]);
    }
    if (st < nst) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (gplain && ok[i]) gplain[idx[i]] = g[i];
            gf[(((size_t)b * ncm + cm) * nst + st) * 64 + (tg & 1) * 32 + 8 * i + (lane >> 3)] = g[i];
        }
    }
}

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- per-device facts and one-time kernel set-up (host) -----------------------------------------
// Launches sit on the hot path of a training step, so nothing below queries the runtime more than
// once per device and kernel: the compute-unit count is cached, and the opt-in to more than 64 KiB
// of dynamic LDS (a per-device function attribute) is made on a kernel's first launch on a device.
constexpr int kMaxDevices = 64;
struct DeviceInfo {
    int dev;  // current device, or -1 when the runtime could not say
    int cus;  // its compute units (256 when unknown)
};
DeviceInfo current_device_info();
struct LdsOptIn {
    unsigned char done[kMaxDevices] = {};  // written once per device; a racing second write stores the same value
};
// Raise the dynamic-LDS limit of `fn` to `bytes` on the current device unless that was done before.
hipError_t ensure_dynamic_lds(LdsOptIn &state, const void *fn, int bytes);

// One-shot event pair armed by nm_conv1d_time_next_main_kernel (thread local, nm_conv1d_api.hip).
// Construct right before the launch of a call's main kernel, destroy right after it.
struct MainKernelTimer {
    explicit MainKernelTimer(hipStream_t s);
    ~MainKernelTimer();
    hipStream_t stream;
    hipEvent_t stop;
};

// ---- plain kernels (direct_kernels.hip); is_bf16 selects the storage type ---------------
hipError_t launch_direct_fwd(const Geom &g, bool is_bf16, const void *x, const void *w,
                             const float *scale, const float *shift, const void *res, void *y,
                             bool relu, hipStream_t s);
// dz = dy*[y>0]*scale (any of dz/dres may be NULL); y may be NULL when !relu.
hipError_t launch_epilogue_bwd(const Geom &g, bool is_bf16, const void *dy, const void *y,
                               const float *scale, bool relu, void *dz, void *dres, hipStream_t s);
// Same for bf16 tensors with To % 8 == 0 and 16-byte aligned pointers (8 elements per thread).
hipError_t launch_epilogue_bwd_vec8(const Geom &g, const void *dy, const void *y, const float *scale, bool relu,
                                    void *dz, void *dres, hipStream_t s);
// accumulate: dx = storage(dx + gradient) (positions at or beyond a sample's length keep their value)
hipError_t launch_direct_dgrad(const Geom &g, bool is_bf16, const void *dz, const void *w, void *dx, bool accumulate,
                               hipStream_t s);
// dw = (accumulate ? dw : 0) + scale[co] * sum (scale may be NULL: 1)
hipError_t launch_direct_wgrad(const Geom &g, bool is_bf16, const void *x, const void *dz, const float *scale, float *dw,
                               bool accumulate, hipStream_t s);

// ---- matrix-core kernels (mfma_*.hip), bf16 storage only -------------------------------
// Each *_supported says whether the matrix-core path can serve the geometry; the
// *_workspace functions give its scratch need; launches return hipSuccess or the error.
bool mfma_fwd_supported(const Geom &g);
size_t mfma_fwd_workspace(const Geom &g);
// stats (optional, only where mfma_fwd_stats_parts(g) > 0): [parts][Cout][3] doubles that receive count, mean and
// centred second moment of the stored outputs of every (batch item, 160-step time tile) part and channel
hipError_t launch_mfma_fwd(const Geom &g, const void *x, const void *w, const float *scale,
                           const float *shift, const void *res, void *y, bool relu, void *ws,
                           hipStream_t s, double *stats = nullptr);
int mfma_fwd_stats_parts(const Geom &g);

// pointwise forward with at most 32 output channels: bound by reading x once (decoder_logsoftmax.hip)
bool skinny_fwd_supported(const Geom &g);
hipError_t launch_skinny_fwd(const Geom &g, const void *x, const void *w, const float *scale, const float *shift,
                             const void *res, void *y, bool relu, hipStream_t s);

bool mfma_dgrad_supported(const Geom &g);
size_t mfma_dgrad_workspace(const Geom &g);
// g_used (optional, stride 1): receives the tensor the kernel contracted, g = dy*[y>0] -- dy itself without
// ReLU, else dres or a buffer inside ws -- so that a weight gradient launched next need not form it again
hipError_t launch_mfma_dgrad(const Geom &g, const void *dy, const void *y, const float *scale,
                             const void *w, void *dx, void *dres, bool relu, bool accumulate, void *ws,
                             hipStream_t s, const void **g_used = nullptr);

bool mfma_wgrad_supported(const Geom &g);
size_t mfma_wgrad_workspace(const Geom &g, bool need_dz);
hipError_t launch_mfma_wgrad(const Geom &g, const void *x, const void *dy, const void *y,
                             const float *scale, float *dw, bool relu, bool accumulate, void *ws,
                             hipStream_t s);

// dw[co][ci][k] = (accumulate ? dw : 0) + scale[co] * sum_s part[s][k][co][ci] (scale NULL: 1), fixed order
hipError_t launch_wgrad_reduce(const Geom &g, const float *part, float *dw, const float *scale, int S, bool accumulate,
                               hipStream_t s);
// pointwise (K = 1) weight gradient as a GEMM over plain rows (mfma_wgrad_k1.hip); never with lengths
bool wgrad_k1_supported(const Geom &g);
size_t wgrad_k1_part_bytes(const Geom &g);
hipError_t launch_wgrad_k1(const Geom &g, const void *x, const void *gplain, const float *scale, float *dw, bool accumulate,
                           void *ws, hipStream_t s);

// ---- fused backward: one pass over dy / y feeds both gradients --------------------------------
// The stride-1 weight-gradient kernels read g = dy*[y>0] in MFMA fragment order
// [B][ncm = 2*ceil(Cout/64)][nst][64 lanes][8]: lane l of block (b, cm, st) holds channel cm*32 + l%32,
// time steps 16*st + 8*(l/32) .. +7 (zeros outside the tensor).  It lives `offset` bytes into that
// kernel's workspace (mfma_wgrad_workspace(g, true) bytes in all).
struct DzfLayout {
    int ncm, nst;
    size_t offset, bytes;
};
bool mfma_wgrad_fast_supported(const Geom &g);
DzfLayout mfma_wgrad_dzf_layout(const Geom &g);
// weight gradient from a workspace whose fragment-order g has been written already; scale[co] (or NULL)
// multiplies the float32 sums
hipError_t launch_mfma_wgrad_prepared(const Geom &g, const void *x, const float *scale, float *dw, bool accumulate,
                                      void *ws, hipStream_t s);
// packs the flipped weights times scale into ws (as launch_mfma_dgrad does) and, in the same launch, forms
// g plain (into dres, else behind the packed weights in ws, else nowhere) and in fragment order (gf);
// *g_plain: the tensor the input gradient contracts
hipError_t launch_bwd_prepare(const Geom &g, const void *dy, const void *y, const float *scale, const void *w,
                              bool relu, void *ws, void *gf, const DzfLayout &layout, void *dres, const void **g_plain,
                              hipStream_t s);
// input gradient from a workspace prepared by launch_bwd_prepare
hipError_t launch_mfma_dgrad_prepared(const Geom &g, const void *g_plain, void *dx, bool accumulate, void *ws,
                                      hipStream_t s);

// ---- training-mode BatchNorm passes (bn_train.hip) ---------------------------------------------
size_t bn_fwd_scratch_bytes(int B, int C, int T);
size_t bn_bwd_scratch_bytes(int B, int C);
hipError_t launch_bn_fwd(int B, int C, int T, bool is_bf16, const void *z, const float *gamma, const float *beta, float eps,
                         const void *residual, bool relu, void *y, float *mean, float *invstd, void *scratch, hipStream_t s,
                         int given_parts = 0);
hipError_t launch_bn_bwd(int B, int C, int T, bool is_bf16, const void *dy, const void *y, const void *z, const float *gamma,
                         const float *mean, const float *invstd, bool relu, void *dz, void *dres, float *dgamma,
                         float *dbeta, bool accumulate, void *scratch, hipStream_t s);

}  // namespace nm
