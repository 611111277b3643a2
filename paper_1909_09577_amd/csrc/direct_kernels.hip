// Plain one-thread-per-output kernels for the conv1d sub-block (any stride, dilation,
// padding; float or bfloat16 storage; float32 arithmetic).  They serve the float32
// mode and every geometry the matrix-core kernels do not cover.  The sums are taken
// in short float32 blocks that are then added together, which keeps the rounding
// error of an n-term sum near sqrt(n)^(1/2) ulp instead of sqrt(n) ulp.
#include "nm_common.h"

namespace nm {
namespace {

constexpr int kThreads = 256;
constexpr int kChanPerThread = 4;  // output channels sharing one activation load
constexpr int kBlockChannels = 8;  // reduction channels per partial sum

// z = sum_ci sum_k w[co,ci,k] x[b,ci,t*stride-pad+k*dil]; then affine, residual, ReLU.
template <typename TS>
__global__ __launch_bounds__(kThreads) void direct_fwd_kernel(Geom g, const TS *__restrict__ x,
                                                              const TS *__restrict__ w,
                                                              const float *__restrict__ scale,
                                                              const float *__restrict__ shift,
                                                              const TS *__restrict__ res,
                                                              TS *__restrict__ y, int relu)
{
    const int t = blockIdx.x * kThreads + threadIdx.x;
    const int co0 = blockIdx.y * kChanPerThread;
    const int b = blockIdx.z;
    if (t >= g.To) return;
    const TS *xb = x + (size_t)b * g.Cin * g.T;
    const int tau0 = t * g.stride - g.pad;
    const int len = valid_len(g, b);
    float acc[kChanPerThread];
#pragma unroll
    for (int c = 0; c < kChanPerThread; ++c) acc[c] = 0.f;
    for (int ci0 = 0; ci0 < g.Cin; ci0 += kBlockChannels) {
        const int ci1 = min(ci0 + kBlockChannels, g.Cin);
        float part[kChanPerThread];
#pragma unroll
        for (int c = 0; c < kChanPerThread; ++c) part[c] = 0.f;
        for (int ci = ci0; ci < ci1; ++ci) {
            for (int k = 0; k < g.K; ++k) {
                const int tau = tau0 + k * g.dil;
                if (tau < 0 || tau >= len) continue;
                const float xv = load_as_f32(xb, (size_t)ci * g.T + tau);
#pragma unroll
                for (int c = 0; c < kChanPerThread; ++c) {
                    if (co0 + c < g.Cout)
                        part[c] = fmaf(load_as_f32(w, ((size_t)(co0 + c) * g.Cin + ci) * g.K + k), xv, part[c]);
                }
            }
        }
#pragma unroll
        for (int c = 0; c < kChanPerThread; ++c) acc[c] += part[c];
    }
#pragma unroll
    for (int c = 0; c < kChanPerThread; ++c) {
        const int co = co0 + c;
        if (co >= g.Cout) break;
        const size_t o = ((size_t)b * g.Cout + co) * g.To + t;
        float v = acc[c];
        if (scale) v *= scale[co];
        if (shift) v += shift[co];
        if (res) v += load_as_f32(res, o);
        if (relu) v = v > 0.f ? v : 0.f;
        store_from_f32(y, o, v);
    }
}

// dres = dy*[y>0];  dz = dres*scale[co]  (either output may be absent).
template <typename TS>
__global__ __launch_bounds__(kThreads) void epilogue_bwd_kernel(size_t n, int Cout, int To,
                                                                const TS *__restrict__ dy,
                                                                const TS *__restrict__ y,
                                                                const float *__restrict__ scale, int relu,
                                                                TS *__restrict__ dz, TS *__restrict__ dres)
{
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) {
        float gval = load_as_f32(dy, i);
        if (relu && !(load_as_f32(y, i) > 0.f)) gval = 0.f;
        if (dres) store_from_f32(dres, i, gval);
        if (dz) {
            const int co = (int)((i / (size_t)To) % (size_t)Cout);
            store_from_f32(dz, i, scale ? gval * scale[co] : gval);
        }
    }
}

// dx[b,ci,tau] = sum_co sum_k [ (tau+pad-k*dil) = t*stride, 0<=t<To ] w[co,ci,k] dz[b,co,t].
template <typename TS>
__global__ __launch_bounds__(kThreads) void direct_dgrad_kernel(Geom g, const TS *__restrict__ dz,
                                                                const TS *__restrict__ w,
                                                                TS *__restrict__ dx, int accumulate)
{
    const int tau = blockIdx.x * kThreads + threadIdx.x;
    const int ci0 = blockIdx.y * kChanPerThread;
    const int b = blockIdx.z;
    if (tau >= g.T) return;
    const TS *dzb = dz + (size_t)b * g.Cout * g.To;
    float acc[kChanPerThread];
#pragma unroll
    for (int c = 0; c < kChanPerThread; ++c) acc[c] = 0.f;
    for (int co0 = 0; co0 < g.Cout; co0 += kBlockChannels) {
        const int co1 = min(co0 + kBlockChannels, g.Cout);
        float part[kChanPerThread];
#pragma unroll
        for (int c = 0; c < kChanPerThread; ++c) part[c] = 0.f;
        for (int co = co0; co < co1; ++co) {
            for (int k = 0; k < g.K; ++k) {
                const int num = tau + g.pad - k * g.dil;
                if (num < 0) continue;
                const int t = num / g.stride;
                if (t * g.stride != num || t >= g.To) continue;
                const float gv = load_as_f32(dzb, (size_t)co * g.To + t);
#pragma unroll
                for (int c = 0; c < kChanPerThread; ++c) {
                    if (ci0 + c < g.Cin)
                        part[c] = fmaf(load_as_f32(w, ((size_t)co * g.Cin + ci0 + c) * g.K + k), gv, part[c]);
                }
            }
        }
#pragma unroll
        for (int c = 0; c < kChanPerThread; ++c) acc[c] += part[c];
    }
    const bool padding = tau >= valid_len(g, b);
#pragma unroll
    for (int c = 0; c < kChanPerThread; ++c) {
        if (ci0 + c >= g.Cin) break;
        const size_t o = ((size_t)b * g.Cin + ci0 + c) * g.T + tau;
        const float v = padding ? 0.f : acc[c];
        store_from_f32(dx, o, accumulate ? load_as_f32(dx, o) + v : v);
    }
}

// dw[co,ci,k] = sum_b sum_t dz[b,co,t] x[b,ci,t*stride-pad+k*dil]; one thread per (ci,k).
template <typename TS>
__global__ __launch_bounds__(kThreads) void direct_wgrad_kernel(Geom g, const TS *__restrict__ x,
                                                                const TS *__restrict__ dz,
                                                                const float *__restrict__ scale,
                                                                float *__restrict__ dw, int accumulate)
{
    const int n = blockIdx.x * kThreads + threadIdx.x;
    const int co = blockIdx.y;
    if (n >= g.Cin * g.K) return;
    const int ci = n / g.K;
    const int k = n - ci * g.K;
    const int off = k * g.dil - g.pad;
    // valid t: 0 <= t*stride + off < T
    int t_lo = 0;
    if (off < 0) t_lo = (-off + g.stride - 1) / g.stride;
    int t_hi = g.To;  // exclusive
    if (g.T - 1 - off < 0) t_hi = 0;
    else t_hi = min(g.To, (g.T - 1 - off) / g.stride + 1);
    float acc = 0.f;
    for (int b = 0; b < g.B; ++b) {
        const TS *dzr = dz + ((size_t)b * g.Cout + co) * g.To;
        const TS *xr = x + ((size_t)b * g.Cin + ci) * g.T;
        // with lengths: t*stride + off < len[b]
        const int len = valid_len(g, b);
        const int t_hi_b = len - 1 - off < 0 ? 0 : min(t_hi, (len - 1 - off) / g.stride + 1);
        for (int t0 = t_lo; t0 < t_hi_b; t0 += 64) {
            const int t1 = min(t0 + 64, t_hi_b);
            float part = 0.f;
            for (int t = t0; t < t1; ++t)
                part = fmaf(load_as_f32(dzr, t), load_as_f32(xr, (size_t)(t * g.stride + off)), part);
            acc += part;
        }
    }
    const size_t o = ((size_t)co * g.Cin + ci) * g.K + k;
    if (scale) acc *= scale[co];
    dw[o] = accumulate ? dw[o] + acc : acc;
}

// Vectorised form of epilogue_bwd_kernel for bf16 tensors whose rows are 16-byte aligned
// (To % 8 == 0): 8 elements per thread.
__global__ __launch_bounds__(kThreads) void epilogue_bwd_vec8_kernel(size_t n8, int Cout, int To8,
                                                                     const u32x4_t *__restrict__ dy,
                                                                     const u32x4_t *__restrict__ y,
                                                                     const float *__restrict__ scale, int relu,
                                                                     u32x4_t *__restrict__ dz,
                                                                     u32x4_t *__restrict__ dres)
{
    const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n8) epilogue_bwd_vec8_item(i, Cout, To8, dy, y, scale, relu, dz, dres);
}

template <typename TS>
hipError_t fwd_t(const Geom &g, const void *x, const void *w, const float *scale, const float *shift,
                 const void *res, void *y, bool relu, hipStream_t s)
{
    dim3 grid((g.To + kThreads - 1) / kThreads, (g.Cout + kChanPerThread - 1) / kChanPerThread, g.B);
    hipLaunchKernelGGL(direct_fwd_kernel<TS>, grid, dim3(kThreads), 0, s, g, (const TS *)x, (const TS *)w,
                       scale, shift, (const TS *)res, (TS *)y, relu ? 1 : 0);
    return hipGetLastError();
}

template <typename TS>
hipError_t dgrad_t(const Geom &g, const void *dz, const void *w, void *dx, bool accumulate, hipStream_t s)
{
    dim3 grid((g.T + kThreads - 1) / kThreads, (g.Cin + kChanPerThread - 1) / kChanPerThread, g.B);
    hipLaunchKernelGGL(direct_dgrad_kernel<TS>, grid, dim3(kThreads), 0, s, g, (const TS *)dz,
                       (const TS *)w, (TS *)dx, accumulate ? 1 : 0);
    return hipGetLastError();
}

template <typename TS>
hipError_t wgrad_t(const Geom &g, const void *x, const void *dz, const float *scale, float *dw, bool accumulate,
                   hipStream_t s)
{
    dim3 grid((g.Cin * g.K + kThreads - 1) / kThreads, g.Cout, 1);
    hipLaunchKernelGGL(direct_wgrad_kernel<TS>, grid, dim3(kThreads), 0, s, g, (const TS *)x,
                       (const TS *)dz, scale, dw, accumulate ? 1 : 0);
    return hipGetLastError();
}

template <typename TS>
hipError_t epi_t(const Geom &g, const void *dy, const void *y, const float *scale, bool relu, void *dz,
                 void *dres, hipStream_t s)
{
    const size_t n = (size_t)g.B * g.Cout * g.To;
    size_t blocks = (n + kThreads - 1) / kThreads;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(epilogue_bwd_kernel<TS>, dim3((unsigned)blocks), dim3(kThreads), 0, s, n, g.Cout,
                       g.To, (const TS *)dy, (const TS *)y, scale, relu ? 1 : 0, (TS *)dz, (TS *)dres);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_direct_fwd(const Geom &g, bool is_bf16, const void *x, const void *w, const float *scale,
                             const float *shift, const void *res, void *y, bool relu, hipStream_t s)
{
    return is_bf16 ? fwd_t<bf16_t>(g, x, w, scale, shift, res, y, relu, s)
                   : fwd_t<float>(g, x, w, scale, shift, res, y, relu, s);
}

hipError_t launch_epilogue_bwd(const Geom &g, bool is_bf16, const void *dy, const void *y,
                               const float *scale, bool relu, void *dz, void *dres, hipStream_t s)
{
    return is_bf16 ? epi_t<bf16_t>(g, dy, y, scale, relu, dz, dres, s)
                   : epi_t<float>(g, dy, y, scale, relu, dz, dres, s);
}

hipError_t launch_epilogue_bwd_vec8(const Geom &g, const void *dy, const void *y, const float *scale, bool relu,
                                    void *dz, void *dres, hipStream_t s)
{
    const size_t n8 = (size_t)g.B * g.Cout * g.To / 8;
    hipLaunchKernelGGL(epilogue_bwd_vec8_kernel, dim3((unsigned)((n8 + kThreads - 1) / kThreads)), dim3(kThreads), 0, s,
                       n8, g.Cout, g.To / 8, (const u32x4_t *)dy, (const u32x4_t *)y, scale, relu ? 1 : 0,
                       (u32x4_t *)dz, (u32x4_t *)dres);
    return hipGetLastError();
}

hipError_t launch_direct_dgrad(const Geom &g, bool is_bf16, const void *dz, const void *w, void *dx, bool accumulate,
                               hipStream_t s)
{
    return is_bf16 ? dgrad_t<bf16_t>(g, dz, w, dx, accumulate, s) : dgrad_t<float>(g, dz, w, dx, accumulate, s);
}

hipError_t launch_direct_wgrad(const Geom &g, bool is_bf16, const void *x, const void *dz, const float *scale, float *dw,
                               bool accumulate, hipStream_t s)
{
    return is_bf16 ? wgrad_t<bf16_t>(g, x, dz, scale, dw, accumulate, s)
                   : wgrad_t<float>(g, x, dz, scale, dw, accumulate, s);
}

}  // namespace nm
