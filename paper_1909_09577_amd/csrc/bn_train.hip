// Training-mode BatchNorm of the conv1d sub-block: batch statistics over (batch, time) of the stored
// pre-activation z, the normalise + affine + residual + ReLU pass, and the backward pass through the
// statistics (dgamma, dbeta and the corrected dz that the two convolution gradients then contract).
//
//   mean[c] = (1/N) sum z,  var[c] = (1/N) sum (z-mean)^2,  invstd = 1/sqrt(var+eps),  zhat = (z-mean)*invstd
//   y  = relu?( gamma*zhat + beta + residual )
//   g  = dy*[y>0];  dbeta = sum g;  dgamma = sum g*zhat;  dz = gamma*invstd*( g - dbeta/N - zhat*dgamma/N )
//
// All of these are bandwidth-bound passes over [B][C][T] tensors.  Sums are deterministic: every block
// owns one channel and a fixed subset of the batch items, reduces in a fixed tree (in double, so that
// var = M2/N does not cancel), and a one-thread-per-channel kernel combines the per-block results in a
// fixed order (block means and centred second moments, merged pairwise as in a streaming variance).
// Elements move in groups of VEC: 8 bf16 (16 bytes) when rows are 16-byte aligned, else one at a time.
#include "nm_common.h"

#include <initializer_list>

namespace nm {
namespace {

constexpr int kThreads = 256;

template <typename TS, int VEC>
struct Group {
    float v[VEC];
};
template <typename TS, int VEC>
__device__ __forceinline__ Group<TS, VEC> load_group(const TS *p, size_t group)
{
    Group<TS, VEC> r;
    if constexpr (VEC == 8) {
        const u32x4_t raw = reinterpret_cast<const u32x4_t *>(p)[group];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            r.v[2 * j] = __uint_as_float(raw[j] << 16);
            r.v[2 * j + 1] = __uint_as_float(raw[j] & 0xffff0000u);
        }
    } else {
        r.v[0] = load_as_f32(p, group);
    }
    return r;
}
template <typename TS, int VEC>
__device__ __forceinline__ void store_group(TS *p, size_t group, const Group<TS, VEC> &g)
{
    if constexpr (VEC == 8) {
        u32x4_t raw;
#pragma unroll
        for (int j = 0; j < 4; ++j) raw[j] = pack_bf16x2(g.v[2 * j], g.v[2 * j + 1]);
        reinterpret_cast<u32x4_t *>(p)[group] = raw;
    } else {
        store_from_f32(p, group, g.v[0]);
    }
}

// Sum of `a` and of `b` over the block, in a fixed tree, returned to thread 0.
__device__ __forceinline__ void block_sum2(double &a, double &b)
{
    __shared__ double red[2][kThreads];
    red[0][threadIdx.x] = a;
    red[1][threadIdx.x] = b;
    __syncthreads();
    for (int s = kThreads / 2; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) {
            red[0][threadIdx.x] += red[0][threadIdx.x + s];
            red[1][threadIdx.x] += red[1][threadIdx.x + s];
        }
        __syncthreads();
    }
    a = red[0][0];
    b = red[1][0];
}

// Block (c, g): batch items g, g+G, ... of channel c -> part[(g*C + c)*3] = {count, mean, centred second moment}.
template <typename TS, int VEC>
__global__ __launch_bounds__(kThreads) void bn_stats_kernel(const TS *__restrict__ z, int B, int C, int T, int G,
                                                            double *__restrict__ part)
{
    const int c = blockIdx.x, g = blockIdx.y;
    const int ng = T / VEC;
    float s1 = 0.f, s2 = 0.f;
    int rows = 0;
    for (int b = g; b < B; b += G, ++rows) {
        const size_t row = ((size_t)b * C + c) * ng;
        for (int i = threadIdx.x; i < ng; i += kThreads) {
            const Group<TS, VEC> v = load_group<TS, VEC>(z, row + i);
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                s1 += v.v[e];
                s2 = fmaf(v.v[e], v.v[e], s2);
            }
        }
    }
    double a = s1, q = s2;
    block_sum2(a, q);
    if (threadIdx.x == 0) {
        const double n = (double)rows * T;
        double *o = part + ((size_t)g * C + c) * 3;
        o[0] = n;
        o[1] = n > 0 ? a / n : 0.0;
        o[2] = n > 0 ? q - a * a / n : 0.0;
    }
}

// One wavefront per channel: lane l merges parts l, l+64, ... in order (Chan's update), then the lanes merge in a
// fixed tree; mean, invstd, and the affine they imply.
__global__ __launch_bounds__(64) void bn_finalize_kernel(const double *__restrict__ part, int G, int C,
                                                         const float *__restrict__ gamma, const float *__restrict__ beta,
                                                         float eps, float *__restrict__ mean, float *__restrict__ invstd,
                                                         float *__restrict__ scale, float *__restrict__ shift)
{
    const int c = blockIdx.x, lane = threadIdx.x;
    double n = 0.0, mu = 0.0, m2 = 0.0;
    auto merge = [&](double nb, double mb, double qb) {
        if (nb <= 0.0) return;
        const double delta = mb - mu, tot = n + nb;
        mu += delta * nb / tot;
        m2 += qb + delta * delta * n * nb / tot;
        n = tot;
    };
    for (int g = lane; g < G; g += 64) {
        const double *p = part + ((size_t)g * C + c) * 3;
        merge(p[0], p[1], p[2]);
    }
    for (int off = 32; off > 0; off >>= 1) {
        const double nb = __shfl_down(n, off, 64), mb = __shfl_down(mu, off, 64), qb = __shfl_down(m2, off, 64);
        if (lane < off) merge(nb, mb, qb);
    }
    if (lane != 0) return;
    const double var = n > 0 ? (m2 > 0 ? m2 / n : 0.0) : 0.0;
    const double is = 1.0 / sqrt(var + (double)eps);
    const double ga = gamma ? (double)gamma[c] : 1.0, be = beta ? (double)beta[c] : 0.0;
    mean[c] = (float)mu;
    invstd[c] = (float)is;
    scale[c] = (float)(ga * is);
    shift[c] = (float)(be - mu * ga * is);
}

// y = relu?(scale[c]*z + shift[c] + residual)
template <typename TS, int VEC>
__global__ __launch_bounds__(kThreads) void bn_apply_fwd_kernel(size_t ngroups, int C, int ng, const TS *__restrict__ z,
                                                                const float *__restrict__ scale,
                                                                const float *__restrict__ shift,
                                                                const TS *__restrict__ res, int relu, TS *__restrict__ y)
{
    const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= ngroups) return;
    const int c = (int)((i / (size_t)ng) % (size_t)C);
    const float sc = scale[c], sh = shift[c];
    const Group<TS, VEC> zv = load_group<TS, VEC>(z, i);
    Group<TS, VEC> out;
    if (res) {
        const Group<TS, VEC> rv = load_group<TS, VEC>(res, i);
#pragma unroll
        for (int e = 0; e < VEC; ++e) out.v[e] = fmaf(zv.v[e], sc, sh) + rv.v[e];
    } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) out.v[e] = fmaf(zv.v[e], sc, sh);
    }
    if (relu) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) out.v[e] = out.v[e] > 0.f ? out.v[e] : 0.f;
    }
    store_group<TS, VEC>(y, i, out);
}

// Block (c, g): part[(g*C + c)*2] = {sum g, sum g*zhat} over its batch items, g = dy*[y>0].
template <typename TS, int VEC>
__global__ __launch_bounds__(kThreads) void bn_bwd_stats_kernel(const TS *__restrict__ dy, const TS *__restrict__ y,
                                                                const TS *__restrict__ z, const float *__restrict__ mean,
                                                                const float *__restrict__ invstd, int relu, int B, int C,
                                                                int T, int G, double *__restrict__ part)
{
    const int c = blockIdx.x, g = blockIdx.y;
    const int ng = T / VEC;
    const float mu = mean[c], is = invstd[c];
    float s1 = 0.f, s2 = 0.f;
    for (int b = g; b < B; b += G) {
        const size_t row = ((size_t)b * C + c) * ng;
        for (int i = threadIdx.x; i < ng; i += kThreads) {
            const Group<TS, VEC> dv = load_group<TS, VEC>(dy, row + i);
            const Group<TS, VEC> zv = load_group<TS, VEC>(z, row + i);
            Group<TS, VEC> yv;
            if (relu) yv = load_group<TS, VEC>(y, row + i);
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const float gv = (!relu || yv.v[e] > 0.f) ? dv.v[e] : 0.f;
                s1 += gv;
                s2 = fmaf(gv, (zv.v[e] - mu) * is, s2);
            }
        }
    }
    double a = s1, q = s2;
    block_sum2(a, q);
    if (threadIdx.x == 0) {
        double *o = part + ((size_t)g * C + c) * 2;
        o[0] = a;
        o[1] = q;
    }
}

// One thread per channel: dbeta, dgamma (added to the old values when accumulating) and the three
// per-channel numbers the elementwise pass needs: coef[c] = {gamma*invstd, dbeta/N, dgamma/N}.
__global__ void bn_bwd_finalize_kernel(const double *__restrict__ part, int G, int C, double N,
                                       const float *__restrict__ gamma, const float *__restrict__ invstd,
                                       float *__restrict__ dgamma, float *__restrict__ dbeta, int accumulate,
                                       float *__restrict__ coef)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    double sb = 0.0, sg = 0.0;
    for (int g = 0; g < G; ++g) {
        sb += part[((size_t)g * C + c) * 2];
        sg += part[((size_t)g * C + c) * 2 + 1];
    }
    if (dbeta) dbeta[c] = accumulate ? dbeta[c] + (float)sb : (float)sb;
    if (dgamma) dgamma[c] = accumulate ? dgamma[c] + (float)sg : (float)sg;
    coef[3 * c] = (gamma ? gamma[c] : 1.f) * invstd[c];
    coef[3 * c + 1] = (float)(sb / N);
    coef[3 * c + 2] = (float)(sg / N);
}

// dz = coef0*(g - coef1 - zhat*coef2) in the storage type; dres = g (optional).
template <typename TS, int VEC>
__global__ __launch_bounds__(kThreads) void bn_bwd_apply_kernel(size_t ngroups, int C, int ng, const TS *__restrict__ dy,
                                                                const TS *__restrict__ y, const TS *__restrict__ z,
                                                                const float *__restrict__ mean,
                                                                const float *__restrict__ invstd,
                                                                const float *__restrict__ coef, int relu,
                                                                TS *__restrict__ dz, TS *__restrict__ dres)
{
    const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= ngroups) return;
    const int c = (int)((i / (size_t)ng) % (size_t)C);
    const float mu = mean[c], is = invstd[c];
    const float k0 = coef[3 * c], k1 = coef[3 * c + 1], k2 = coef[3 * c + 2];
    const Group<TS, VEC> dv = load_group<TS, VEC>(dy, i);
    const Group<TS, VEC> zv = load_group<TS, VEC>(z, i);
    Group<TS, VEC> yv, gout, zout;
    if (relu) yv = load_group<TS, VEC>(y, i);
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        const float gv = (!relu || yv.v[e] > 0.f) ? dv.v[e] : 0.f;
        gout.v[e] = gv;
        zout.v[e] = k0 * (gv - k1 - (zv.v[e] - mu) * is * k2);
    }
    store_group<TS, VEC>(dz, i, zout);
    if (dres) store_group<TS, VEC>(dres, i, gout);
}

int batch_groups(int B) { return B < 8 ? B : 8; }

bool vec8_ok(bool is_bf16, int T, std::initializer_list<const void *> ptrs)
{
    if (!is_bf16 || T % 8 != 0) return false;
    for (const void *p : ptrs)
        if (p && ((uintptr_t)p % 16) != 0) return false;
    return true;
}

// parts of a channel's statistics: the groups of batch items of bn_stats_kernel, or one per (batch item, 160-step
// time tile) when the convolution kernel writes them from its epilogue
size_t bn_parts_cap(int B, int T)
{
    const size_t tiles = (size_t)B * ((T + 159) / 160);
    return tiles > (size_t)batch_groups(B) ? tiles : (size_t)batch_groups(B);
}

}  // namespace

size_t bn_fwd_scratch_bytes(int B, int C, int T)
{
    return align_up(bn_parts_cap(B, T) * C * 3 * sizeof(double), 256) + 2 * align_up((size_t)C * sizeof(float), 256);
}

size_t bn_bwd_scratch_bytes(int B, int C)
{
    return align_up((size_t)batch_groups(B) * C * 2 * sizeof(double), 256) + align_up((size_t)3 * C * sizeof(float), 256);
}

// Statistics of z [B][C][T], then y = relu?(gamma*zhat + beta + residual).  scratch: bn_fwd_scratch_bytes.
hipError_t launch_bn_fwd(int B, int C, int T, bool is_bf16, const void *z, const float *gamma, const float *beta, float eps,
                         const void *residual, bool relu, void *y, float *mean, float *invstd, void *scratch, hipStream_t s,
                         int given_parts)
{
    // given_parts > 0: the part array already holds that many parts per channel (written by the convolution kernel)
    const int G = given_parts > 0 ? given_parts : batch_groups(B);
    double *part = (double *)scratch;
    float *scale = (float *)((unsigned char *)scratch + align_up(bn_parts_cap(B, T) * C * 3 * sizeof(double), 256));
    float *shift = (float *)((unsigned char *)scale + align_up((size_t)C * sizeof(float), 256));
    const bool v8 = vec8_ok(is_bf16, T, {z, residual, y});
    const dim3 sgrid(C, G);
    if (given_parts > 0)
        ;
    else if (v8)
        hipLaunchKernelGGL((bn_stats_kernel<bf16_t, 8>), sgrid, dim3(kThreads), 0, s, (const bf16_t *)z, B, C, T, G, part);
    else if (is_bf16)
        hipLaunchKernelGGL((bn_stats_kernel<bf16_t, 1>), sgrid, dim3(kThreads), 0, s, (const bf16_t *)z, B, C, T, G, part);
    else
        hipLaunchKernelGGL((bn_stats_kernel<float, 1>), sgrid, dim3(kThreads), 0, s, (const float *)z, B, C, T, G, part);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(bn_finalize_kernel, dim3(C), dim3(64), 0, s, part, G, C, gamma, beta, eps, mean, invstd, scale, shift);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int ng = v8 ? T / 8 : T;
    const size_t ngroups = (size_t)B * C * ng;
    const dim3 agrid((unsigned)((ngroups + kThreads - 1) / kThreads));
    if (v8)
        hipLaunchKernelGGL((bn_apply_fwd_kernel<bf16_t, 8>), agrid, dim3(kThreads), 0, s, ngroups, C, ng, (const bf16_t *)z,
                           scale, shift, (const bf16_t *)residual, relu ? 1 : 0, (bf16_t *)y);
    else if (is_bf16)
        hipLaunchKernelGGL((bn_apply_fwd_kernel<bf16_t, 1>), agrid, dim3(kThreads), 0, s, ngroups, C, ng, (const bf16_t *)z,
                           scale, shift, (const bf16_t *)residual, relu ? 1 : 0, (bf16_t *)y);
    else
        hipLaunchKernelGGL((bn_apply_fwd_kernel<float, 1>), agrid, dim3(kThreads), 0, s, ngroups, C, ng, (const float *)z,
                           scale, shift, (const float *)residual, relu ? 1 : 0, (float *)y);
    return hipGetLastError();
}

// dgamma, dbeta, dres and the corrected dz (storage type) from dy, the saved y and z and the saved statistics.
hipError_t launch_bn_bwd(int B, int C, int T, bool is_bf16, const void *dy, const void *y, const void *z, const float *gamma,
                         const float *mean, const float *invstd, bool relu, void *dz, void *dres, float *dgamma,
                         float *dbeta, bool accumulate, void *scratch, hipStream_t s)
{
    const int G = batch_groups(B);
    double *part = (double *)scratch;
    float *coef = (float *)((unsigned char *)scratch + align_up((size_t)G * C * 2 * sizeof(double), 256));
    const bool v8 = vec8_ok(is_bf16, T, {dy, y, z, dz, dres});
    const dim3 sgrid(C, G);
    if (v8)
        hipLaunchKernelGGL((bn_bwd_stats_kernel<bf16_t, 8>), sgrid, dim3(kThreads), 0, s, (const bf16_t *)dy, (const bf16_t *)y,
                           (const bf16_t *)z, mean, invstd, relu ? 1 : 0, B, C, T, G, part);
    else if (is_bf16)
        hipLaunchKernelGGL((bn_bwd_stats_kernel<bf16_t, 1>), sgrid, dim3(kThreads), 0, s, (const bf16_t *)dy, (const bf16_t *)y,
                           (const bf16_t *)z, mean, invstd, relu ? 1 : 0, B, C, T, G, part);
    else
        hipLaunchKernelGGL((bn_bwd_stats_kernel<float, 1>), sgrid, dim3(kThreads), 0, s, (const float *)dy, (const float *)y,
                           (const float *)z, mean, invstd, relu ? 1 : 0, B, C, T, G, part);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(bn_bwd_finalize_kernel, dim3((C + 127) / 128), dim3(128), 0, s, part, G, C, (double)B * T, gamma, invstd,
                       dgamma, dbeta, accumulate ? 1 : 0, coef);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int ng = v8 ? T / 8 : T;
    const size_t ngroups = (size_t)B * C * ng;
    const dim3 agrid((unsigned)((ngroups + kThreads - 1) / kThreads));
    if (v8)
        hipLaunchKernelGGL((bn_bwd_apply_kernel<bf16_t, 8>), agrid, dim3(kThreads), 0, s, ngroups, C, ng, (const bf16_t *)dy,
                           (const bf16_t *)y, (const bf16_t *)z, mean, invstd, coef, relu ? 1 : 0, (bf16_t *)dz, (bf16_t *)dres);
    else if (is_bf16)
        hipLaunchKernelGGL((bn_bwd_apply_kernel<bf16_t, 1>), agrid, dim3(kThreads), 0, s, ngroups, C, ng, (const bf16_t *)dy,
                           (const bf16_t *)y, (const bf16_t *)z, mean, invstd, coef, relu ? 1 : 0, (bf16_t *)dz, (bf16_t *)dres);
    else
        hipLaunchKernelGGL((bn_bwd_apply_kernel<float, 1>), agrid, dim3(kThreads), 0, s, ngroups, C, ng, (const float *)dy,
                           (const float *)y, (const float *)z, mean, invstd, coef, relu ? 1 : 0, (float *)dz, (float *)dres);
    return hipGetLastError();
}

}  // namespace nm
