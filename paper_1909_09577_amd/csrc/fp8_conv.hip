// Block forward on 8-bit floating-point (E4M3) operands: quantisation kernels, the matrix-core
// convolution kernel and the entry points declared in include/nm_conv1d_fp8.h.
//
//   q = E4M3(v * (1/s))  (float32 arithmetic, round to nearest even, saturating at +-448)
//   z[b,co,t] = sum_ci sum_k decode(wq[co,ci,k]) * decode(xq[b,ci,t - pad + k*dil])      (stride 1)
//   y = relu?( scale[co]*sx*sw[co]*z + shift[co] + residual )
//
// The contraction runs on v_mfma_f32_32x32x64_f8f6f4 (both operands E4M3, no block scaling): one
// instruction multiplies a 32x64 by a 64x32 tile, four times the work of the bfloat16 instruction at
// twice its rate.  Products of two E4M3 values have at most 8 significant bits and are exact in float32.
//
// Data layout chosen for this kernel (both tensors are written by the quantisation kernels below, so
// nothing has to follow the [B][C][T] order of the inputs):
//   * activations  xq[B][Cin/64][Tp][64]: time-major rows of 64 channels, Tp = 160*ceil(T_out/160) +
//     (K-1)*dil rows per (batch item, channel group), row r standing for input time r - pad; rows outside
//     [0, T) are zero.  The window of a chunk (all rows the K taps of a 160-step tile touch) is one
//     contiguous piece of memory, copied to LDS with 16-byte accesses and no shuffling, and every tap is
//     a row offset;
//   * weights  wq[Cout/64][Cin/64][K][2][64 lanes][32 B]: A fragments in register order, so a wavefront
//     reads 2 KiB contiguous per fragment straight from L2 into registers.
//
// Work decomposition: an output tile is 64 channels x 160 time steps of one batch item, held by one
// wavefront in ten 32x32 accumulators; a workgroup is four wavefronts that own four tiles of the same
// channel tile (so their weight loads hit L1) with private LDS windows -- no workgroup barrier anywhere.
// Wavefronts are persistent and run through their tiles with one pipeline: weight fragments live in
// 4 (+ K mod 4) register sets, each reloaded right after its last use with the tap that needs it
// next, four taps ahead, across chunk and tile boundaries; the window of the next chunk (or of the next
// tile's first chunk) is requested piece by piece during the current chunk and written to the other LDS
// buffer four taps later; a B fragment register is reloaded for the next tap right after the two
// MFMAs that read it.  A small last round of tiles is shared by the four wavefronts of a workgroup: each
// takes every fourth chunk of the tile and the partial tiles are summed through LDS in a fixed order.
#include "../../include/nm_conv1d.h"
#include "../../include/nm_conv1d_fp8.h"
#include "nm_common.h"

#include <type_traits>
#include <utility>

namespace nm {
namespace {

typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWaves = 4;
constexpr int kThreads = 64 * kWaves;
constexpr int kTileCo = 64;
constexpr int kNT = 5;                     // 32-step blocks per tile
constexpr int kTileT = 32 * kNT;           // 160
constexpr int kChunk = 64;                 // reduction channels per chunk = bytes of a window row
constexpr int kRowBytes = 80;              // LDS row: 64 B + 16 B pad
constexpr int kFragBytes = 64 * 32;        // one A fragment
constexpr int kTapBytes = 2 * kFragBytes;  // the two fragments (rows 0-31, 32-63) of one tap and chunk
constexpr int kAhead = 4;                  // taps between the request of a window piece and its LDS write
constexpr size_t kSlack = 8192;            // bytes behind each quantised tensor that prefetches may read
constexpr float kE4M3Max = 448.0f;

// ---------------------------------------------------------------------------------------------
// E4M3 conversion: round to nearest, ties to even, saturating at +-448.  The hardware conversion
// (v_cvt_pk_fp8_f32, two values per instruction) rounds to nearest even; the saturation is made explicit by
// clamping first.  Inputs are finite by contract (a NaN gives a NaN code).
__device__ __forceinline__ float clamp_e4m3(float v) { return __builtin_fminf(__builtin_fmaxf(v, -448.0f), 448.0f); }
// codes of a, b, c, d in bytes 0..3
__device__ __forceinline__ uint32_t e4m3_pack4(float a, float b, float c, float d)
{
    int r = __builtin_amdgcn_cvt_pk_fp8_f32(clamp_e4m3(a), clamp_e4m3(b), 0, false);
    r = __builtin_amdgcn_cvt_pk_fp8_f32(clamp_e4m3(c), clamp_e4m3(d), r, true);
    return (uint32_t)r;
}
__device__ __forceinline__ uint32_t f32_to_e4m3(float f) { return e4m3_pack4(f, 0.f, 0.f, 0.f) & 0xffu; }

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

__global__ __launch_bounds__(256) void fill_u32_kernel(uint32_t *p, int n, uint32_t v)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = v;
}

// amax[r] (as the bit pattern of a non-negative float, which orders like an unsigned integer)
__global__ __launch_bounds__(256) void row_amax_kernel(const bf16_t *__restrict__ x, size_t row_len, uint32_t *amax)
{
    const int r = blockIdx.y;
    const bf16_t *row = x + (size_t)r * row_len;
    float m = 0.f;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < row_len; i += (size_t)gridDim.x * 256)
        m = fmaxf(m, fabsf(bf16_to_f32(row[i])));
    m = wave_max(m);
    if ((threadIdx.x & 63) == 0) atomicMax(amax + r, __float_as_uint(m));
}

__global__ __launch_bounds__(256) void amax_to_scale_kernel(float *s, int n)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const float a = s[i];
    s[i] = a == 0.f ? 1.f : a / kE4M3Max;
}

__global__ __launch_bounds__(256) void quantize_rows_kernel(const bf16_t *__restrict__ x, size_t row_len, size_t total,
                                                            const float *__restrict__ scales, unsigned char *__restrict__ q)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const float inv = 1.0f / scales[i / row_len];
    q[i] = (unsigned char)f32_to_e4m3(bf16_to_f32(x[i]) * inv);
}

// x [B][Cin][T] bf16 -> xq[B][Cin/64][Tp][64] codes; row r stands for input time r - pad, zero outside [0,T).
// grid (ceil(Tp/64), Cin/64, B); thread (tl, cg): row blockIdx.x*64 + tl, channels 16*cg .. 16*cg+15.
__global__ __launch_bounds__(256) void quant_x_kernel(const bf16_t *__restrict__ x, const float *__restrict__ xs,
                                                      unsigned char *__restrict__ xq, int Cin, int T, int Tp, int pad)
{
    const int tl = threadIdx.x & 63, cg = threadIdx.x >> 6;
    const int r = blockIdx.x * 64 + tl;
    if (r >= Tp) return;
    const int c = blockIdx.y, b = blockIdx.z;
    const int t = r - pad;
    u32x4 out = {0u, 0u, 0u, 0u};
    if (t >= 0 && t < T) {
        const float inv = 1.0f / xs[0];
        const bf16_t *src = x + ((size_t)b * Cin + c * 64 + cg * 16) * T + t;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            out[j] = e4m3_pack4(bf16_to_f32(src[(size_t)(4 * j) * T]) * inv, bf16_to_f32(src[(size_t)(4 * j + 1) * T]) * inv,
                                bf16_to_f32(src[(size_t)(4 * j + 2) * T]) * inv, bf16_to_f32(src[(size_t)(4 * j + 3) * T]) * inv);
    }
    *reinterpret_cast<u32x4 *>(xq + (((size_t)b * gridDim.y + c) * Tp + r) * 64 + cg * 16) = out;
}

// The same for T % 8 == 0 and 16-byte aligned x: 16-byte loads along T, the transposition to time-major rows goes
// through LDS.  grid (ceil(T/128), Cin/64, B); a block converts 64 channels x 128 time steps.  Thread (g, tv) loads 8
// time steps of the four channels 4g..4g+3 and writes eight dwords (four channel codes of one time step each); then
// every thread copies 16-byte pieces of finished rows out.  The first and the last block of a row of blocks also
// write the zero rows before time 0 and behind time T.
constexpr int kQxT = 128;
__global__ __launch_bounds__(256) void quant_x_vec_kernel(const bf16_t *__restrict__ x, const float *__restrict__ xs,
                                                          unsigned char *__restrict__ xq, int Cin, int T, int Tp, int pad)
{
    __shared__ __align__(16) unsigned char tile[kQxT * kRowBytes];
    const int c = blockIdx.y, b = blockIdx.z, nck = gridDim.y;
    const int t0 = blockIdx.x * kQxT;
    const int g = threadIdx.x & 15, tv = threadIdx.x >> 4;
    const float inv = 1.0f / xs[0];
    const int t = t0 + tv * 8;
    if (t < T) {
        const bf16_t *src = x + ((size_t)b * Cin + c * 64 + g * 4) * T + t;
        u32x4 raw[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) raw[j] = *reinterpret_cast<const u32x4 *>(src + (size_t)j * T);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = bf16_to_f32((bf16_t)((raw[j][e >> 1] >> (16 * (e & 1))) & 0xffffu)) * inv;
            *reinterpret_cast<uint32_t *>(tile + (tv * 8 + e) * kRowBytes + g * 4) = e4m3_pack4(v[0], v[1], v[2], v[3]);
        }
    }
    __syncthreads();
    unsigned char *const slab = xq + ((size_t)b * nck + c) * Tp * 64;
    const int rows = min(kQxT, T - t0);
    for (int i = threadIdx.x; i < rows * 4; i += 256) {
        const int row = i >> 2, q = i & 3;
        *reinterpret_cast<u32x4 *>(slab + (size_t)(t0 + row + pad) * 64 + q * 16) =
            *reinterpret_cast<const u32x4 *>(tile + row * kRowBytes + q * 16);
    }
    const u32x4 zero = {0u, 0u, 0u, 0u};
    if (blockIdx.x == 0)
        for (int i = threadIdx.x; i < pad * 4; i += 256) *reinterpret_cast<u32x4 *>(slab + (size_t)i * 16) = zero;
    if (blockIdx.x == gridDim.x - 1)
        for (int i = threadIdx.x; i < (Tp - T - pad) * 4; i += 256)
            *reinterpret_cast<u32x4 *>(slab + (size_t)(T + pad) * 64 + (size_t)i * 16) = zero;
}

// w [Cout][Cin][K] bf16 -> wq[Cout/64][Cin/64][K][2][64][32] codes.  One block per (channel tile, chunk,
// row half): its 32 rows of 64*K weights are contiguous pieces of memory; they go through LDS as codes.
// Lane l of a fragment holds row l%32 and the 32 channels 32*(l/32) .. +31 of the chunk.
constexpr int kPackThreads = 1024;
__global__ __launch_bounds__(kPackThreads) void pack_w_kernel(const bf16_t *__restrict__ w, const float *__restrict__ wsc,
                                                              unsigned char *__restrict__ wq, int Cin, int K)
{
    extern __shared__ __align__(16) unsigned char codes[];  // [32][pitch]
    const int mi = blockIdx.x & 1, c = blockIdx.y, cot = blockIdx.z;
    const int nck = gridDim.y;
    const int rowlen = 64 * K;       // codes per row
    const int pitch = rowlen + 8;    // keeps the 8-byte writes aligned
    const int vec_per_row = rowlen / 8;
    const int nvec = 32 * vec_per_row;
    for (int base = 0; base < nvec; base += 4 * kPackThreads) {
        u32x4 raw[4];
        int row[4], col[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {  // four loads in flight
            const int v = base + u * kPackThreads + threadIdx.x;
            row[u] = v / vec_per_row;
            col[u] = v - row[u] * vec_per_row;
            if (v < nvec)
                raw[u] = *reinterpret_cast<const u32x4 *>(w + ((size_t)(cot * 64 + mi * 32 + row[u]) * Cin + c * 64) * K + col[u] * 8);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (base + u * kPackThreads + (int)threadIdx.x >= nvec) continue;
            const float inv = 1.0f / wsc[cot * 64 + mi * 32 + row[u]];
            float v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = bf16_to_f32((bf16_t)((raw[u][j >> 1] >> (16 * (j & 1))) & 0xffffu)) * inv;
            const u32x2 o = {e4m3_pack4(v[0], v[1], v[2], v[3]), e4m3_pack4(v[4], v[5], v[6], v[7])};
            *reinterpret_cast<u32x2 *>(codes + row[u] * pitch + col[u] * 8) = o;
        }
    }
    __syncthreads();
    for (int it = threadIdx.x; it < K * 64; it += kPackThreads) {
        const int k = it >> 6, lane = it & 63;
        const unsigned char *src = codes + (lane & 31) * pitch + (32 * (lane >> 5)) * K + k;
        u32x4 lo = {0u, 0u, 0u, 0u}, hi = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            lo[j >> 2] |= (uint32_t)src[j * K] << (8 * (j & 3));
            hi[j >> 2] |= (uint32_t)src[(16 + j) * K] << (8 * (j & 3));
        }
        u32x4 *dst = reinterpret_cast<u32x4 *>(wq + ((((size_t)(cot * nck + c) * K + k) * 2 + mi) * 64 + lane) * 32);
        dst[0] = lo;
        dst[1] = hi;
    }
}

// ---- operands of the input gradient ------------------------------------------------------------
// out[ci] = max over (co, k) of |w[co,ci,k]*scale[co]| / 448 (1 if that maximum is 0); one block per input channel
__global__ __launch_bounds__(256) void dgrad_wscale_kernel(const bf16_t *__restrict__ w, const float *__restrict__ scale,
                                                           float *__restrict__ out, int Cin, int Cout, int K)
{
    __shared__ float part[4];
    const int ci = blockIdx.x;
    float m = 0.f;
    for (int co = threadIdx.x; co < Cout; co += 256) {
        const float f = scale ? scale[co] : 1.f;
        const bf16_t *row = w + ((size_t)co * Cin + ci) * K;
        for (int k = 0; k < K; ++k) m = fmaxf(m, fabsf(bf16_to_f32(row[k]) * f));
    }
    m = wave_max(m);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        const float a = fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3]));
        out[ci] = a == 0.f ? 1.f : a / kE4M3Max;
    }
}

// g = dy*[y>0] -> codes in the time-major layout of the activations (row r stands for time r - pad), and g itself
// to dres when that is wanted.  Same structure as quant_x_vec_kernel; T % 8 == 0 and 16-byte aligned tensors.
__global__ __launch_bounds__(256) void quant_g_vec_kernel(const bf16_t *__restrict__ dy, const bf16_t *__restrict__ y,
                                                          const float *__restrict__ gs, unsigned char *__restrict__ gq,
                                                          bf16_t *__restrict__ dres, int C, int T, int Tp, int pad)
{
    __shared__ __align__(16) unsigned char tile[kQxT * kRowBytes];
    const int c = blockIdx.y, b = blockIdx.z, nck = gridDim.y;
    const int t0 = blockIdx.x * kQxT;
    const int g4 = threadIdx.x & 15, tv = threadIdx.x >> 4;
    const float inv = 1.0f / gs[0];
    const int t = t0 + tv * 8;
    if (t < T) {
        const size_t off = ((size_t)b * C + c * 64 + g4 * 4) * T + t;
        u32x4 raw[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) raw[j] = *reinterpret_cast<const u32x4 *>(dy + off + (size_t)j * T);
        if (y) {
#pragma unroll
            for (int j = 0; j < 4; ++j) raw[j] = masked_grad8(raw[j], *reinterpret_cast<const u32x4 *>(y + off + (size_t)j * T));
        }
        if (dres) {
#pragma unroll
            for (int j = 0; j < 4; ++j) *reinterpret_cast<u32x4 *>(dres + off + (size_t)j * T) = raw[j];
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = bf16_to_f32((bf16_t)((raw[j][e >> 1] >> (16 * (e & 1))) & 0xffffu)) * inv;
            *reinterpret_cast<uint32_t *>(tile + (tv * 8 + e) * kRowBytes + g4 * 4) = e4m3_pack4(v[0], v[1], v[2], v[3]);
        }
    }
    __syncthreads();
    unsigned char *const slab = gq + ((size_t)b * nck + c) * Tp * 64;
    const int rows = min(kQxT, T - t0);
    for (int i = threadIdx.x; i < rows * 4; i += 256) {
        const int row = i >> 2, q = i & 3;
        *reinterpret_cast<u32x4 *>(slab + (size_t)(t0 + row + pad) * 64 + q * 16) =
            *reinterpret_cast<const u32x4 *>(tile + row * kRowBytes + q * 16);
    }
    const u32x4 zero = {0u, 0u, 0u, 0u};
    if (blockIdx.x == 0)
        for (int i = threadIdx.x; i < pad * 4; i += 256) *reinterpret_cast<u32x4 *>(slab + (size_t)i * 16) = zero;
    if (blockIdx.x == gridDim.x - 1)
        for (int i = threadIdx.x; i < (Tp - T - pad) * 4; i += 256)
            *reinterpret_cast<u32x4 *>(slab + (size_t)(T + pad) * 64 + (size_t)i * 16) = zero;
}

// The same element by element (any T and alignment); grid (ceil(Tp/64), C/64, B) as quant_x_kernel.
__global__ __launch_bounds__(256) void quant_g_kernel(const bf16_t *__restrict__ dy, const bf16_t *__restrict__ y,
                                                      const float *__restrict__ gs, unsigned char *__restrict__ gq,
                                                      bf16_t *__restrict__ dres, int C, int T, int Tp, int pad)
{
    const int tl = threadIdx.x & 63, cg = threadIdx.x >> 6;
    const int r = blockIdx.x * 64 + tl;
    if (r >= Tp) return;
    const int c = blockIdx.y, b = blockIdx.z;
    const int t = r - pad;
    u32x4 out = {0u, 0u, 0u, 0u};
    if (t >= 0 && t < T) {
        const float inv = 1.0f / gs[0];
        const size_t off = ((size_t)b * C + c * 64 + cg * 16) * T + t;
        float v[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            bf16_t gb = dy[off + (size_t)j * T];
            if (y && !((uint32_t)y[off + (size_t)j * T] - 1u < 0x7f80u)) gb = 0;
            if (dres) dres[off + (size_t)j * T] = gb;
            v[j] = bf16_to_f32(gb) * inv;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) out[j] = e4m3_pack4(v[4 * j], v[4 * j + 1], v[4 * j + 2], v[4 * j + 3]);
    }
    *reinterpret_cast<u32x4 *>(gq + (((size_t)b * gridDim.y + c) * Tp + r) * 64 + cg * 16) = out;
}

// Weight operand of the input gradient: W'[ci][co][k'] = w[co][ci][K-1-k'] * scale[co], quantised with the scale of
// its row ci, in fragment order wtq[Cin/64][Cout/64][K][2][64][32].  One block per (input-channel tile, chunk of 64
// output channels, row half): for every output channel of the chunk the 32*K weights of the block's 32 input
// channels are one contiguous piece of memory; they go through LDS as codes [co][ci*K + k].
__global__ __launch_bounds__(kPackThreads) void pack_wt_kernel(const bf16_t *__restrict__ w, const float *__restrict__ scale,
                                                               const float *__restrict__ wts, unsigned char *__restrict__ wtq,
                                                               int Cin, int K)
{
    extern __shared__ __align__(16) unsigned char codes[];  // [64][pitch]
    const int mi = blockIdx.x & 1, c = blockIdx.y, cit = blockIdx.z;
    const int nck = gridDim.y;
    const int rowlen = 32 * K;       // codes per output channel
    const int pitch = rowlen + 8;
    const int vec_per_row = rowlen / 8;
    const int nvec = 64 * vec_per_row;
    const int ci0 = cit * 64 + mi * 32;
    for (int base = 0; base < nvec; base += 4 * kPackThreads) {
        u32x4 raw[4];
        int row[4], col[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int v = base + u * kPackThreads + threadIdx.x;
            row[u] = v / vec_per_row;
            col[u] = v - row[u] * vec_per_row;
            if (v < nvec) raw[u] = *reinterpret_cast<const u32x4 *>(w + ((size_t)(c * 64 + row[u]) * Cin + ci0) * K + col[u] * 8);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (base + u * kPackThreads + (int)threadIdx.x >= nvec) continue;
            const float f = scale ? scale[c * 64 + row[u]] : 1.f;
            float v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int e = col[u] * 8 + j;  // element (ci_l, k) = (e / K, e % K) of this output channel's piece
                const float inv = 1.0f / wts[ci0 + e / K];
                v[j] = (bf16_to_f32((bf16_t)((raw[u][j >> 1] >> (16 * (j & 1))) & 0xffffu)) * f) * inv;
            }
            const u32x2 o = {e4m3_pack4(v[0], v[1], v[2], v[3]), e4m3_pack4(v[4], v[5], v[6], v[7])};
            *reinterpret_cast<u32x2 *>(codes + row[u] * pitch + col[u] * 8) = o;
        }
    }
    __syncthreads();
    for (int it = threadIdx.x; it < K * 64; it += kPackThreads) {
        const int k = it >> 6, lane = it & 63;  // fragment of tap k' = k: row ci_l = lane % 32, output channels 32*(lane/32) .. +31
        const unsigned char *src = codes + (32 * (lane >> 5)) * pitch + (lane & 31) * K + (K - 1 - k);
        u32x4 lo = {0u, 0u, 0u, 0u}, hi = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            lo[j >> 2] |= (uint32_t)src[j * pitch] << (8 * (j & 3));
            hi[j >> 2] |= (uint32_t)src[(16 + j) * pitch] << (8 * (j & 3));
        }
        u32x4 *dst = reinterpret_cast<u32x4 *>(wtq + ((((size_t)(cit * nck + c) * K + k) * 2 + mi) * 64 + lane) * 32);
        dst[0] = lo;
        dst[1] = hi;
    }
}

// ---------------------------------------------------------------------------------------------
struct Fp8Params {
    int B, Cin, Cout, To, K;
    int ncot, nck, ntt, Tp;
    int nbt;     // B * ntt (batch item, time tile) pairs
    int ntiles;  // ncot * 4 * ceil(nbt / 4): tile ids, some of them empty when nbt % 4 != 0
    int priv_rounds;    // tiles below shared_first are private: wavefront w takes w, w + nwaves, ... (this many rounds)
    int shared_first;   // tiles from here on are shared by the four wavefronts of a workgroup (ntiles: none)
    int shared_rounds;  // ceil((ntiles - shared_first) / grid)
    int relu;
    int vec_io;  // T_out % 8 == 0 and y, residual 16-byte aligned: rows are read and written in 16-byte pieces
    const unsigned char *xq;
    const unsigned char *wq;
    const float *xs, *ws, *scale, *shift;
    const bf16_t *res;
    bf16_t *y;
};

struct TileCoords {
    int cot, b, tt;
    bool valid;
};
// tile ids are numbered so that four consecutive ids share the channel tile: id = (group*ncot + cot)*4 + j,
// (b, tt) pair number group*4 + j
__device__ __forceinline__ TileCoords decode_tile(const Fp8Params &p, int id)
{
    TileCoords c;
    const int q = id >> 2, j = id & 3;
    c.cot = q % p.ncot;
    const int bt = (q / p.ncot) * 4 + j;
    c.valid = id < p.ntiles && bt < p.nbt;
    c.b = bt / p.ntt;
    c.tt = bt - c.b * p.ntt;
    return c;
}

template <int N, typename F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl<N>(f, std::make_integer_sequence<int, N>{});
}

// The lane number, recomputed where it is needed (two ALU operations).
__device__ __forceinline__ int fresh_lane()
{
    int l = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    asm volatile("" : "+v"(l));
    return l;
}

__device__ __forceinline__ void wave_lds_fence()
{
    // LDS operations of one wavefront execute in order; this only keeps the compiler from moving LDS
    // accesses across the point where other lanes' data must be visible.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int KT, int DIL>
struct Plan {
    static constexpr int Q4 = (KT / 4) * 4, R = KT - Q4, NSETS = 4 + R;
    static constexpr int ROWS = kTileT + (KT - 1) * DIL;
    static constexpr int NIT = (ROWS * 4 + 63) / 64;  // 16-byte window pieces per lane
    static constexpr int BUF = NIT * 16 * kRowBytes;  // one LDS window buffer of a wavefront
    static constexpr int SPAN = KT - 1 - kAhead;      // taps over which the window requests are spread
    static_assert(SPAN >= 1, "too few taps for the staging schedule");
    static constexpr int XCH = 4 * 40 * 64 * 4;  // LDS for the exchange of partial tiles: 4 wavefronts x 40 floats per lane
    static constexpr bool kShared = kWaves * 2 * BUF + XCH <= 160 * 1024;
    static constexpr int LDS = kWaves * 2 * BUF + (kShared ? XCH : 0);
    static constexpr int set_of(int k) { return k < Q4 ? k % 4 : 4 + (k - Q4); }
    static constexpr int load_tap(int i) { return i * SPAN / NIT; }
};

template <int KT, int DIL>
__global__ __launch_bounds__(kThreads) void fp8_conv_kernel(const Fp8Params p)
{
    using P = Plan<KT, DIL>;
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wid = blockIdx.x * kWaves + wave;
    const int nwaves = gridDim.x * kWaves;
    unsigned char *const lds = smem + wave * (2 * P::BUF);
    const int n = lane & 31, h = lane >> 5;
    const int rd_lane = n * kRowBytes + 32 * h;                    // B fragment: row n, channels 32h..32h+31
    const int wr_lane = (lane >> 2) * kRowBytes + (lane & 3) * 16;  // window piece: row lane/4, quarter lane%4
    const size_t chunk_stride = (size_t)p.Tp * kChunk;              // bytes between the windows of consecutive chunks
    const size_t wchunk_bytes = (size_t)KT * kTapBytes;

    // base pointers are the same for all lanes (scalar registers); the lane's share is a 32-bit offset
    const uint32_t lane16 = lane * 16, lane32 = lane * 32;

    // ---- the wavefront's work items, in order: private tiles (sequence numbers below priv_rounds: tile
    // wid + s*nwaves, all chunks), then the workgroup's shared tiles (tile shared_first + blockIdx + j*grid: the
    // four wavefronts take chunks wave, wave+4, ... and sum their partial tiles through LDS).  Everything here
    // is the same for all lanes, and the list of shared tiles is the same for the four wavefronts of a workgroup.
    struct Item {
        TileCoords t;
        int c0, cs;
        bool shared;
        const unsigned char *x0, *w0;  // window and weights of the item's first chunk
    };
    const int nseq = p.priv_rounds + p.shared_rounds;
    auto item_at = [&](int sq, Item &it) -> bool {
        int id;
        if (sq < p.priv_rounds) {
            id = wid + sq * nwaves;
            if (id >= p.shared_first) return false;
            it.shared = false;
            it.c0 = 0;
            it.cs = 1;
        } else {
            id = p.shared_first + (int)blockIdx.x + (sq - p.priv_rounds) * (int)gridDim.x;
            if (id >= p.ntiles) return false;
            it.shared = true;
            it.c0 = wave;
            it.cs = kWaves;
        }
        it.t = decode_tile(p, id);
        if (!it.t.valid) return false;
        it.x0 = p.xq + (((size_t)it.t.b * p.nck + it.c0) * p.Tp + (size_t)it.t.tt * kTileT) * kChunk;
        it.w0 = p.wq + ((size_t)it.t.cot * p.nck + it.c0) * wchunk_bytes;
        return true;
    };
    auto next_item = [&](int from, Item &it) -> int {  // first sequence number >= from with an item, or nseq
        int sq = from;
        while (sq < nseq && !item_at(sq, it)) ++sq;
        return sq;
    };
    Item item;
    int seq = next_item(0, item);
    if (seq >= nseq) return;  // nothing to do (then the workgroup has no shared tile either)

    u32x4 stage[P::NIT];
    i32x8 aset[P::NSETS][2];
    i32x8 bfr[kNT];
    f32x16 acc[2][kNT];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int tb = 0; tb < kNT; ++tb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][tb][r] = 0.f;

    auto load_a = [&](i32x8(&dst)[2], const unsigned char *src) {
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) {
            const u32x4 lo = *reinterpret_cast<const u32x4 *>(src + lane32 + mi * kFragBytes);
            const u32x4 hi = *reinterpret_cast<const u32x4 *>(src + lane32 + mi * kFragBytes + 16);
            dst[mi] = i32x8{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
        }
    };
    auto load_b = [&](i32x8 &dst, const unsigned char *buf, int row_off) {
        const u32x4 lo = *reinterpret_cast<const u32x4 *>(buf + rd_lane + row_off * kRowBytes);
        const u32x4 hi = *reinterpret_cast<const u32x4 *>(buf + rd_lane + row_off * kRowBytes + 16);
        dst = i32x8{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
    };

    // ---- prologue: the first item's first window, weight sets and B fragments
    const unsigned char *xcur = item.x0;
    const unsigned char *wcur = item.w0;
    static_for<P::NIT>([&](auto ic) {
        constexpr int i = decltype(ic)::value;
        stage[i] = *reinterpret_cast<const u32x4 *>(xcur + lane16 + i * 1024);
    });
    static_for<P::NIT>([&](auto ic) {
        constexpr int i = decltype(ic)::value;
        *reinterpret_cast<u32x4 *>(lds + wr_lane + i * 16 * kRowBytes) = stage[i];
    });
    static_for<KT>([&](auto kc) {
        constexpr int k = decltype(kc)::value;
        if constexpr (k < 4 || k >= P::Q4) load_a(aset[P::set_of(k)], wcur + k * kTapBytes);
    });
    wave_lds_fence();
    static_for<kNT>([&](auto tc5) {
        constexpr int tb = decltype(tc5)::value;
        load_b(bfr[tb], lds, tb * 32);
    });
    int cur = 0;  // LDS buffer that holds the current chunk's window

    for (;;) {
        // the item after this one (if any) supplies the "next chunk" of this item's last chunk
        Item nxt;
        const int nseq_next = next_item(seq + 1, nxt);
        const bool has_next = nseq_next < nseq;
        const unsigned char *xnext_item = has_next ? nxt.x0 : item.x0;
        const unsigned char *wnext_item = has_next ? nxt.w0 : item.w0;
        const TileCoords tc = item.t;

        for (int c = item.c0; c < p.nck; c += item.cs) {
            const bool last = c + item.cs >= p.nck;
            const unsigned char *xnxt = last ? xnext_item : xcur + item.cs * chunk_stride;
            const unsigned char *wnxt = last ? wnext_item : wcur + item.cs * wchunk_bytes;
            unsigned char *const bcur = lds + cur * P::BUF;
            unsigned char *const bnxt = lds + (cur ^ 1) * P::BUF;

            static_for<KT>([&](auto kc) {
                constexpr int k = decltype(kc)::value;
                // window of the next chunk: request pieces, write the ones requested kAhead taps ago
                static_for<P::NIT>([&](auto ic) {
                    constexpr int i = decltype(ic)::value;
                    if constexpr (P::load_tap(i) == k) stage[i] = *reinterpret_cast<const u32x4 *>(xnxt + lane16 + i * 1024);
                });
                static_for<P::NIT>([&](auto ic) {
                    constexpr int i = decltype(ic)::value;
                    if constexpr (P::load_tap(i) + kAhead == k)
                        *reinterpret_cast<u32x4 *>(bnxt + wr_lane + i * 16 * kRowBytes) = stage[i];
                });
                if constexpr (k == KT - 1) wave_lds_fence();  // the next window is complete before its first rows are read
                __builtin_amdgcn_sched_barrier(0);
                constexpr int s = P::set_of(k);
                static_for<kNT>([&](auto tc5) {
                    constexpr int tb = decltype(tc5)::value;
                    acc[0][tb] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(aset[s][0], bfr[tb], acc[0][tb], 0, 0, 0, 0, 0, 0);
                    acc[1][tb] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(aset[s][1], bfr[tb], acc[1][tb], 0, 0, 0, 0, 0, 0);
                    if constexpr (k + 1 < KT)
                        load_b(bfr[tb], bcur, tb * 32 + (k + 1) * DIL);
                    else
                        load_b(bfr[tb], bnxt, tb * 32);
                    __builtin_amdgcn_sched_barrier(0);  // keep the reload here: the scheduler would sink it to its use
                });
                // this tap's weight set is free: fetch the tap that uses it next
                if constexpr (k + 4 < P::Q4)
                    load_a(aset[s], wcur + (k + 4) * kTapBytes);
                else if constexpr (k < P::Q4)
                    load_a(aset[s], wnxt + (k % 4) * kTapBytes);
                else
                    load_a(aset[s], wnxt + k * kTapBytes);
                __builtin_amdgcn_sched_barrier(0);
            });
            xcur = xnxt;
            wcur = wnxt;
            cur ^= 1;
        }

        // ---- a shared tile: the four partial tiles are summed in four rounds, one quarter (16 channels: block row
        // mi = q/2, registers 8*(q%2) .. +7 of every time block) per round -- the other three wavefronts park their
        // 40 values per lane in LDS and wavefront q adds them in a fixed order, position by position.
        if constexpr (P::kShared) {
            if (item.shared) {
                const int l = fresh_lane();
                float *const xch = reinterpret_cast<float *>(smem + kWaves * 2 * P::BUF);
                static_for<4>([&](auto qc) {
                    constexpr int q = decltype(qc)::value, mi = q / 2, r0 = 8 * (q % 2);
                    if (wave != q) {
#pragma unroll
                        for (int rr = 0; rr < 8; ++rr)
#pragma unroll
                            for (int tb = 0; tb < kNT; ++tb) xch[((wave * 40) + rr * kNT + tb) * 64 + l] = acc[mi][tb][r0 + rr];
                    }
                    __syncthreads();
                    if (wave == q) {
                        static_for<4>([&](auto wc) {
                            constexpr int w2 = decltype(wc)::value;
                            if constexpr (w2 != q) {
                                float part[8 * kNT];  // all reads of one partial tile first, then the additions
#pragma unroll
                                for (int e = 0; e < 8 * kNT; ++e) part[e] = xch[((w2 * 40) + e) * 64 + l];
                                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                                for (int rr = 0; rr < 8; ++rr)
#pragma unroll
                                    for (int tb = 0; tb < kNT; ++tb) acc[mi][tb][r0 + rr] += part[rr * kNT + tb];
                                __builtin_amdgcn_sched_barrier(0);
                            }
                        });
                    }
                    __syncthreads();
                });
            }
        }

        // ---- epilogue: register r of block (mi, tb) is channel cot*64 + mi*32 + 8*(r/4) + 4*h + r%4, time tt*160 + tb*32 + n.
        // The tile leaves in quarters of 16 channels (all four for a private tile, quarter `wave` for a shared one): every
        // lane writes the float32 values scale*acc + shift of the 40 elements it owns to a [16][160] LDS tile, then each
        // lane takes 8 consecutive time steps of a row (two 16-byte LDS reads), adds the residual (one 16-byte load,
        // requested a quarter ahead), applies the ReLU, rounds and stores 16 bytes.  The LDS tile is the window of this
        // item's last chunk, which is dead (the other buffer holds the next item's first window).
        {
            // lane-dependent values are recomputed here: kept alive across the main loop they would be spilled, and
            // the reload of a spilled value waits for every memory operation in flight
            const int lane = fresh_lane();
            const int n = lane & 31, h = lane >> 5;
            const float sx = p.xs[0];
            unsigned char *const ebuf = smem + wave * (2 * P::BUF) + (cur ^ 1) * P::BUF;
            constexpr int kQPitch = kTileT * 4 + 16;
            static_assert(16 * kQPitch + 512 <= P::BUF, "the epilogue tile must fit a window buffer");
            constexpr int kVecPerRow = kTileT / 8, kVec = 16 * kVecPerRow / 64;  // 20 per row, 5 per lane
            // per-row factor and shift of the tile's 64 channels: one load per lane, parked behind the tile
            float *const rowf = reinterpret_cast<float *>(ebuf + 16 * kQPitch);
            {
                const int co = tc.cot * kTileCo + lane;
                rowf[lane] = (p.scale ? p.scale[co] : 1.f) * (sx * p.ws[co]);
                rowf[64 + lane] = p.shift ? p.shift[co] : 0.f;
            }
            const bool vec_res = p.res && p.vec_io;
            u32x4 rv[2][kVec];
            auto load_residual = [&](u32x4(&dst)[kVec], int q) {
#pragma unroll
                for (int j = 0; j < kVec; ++j) {
                    const int idx = j * 64 + lane, row = idx / kVecPerRow, col = idx - row * kVecPerRow;
                    const int t = tc.tt * kTileT + col * 8;
                    const size_t off = ((size_t)tc.b * p.Cout + tc.cot * kTileCo + q * 16 + row) * p.To + t;
                    dst[j] = t < p.To ? *reinterpret_cast<const u32x4 *>(p.res + off) : u32x4{0u, 0u, 0u, 0u};
                }
            };
            wave_lds_fence();
            // one quarter; LOAD_OWN: request its residual first, LOAD_NEXT: request the next quarter's in the middle
            auto quarter = [&](auto qc, auto load_own, auto load_next) {
                constexpr int q = decltype(qc)::value, mi = q / 2, r0 = 8 * (q % 2);
                if constexpr (decltype(load_own)::value) {
                    if (vec_res) load_residual(rv[q & 1], q);
                }
                f32x4 e4[2], s4[2];
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    e4[j] = *reinterpret_cast<const f32x4 *>(rowf + q * 16 + 8 * j + 4 * h);
                    s4[j] = *reinterpret_cast<const f32x4 *>(rowf + 64 + q * 16 + 8 * j + 4 * h);
                }
#pragma unroll
                for (int rr = 0; rr < 8; ++rr) {
                    const int j = rr >> 2, i = rr & 3, rl = 8 * j + 4 * h + i;
#pragma unroll
                    for (int tb = 0; tb < kNT; ++tb)
                        *reinterpret_cast<float *>(ebuf + rl * kQPitch + (tb * 32 + n) * 4) = acc[mi][tb][r0 + rr] * e4[j][i] + s4[j][i];
                }
                if constexpr (decltype(load_next)::value) {
                    if (vec_res) load_residual(rv[(q + 1) & 1], q + 1);
                }
                wave_lds_fence();
                if (p.vec_io) {
                    // all LDS reads first, then the arithmetic and the stores: with the reads inside the loop every
                    // piece would wait for its own LDS round trip
                    f32x4 lo[kVec], hi[kVec];
#pragma unroll
                    for (int j = 0; j < kVec; ++j) {
                        const int idx = j * 64 + lane, row = idx / kVecPerRow, col = idx - row * kVecPerRow;
                        lo[j] = *reinterpret_cast<const f32x4 *>(ebuf + row * kQPitch + col * 32);
                        hi[j] = *reinterpret_cast<const f32x4 *>(ebuf + row * kQPitch + col * 32 + 16);
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int j = 0; j < kVec; ++j) {
                        const int idx = j * 64 + lane, row = idx / kVecPerRow, col = idx - row * kVecPerRow;
                        const int t = tc.tt * kTileT + col * 8;
                        float v[8] = {lo[j][0], lo[j][1], lo[j][2], lo[j][3], hi[j][0], hi[j][1], hi[j][2], hi[j][3]};
                        const size_t off = ((size_t)tc.b * p.Cout + tc.cot * kTileCo + q * 16 + row) * p.To + t;
                        if (t < p.To) {
                            if (p.res) {
#pragma unroll
                                for (int e = 0; e < 8; ++e)
                                    v[e] += bf16_to_f32((bf16_t)((rv[q & 1][j][e >> 1] >> (16 * (e & 1))) & 0xffffu));
                            }
                            if (p.relu) {
#pragma unroll
                                for (int e = 0; e < 8; ++e) v[e] = fmaxf(v[e], 0.f);
                            }
                            const u32x4 o = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]),
                                             pack_bf16x2(v[6], v[7])};
                            *reinterpret_cast<u32x4 *>(p.y + off) = o;
                        }
                    }
                } else {  // rows that are not 16-byte pieces: element by element
                    for (int j = 0; j < kVec; ++j) {
                        const int idx = j * 64 + lane, row = idx / kVecPerRow, col = idx - row * kVecPerRow;
                        const int t = tc.tt * kTileT + col * 8;
                        const float *v = reinterpret_cast<const float *>(ebuf + row * kQPitch + col * 32);
                        const size_t off = ((size_t)tc.b * p.Cout + tc.cot * kTileCo + q * 16 + row) * p.To + t;
                        for (int e = 0; e < 8; ++e) {
                            if (t + e < p.To) {
                                float u = v[e];
                                if (p.res) u += bf16_to_f32(p.res[off + e]);
                                if (p.relu) u = fmaxf(u, 0.f);
                                p.y[off + e] = f32_to_bf16(u);
                            }
                        }
                    }
                }
                wave_lds_fence();
            };
            using T = std::true_type;
            using F = std::false_type;
            using std::integral_constant;
            if (!item.shared) {
                quarter(integral_constant<int, 0>{}, T{}, T{});
                quarter(integral_constant<int, 1>{}, F{}, T{});
                quarter(integral_constant<int, 2>{}, F{}, T{});
                quarter(integral_constant<int, 3>{}, F{}, F{});
            } else if (wave == 0) {
                quarter(integral_constant<int, 0>{}, T{}, F{});
            } else if (wave == 1) {
                quarter(integral_constant<int, 1>{}, T{}, F{});
            } else if (wave == 2) {
                quarter(integral_constant<int, 2>{}, T{}, F{});
            } else {
                quarter(integral_constant<int, 3>{}, T{}, F{});
            }
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int tb = 0; tb < kNT; ++tb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[mi][tb][r] = 0.f;
        }
        if (!has_next) break;
        seq = nseq_next;
        item = nxt;
        // The weight sets and B fragments of the next item's first taps are fetched again here rather than kept
        // across the epilogue (120 registers that the epilogue needs; the window itself stays in LDS).
        static_for<KT>([&](auto kc) {
            constexpr int k = decltype(kc)::value;
            if constexpr (k < 4 || k >= P::Q4) load_a(aset[P::set_of(k)], wcur + k * kTapBytes);
        });
        {
            const unsigned char *const bfirst = lds + cur * P::BUF;
            static_for<kNT>([&](auto tc5) {
                constexpr int tb = decltype(tc5)::value;
                load_b(bfr[tb], bfirst, tb * 32);
            });
        }
    }
}

template <int KT, int DIL>
hipError_t launch_fp8_conv(Fp8Params p, hipStream_t s)
{
    using P = Plan<KT, DIL>;
    static LdsOptIn opt_in;
    static_assert(P::LDS <= 160 * 1024, "LDS windows exceed the CU");
    hipError_t e = ensure_dynamic_lds(opt_in, reinterpret_cast<const void *>(fp8_conv_kernel<KT, DIL>), P::LDS);
    if (e != hipSuccess) return e;
    // Tiles are dealt in rounds of one per wavefront.  A last partial round of at most two tiles per workgroup is
    // run in shared form (four wavefronts per tile, a quarter of the reduction each) so that the chip stays full;
    // a larger remainder is cheaper as one more private round.
    const int G = current_device_info().cus, nw_max = G * kWaves;
    const bool can_share = P::kShared && p.nck >= kWaves;
    int grid;
    if (p.ntiles >= nw_max) {
        grid = G;
        const int full = p.ntiles / nw_max, rem = p.ntiles - full * nw_max;
        const bool share = can_share && rem <= 2 * G;
        p.priv_rounds = share ? full : full + (rem > 0 ? 1 : 0);
        p.shared_first = share ? full * nw_max : p.ntiles;
    } else if (can_share && p.ntiles <= 2 * G) {
        grid = min(G, p.ntiles);
        p.priv_rounds = 0;
        p.shared_first = 0;
    } else {
        grid = (p.ntiles + kWaves - 1) / kWaves;
        p.priv_rounds = 1;
        p.shared_first = p.ntiles;
    }
    p.shared_rounds = (p.ntiles - p.shared_first + grid - 1) / grid;
    MainKernelTimer timer(s);
    hipLaunchKernelGGL((fp8_conv_kernel<KT, DIL>), dim3(grid), dim3(kThreads), P::LDS, s, p);
    return hipGetLastError();
}

bool taps_supported(int K, int dil)
{
    return (dil == 1 && (K == 17 || K == 21 || K == 25)) || (dil == 2 && K == 29);
}

struct Fp8Layout {
    int ncot, nck, ntt, Tp;
    size_t xq_bytes, wq_bytes, total;
};
Fp8Layout fp8_layout(int B, int Cin, int Cout, int To, int K, int dil)
{
    Fp8Layout l;
    l.ncot = Cout / kTileCo;
    l.nck = Cin / kChunk;
    l.ntt = (To + kTileT - 1) / kTileT;
    l.Tp = l.ntt * kTileT + (K - 1) * dil;
    l.xq_bytes = align_up((size_t)B * l.nck * l.Tp * kChunk + kSlack, 256);
    l.wq_bytes = align_up((size_t)l.ncot * l.nck * K * kTapBytes + kSlack, 256);
    l.total = l.xq_bytes + l.wq_bytes;
    return l;
}

int fp8_check(int B, int Cin, int Cout, int T, int K, int stride, int dil, int pad, int *To)
{
    if (B <= 0 || Cin <= 0 || Cout <= 0 || T <= 0 || K <= 0 || stride <= 0 || dil <= 0 || pad < 0) return NM_ERR_BAD_ARG;
    const long long span = (long long)T + 2LL * pad - (long long)dil * (K - 1) - 1;
    if (span < 0) return NM_ERR_BAD_ARG;
    const long long to = span / stride + 1;
    if (to > (1LL << 31) - 1) return NM_ERR_BAD_ARG;
    *To = (int)to;
    if (stride != 1 || Cin % kChunk || Cout % kTileCo || !taps_supported(K, dil)) return NM_ERR_UNSUPPORTED;
    if (pad > (K - 1) * dil) return NM_ERR_UNSUPPORTED;  // rows of xq before time 0 are the left padding only
    if ((long long)B * Cin * T > (1LL << 31) - 1 || (long long)B * Cout * to > (1LL << 31) - 1 ||
        (long long)Cout * Cin * K > (1LL << 31) - 1 || B > 65535)
        return NM_ERR_UNSUPPORTED;
    const Fp8Layout l = fp8_layout(B, Cin, Cout, (int)to, K, dil);
    if (l.xq_bytes > (1ull << 31) || l.wq_bytes > (1ull << 31)) return NM_ERR_UNSUPPORTED;
    return NM_OK;
}

bool overlap(const void *a, size_t na, const void *b, size_t nb)
{
    if (!a || !b) return false;
    const char *pa = (const char *)a, *pb = (const char *)b;
    return pa < pb + nb && pb < pa + na;
}

}  // namespace

// ---- quantisation passes shared with the weight-gradient kernel (fp8_wgrad.hip) ------------------
bool fp8_taps_supported(int K, int dil) { return taps_supported(K, dil); }

// x [B][C][T] -> codes [B][C/64][Tp][64], row r standing for time r - pad, zero rows elsewhere
hipError_t fp8_launch_quant_x(const void *x, const float *xs, unsigned char *xq, int B, int C, int T, int Tp, int pad,
                              hipStream_t s)
{
    if (T % 8 == 0 && !((uintptr_t)x & 15))
        hipLaunchKernelGGL(quant_x_vec_kernel, dim3((T + kQxT - 1) / kQxT, C / 64, B), dim3(256), 0, s, (const bf16_t *)x, xs, xq,
                           C, T, Tp, pad);
    else
        hipLaunchKernelGGL(quant_x_kernel, dim3((Tp + 63) / 64, C / 64, B), dim3(256), 0, s, (const bf16_t *)x, xs, xq, C, T, Tp,
                           pad);
    return hipGetLastError();
}

// g = dy*[y>0] (y NULL: dy) -> codes in the same layout; g itself to dres when that is given
hipError_t fp8_launch_quant_g(const void *dy, const void *y, const float *gs, unsigned char *gq, void *dres, int B, int C,
                              int T, int Tp, int pad, hipStream_t s)
{
    const bool vec = T % 8 == 0 && !((uintptr_t)dy & 15) && !((uintptr_t)y & 15) && !((uintptr_t)dres & 15);
    if (vec)
        hipLaunchKernelGGL(quant_g_vec_kernel, dim3((T + kQxT - 1) / kQxT, C / 64, B), dim3(256), 0, s, (const bf16_t *)dy,
                           (const bf16_t *)y, gs, gq, (bf16_t *)dres, C, T, Tp, pad);
    else
        hipLaunchKernelGGL(quant_g_kernel, dim3((Tp + 63) / 64, C / 64, B), dim3(256), 0, s, (const bf16_t *)dy, (const bf16_t *)y,
                           gs, gq, (bf16_t *)dres, C, T, Tp, pad);
    return hipGetLastError();
}

// Input gradient behind the quantisation of g: packs the flipped, scale-folded weights (quantised per input
// channel) into wtq and runs the matrix-core kernel on the codes gq (time-major, Tp rows per batch item and
// 64-channel group, row r standing for output time r - (dil*(K-1) - pad)).
hipError_t fp8_dgrad_run(int B, int Cin, int Cout, int T, int K, int dil, const unsigned char *gq, int Tp, const float *g_scale,
                         const void *w, const float *scale, const float *wt_scales, void *dx, unsigned char *wtq, hipStream_t s)
{
    const int ncit = Cin / kTileCo, nck = Cout / kChunk, ntt = (T + kTileT - 1) / kTileT;
    hipLaunchKernelGGL(pack_wt_kernel, dim3(2, nck, ncit), dim3(kPackThreads), (size_t)64 * (32 * K + 8), s, (const bf16_t *)w,
                       scale, wt_scales, wtq, Cin, K);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    Fp8Params p;
    p.B = B; p.Cin = Cout; p.Cout = Cin; p.To = T; p.K = K;
    p.ncot = ncit; p.nck = nck; p.ntt = ntt; p.Tp = Tp;
    p.nbt = B * ntt;
    p.ntiles = ncit * 4 * ((p.nbt + 3) / 4);
    p.relu = 0;
    p.vec_io = (T % 8 == 0 && !((uintptr_t)dx & 15)) ? 1 : 0;
    p.xq = gq; p.wq = wtq;
    p.xs = g_scale; p.ws = wt_scales; p.scale = nullptr; p.shift = nullptr;
    p.res = nullptr;
    p.y = (bf16_t *)dx;
    if (dil == 2) return launch_fp8_conv<29, 2>(p, s);
    if (K == 17) return launch_fp8_conv<17, 1>(p, s);
    if (K == 21) return launch_fp8_conv<21, 1>(p, s);
    return launch_fp8_conv<25, 1>(p, s);
}
// bytes of the packed weight operand (either direction) including the slack prefetches may read
size_t fp8_packed_weight_bytes(int Cin, int Cout, int K)
{
    return align_up((size_t)(Cout / kTileCo) * (Cin / kChunk) * K * kTapBytes + kSlack, 256);
}

}  // namespace nm

using namespace nm;

extern "C" int nm_fp8_row_scales(const void *x, int rows, size_t row_len, float *scales, void *hip_stream)
{
    if (!x || !scales || rows <= 0 || row_len == 0) return NM_ERR_BAD_ARG;
    if ((unsigned long long)rows * row_len > (1ull << 31) - 1 || rows > 65535) return NM_ERR_UNSUPPORTED;
    hipStream_t s = (hipStream_t)hip_stream;
    hipLaunchKernelGGL(fill_u32_kernel, dim3((rows + 255) / 256), dim3(256), 0, s, reinterpret_cast<uint32_t *>(scales), rows, 0u);
    const int bx = (int)std::min<size_t>((row_len + 2047) / 2048, 1024);
    hipLaunchKernelGGL(row_amax_kernel, dim3(bx, rows), dim3(256), 0, s, (const bf16_t *)x, row_len,
                       reinterpret_cast<uint32_t *>(scales));
    hipLaunchKernelGGL(amax_to_scale_kernel, dim3((rows + 255) / 256), dim3(256), 0, s, scales, rows);
    return hipGetLastError() == hipSuccess ? NM_OK : NM_ERR_DEVICE;
}

extern "C" int nm_fp8_quantize_rows(const void *x, int rows, size_t row_len, const float *scales, unsigned char *codes,
                                    void *hip_stream)
{
    if (!x || !scales || !codes || rows <= 0 || row_len == 0) return NM_ERR_BAD_ARG;
    if ((unsigned long long)rows * row_len > (1ull << 31) - 1) return NM_ERR_UNSUPPORTED;
    const size_t total = (size_t)rows * row_len;
    if (overlap(x, total * 2, codes, total)) return NM_ERR_BAD_ARG;
    hipLaunchKernelGGL(quantize_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, (hipStream_t)hip_stream,
                       (const bf16_t *)x, row_len, total, scales, codes);
    return hipGetLastError() == hipSuccess ? NM_OK : NM_ERR_DEVICE;
}

extern "C" int nm_conv1d_fp8_supported(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad)
{
    int To = 0;
    return fp8_check(B, Cin, Cout, T, K, stride, dilation, pad, &To) == NM_OK ? 1 : 0;
}

extern "C" size_t nm_conv1d_fp8_workspace_bytes(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad)
{
    int To = 0;
    if (fp8_check(B, Cin, Cout, T, K, stride, dilation, pad, &To) != NM_OK) return 0;
    return fp8_layout(B, Cin, Cout, To, K, dilation).total;
}

extern "C" int nm_conv1d_block_fwd_fp8(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad,
                                       const void *x, const float *x_scale, const void *w, const float *w_scales,
                                       const float *scale, const float *shift, const void *residual, void *y,
                                       unsigned flags, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    int To = 0;
    const int st = fp8_check(B, Cin, Cout, T, K, stride, dilation, pad, &To);
    if (st != NM_OK) return st;
    if (!x || !x_scale || !w || !w_scales || !y) return NM_ERR_BAD_ARG;
    if (flags & ~(unsigned)NM_RELU) return NM_ERR_BAD_ARG;
    const Fp8Layout l = fp8_layout(B, Cin, Cout, To, K, dilation);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < l.total) return NM_ERR_WORKSPACE;
    const size_t nx = (size_t)B * Cin * T * 2, ny = (size_t)B * Cout * To * 2, nw = (size_t)Cout * Cin * K * 2;
    if (((uintptr_t)w & 15) || ((uintptr_t)x & 1) || ((uintptr_t)y & 1) || ((uintptr_t)residual & 1)) return NM_ERR_BAD_ARG;
    if (overlap(y, ny, x, nx) || overlap(y, ny, w, nw) || overlap(y, ny, residual, ny) || overlap(y, ny, workspace, l.total) ||
        overlap(x, nx, workspace, l.total) || overlap(w, nw, workspace, l.total) || overlap(residual, ny, workspace, l.total))
        return NM_ERR_BAD_ARG;

    hipStream_t s = (hipStream_t)hip_stream;
    unsigned char *xq = (unsigned char *)workspace;
    unsigned char *wq = xq + l.xq_bytes;
    if (T % 8 == 0 && !((uintptr_t)x & 15))
        hipLaunchKernelGGL(quant_x_vec_kernel, dim3((T + kQxT - 1) / kQxT, l.nck, B), dim3(256), 0, s, (const bf16_t *)x,
                           x_scale, xq, Cin, T, l.Tp, pad);
    else
        hipLaunchKernelGGL(quant_x_kernel, dim3((l.Tp + 63) / 64, l.nck, B), dim3(256), 0, s, (const bf16_t *)x, x_scale, xq,
                           Cin, T, l.Tp, pad);
    hipLaunchKernelGGL(pack_w_kernel, dim3(2, l.nck, l.ncot), dim3(kPackThreads), (size_t)32 * (64 * K + 8), s,
                       (const bf16_t *)w, w_scales, wq, Cin, K);
    if (hipGetLastError() != hipSuccess) return NM_ERR_DEVICE;

    Fp8Params p;
    p.B = B; p.Cin = Cin; p.Cout = Cout; p.To = To; p.K = K;
    p.ncot = l.ncot; p.nck = l.nck; p.ntt = l.ntt; p.Tp = l.Tp;
    p.nbt = B * l.ntt;
    p.ntiles = l.ncot * 4 * ((p.nbt + 3) / 4);
    p.relu = (flags & NM_RELU) ? 1 : 0;
    p.vec_io = (To % 8 == 0 && !((uintptr_t)y & 15) && !((uintptr_t)residual & 15)) ? 1 : 0;
    p.xq = xq; p.wq = wq;
    p.xs = x_scale; p.ws = w_scales; p.scale = scale; p.shift = shift;
    p.res = (const bf16_t *)residual;
    p.y = (bf16_t *)y;
    hipError_t e;
    if (dilation == 2) e = launch_fp8_conv<29, 2>(p, s);
    else if (K == 17) e = launch_fp8_conv<17, 1>(p, s);
    else if (K == 21) e = launch_fp8_conv<21, 1>(p, s);
    else e = launch_fp8_conv<25, 1>(p, s);
    return e == hipSuccess ? NM_OK : NM_ERR_DEVICE;
}

// ---- input gradient ---------------------------------------------------------------------------------
namespace {
// the input gradient is the forward engine with the channel roles swapped, the taps flipped and the left padding
// dil*(K-1) - pad: checks and layout in those terms
int fp8_dgrad_check(int B, int Cin, int Cout, int T, int K, int stride, int dil, int pad, int *To)
{
    return fp8_check(B, Cin, Cout, T, K, stride, dil, pad, To);
}
Fp8Layout fp8_dgrad_layout(int B, int Cin, int Cout, int T, int K, int dil)
{
    return fp8_layout(B, /*reduction channels*/ Cout, /*output channels*/ Cin, /*output length*/ T, K, dil);
}
}  // namespace

extern "C" int nm_fp8_dgrad_weight_scales(int Cin, int Cout, int K, const void *w, const float *scale, float *scales,
                                          void *hip_stream)
{
    if (!w || !scales || Cin <= 0 || Cout <= 0 || K <= 0) return NM_ERR_BAD_ARG;
    if ((long long)Cin * Cout * K > (1LL << 31) - 1) return NM_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(dgrad_wscale_kernel, dim3(Cin), dim3(256), 0, (hipStream_t)hip_stream, (const bf16_t *)w, scale, scales,
                       Cin, Cout, K);
    return hipGetLastError() == hipSuccess ? NM_OK : NM_ERR_DEVICE;
}

extern "C" size_t nm_conv1d_fp8_bwd_data_workspace_bytes(int B, int Cin, int Cout, int T, int K, int stride, int dilation,
                                                         int pad)
{
    int To = 0;
    if (fp8_dgrad_check(B, Cin, Cout, T, K, stride, dilation, pad, &To) != NM_OK) return 0;
    return fp8_dgrad_layout(B, Cin, Cout, T, K, dilation).total;
}

extern "C" int nm_conv1d_bwd_data_fp8(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad,
                                      const void *dy, const void *y, const float *g_scale, const void *w, const float *scale,
                                      const float *wt_scales, void *dx, void *dres, unsigned flags, void *workspace,
                                      size_t workspace_bytes, void *hip_stream)
{
    int To = 0;
    const int st = fp8_dgrad_check(B, Cin, Cout, T, K, stride, dilation, pad, &To);
    if (st != NM_OK) return st;
    if (!dy || !g_scale || !w || !wt_scales || !dx) return NM_ERR_BAD_ARG;
    if (flags & ~(unsigned)NM_RELU) return NM_ERR_BAD_ARG;
    const bool relu = (flags & NM_RELU) != 0;
    if (relu && !y) return NM_ERR_BAD_ARG;
    const Fp8Layout l = fp8_dgrad_layout(B, Cin, Cout, T, K, dilation);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < l.total) return NM_ERR_WORKSPACE;
    const size_t nx = (size_t)B * Cin * T * 2, ny = (size_t)B * Cout * To * 2, nw = (size_t)Cout * Cin * K * 2;
    if (((uintptr_t)w & 15) || ((uintptr_t)dy & 1) || ((uintptr_t)y & 1) || ((uintptr_t)dx & 1) || ((uintptr_t)dres & 1))
        return NM_ERR_BAD_ARG;
    if (overlap(dx, nx, dy, ny) || overlap(dx, nx, y, ny) || overlap(dx, nx, w, nw) || overlap(dx, nx, dres, ny) ||
        overlap(dres, ny, dy, ny) || overlap(dres, ny, y, ny) || overlap(dres, ny, w, nw) || overlap(dx, nx, workspace, l.total) ||
        overlap(dres, ny, workspace, l.total) || overlap(dy, ny, workspace, l.total) || overlap(y, ny, workspace, l.total) ||
        overlap(w, nw, workspace, l.total))
        return NM_ERR_BAD_ARG;

    hipStream_t s = (hipStream_t)hip_stream;
    unsigned char *gq = (unsigned char *)workspace;
    unsigned char *wtq = gq + l.xq_bytes;
    const int padL = dilation * (K - 1) - pad;
    const bf16_t *ym = relu ? (const bf16_t *)y : nullptr;
    const bool vec = To % 8 == 0 && !((uintptr_t)dy & 15) && !((uintptr_t)y & 15) && !((uintptr_t)dres & 15);
    if (vec)
        hipLaunchKernelGGL(quant_g_vec_kernel, dim3((To + kQxT - 1) / kQxT, l.nck, B), dim3(256), 0, s, (const bf16_t *)dy, ym,
                           g_scale, gq, (bf16_t *)dres, Cout, To, l.Tp, padL);
    else
        hipLaunchKernelGGL(quant_g_kernel, dim3((l.Tp + 63) / 64, l.nck, B), dim3(256), 0, s, (const bf16_t *)dy, ym, g_scale, gq,
                           (bf16_t *)dres, Cout, To, l.Tp, padL);
    if (hipGetLastError() != hipSuccess) return NM_ERR_DEVICE;
    return fp8_dgrad_run(B, Cin, Cout, T, K, dilation, gq, l.Tp, g_scale, w, scale, wt_scales, dx, wtq, s) == hipSuccess
               ? NM_OK
               : NM_ERR_DEVICE;
}
