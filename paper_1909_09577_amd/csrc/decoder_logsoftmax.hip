// Decoder tail: 1x1 convolution from the encoder channels to the vocabulary fused with the
// log-softmax over the classes of every frame (the log_probs that the CTC decoder module of the
// paper's ASR example, Section 4.1.1, hands to the CTC loss):
//
//   z[b,c,t]    = sum_ci w[c,ci] * x[b,ci,t] + bias[c]
//   logp[b,c,t] = z[b,c,t] - log(sum_c' exp(z[b,c',t]))          (float32 out)
//
// The step is bound by reading x once (Cin >> Ncls: 52 MB in, 3 MB out at the encoder's size), so the
// kernel is built around the load stream, not the arithmetic:
//   * a wavefront owns 32 frames of one batch item and all classes (Ncls <= 32: one 32x32 MFMA
//     accumulator), so the softmax needs no exchange between wavefronts -- the two lanes that hold
//     the halves of a frame's classes swap one value twice; the four wavefronts of a workgroup sit
//     side by side (256 contiguous bytes of every channel row);
//   * x is copied as it lies in memory: per 16 channels one 16-byte load and one 16-byte LDS write
//     per lane (16 rows of 64 bytes, wave-private, two buffers), and the MFMA B fragment (8
//     consecutive channels of one frame) is read back with the transposing LDS read
//     ds_read_b64_tr_b16 -- no shuffling instructions at all;
//   * sixteen x loads and sixteen weight loads per lane are kept in flight (register rings), LDS write,
//     LDS read and MFMA of consecutive steps overlap;
//   * the weight rows are read straight from w ([Ncls][Cin]: 8 consecutive channels of one class are
//     16 contiguous bytes), classes beyond Ncls read zeros.
// Shapes the matrix-core kernel does not take (Ncls > 32, Cin % 16 != 0, T % 8 != 0, float32
// storage, misaligned tensors) use a plain kernel: one thread per frame, two passes over the classes.
#include "../../include/nm_conv1d.h"
#include "nm_common.h"

namespace nm {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

constexpr uint32_t kFar = 0x80000000u;  // buffer offset beyond any tensor taken here (<= 1 GiB): reads zeros
constexpr int kRing = 16;               // loads in flight per lane and operand
constexpr int kFramesPerWave = 32;
constexpr int kStepBytes = 16 * 64;     // one step in LDS: 16 channels x 32 frames of bf16

__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// BLOCK == false: the decoder tail (bias, log-softmax, float32 out).  BLOCK == true: the same load stream as the
// forward pass of a pointwise conv1d sub-block with at most 32 output channels (the 1024 -> 29 projection in
// front of the decoder): `bias` is the shift, and the epilogue is scale, shift, residual, ReLU, bf16 out.
template <bool BLOCK>
__global__ __launch_bounds__(256) void decoder_mfma_kernel(int B, int Cin, int Ncls, int T, const bf16_t *__restrict__ x,
                                                           const bf16_t *__restrict__ w, const float *__restrict__ bias,
                                                           float *__restrict__ logp, const float *__restrict__ scale,
                                                           const bf16_t *__restrict__ res, int relu,
                                                           bf16_t *__restrict__ y)
{
    __shared__ __align__(16) unsigned char smem[4 * 2 * kStepBytes];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int b = blockIdx.y;
    const int t0 = (blockIdx.x * 4 + wave) * kFramesPerWave;
    if (t0 >= T) return;
    unsigned char *buf = smem + wave * 2 * kStepBytes;
    const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc((void *)x, 0, (int)((size_t)B * Cin * T * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc((void *)w, 0, (int)((size_t)Ncls * Cin * 2), 0x00020000);
    const int first = 0, last = Cin / 16, per_wave = last;  // steps of 16 channels

    // x: lane = (channel lane/4 of the step, frames 8*(lane%4) .. +7); frames beyond T read zeros
    const int xt = t0 + 8 * (lane & 3);
    const uint32_t x_lane = xt + 8 <= T ? (uint32_t)((((size_t)b * Cin + (lane >> 2)) * T + xt) * 2) : kFar;
    const uint32_t x_step = (uint32_t)(16 * T * 2);
    // w: lane = (class lane%32, channels 8*(lane/32) .. +7 of the step)
    const uint32_t w_lane = (lane & 31) < Ncls ? (uint32_t)(((lane & 31) * Cin + 8 * (lane >> 5)) * 2) : kFar;
    auto load_x = [&](int i) { return __builtin_amdgcn_raw_buffer_load_b128(rs_x, first + i < last ? x_lane : kFar, (uint32_t)(first + i) * x_step, 0); };
    auto load_w = [&](int i) { return __builtin_amdgcn_raw_buffer_load_b128(rs_w, first + i < last ? w_lane : kFar, (uint32_t)(first + i) * 32u, 0); };
    // transposing read of a step: lane addresses 4 frames 16*((lane/16)&1) + 4*(lane&3) of channel row
    // 8*(lane/32) + (lane&15)/4 (+4 for the second read) and receives frame lane%32, 4 channels each
    const int g4 = lane >> 4, i16 = lane & 15;
    const uint32_t tr_off = (uint32_t)((8 * (g4 >> 1) + (i16 >> 2)) * 64 + (16 * (g4 & 1) + 4 * (i16 & 3)) * 2);
    auto read_b = [&](int par) {
        union {
            s16x4 h[2];
            bf16x8 v;
        } cvt;
        const unsigned char *p = buf + par * kStepBytes + tr_off;
        cvt.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p));
        cvt.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p + 4 * 64));
        return cvt.v;
    };
    auto write_x = [&](int par, const u32x4 &v) { *reinterpret_cast<u32x4 *>(buf + par * kStepBytes + lane * 16) = v; };

    u32x4 xr[kRing], wr[kRing];
#pragma unroll
    for (int i = 0; i < kRing; ++i) {
        xr[i] = load_x(i);
        wr[i] = load_w(i);
    }
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;

    // steps run in rounds of kRing so that the rings are indexed statically; a last partial round
    // multiplies zeros.  Step s: LDS write of step s+1, LDS read of step s+1, MFMA of step s.
    write_x(0, xr[0]);
    xr[0] = load_x(kRing);
    wave_lds_fence();
    bf16x8 bcur = read_b(0);
    const int rounds = (per_wave + kRing - 1) / kRing;
    for (int rd = 0; rd < rounds; ++rd) {
#pragma unroll
        for (int i = 0; i < kRing; ++i) {
            const int s = rd * kRing + i;
            // next step into the other buffer (its ring slot is i+1, already reloaded when i+1 wraps)
            const int in = (i + 1) % kRing;
            write_x((i + 1) & 1, xr[in]);
            xr[in] = load_x(s + 1 + kRing);
            wave_lds_fence();
            const bf16x8 bnext = read_b((i + 1) & 1);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wr[i]), bcur, acc, 0, 0, 0);
            wr[i] = load_w(s + kRing);
            bcur = bnext;
        }
    }

    // Register r of the accumulator is class 8*(r/4) + 4*(lane/32) + r%4, frame lane%32.
    const int t = t0 + (lane & 31);
    if constexpr (BLOCK) {
        if (t < T) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int c = 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (c < Ncls) {
                    const size_t o = ((size_t)b * Ncls + c) * T + t;
                    float v = acc[r];
                    if (scale) v *= scale[c];
                    if (bias) v += bias[c];
                    if (res) v += bf16_to_f32(res[o]);
                    if (relu) v = v > 0.f ? v : 0.f;
                    y[o] = f32_to_bf16(v);
                }
            }
        }
        return;
    }
    // ---- log-softmax over the classes of this lane's frame: a frame's classes sit in two lanes, 32 apart.
    float z[16];
    float m = -INFINITY;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int c = 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        const bool ok = c < Ncls;
        z[r] = ok ? acc[r] + (bias ? bias[c] : 0.f) : -INFINITY;
        m = fmaxf(m, z[r]);
    }
    m = fmaxf(m, __shfl_xor(m, 32));
    float sum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) sum += expf(z[r] - m);  // exp(-inf) = 0 for the padded classes
    sum += __shfl_xor(sum, 32);
    const float lse = m + logf(sum);
    if (t < T) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int c = 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            if (c < Ncls) logp[((size_t)b * Ncls + c) * T + t] = z[r] - lse;
        }
    }
}

// One thread per frame: a first pass over the classes finds max and sum of exponentials (running
// form), a second one recomputes the logits and writes the result.  Any size, both storage types.
template <typename TS>
__global__ __launch_bounds__(256) void decoder_plain_kernel(int B, int Cin, int Ncls, int T, const TS *__restrict__ x,
                                                            const TS *__restrict__ w, const float *__restrict__ bias,
                                                            float *__restrict__ logp)
{
    const int t = blockIdx.x * 256 + threadIdx.x;
    const int b = blockIdx.y;
    if (t >= T) return;
    const TS *xb = x + (size_t)b * Cin * T + t;
    auto logit = [&](int c) {
        float acc = 0.f;
        for (int c0 = 0; c0 < Cin; c0 += 64) {  // short blocks keep the float32 sum accurate
            float part = 0.f;
            const int c1 = min(c0 + 64, Cin);
            for (int ci = c0; ci < c1; ++ci) part = fmaf(load_as_f32(w, (size_t)c * Cin + ci), load_as_f32(xb, (size_t)ci * T), part);
            acc += part;
        }
        return acc + (bias ? bias[c] : 0.f);
    };
    float m = -INFINITY, sum = 0.f;
    for (int c = 0; c < Ncls; ++c) {
        const float z = logit(c);
        const float mn = fmaxf(m, z);
        sum = sum * expf(m - mn) + expf(z - mn);
        m = mn;
    }
    const float lse = m + logf(sum);
    for (int c = 0; c < Ncls; ++c) logp[((size_t)b * Ncls + c) * T + t] = logit(c) - lse;
}

}  // namespace

// Forward of a pointwise sub-block with few output channels on the decoder's load stream.
bool skinny_fwd_supported(const Geom &g)
{
    return g.K == 1 && g.stride == 1 && g.pad == 0 && g.To == g.T && g.len == nullptr && g.Cout <= 32 && g.Cin % 16 == 0 &&
           g.T % 8 == 0 && (size_t)g.B * g.Cin * g.T * 2 <= ((size_t)1 << 30);
}

hipError_t launch_skinny_fwd(const Geom &g, const void *x, const void *w, const float *scale, const float *shift,
                             const void *res, void *y, bool relu, hipStream_t s)
{
    dim3 grid((g.T + 4 * kFramesPerWave - 1) / (4 * kFramesPerWave), g.B);
    MainKernelTimer timer(s);
    hipLaunchKernelGGL(decoder_mfma_kernel<true>, grid, dim3(256), 0, s, g.B, g.Cin, g.Cout, g.T, (const bf16_t *)x,
                       (const bf16_t *)w, shift, (float *)nullptr, scale, (const bf16_t *)res, relu ? 1 : 0, (bf16_t *)y);
    return hipGetLastError();
}

}  // namespace nm

using namespace nm;

extern "C" int nm_decoder_logsoftmax_fwd(int B, int Cin, int Ncls, int T, const void *x, const void *w, const float *bias,
                                         float *logp, unsigned flags, int dtype, void *hip_stream)
{
    if (B <= 0 || Cin <= 0 || Ncls <= 0 || T <= 0) return NM_ERR_BAD_ARG;
    if (dtype != NM_BF16 && dtype != NM_F32) return NM_ERR_BAD_ARG;
    if (flags & ~(unsigned)NM_FORCE_DIRECT) return NM_ERR_BAD_ARG;
    if (!x || !w || !logp) return NM_ERR_BAD_ARG;
    const long long lim = (1LL << 31) - 1;
    if ((long long)B * Cin * T > lim || (long long)B * Ncls * T > lim || (long long)Ncls * Cin > lim || B > 65535)
        return NM_ERR_UNSUPPORTED;
    hipStream_t s = (hipStream_t)hip_stream;
    const bool fast = dtype == NM_BF16 && !(flags & NM_FORCE_DIRECT) && Ncls <= 32 && Cin % 16 == 0 && T % 8 == 0 &&
                      ((uintptr_t)x % 16) == 0 && ((uintptr_t)w % 16) == 0 &&
                      (size_t)B * Cin * T * 2 <= ((size_t)1 << 30);
    if (fast) {
        dim3 grid((T + 4 * kFramesPerWave - 1) / (4 * kFramesPerWave), B);
        hipLaunchKernelGGL(decoder_mfma_kernel<false>, grid, dim3(256), 0, s, B, Cin, Ncls, T, (const bf16_t *)x,
                           (const bf16_t *)w, bias, logp, (const float *)nullptr, (const bf16_t *)nullptr, 0, (bf16_t *)nullptr);
    } else {
        dim3 grid((T + 255) / 256, B);
        if (dtype == NM_BF16)
            hipLaunchKernelGGL(decoder_plain_kernel<bf16_t>, grid, dim3(256), 0, s, B, Cin, Ncls, T, (const bf16_t *)x,
                               (const bf16_t *)w, bias, logp);
        else
            hipLaunchKernelGGL(decoder_plain_kernel<float>, grid, dim3(256), 0, s, B, Cin, Ncls, T, (const float *)x,
                               (const float *)w, bias, logp);
    }
    return hipGetLastError() == hipSuccess ? NM_OK : NM_ERR_DEVICE;
}
