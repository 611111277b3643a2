// Stand-alone probe: sustained v_mfma_f32_32x32x16_bf16 rate of the whole chip with nothing else
// running (no LDS, no memory traffic in the loop), for three kinds of operand data.  The shader clock
// under a full MFMA load depends on how many operand bits toggle, so the rate on realistic (random)
// data is the practical ceiling for any bf16 matrix-core kernel on the same machine; the rate on
// constant data shows the nominal one.  Prints TFLOP/s and the core clock seen by wave 0
// (clock64 ticks per wall-clock nanosecond).
//
// Build and run:  python -m paper_1909_09577_amd.build probe && paper_1909_09577_amd/probes/mfma_rate
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define CHECK(x)                                                                        \
    do {                                                                                \
        hipError_t e_ = (x);                                                            \
        if (e_ != hipSuccess) {                                                         \
            std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);  \
            std::exit(1);                                                               \
        }                                                                               \
    } while (0)

// 20 MFMAs per iteration on 10 accumulators, 4 A and 5 B fragments held in registers.
__global__ __launch_bounds__(256) void mfma_loop(const u32x4 *__restrict__ g, float *out, long long *clk, int iters)
{
    const int tid = blockIdx.x * 256 + threadIdx.x;
    f32x16 acc[10];
    for (int t = 0; t < 10; ++t)
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
    union U {
        u32x4 u;
        bf16x8 b;
    };
    U a[4], b[5];
    for (int i = 0; i < 4; ++i) a[i].u = g[(size_t)tid * 9 + i];
    for (int i = 0; i < 5; ++i) b[i].u = g[(size_t)tid * 9 + 4 + i];
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
        for (int i = 0; i < 5; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0].b, b[i].b, acc[i], 0, 0, 0);
        for (int i = 0; i < 5; ++i) acc[5 + i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1].b, b[i].b, acc[5 + i], 0, 0, 0);
        for (int i = 0; i < 5; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[2].b, b[i].b, acc[i], 0, 0, 0);
        for (int i = 0; i < 5; ++i) acc[5 + i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[3].b, b[i].b, acc[5 + i], 0, 0, 0);
    }
    const long long c1 = clock64(), w1 = wall_clock64();
    float s = 0;
    for (int t = 0; t < 10; ++t)
        for (int r = 0; r < 16; ++r) s += acc[t][r];
    out[tid] = s;
    if ((threadIdx.x & 63) == 0) {
        clk[(tid >> 6) * 2] = c1 - c0;
        clk[(tid >> 6) * 2 + 1] = w1 - w0;
    }
}

int main()
{
    int dev = 0, cus = 0;
    CHECK(hipGetDevice(&dev));
    CHECK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    const int grid = cus, iters = 20000;
    const size_t n = (size_t)grid * 256 * 9;
    u32x4 *h = (u32x4 *)std::malloc(n * 16);
    u32x4 *g;
    float *out;
    long long *clk;
    CHECK(hipMalloc(&g, n * 16));
    CHECK(hipMalloc(&out, (size_t)grid * 256 * 4));
    CHECK(hipMalloc(&clk, (size_t)grid * 4 * 2 * 8));
    const char *names[3] = {"all ones", "all zeros", "random in [-2,2]"};
    for (int mode = 0; mode < 3; ++mode) {
        uint32_t st = 12345u;
        auto rnd_bf16 = [&]() {  // random sign and mantissa, exponent 0x7a..0x81
            st = st * 1664525u + 1013904223u;
            const uint32_t r = st >> 8;
            return (uint16_t)(((r & 1) << 15) | ((0x7a + ((r >> 1) & 7)) << 7) | ((r >> 4) & 0x7f));
        };
        for (size_t i = 0; i < n * 4; ++i) {
            uint32_t v = 0;
            if (mode == 0) v = 0x3f803f80u;
            if (mode == 2) {
                const uint32_t lo = rnd_bf16();
                v = lo | ((uint32_t)rnd_bf16() << 16);
            }
            ((uint32_t *)h)[i] = v;
        }
        CHECK(hipMemcpy(g, h, n * 16, hipMemcpyHostToDevice));
        hipEvent_t e0, e1;
        CHECK(hipEventCreate(&e0));
        CHECK(hipEventCreate(&e1));
        mfma_loop<<<grid, 256>>>(g, out, clk, iters);
        CHECK(hipDeviceSynchronize());
        CHECK(hipEventRecord(e0));
        for (int r = 0; r < 10; ++r) mfma_loop<<<grid, 256>>>(g, out, clk, iters);
        CHECK(hipEventRecord(e1));
        CHECK(hipEventSynchronize(e1));
        float ms = 0;
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        ms /= 10;
        long long hc[2];
        CHECK(hipMemcpy(hc, clk, 16, hipMemcpyDeviceToHost));
        const double flops = (double)grid * 4 * iters * 20 * 32768.0;
        std::printf("%-18s %8.3f ms/launch  %7.1f TFLOP/s  core clock %.2f GHz  %.2f ns per MFMA and wave\n", names[mode], ms,
                    flops / ms / 1e9, (double)hc[0] / (hc[1] * 10.0), ms * 1e6 / (iters * 20.0));
    }
    return 0;
}
