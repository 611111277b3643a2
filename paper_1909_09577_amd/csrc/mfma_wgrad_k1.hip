// Weight gradient of a pointwise (K = 1, stride 1, no padding) convolution:
//
//   dw[co, ci] = scale[co] * sum_b sum_t g[b, co, t] * x[b, ci, t],      g = dy * [y > 0]
//
// a plain GEMM whose reduction index (time) is the contiguous one in both operands, so neither needs a
// transpose or a fragment-order copy: rows of g and x go to LDS as they lie in memory and every MFMA
// fragment (8 consecutive time steps of one channel) is one aligned 16-byte LDS read.
//
// A workgroup owns a 256 (co) x 128 (ci) output tile and a share of the reduction (units of one batch
// item x 128 time steps, every S-th unit); its four wavefronts form a 2 x 2 grid of 128 x 64 sub-tiles
// (4 x 2 accumulator blocks each).  The 384 operand rows of a unit are staged cooperatively: 16-byte loads
// along time (16 lanes cover 256 contiguous bytes of a row: the longer the run, the fewer cache lines are
// fetched for bytes nobody asked for, rows of 800 steps not being line aligned), held in registers while
// the previous unit multiplies, then written to one LDS buffer of 272-byte rows (conflict-free 16-byte
// reads) between two barriers; a unit is 64 MFMAs per wavefront.  A staged byte feeds 8 (g) resp. 16 (x)
// MFMA rows, which keeps the L2 traffic at about 0.4 KiB per MFMA.  The S partial tiles go to the
// [S][Cout][Cin] float32 scratch and the common reduction kernel adds them in a fixed order and applies
// scale[co]: deterministic.
#include "nm_common.h"

namespace nm {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kTileCo = 256, kTileCi = 128;
constexpr int kTK = 128, kSteps = kTK / 16, kGran = kTK / 8;    // time steps, MFMA steps, 16-byte granules per row and unit
constexpr int kRowBytes = kTK * 2 + 16;                         // 272: 68 dwords, 8 consecutive rows hit disjoint bank groups
constexpr int kRows = kTileCo + kTileCi;
constexpr int kBufBytes = kRows * kRowBytes;                    // 104 448
constexpr int kRowsPerPass = kThreads / kGran;                  // 16 rows per staging pass (lane = row x granule)
constexpr int kGranA = kTileCo / kRowsPerPass;                  // 16 granules per thread and unit (g rows)
constexpr int kGranB = kTileCi / kRowsPerPass;                  // 8 (x rows)
constexpr size_t kLds = (size_t)kBufBytes;
constexpr uint32_t kFar = 0x80000000u;                          // beyond every tensor addressed here (the host keeps them below 1 GiB)

struct K1Params {
    int B, Cin, Cout, T;
    int ncot, ncit, S, nchunk, units, total, per_xcd;
    const bf16_t *x;  // [B][Cin][T]
    const bf16_t *g;  // [B][Cout][T]
    float *part;      // [S][Cout][Cin]
};

__global__ __launch_bounds__(kThreads) void wgrad_k1_kernel(const K1Params p)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // work items: the workgroups that the hardware places on one XCD (blockIdx mod 8) take a contiguous
    // range of items, ci tile fastest, so neighbouring tiles of one reduction share meet in one L2
    const int v = ((int)blockIdx.x & 7) * p.per_xcd + ((int)blockIdx.x >> 3);
    if (((int)blockIdx.x >> 3) >= p.per_xcd || v >= p.total) return;
    const int cit = v % p.ncit, cot = (v / p.ncit) % p.ncot, sp = v / (p.ncit * p.ncot);
    const int co0 = cot * kTileCo, ci0 = cit * kTileCi;
    const int wm = wave >> 1, wn = wave & 1;

    const __amdgpu_buffer_rsrc_t rs_g =
        __builtin_amdgcn_make_buffer_rsrc((void *)p.g, 0, (int)((size_t)p.B * p.Cout * p.T * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_x =
        __builtin_amdgcn_make_buffer_rsrc((void *)p.x, 0, (int)((size_t)p.B * p.Cin * p.T * 2), 0x00020000);

    // staging granule i of this thread: row 16*i + tid/16 of the operand's tile, 16-byte column tid%16
    u32x4 ra[kGranA], rb[kGranB];
    const int srow = (int)threadIdx.x / kGran, scol = (int)threadIdx.x % kGran;
    const uint32_t va0 = (uint32_t)(((co0 + srow) * p.T + 8 * scol) * 2), vb0 = (uint32_t)(((ci0 + srow) * p.T + 8 * scol) * 2);
    const uint32_t vstep = (uint32_t)(kRowsPerPass * p.T * 2);
    const int na_ok = (p.Cout - co0 - srow + kRowsPerPass - 1) / kRowsPerPass;  // granules i < na_ok lie inside the tensor
    const int nb_ok = (p.Cin - ci0 - srow + kRowsPerPass - 1) / kRowsPerPass;
    const int lds0 = srow * kRowBytes + scol * 16;
    auto load_unit = [&](int u) {
        const bool live = u < p.units;
        const int uu = live ? u : 0;
        const int b = uu / p.nchunk, t0 = (uu - b * p.nchunk) * kTK;
        const uint32_t sg = (uint32_t)(((size_t)b * p.Cout * p.T + t0) * 2);
        const uint32_t sx = (uint32_t)(((size_t)b * p.Cin * p.T + t0) * 2);
        const bool col_ok = live && t0 + 8 * scol < p.T;  // (T % 8 == 0: a granule lies inside the row or outside)
#pragma unroll
        for (int i = 0; i < kGranA; ++i)
            ra[i] = __builtin_amdgcn_raw_buffer_load_b128(rs_g, (col_ok && i < na_ok) ? va0 + (uint32_t)i * vstep : kFar, sg, 0);
#pragma unroll
        for (int i = 0; i < kGranB; ++i)
            rb[i] = __builtin_amdgcn_raw_buffer_load_b128(rs_x, (col_ok && i < nb_ok) ? vb0 + (uint32_t)i * vstep : kFar, sx, 0);
    };
    auto write_unit = [&]() {
#pragma unroll
        for (int i = 0; i < kGranA; ++i) *reinterpret_cast<u32x4 *>(smem + lds0 + i * kRowsPerPass * kRowBytes) = ra[i];
#pragma unroll
        for (int i = 0; i < kGranB; ++i)
            *reinterpret_cast<u32x4 *>(smem + lds0 + (kTileCo + i * kRowsPerPass) * kRowBytes) = rb[i];
    };
    // MFMA steps of unit u that lie inside the row (the last unit of a row may be short)
    auto steps_of = [&](int u) {
        const int c = u % p.nchunk;
        const int left = p.T - c * kTK;
        return left >= kTK ? kSteps : (left + 15) / 16;
    };

    f32x16 acc[4][2];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

    // fragment addresses of this lane: row lane%32 of a 32-row block, time half lane/32
    const int a_off = (wm * 128 + (lane & 31)) * kRowBytes + (lane >> 5) * 16;
    const int b_off = (kTileCo + wn * 64 + (lane & 31)) * kRowBytes + (lane >> 5) * 16;

    const int my_units = sp < p.units ? (p.units - sp + p.S - 1) / p.S : 0;  // the same for all four wavefronts
    if (my_units > 0) load_unit(sp);
    for (int i = 0, u = sp; i < my_units; ++i, u += p.S) {
        if (i > 0) __syncthreads();  // every wavefront has finished reading the previous unit
        write_unit();
        __syncthreads();
        load_unit(u + p.S);  // requested now, held in registers while this unit multiplies (zeros past the end)
        const int nsteps = steps_of(u);
        // fragments of step ks+1 are read while step ks multiplies
        bf16x8 af[2][4], bfr[2][2];
        auto read_frags = [&](int ks, bf16x8(&a)[4], bf16x8(&bb)[2]) {
#pragma unroll
            for (int mi = 0; mi < 4; ++mi)
                a[mi] = *reinterpret_cast<const bf16x8 *>(smem + a_off + mi * 32 * kRowBytes + ks * 32);
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
                bb[ni] = *reinterpret_cast<const bf16x8 *>(smem + b_off + ni * 32 * kRowBytes + ks * 32);
        };
        read_frags(0, af[0], bfr[0]);
#pragma unroll
        for (int ks = 0; ks < kSteps; ++ks) {
            if (ks < nsteps) {  // (wave-uniform)
                if (ks + 1 < kSteps) read_frags(ks + 1, af[(ks + 1) & 1], bfr[(ks + 1) & 1]);
#pragma unroll
                for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                    for (int ni = 0; ni < 2; ++ni)
                        acc[mi][ni] =
                            __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks & 1][mi], bfr[ks & 1][ni], acc[mi][ni], 0, 0, 0);
            }
        }
    }

    // register r of a block: output channel 8*(r/4) + 4*(lane/32) + r%4, input channel lane%32
    const int ci = ci0 + wn * 64 + (lane & 31);
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
            const int cc = ci + ni * 32;
            if (cc >= p.Cin) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int co = co0 + wm * 128 + mi * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (co < p.Cout) p.part[((size_t)sp * p.Cout + co) * p.Cin + cc] = acc[mi][ni][r];
            }
        }
}

struct K1Plan {
    int ncot, ncit, S, nchunk, units;
};
K1Plan make_k1_plan(const Geom &g)
{
    K1Plan q;
    q.ncot = (g.Cout + kTileCo - 1) / kTileCo;
    q.ncit = (g.Cin + kTileCi - 1) / kTileCi;
    q.nchunk = (g.T + kTK - 1) / kTK;
    q.units = g.B * q.nchunk;
    const int tiles = q.ncot * q.ncit;
    const int cus = 256;  // a planning target only: any count works
    int S = cus / tiles;
    if (S > 64) S = 64;
    if (S > q.units) S = q.units;
    if (S < 1) S = 1;
    q.S = S;
    return q;
}

}  // namespace

bool wgrad_k1_supported(const Geom &g)
{
    if (!(g.K == 1 && g.stride == 1 && g.pad == 0 && g.To == g.T && g.T % 8 == 0 && g.len == nullptr)) return false;
    const size_t lim = (size_t)1 << 30;  // both operands are addressed through buffer descriptors
    if ((size_t)g.B * g.Cin * g.T * sizeof(bf16_t) > lim || (size_t)g.B * g.Cout * g.T * sizeof(bf16_t) > lim) return false;
    return g.Cout >= 64 && g.Cin >= 64;  // smaller layers are bandwidth bound and stay on the general kernels
}

size_t wgrad_k1_part_bytes(const Geom &g)
{
    return align_up((size_t)make_k1_plan(g).S * g.Cout * g.Cin * sizeof(float), 256);
}

// gplain: g = dy*[y>0] in the layout of dy (dy itself without a ReLU).  ws: wgrad_k1_part_bytes(g) bytes.
hipError_t launch_wgrad_k1(const Geom &g, const void *x, const void *gplain, const float *scale, float *dw, bool accumulate,
                           void *ws, hipStream_t s)
{
    const K1Plan q = make_k1_plan(g);
    K1Params p = {};
    p.B = g.B; p.Cin = g.Cin; p.Cout = g.Cout; p.T = g.T;
    p.ncot = q.ncot; p.ncit = q.ncit; p.S = q.S; p.nchunk = q.nchunk; p.units = q.units;
    p.total = q.ncot * q.ncit * q.S;
    p.per_xcd = (p.total + 7) / 8;
    p.x = (const bf16_t *)x; p.g = (const bf16_t *)gplain; p.part = (float *)ws;
    static LdsOptIn opt_in;
    hipError_t e = ensure_dynamic_lds(opt_in, reinterpret_cast<const void *>(wgrad_k1_kernel), (int)kLds);
    if (e != hipSuccess) return e;
    {
        MainKernelTimer timer(s);
        hipLaunchKernelGGL(wgrad_k1_kernel, dim3(p.per_xcd * 8), dim3(kThreads), kLds, s, p);
        e = hipGetLastError();
    }
    if (e != hipSuccess) return e;
    return launch_wgrad_reduce(g, (const float *)ws, dw, scale, q.S, accumulate, s);
}

}  // namespace nm
