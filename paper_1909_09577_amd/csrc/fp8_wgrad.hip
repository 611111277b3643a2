// Weight gradient on 8-bit floating-point (E4M3) operands.
//
//   dw[co,ci,k] = scale[co]*sg*sx * sum_b sum_t decode(gq[b,co,t]) * decode(xq[b,ci,t - pad + k*dil])      (stride 1)
//
// Per tap a GEMM with M = co, N = ci and the reduction over (b, t), on v_mfma_f32_32x32x64_f8f6f4: 64 time steps
// per instruction.  Both operands come in the time-major layout the other 8-bit kernels use (rows of 64 channels,
// row r of x standing for input time r - pad, zero rows for the padding; rows of g standing for output time r), so a
// tap is a row offset.  The matrix cores want, per lane, 32 consecutive reduction indices (time steps) of one channel
// -- a column of that layout -- which the gfx950 transposing LDS read delivers: ds_read_b64_tr_b8 lets 16 lanes read
// an 8 x 16 byte block (lane j supplies row j/2, columns 8*(j%2) .. +7) and gives lane c the 8 bytes of column c.
// Four such reads fill a 32-byte operand; A and B use the same (lane half, byte) -> time step assignment, which is
// all the contraction needs.
//
// Work decomposition: an output tile is 64 output channels x 32 input channels x all K taps.  A workgroup (four
// wavefronts) takes the tile's taps -- for K > 20 every second of them, two workgroups sharing the tile -- and
// wavefront w every fourth of those (two 32x32 accumulators per tap), so that no wavefront holds more than five taps
// and two workgroups fit a CU: the second one's MFMAs cover the first one's waits.  The taps of a wavefront are
// 4 or 8 rows apart, so the 8-row blocks their operands are made of lie on one grid: each block is read once per
// unit and every tap picks its four from the registers.  The reduction is cut into units of one batch item x 64
// time steps; the S workgroups that share a (tile, tap group) take every S-th unit.  Per unit the workgroup stages
// the 64 x 64 window of g and the (64 + (K-1)*dil) x 32 window of x in LDS (one 16-byte load per thread and window,
// requested a unit ahead, double buffered, one barrier per unit).  Every workgroup writes its float32 partial tile
// to [S][K][Cout][Cin]; the reduction kernel of the bfloat16 path adds the S partials in a fixed order, applies the
// per-channel factor and writes dw[co][ci][k]: deterministic.
#include "../../include/nm_conv1d.h"
#include "../../include/nm_conv1d_fp8.h"
#include "nm_common.h"

#include <type_traits>
#include <utility>

namespace nm {
// quantisation passes of fp8_conv.hip
hipError_t fp8_launch_quant_x(const void *x, const float *xs, unsigned char *xq, int B, int C, int T, int Tp, int pad,
                              hipStream_t s);
hipError_t fp8_launch_quant_g(const void *dy, const void *y, const float *gs, unsigned char *gq, void *dres, int B, int C,
                              int T, int Tp, int pad, hipStream_t s);
bool fp8_taps_supported(int K, int dil);
hipError_t fp8_dgrad_run(int B, int Cin, int Cout, int T, int K, int dil, const unsigned char *gq, int Tp, const float *g_scale,
                         const void *w, const float *scale, const float *wt_scales, void *dx, unsigned char *wtq, hipStream_t s);
size_t fp8_packed_weight_bytes(int Cin, int Cout, int K);

namespace {

typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef int i32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) i32x2 lds_i32x2;

constexpr int kThreads = 256;
constexpr int kUnitT = 64;   // time steps per unit = reduction length of one MFMA
constexpr int kTileCo = 64;
constexpr int kTileCi = 32;
constexpr int kGPitch = 80;  // LDS row of the g window: 64 B + 16 B pad
constexpr int kXPitch = 48;  // LDS row of the x window: 32 B + 16 B pad
constexpr size_t kSlack = 8192;

struct WgParams {
    int B, Cin, Cout, K;
    int ncit, S;         // input-channel tiles (of 32); workgroups per output tile
    int nu, units;       // units per batch item; B * nu
    int Tpg, Tpx;        // rows per (batch item, 64-channel group) of gq / xq
    int g_row0;          // row of gq that stands for output time 0
    const unsigned char *gq;  // [B][Cout/64][Tpg][64]
    const unsigned char *xq;  // [B][Cin/64][Tpx][64]
    float *part;              // [S][K][Cout][Cin]
};

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

// One transposing read: rows row0 + 32*(lane/32) .. +7 of channel col0 + lane%32 (8 reduction indices per lane)
__device__ __forceinline__ i32x2 read_block(const unsigned char *win, int pitch, int row0, int col0, int lane)
{
    const int gi = lane >> 4, j = lane & 15;
    const unsigned char *a = win + (row0 + 32 * (gi >> 1) + (j >> 1)) * pitch + col0 + 16 * (gi & 1) + 8 * (j & 1);
    return __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_i32x2 *)a);
}
// 32 reduction indices (rows row0 + 32*(lane/32) .. +31) of channel col0 + lane%32 from a time-major LDS window
__device__ __forceinline__ i32x8 read_operand(const unsigned char *win, int pitch, int row0, int col0, int lane)
{
    i32x8 r;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const i32x2 v = read_block(win, pitch, row0 + 8 * q, col0, lane);
        r[2 * q] = v[0];
        r[2 * q + 1] = v[1];
    }
    return r;
}

// TG workgroups share the taps of a tile (workgroup G of them takes the taps G, G+TG, ...); inside a workgroup
// wavefront W takes every fourth of those: taps K0 + KS*i with K0 = G + TG*W, KS = 4*TG.
template <int KT, int DIL, int TG, int G, int W>
__device__ __forceinline__ void wgrad_units(const WgParams &p, unsigned char *gbuf, unsigned char *xbuf, int sp, int cot, int cit)
{
    constexpr int XROWS = kUnitT + (KT - 1) * DIL;
    constexpr int K0 = G + TG * W, KS = 4 * TG;
    constexpr int NTW = K0 < KT ? (KT - K0 + KS - 1) / KS : 0;  // taps of this wavefront
    if constexpr (NTW == 0) {
        // no tap for this wavefront: it still takes part in the staging and the barriers below
    }
    // The operand of tap K0+KS*i is the four 8-row blocks at rows (K0+KS*i)*DIL + 8q.  All those rows lie on the grid
    // K0*DIL + STEP*j, so every block is read once per unit and the taps pick their four from the registers.
    constexpr int STEP = (KS * DIL) % 8 == 0 ? 8 : 4;
    static_assert((KS * DIL) % STEP == 0 && 8 % STEP == 0, "block grid");
    constexpr int PER_TAP = KS * DIL / STEP, PER_Q = 8 / STEP;
    constexpr int NB = NTW > 0 ? PER_TAP * (NTW - 1) + PER_Q * 3 + 1 : 1;
    constexpr int NACC = NTW > 0 ? NTW : 1;
    const int tid = threadIdx.x, lane = tid & 63;
    f32x16 acc[NACC][2];
#pragma unroll
    for (int i = 0; i < NACC; ++i)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][cb][r] = 0.f;

    const int nckg = p.Cout / 64, nckx = p.Cin / 64;
    // this thread's piece of the two windows: g row tid/4, quarter tid%4; x row tid/2, half tid%2 (threads below 2*XROWS)
    const bool has_x = tid < 2 * XROWS;
    auto g_src = [&](int u) {
        const int b = u / p.nu, tu = u - b * p.nu;
        return p.gq + (((size_t)b * nckg + cot) * p.Tpg + (size_t)tu * kUnitT + p.g_row0) * 64 + tid * 16;
    };
    auto x_src = [&](int u) {
        const int b = u / p.nu, tu = u - b * p.nu;
        return p.xq + (((size_t)b * nckx + (cit >> 1)) * p.Tpx + (size_t)tu * kUnitT + (tid >> 1)) * 64 + (cit & 1) * 32 + (tid & 1) * 16;
    };
    unsigned char *const g_dst = gbuf + (tid >> 2) * kGPitch + (tid & 3) * 16;
    unsigned char *const x_dst = xbuf + (tid >> 1) * kXPitch + (tid & 1) * 16;
    constexpr int GBUF = kUnitT * kGPitch, XBUF = XROWS * kXPitch;

    int u = sp;
    u32x4 gv = {0u, 0u, 0u, 0u}, xv = {0u, 0u, 0u, 0u};
    if (u < p.units) {
        gv = *reinterpret_cast<const u32x4 *>(g_src(u));
        if (has_x) xv = *reinterpret_cast<const u32x4 *>(x_src(u));
        *reinterpret_cast<u32x4 *>(g_dst) = gv;
        if (has_x) *reinterpret_cast<u32x4 *>(x_dst) = xv;
    }
    __syncthreads();
    int cur = 0;
    for (; u < p.units; u += p.S) {
        const int un = u + p.S;
        const bool more = un < p.units;
        if (more) {  // the next unit's pieces travel while this unit is multiplied
            gv = *reinterpret_cast<const u32x4 *>(g_src(un));
            if (has_x) xv = *reinterpret_cast<const u32x4 *>(x_src(un));
        }
        const unsigned char *gw = gbuf + cur * GBUF, *xw = xbuf + cur * XBUF;
        const i32x8 a0 = read_operand(gw, kGPitch, 0, 0, lane);
        const i32x8 a1 = read_operand(gw, kGPitch, 0, 32, lane);
        i32x2 blk[NB];
        static_for<NB>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            if constexpr (NTW > 0) blk[j] = read_block(xw, kXPitch, K0 * DIL + STEP * j, 0, lane);
        });
        static_for<NTW>([&](auto ic) {
            constexpr int i = decltype(ic)::value, j0 = PER_TAP * i;
            const i32x8 bk = {blk[j0][0], blk[j0][1], blk[j0 + PER_Q][0], blk[j0 + PER_Q][1],
                              blk[j0 + 2 * PER_Q][0], blk[j0 + 2 * PER_Q][1], blk[j0 + 3 * PER_Q][0], blk[j0 + 3 * PER_Q][1]};
            acc[i][0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a0, bk, acc[i][0], 0, 0, 0, 0, 0, 0);
            acc[i][1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a1, bk, acc[i][1], 0, 0, 0, 0, 0, 0);
        });
        if (more) {
            *reinterpret_cast<u32x4 *>(g_dst + (cur ^ 1) * GBUF) = gv;
            if (has_x) *reinterpret_cast<u32x4 *>(x_dst + (cur ^ 1) * XBUF) = xv;
        }
        cur ^= 1;
        __syncthreads();  // the next window is complete; the one just read may be overwritten in the next round
    }

    // register r of block (tap, cb) is output channel cot*64 + cb*32 + 8*(r/4) + 4*(lane/32) + r%4, input channel cit*32 + lane%32
    const int ci = cit * kTileCi + (lane & 31);
#pragma unroll
    for (int i = 0; i < NTW; ++i) {
        const int k = K0 + KS * i;
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int co = cot * kTileCo + cb * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                p.part[(((size_t)sp * p.K + k) * p.Cout + co) * p.Cin + ci] = acc[i][cb][r];
            }
    }
}

template <int KT, int DIL, int TG>
__global__ __launch_bounds__(kThreads) void fp8_wgrad_kernel(const WgParams p)
{
    constexpr int XROWS = kUnitT + (KT - 1) * DIL;
    static_assert(2 * XROWS <= kThreads, "one 16-byte piece of the x window per thread");
    static_assert(TG == 1 || TG == 2, "tap groups");
    __shared__ __align__(16) unsigned char gbuf[2 * kUnitT * kGPitch];
    __shared__ __align__(16) unsigned char xbuf[2 * XROWS * kXPitch];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int id = blockIdx.x;
    const int grp = id % TG;
    id /= TG;
    const int sp = id % p.S, tile = id / p.S;
    const int cit = tile % p.ncit, cot = tile / p.ncit;
    // one copy per (tap group, wavefront number): the tap lists are static
    if (TG == 1 || grp == 0) {
        switch (wave) {
        case 0: wgrad_units<KT, DIL, TG, 0, 0>(p, gbuf, xbuf, sp, cot, cit); break;
        case 1: wgrad_units<KT, DIL, TG, 0, 1>(p, gbuf, xbuf, sp, cot, cit); break;
        case 2: wgrad_units<KT, DIL, TG, 0, 2>(p, gbuf, xbuf, sp, cot, cit); break;
        default: wgrad_units<KT, DIL, TG, 0, 3>(p, gbuf, xbuf, sp, cot, cit); break;
        }
    } else {
        switch (wave) {
        case 0: wgrad_units<KT, DIL, TG, TG - 1, 0>(p, gbuf, xbuf, sp, cot, cit); break;
        case 1: wgrad_units<KT, DIL, TG, TG - 1, 1>(p, gbuf, xbuf, sp, cot, cit); break;
        case 2: wgrad_units<KT, DIL, TG, TG - 1, 2>(p, gbuf, xbuf, sp, cot, cit); break;
        default: wgrad_units<KT, DIL, TG, TG - 1, 3>(p, gbuf, xbuf, sp, cot, cit); break;
        }
    }
}

// eff[co] = scale[co] * sg * sx
__global__ __launch_bounds__(256) void wgrad_factor_kernel(const float *scale, const float *sg, const float *sx, float *eff, int Cout)
{
    const int co = blockIdx.x * 256 + threadIdx.x;
    if (co < Cout) eff[co] = (scale ? scale[co] : 1.f) * (sg[0] * sx[0]);
}

struct WgLayout {
    int nu, Tpg, Tpx, S, TG, ntiles;
    size_t gq_bytes, xq_bytes, part_bytes, eff_bytes, total;
};
WgLayout wg_layout(int B, int Cin, int Cout, int To, int K, int dil)
{
    WgLayout l;
    l.nu = (To + kUnitT - 1) / kUnitT;
    l.Tpg = l.nu * kUnitT;
    l.Tpx = l.nu * kUnitT + (K - 1) * dil;
    l.ntiles = (Cout / kTileCo) * (Cin / kTileCi);
    const int cus = current_device_info().cus;
    // Two workgroups fit a CU when a wavefront holds at most five taps (registers), which hides the load latency:
    // K = 17 as it is, longer filters with their taps dealt to two workgroups per tile.
    l.TG = K > 20 ? 2 : 1;
    // Workgroups per (tile, tap group): the count that minimises the number of rounds over the 2*cus slots, per
    // split, with a charge for the float32 partial tiles every split writes and the reduction reads again.
    const int items = l.ntiles * l.TG, slots = 2 * cus;
    double best = 1e30;
    l.S = 1;
    for (int sc = 1; sc <= 8; ++sc) {
        const double cost = (double)((items * sc + slots - 1) / slots) / sc + 0.05 * sc;
        if (cost < best - 1e-9) {
            best = cost;
            l.S = sc;
        }
    }
    l.S = std::min(l.S, std::max(1, B * l.nu));
    l.gq_bytes = align_up((size_t)B * (Cout / 64) * l.Tpg * 64 + kSlack, 256);
    l.xq_bytes = align_up((size_t)B * (Cin / 64) * l.Tpx * 64 + kSlack, 256);
    l.part_bytes = align_up((size_t)8 * K * Cout * Cin * sizeof(float), 256);  // sized for the largest split
    l.eff_bytes = align_up((size_t)Cout * sizeof(float), 256);
    l.total = l.gq_bytes + l.xq_bytes + l.part_bytes + l.eff_bytes;
    return l;
}

int wg_check(int B, int Cin, int Cout, int T, int K, int stride, int dil, int pad, int *To)
{
    if (B <= 0 || Cin <= 0 || Cout <= 0 || T <= 0 || K <= 0 || stride <= 0 || dil <= 0 || pad < 0) return NM_ERR_BAD_ARG;
    const long long span = (long long)T + 2LL * pad - (long long)dil * (K - 1) - 1;
    if (span < 0) return NM_ERR_BAD_ARG;
    const long long to = span / stride + 1;
    if (to > (1LL << 31) - 1) return NM_ERR_BAD_ARG;
    *To = (int)to;
    if (stride != 1 || Cin % 64 || Cout % 64 || !fp8_taps_supported(K, dil) || pad > (K - 1) * dil) return NM_ERR_UNSUPPORTED;
    if ((long long)B * Cin * T > (1LL << 31) - 1 || (long long)B * Cout * to > (1LL << 31) - 1 ||
        (long long)Cout * Cin * K > (1LL << 28) || B > 65535)
        return NM_ERR_UNSUPPORTED;
    return NM_OK;
}

bool overlap(const void *a, size_t na, const void *b, size_t nb)
{
    if (!a || !b) return false;
    const char *pa = (const char *)a, *pb = (const char *)b;
    return pa < pb + nb && pb < pa + na;
}

template <int KT, int DIL, int TG>
hipError_t launch_wgrad(const WgParams &p, int grid, hipStream_t s)
{
    MainKernelTimer timer(s);
    hipLaunchKernelGGL((fp8_wgrad_kernel<KT, DIL, TG>), dim3(grid), dim3(kThreads), 0, s, p);
    return hipGetLastError();
}

// The weight gradient behind the quantisation of g: quantises x into `rest`, runs the matrix-core kernel on the
// codes gq (Tpg rows per batch item and channel group, row g_row0 standing for output time 0) and reduces the
// partial tiles into dw.  `rest`: xq, partial tiles, per-channel factors (sizes of `l`).
hipError_t wgrad_run(int B, int Cin, int Cout, int T, int To, int K, int dil, int pad, const WgLayout &l, const unsigned char *gq,
                     int Tpg, int g_row0, const void *x, const float *x_scale, const float *g_scale, const float *scale, float *dw,
                     bool accumulate, unsigned char *rest, hipStream_t s)
{
    unsigned char *xq = rest;
    float *part = reinterpret_cast<float *>(xq + l.xq_bytes);
    float *eff = reinterpret_cast<float *>(reinterpret_cast<unsigned char *>(part) + l.part_bytes);
    hipError_t e = fp8_launch_quant_x(x, x_scale, xq, B, Cin, T, l.Tpx, pad, s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(wgrad_factor_kernel, dim3((Cout + 255) / 256), dim3(256), 0, s, scale, g_scale, x_scale, eff, Cout);
    WgParams p;
    p.B = B; p.Cin = Cin; p.Cout = Cout; p.K = K;
    p.ncit = Cin / kTileCi; p.S = l.S;
    p.nu = l.nu; p.units = B * l.nu;
    p.Tpg = Tpg; p.Tpx = l.Tpx; p.g_row0 = g_row0;
    p.gq = gq; p.xq = xq; p.part = part;
    const int grid = l.ntiles * l.S * l.TG;
    if (dil == 2) e = launch_wgrad<29, 2, 2>(p, grid, s);
    else if (K == 17) e = launch_wgrad<17, 1, 1>(p, grid, s);
    else if (K == 21) e = launch_wgrad<21, 1, 2>(p, grid, s);
    else e = launch_wgrad<25, 1, 2>(p, grid, s);
    if (e != hipSuccess) return e;
    Geom g;
    g.B = B; g.Cin = Cin; g.Cout = Cout; g.T = T; g.K = K; g.stride = 1; g.dil = dil; g.pad = pad; g.To = To;
    g.len = nullptr;
    return launch_wgrad_reduce(g, part, dw, eff, l.S, accumulate, s);
}

}  // namespace
}  // namespace nm

using namespace nm;

extern "C" size_t nm_conv1d_fp8_bwd_weight_workspace_bytes(int B, int Cin, int Cout, int T, int K, int stride, int dilation,
                                                           int pad)
{
    int To = 0;
    if (wg_check(B, Cin, Cout, T, K, stride, dilation, pad, &To) != NM_OK) return 0;
    return wg_layout(B, Cin, Cout, To, K, dilation).total;
}

extern "C" int nm_conv1d_bwd_weight_fp8(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad, const void *x,
                                        const float *x_scale, const void *dy, const void *y, const float *g_scale,
                                        const float *scale, float *dw, unsigned flags, void *workspace, size_t workspace_bytes,
                                        void *hip_stream)
{
    int To = 0;
    const int st = wg_check(B, Cin, Cout, T, K, stride, dilation, pad, &To);
    if (st != NM_OK) return st;
    if (!x || !x_scale || !dy || !g_scale || !dw) return NM_ERR_BAD_ARG;
    if (flags & ~(unsigned)(NM_RELU | NM_ACCUM_DW)) return NM_ERR_BAD_ARG;
    const bool relu = (flags & NM_RELU) != 0;
    if (relu && !y) return NM_ERR_BAD_ARG;
    if (((uintptr_t)x & 1) || ((uintptr_t)dy & 1) || ((uintptr_t)y & 1) || ((uintptr_t)dw & 3)) return NM_ERR_BAD_ARG;
    const WgLayout l = wg_layout(B, Cin, Cout, To, K, dilation);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < l.total) return NM_ERR_WORKSPACE;
    const size_t nx = (size_t)B * Cin * T * 2, ny = (size_t)B * Cout * To * 2, nw = (size_t)Cout * Cin * K * 4;
    if (overlap(dw, nw, x, nx) || overlap(dw, nw, dy, ny) || overlap(dw, nw, y, ny) || overlap(dw, nw, workspace, l.total) ||
        overlap(x, nx, workspace, l.total) || overlap(dy, ny, workspace, l.total) || overlap(y, ny, workspace, l.total))
        return NM_ERR_BAD_ARG;

    hipStream_t s = (hipStream_t)hip_stream;
    unsigned char *gq = (unsigned char *)workspace;
    unsigned char *rest = gq + l.gq_bytes;
    if (fp8_launch_quant_g(dy, relu ? y : nullptr, g_scale, gq, nullptr, B, Cout, To, l.Tpg, 0, s) != hipSuccess) return NM_ERR_DEVICE;
    return wgrad_run(B, Cin, Cout, T, To, K, dilation, pad, l, gq, l.Tpg, 0, x, x_scale, g_scale, scale, dw,
                     (flags & NM_ACCUM_DW) != 0, rest, s) == hipSuccess
               ? NM_OK
               : NM_ERR_DEVICE;
}

// ---- both gradients in one call: g is masked and quantised once ------------------------------------------
namespace {
struct BwdLayout {
    WgLayout wg;
    int Tp;  // rows of the shared codes of g: the input gradient's window rows and the weight gradient's units behind padL
    size_t gq_bytes, wtq_bytes, total;
};
BwdLayout bwd_layout(int B, int Cin, int Cout, int T, int To, int K, int dil, int pad)
{
    BwdLayout l;
    l.wg = wg_layout(B, Cin, Cout, To, K, dil);
    const int padL = dil * (K - 1) - pad;
    l.Tp = std::max((T + 159) / 160 * 160 + (K - 1) * dil, l.wg.nu * kUnitT + padL);
    l.gq_bytes = align_up((size_t)B * (Cout / 64) * l.Tp * 64 + kSlack, 256);
    l.wtq_bytes = fp8_packed_weight_bytes(Cout, Cin, K);
    l.total = l.gq_bytes + l.wtq_bytes + l.wg.xq_bytes + l.wg.part_bytes + l.wg.eff_bytes;
    return l;
}
}  // namespace

extern "C" size_t nm_conv1d_fp8_bwd_workspace_bytes(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad)
{
    int To = 0;
    if (wg_check(B, Cin, Cout, T, K, stride, dilation, pad, &To) != NM_OK) return 0;
    return bwd_layout(B, Cin, Cout, T, To, K, dilation, pad).total;
}

extern "C" int nm_conv1d_bwd_fp8(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad, const void *x,
                                 const float *x_scale, const void *dy, const void *y, const float *g_scale, const void *w,
                                 const float *scale, const float *wt_scales, void *dx, void *dres, float *dw, unsigned flags,
                                 void *workspace, size_t workspace_bytes, void *hip_stream)
{
    int To = 0;
    const int st = wg_check(B, Cin, Cout, T, K, stride, dilation, pad, &To);
    if (st != NM_OK) return st;
    if (!x || !x_scale || !dy || !g_scale || !w || !wt_scales || !dx || !dw) return NM_ERR_BAD_ARG;
    if (flags & ~(unsigned)(NM_RELU | NM_ACCUM_DW)) return NM_ERR_BAD_ARG;
    const bool relu = (flags & NM_RELU) != 0;
    if (relu && !y) return NM_ERR_BAD_ARG;
    if (((uintptr_t)w & 15) || ((uintptr_t)x & 1) || ((uintptr_t)dy & 1) || ((uintptr_t)y & 1) || ((uintptr_t)dx & 1) ||
        ((uintptr_t)dres & 1) || ((uintptr_t)dw & 3))
        return NM_ERR_BAD_ARG;
    const BwdLayout l = bwd_layout(B, Cin, Cout, T, To, K, dilation, pad);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < l.total) return NM_ERR_WORKSPACE;
    const size_t nx = (size_t)B * Cin * T * 2, ny = (size_t)B * Cout * To * 2, nw = (size_t)Cout * Cin * K * 2, ndw = nw * 2;
    const void *ins[] = {x, dy, y, w};
    const size_t in_bytes[] = {nx, ny, ny, nw};
    void *outs[] = {dx, dres, dw};
    const size_t out_bytes[] = {nx, ny, ndw};
    for (int o = 0; o < 3; ++o) {
        if (overlap(outs[o], out_bytes[o], workspace, l.total)) return NM_ERR_BAD_ARG;
        for (int i = 0; i < 4; ++i)
            if (overlap(outs[o], out_bytes[o], ins[i], in_bytes[i])) return NM_ERR_BAD_ARG;
        for (int o2 = o + 1; o2 < 3; ++o2)
            if (overlap(outs[o], out_bytes[o], outs[o2], out_bytes[o2])) return NM_ERR_BAD_ARG;
    }
    for (int i = 0; i < 4; ++i)
        if (overlap(ins[i], in_bytes[i], workspace, l.total)) return NM_ERR_BAD_ARG;

    hipStream_t s = (hipStream_t)hip_stream;
    unsigned char *gq = (unsigned char *)workspace;
    unsigned char *wtq = gq + l.gq_bytes;
    unsigned char *rest = wtq + l.wtq_bytes;
    const int padL = dilation * (K - 1) - pad;
    // one pass over dy and y: dres and the codes of g, laid out for the input gradient (row = time + padL)
    if (fp8_launch_quant_g(dy, relu ? y : nullptr, g_scale, gq, dres, B, Cout, To, l.Tp, padL, s) != hipSuccess) return NM_ERR_DEVICE;
    if (fp8_dgrad_run(B, Cin, Cout, T, K, dilation, gq, l.Tp, g_scale, w, scale, wt_scales, dx, wtq, s) != hipSuccess)
        return NM_ERR_DEVICE;
    return wgrad_run(B, Cin, Cout, T, To, K, dilation, pad, l.wg, gq, l.Tp, padL, x, x_scale, g_scale, scale, dw,
                     (flags & NM_ACCUM_DW) != 0, rest, s) == hipSuccess
               ? NM_OK
               : NM_ERR_DEVICE;
}
