// Matrix-core implicit-GEMM engine for the forward pass and the input gradient.
//
// Both passes are the same contraction
//     out[b, m, t] = sum_r sum_k  W'[m, r, k] * in[b, r, t*stride - padL + k*dil]
// with (m, r) = (co, ci), W' = w, padL = pad for the forward pass and, for the input gradient
// of a stride-1 convolution, (m, r) = (ci, co), W'[ci,co,k] = w[co,ci,K-1-k],
// padL = dil*(K-1) - pad, in = dz (materialised by the caller of this engine).
//
// Work decomposition (one workgroup = 4 wavefronts of 64 lanes, one workgroup per CU, one
// wavefront per SIMD with up to 512 registers, persistent over work items):
//   * an output tile is 64 channels x NT*32 time steps of one batch item, accumulated by one
//     wavefront in 2*NT 32x32 MFMA accumulators;
//   * work items: every wavefront first computes some tiles on its own over all reduction chunks
//     (no exchange with the others: the unrolled kernels only), then the four wavefronts of a
//     workgroup share tiles by splitting the reduction channels in chunks of 32 (wave w takes chunks
//     w, w+4, ...), sum the four partial tiles through LDS at the end of the tile and finish a
//     quarter of the rows each; neither form has a workgroup barrier in its main loop;
//   * the activation window of a chunk (32 channels x all time steps the K taps touch) is read
//     once with 16-byte buffer loads along T (lanes outside the row are sent out of range and read
//     zeros) and written to the wavefront's private LDS region transposed to [time][channel], so
//     that every tap is a row offset and each MFMA B fragment (8 consecutive channels of one time
//     step) is one aligned 16-byte LDS read; the next chunk (of this work item or the next one) is
//     staged while the current one is multiplied;
//   * weights are prepacked once per call into MFMA A-fragment order and stream from L2 straight
//     into registers (each lane reads 16 contiguous bytes, a wavefront 1 KiB); a fragment register
//     set is reloaded right after its last use with the data of its next use, across chunks and
//     work items;
//   * tiles are numbered channel-tile fastest, so the workgroups that the hardware places on one
//     XCD (blockIdx mod 8) keep reusing the same slice of the packed weights in that L2.
// Two forms of the main loop: for the tap counts of the Jasper blocks (KT > 0) a chunk is one
// straight-line block of 4*NT*KT MFMAs with every load, LDS write and wait placed between them;
// for any other K (KT == 0) tap pairs run in a loop with staging in out-of-line blocks.
#include "nm_common.h"

#include <type_traits>
#include <utility>

namespace nm {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWaves = 4;
constexpr int kThreads = 64 * kWaves;
constexpr int kTileM = 64;       // output channels per tile
constexpr int kChunk = 32;       // reduction channels per staged chunk
constexpr int kRowBytes = 80;    // LDS row: 32 channels * 2 B + 16 B pad (bank-conflict-free 16 B reads)
constexpr int kRowDwords = kRowBytes / 4;
constexpr int kDumpRows = 8;     // rows at the end of a staging buffer that absorb idle staging writes
constexpr int kMaxLds = 160 * 1024;

struct ConvGemmParams {
    int B, M, R, Tin, Tout, K, Kp, dil, padL;  // Kp: K rounded up to even (packed weights)
    int nmt, nch, ntt, num_tiles;
    int nitems;      // staging items per lane and chunk = ceil(rows/8 * 16 / 64)
    int buf_bytes;   // bytes of one staging buffer: (nitems*32 + kDumpRows) rows of kRowBytes
    int overlap;     // the next tile's first chunk is staged during the current tile
    int full;        // tiles every wavefront computes on its own, over the whole reduction, before the shared ones
    int relu;
    const bf16_t *in;       // [B][R][Tin]
    const int *len_in;      // [B] valid input lengths (samples beyond read as zero) or NULL
    const int *len_out;     // [B] lengths beyond which the output is written as zero, or NULL; the limit of
    int len_out_sub, len_out_div;  // batch item b is ceil((len_out[b] - sub) / div) (phases of a strided gradient)
    const bf16x8 *wp;       // packed weights
    size_t wp_bytes;        // size of the packed weights including the zero pair (< 2 GiB)
    size_t wp_zero;         // offset (in fragments of 16 bytes) of one tap pair of zero weights
    const float *scale;     // epilogue (may be NULL)
    const float *shift;     // epilogue (may be NULL)
    const bf16_t *res;      // epilogue (may be NULL)
    bf16_t *out;            // [B][M][Tout]
    double *stats;          // optional [B*ntt][M][3]: count, mean and centred second moment of the stored outputs of
                            // every (batch item, time tile, channel) -- the partial statistics of a BatchNorm over out
};

__device__ __forceinline__ void wave_lds_fence()
{
    // LDS operations of one wavefront execute in order; this only stops the compiler from
    // moving LDS accesses across the point where other lanes' data must be visible.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Buffer offset beyond any tensor this engine accepts (the host limits them to 1 GiB): the load
// returns zeros.  Small additions to it neither wrap nor come back into range.
constexpr uint32_t kOutOfRange = 0x80000000u;

// The lane number, recomputed where it is needed.  The staging code runs once per chunk inside a
// loop whose registers are all taken; values derived from a long-lived lane id would be spilled
// and their reload would wait for every load in flight.  Two ALU operations avoid that.
__device__ __forceinline__ int fresh_lane()
{
    int l = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    asm volatile("" : "+v"(l));
    return l;
}

// f(integral_constant<0>), f(integral_constant<1>), ... in order
template <class F, int... Is>
__device__ __forceinline__ void for_each_index(F &&f, std::integer_sequence<int, Is...>)
{
    (f(std::integral_constant<int, Is>{}), ...);
}

// Staging items the unrolled kernel built for K taps keeps in registers; 0: no such kernel.
__host__ __device__ constexpr int unrolled_slots(int K) { return K == 29 ? 7 : (K == 11 || K == 13 || K == 17 || K == 21 || K == 25) ? 6 : 0; }

// ---- epilogue shared by the engines of this file ------------------------------------------------
// The sums leave the accumulators through a wave-private LDS tile [16 rows][NT*32] (float32) so that
// each lane finishes 8 consecutive time steps of one channel: one 16-byte residual load, one scale,
// one shift, one 16-byte store per item (rows of out and res are 16-byte aligned: checked by the
// host).  All of these are buffer accesses without branches: absent operands have empty descriptors
// and read zeros, masked lanes go out of range.
template <int NT>
struct Epilogue {
    static constexpr int TN = NT * 32;
    static constexpr int kItems = NT;  // 16 rows * (TN/8) groups / 64 lanes
    __amdgpu_buffer_rsrc_t rs_out, rs_res, rs_scale, rs_shift;
    int M, Tout;
    bool has_scale, relu;
    const int *len_out;  // optional [B]: outputs at t >= ceil((len_out[b] - sub) / div) are written as zero
    int len_sub, len_div;
    double *stats;       // see ConvGemmParams::stats (used by the STATS instances only)
    static constexpr int kStatsOffset = 16 * TN;  // float2 [16 rows][TN/8] behind the tile (in floats)
    static constexpr int kTileBytesWithStats = 16 * TN * (int)sizeof(float) + 16 * (TN / 8) * 2 * (int)sizeof(float);

    struct RowLoads {
        u32x4 rvec[kItems];
        float scv[kItems], shv[kItems];
        uint32_t ooff[kItems];
        int tlim_rel;  // output limit of the batch item relative to the tile's first time step (wave-uniform)
    };
    // first time step of batch item b that is written as zero (Tout without lengths)
    __device__ __forceinline__ int out_limit(int b) const
    {
        if (!len_out) return Tout;
        const int n = (len_out[b] - len_sub + len_div - 1) / len_div;
        return n < 0 ? 0 : (n > Tout ? Tout : n);
    }

    __device__ __forceinline__ void init(const bf16_t *out, const bf16_t *res, const float *scale, const float *shift, int B,
                                         int M_, int Tout_, int relu_, const int *len_out_ = nullptr, int sub = 0, int div = 1,
                                         double *stats_ = nullptr)
    {
        stats = stats_;
        len_out = len_out_;
        len_sub = sub;
        len_div = div < 1 ? 1 : div;
        const int out_bytes = (int)((size_t)B * M_ * Tout_ * 2);
        M = M_;
        Tout = Tout_;
        has_scale = scale != nullptr;
        relu = relu_ != 0;
        rs_out = __builtin_amdgcn_make_buffer_rsrc((void *)out, 0, out_bytes, 0x00020000);
        rs_res = __builtin_amdgcn_make_buffer_rsrc((void *)res, 0, res ? out_bytes : 0, 0x00020000);
        rs_scale = __builtin_amdgcn_make_buffer_rsrc((void *)scale, 0, scale ? M_ * 4 : 0, 0x00020000);
        rs_shift = __builtin_amdgcn_make_buffer_rsrc((void *)shift, 0, shift ? M_ * 4 : 0, 0x00020000);
    }
    // operands of the 16 tile rows whose first channel is m0 (tile row r is channel m0 + r, or
    // m0 + 32*(r/8) + r%8 when `split`: eight rows from each row of blocks); el: the lane number
    __device__ __forceinline__ RowLoads request_rows(int el, int b, int t0, int m0, bool split) const
    {
        RowLoads ld;
        ld.tlim_rel = out_limit(b) - t0;
#pragma unroll
        for (int q = 0; q < kItems; ++q) {
            const int idx = el + 64 * q;
            const int r = idx / (TN / 8), c8 = idx - r * (TN / 8);
            const int m = m0 + (split ? (r >> 3) * 32 + (r & 7) : r);
            const int t = t0 + c8 * 8;
            const bool ok = m < M && t < Tout;
            ld.ooff[q] = ok ? (uint32_t)((((size_t)b * M + m) * Tout + t) * 2) : kOutOfRange;
            const uint32_t moff = ok ? (uint32_t)m * 4u : kOutOfRange;
            ld.rvec[q] = __builtin_amdgcn_raw_buffer_load_b128(rs_res, ld.ooff[q], 0, 0);
            ld.scv[q] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs_scale, moff, 0, 0));
            ld.shv[q] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs_shift, moff, 0, 0));
        }
        return ld;
    }
    // affine, residual, ReLU, rounding and the stores of the 16 rows that sit in the LDS tile tp
    template <bool STATS = false>
    __device__ __forceinline__ void finish_rows(int el, float *tp, const RowLoads &ld) const
    {
#pragma unroll
        for (int q = 0; q < kItems; ++q) {
            const int idx = el + 64 * q;
            const int r = idx / (TN / 8), c8 = idx - r * (TN / 8);
            const f32x4 lo = *reinterpret_cast<const f32x4 *>(tp + r * TN + c8 * 8);
            const f32x4 hi = *reinterpret_cast<const f32x4 *>(tp + r * TN + c8 * 8 + 4);
            const float sc = has_scale ? ld.scv[q] : 1.f;
            u32x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float a0 = (e < 2 ? lo[2 * e] : hi[2 * e - 4]), a1 = (e < 2 ? lo[2 * e + 1] : hi[2 * e - 3]);
                float v0 = a0 * sc + ld.shv[q] + __uint_as_float(ld.rvec[q][e] << 16);
                float v1 = a1 * sc + ld.shv[q] + __uint_as_float(ld.rvec[q][e] & 0xffff0000u);
                if (relu) {
                    v0 = v0 > 0.f ? v0 : 0.f;
                    v1 = v1 > 0.f ? v1 : 0.f;
                }
                o[e] = pack_bf16x2(v0, v1);
            }
            if (len_out) {  // zeros from the output limit on (a uniform branch: nothing to do without lengths)
                const int nvalid = ld.tlim_rel - c8 * 8;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] &= nvalid >= 2 * e + 2 ? 0xffffffffu : (nvalid == 2 * e + 1 ? 0x0000ffffu : 0u);
            }
            __builtin_amdgcn_raw_buffer_store_b128(o, rs_out, ld.ooff[q], 0, 0);
            if constexpr (STATS) {  // sums of the eight stored (rounded) values; an item outside the tensor adds nothing
                float s1 = 0.f, s2 = 0.f;
                if (ld.ooff[q] != kOutOfRange) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float v0 = __uint_as_float(o[e] << 16), v1 = __uint_as_float(o[e] & 0xffff0000u);
                        s1 += v0 + v1;
                        s2 = fmaf(v0, v0, fmaf(v1, v1, s2));
                    }
                }
                reinterpret_cast<f32x2 *>(tp + kStatsOffset)[idx] = f32x2{s1, s2};
            }
        }
    }
    // (STATS instances) after finish_rows<true> and a fence: lane r < 16 adds the TN/8 partial sums of tile row r in
    // order and writes count, mean and centred second moment of that row's part of channel m_of_row
    __device__ __forceinline__ void emit_row_stats(int el, const float *tp, int m_of_row, int part, int t0) const
    {
        if (el >= 16 || m_of_row >= M) return;
        const f32x2 *sp = reinterpret_cast<const f32x2 *>(tp + kStatsOffset) + el * (TN / 8);
        double a = 0.0, b2 = 0.0;
#pragma unroll
        for (int i = 0; i < TN / 8; ++i) {
            const f32x2 v = sp[i];
            a += (double)v[0];
            b2 += (double)v[1];
        }
        const int left = Tout - t0;
        const double n = (double)(left < TN ? (left > 0 ? left : 0) : TN);
        double *o = stats + ((size_t)part * M + m_of_row) * 3;
        o[0] = n;
        o[1] = n > 0 ? a / n : 0.0;
        o[2] = n > 0 ? b2 - a * a / n : 0.0;
    }
    // A whole 64-row tile held by one wavefront (rows m_first .. m_first+63): four rounds of 16 rows
    // (row of blocks mi, accumulator registers 8*gp .. 8*gp+7) through tp; the operands of a round
    // are requested two rounds ahead.
    template <bool STATS = false>
    __device__ __forceinline__ void store_private_tile(const f32x16 (&acc)[2][NT], float *tp, int el, int b, int t0,
                                                       int m_first, int part = 0) const
    {
        const int tcol = el & 31, thalf = el >> 5;
        RowLoads ld[2] = {request_rows(el, b, t0, m_first, false), request_rows(el, b, t0, m_first + 16, false)};
#pragma unroll
        for (int rd = 0; rd < 4; ++rd) {
            const int mi = rd >> 1, gp = rd & 1;
#pragma unroll
            for (int g = 0; g < 2; ++g)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int r = g * 8 + 4 * thalf + j;
#pragma unroll
                    for (int ni = 0; ni < NT; ++ni) tp[r * TN + ni * 32 + tcol] = acc[mi][ni][4 * (2 * gp + g) + j];
                }
            wave_lds_fence();
            finish_rows<STATS>(el, tp, ld[rd & 1]);
            if (rd + 2 < 4) ld[rd & 1] = request_rows(el, b, t0, m_first + (rd + 2) * 16, false);
            wave_lds_fence();
            if constexpr (STATS) emit_row_stats(el, tp, m_first + rd * 16 + el, part, t0);
        }
    }
};

// valid length of batch item b from an optional device array, clipped to [0, T]
__device__ __forceinline__ int clipped_len(const int *len, int b, int T)
{
    if (!len) return T;
    const int n = len[b];
    return n < 0 ? 0 : (n > T ? T : n);
}

struct TileCoords {
    int mt, b, t0, ws_al, off0;
};

// KT > 0: the number of taps is a compile-time constant and a chunk is one straight-line block
// (see the unrolled main loop below); KT == 0: any K, tap pairs in a loop.
// LEN: the instance for calls with per-sample lengths; it alone carries the test for tiles in the padding.
// STATS: the instance that also writes the per-tile statistics of its stored outputs (ConvGemmParams::stats).
template <int NT, int STRIDE, int KT, bool LEN = false, bool STATS = false>
__global__ __launch_bounds__(kThreads) void conv_gemm_kernel(const ConvGemmParams p)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    constexpr int TN = NT * 32;

    const int nitems = p.nitems;                           // staging items per lane and chunk
    const int nmy = (p.nch - wave + kWaves - 1) / kWaves;  // chunks of this wavefront (may be 0)
    const int P = p.Kp >> 1;                               // tap pairs per chunk
    const int tap_bytes = p.dil * kRowBytes;
    const int gstep = (int)(gridDim.x % (unsigned)p.nmt);  // tile += gridDim.x moves the channel tile by this much
    const __amdgpu_buffer_rsrc_t rs_in =
        __builtin_amdgcn_make_buffer_rsrc((void *)p.in, 0, (int)((size_t)p.B * p.R * p.Tin * 2), 0x00020000);

    // staging item `it` of a lane: channel pair pp = lane & 15, time group q0 + 4*it (8 steps)
    auto buf_ptr = [&](int par) { return smem + ((size_t)(par & 1) * kWaves + wave) * p.buf_bytes; };

    auto finish_coords = [&](TileCoords &tc, int tt) {
        tc.t0 = tt * TN;
        const int ws = tc.t0 * STRIDE - p.padL;
        tc.ws_al = (ws >> 3) * 8;  // arithmetic shift: floor
        tc.off0 = ws - tc.ws_al;
    };
    auto tile_coords = [&](int tile, int &tt) {
        TileCoords tc;
        tc.mt = tile % p.nmt;
        const int ntile = tile / p.nmt;
        tc.b = ntile / p.ntt;
        tt = ntile - tc.b * p.ntt;
        finish_coords(tc, tt);
        return tc;
    };
    // Staging loads of chunk c of batch item b, window start ws_al.  The scalar part of the address
    // (batch item, chunk) travels as the scalar offset of the buffer load; lanes whose 8 time steps
    // or whose channel lie outside the tensor get an offset beyond the buffer and read zeros.
    struct StageAddr {
        uint32_t soff, va, vb;  // scalar offset; lane offsets of the even / odd channel (or out of range)
        int tq;                 // first time step of item 0 of this lane
        int tlen;               // valid length of the batch item (Tin without lengths)
        int ws_al;              // time step of window row 0
    };
    auto stage_addr = [&](int b, int c, int ws_al) {
        StageAddr a;
        a.soff = (uint32_t)(((size_t)b * p.R + (size_t)c * kChunk) * p.Tin * 2);
        const int rem = p.R - c * kChunk;  // channels left from this chunk on
        const int l = fresh_lane();
        const int pp = l & 15, q0 = l >> 4;
        const uint32_t base = (uint32_t)(((2 * pp) * p.Tin + 8 * q0 + ws_al) * 2);
        const int tq = ws_al + 8 * q0;
        a.va = 2 * pp < rem ? base : kOutOfRange;
        a.vb = 2 * pp + 1 < rem ? base + (uint32_t)(p.Tin * 2) : kOutOfRange;
        a.tq = tq;
        a.tlen = __builtin_amdgcn_readfirstlane(clipped_len(p.len_in, b, p.Tin));
        a.ws_al = ws_al;
        return a;
    };
    auto stage_load = [&](const StageAddr &a, int it, bool active, u32x4 &xa, u32x4 &xb) {
        const int t = a.tq + 32 * it;
        // a group is requested when it starts inside [0, tlen) (groups are 8-aligned and Tin % 8 == 0, so it
        // then ends inside the row); what lies at or beyond tlen in it is cleared when it is written to LDS
        const bool t_ok = active && (unsigned)t < (unsigned)a.tlen;
        // a lane of a missing channel holds kOutOfRange: adding 64*it keeps it beyond the buffer
        xa = __builtin_amdgcn_raw_buffer_load_b128(rs_in, t_ok ? a.va + (uint32_t)(64 * it) : kOutOfRange, a.soff, 0);
        xb = __builtin_amdgcn_raw_buffer_load_b128(rs_in, t_ok ? a.vb + (uint32_t)(64 * it) : kOutOfRange, a.soff, 0);
    };
    // transposing write of an item: one dword (channel pair) per time step
    auto stage_write = [&](unsigned char *buf, int it, bool active, const u32x4 &xa, const u32x4 &xb) {
        const int l = fresh_lane();
        const int pp = l & 15, q0 = l >> 4;
        const uint32_t row = active ? (uint32_t)(q0 * 8 + it * 32) : (uint32_t)(nitems * 32);  // idle writes go to the dump rows
        uint32_t *dst = reinterpret_cast<uint32_t *>(buf + row * kRowBytes + pp * 4);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            dst[(2 * j) * kRowDwords] = zip_lo16(xa[j], xb[j]);
            dst[(2 * j + 1) * kRowDwords] = zip_hi16(xa[j], xb[j]);
        }
    };
    // the same with the lane's LDS offsets computed by the caller: lane_lds = ((lane/16)*8 rows,
    // channel pair lane%16) for real items, lane_dump = (first dump row, channel pair) for idle ones
    auto stage_write_at = [&](unsigned char *buf, uint32_t lane_lds, uint32_t lane_dump, int it, bool active,
                              const u32x4 &xa, const u32x4 &xb) {
        uint32_t *dst = reinterpret_cast<uint32_t *>(buf + (active ? lane_lds + (uint32_t)(it * 32 * kRowBytes) : lane_dump));
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            dst[(2 * j) * kRowDwords] = zip_lo16(xa[j], xb[j]);
            dst[(2 * j + 1) * kRowDwords] = zip_hi16(xa[j], xb[j]);
        }
    };
    // With lengths, the 8-step group that contains the first padding sample has been staged whole: its
    // rows from the valid length on are cleared here, after the chunk's items are in LDS and before it
    // is read (groups that start in the padding were never requested).  ws_al: time of buffer row 0.
    auto clear_padding_rows = [&](unsigned char *buf, int tlen, int ws_al) {
        const int r0 = tlen - ws_al;                 // first padding row of the window
        const int nr = ((tlen + 7) & ~7) - tlen;     // rows up to the end of its group (0 when tlen % 8 == 0)
        if (tlen < p.Tin && nr > 0 && r0 >= 0 && r0 < nitems * 32) {
            const int l = fresh_lane();
            for (int r = l >> 4; r < nr; r += 4)
                *reinterpret_cast<uint32_t *>(buf + (size_t)(r0 + r) * kRowBytes + (l & 15) * 4) = 0u;
        }
    };
    constexpr int kSlots = KT > 0 ? unrolled_slots(KT) : 6;  // staging items of the next chunk held in registers
    u32x4 sxa[kSlots], sxb[kSlots];
    // a whole chunk, nothing to overlap with (first tile, or every tile without cross-tile staging)
    auto stage_chunk_now = [&](int b, int c, int ws_al, unsigned char *buf) {
        const StageAddr sa = stage_addr(b, c, ws_al);
        for (int it0 = 0; it0 < nitems; it0 += kSlots) {
#pragma unroll
            for (int q = 0; q < kSlots; ++q) stage_load(sa, it0 + q, it0 + q < nitems, sxa[q], sxb[q]);
#pragma unroll
            for (int q = 0; q < kSlots; ++q) stage_write(buf, it0 + q, it0 + q < nitems, sxa[q], sxb[q]);
        }
        clear_padding_rows(buf, sa.tlen, sa.ws_al);
    };

    // ---- weight fragment stream: buffer loads whose scalar offset is a cursor into the packed weights
    const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc((void *)p.wp, 0, (int)p.wp_bytes, 0x00020000);
    const uint32_t w_lane = (uint32_t)lane * 16;
    auto w_load = [&](uint32_t soff, int f) {
        return __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(rs_w, w_lane + (uint32_t)f * 1024u, soff, 0));
    };

    // (KT == 0)  Tap pairs are multiplied alternately from two register sets
    // (afA, afB: [tap 2][ks 2][mi 2] fragments each); a set is reloaded right after its last use
    // with the pair that comes two pairs later in this wavefront's stream, which runs across
    // chunks and tiles, so the loads have about two pairs of MFMA work to arrive.  A tile with an
    // odd number of pairs gets one pair of zero weights, so that tiles start on afA.  The cursor
    // is kept in scalar registers and moves without branches except at a tile end; the loads are
    // buffer loads whose scalar offset is the cursor.
    bf16x8 afA[8], afB[8];
    const int total_pairs = nmy * P;
    const int slots = total_pairs + (total_pairs & 1);  // pairs per tile including the zero pair
    constexpr uint32_t kPairBytes = 512 * 16;           // one tap pair of one chunk
    const uint32_t zero_soff = (uint32_t)(p.wp_zero * 16);
    const uint32_t chunk_jump = kPairBytes * (uint32_t)(1 + (kWaves - 1) * P);  // last pair of a chunk -> first of the next
    auto w_base = [&](int mt) { return (uint32_t)(mt * p.nch + wave) * (uint32_t)P * kPairBytes; };
    int w_tile = blockIdx.x, w_mt = (int)(blockIdx.x % (unsigned)p.nmt), w_pr = 0, w_s = 0;
    bool w_live = w_tile < p.num_tiles && nmy > 0;
    uint32_t w_soff = w_base(w_mt);
    auto w_next = [&]() -> uint32_t {  // offset of the cursor pair; moves the cursor on
        const uint32_t off = (w_live && w_s < total_pairs) ? w_soff : zero_soff;
        ++w_s;
        ++w_pr;
        const bool chunk_end = w_pr == P;
        w_soff += chunk_end ? chunk_jump : kPairBytes;
        w_pr = chunk_end ? 0 : w_pr;
        if (__builtin_expect(w_s == slots, 0)) {  // tile end
            w_s = 0;
            w_pr = 0;
            w_tile += gridDim.x;
            w_mt += gstep;
            w_mt -= w_mt >= p.nmt ? p.nmt : 0;
            w_live = w_live && w_tile < p.num_tiles;
            w_soff = w_base(w_mt);
        }
        return off;
    };
    if constexpr (KT == 0) {
        const uint32_t s0 = w_next();
#pragma unroll
        for (int f = 0; f < 8; ++f) afA[f] = w_load(s0, f);
        const uint32_t s1 = w_next();
#pragma unroll
        for (int f = 0; f < 8; ++f) afB[f] = w_load(s1, f);
    }


    // (KT > 0)  One register set of four fragments ([ks 2][mi 2]) per tap, rotating over NS sets
    // plus one extra set for each of the KT % NS last taps, so that the assignment of taps to sets
    // is the same in every chunk.  A set is reloaded right after its last multiplication with the
    // tap that uses it next: NS taps later in this chunk, or in the next chunk of this wavefront's
    // stream (w_cur / w_nxt: byte offsets of the current and the next chunk), which runs across
    // tiles.  The zero tap that pads an odd K in the packed tensor is never touched.
    constexpr int NS = 4, NQ = KT / NS, NR = KT % NS, NSETS = KT > 0 ? NS + NR : 1;
    bf16x8 wf[NSETS][4];
    constexpr uint32_t kTapBytes = 4 * 64 * 16;
    const uint32_t chunk_bytes = (uint32_t)p.Kp * kTapBytes;
    auto chunk_off = [&](int mt, int c) { return (uint32_t)(mt * p.nch + c) * chunk_bytes; };
    uint32_t w_cur = 0;

    Epilogue<NT> epi;
    epi.init(p.out, p.res, p.scale, p.shift, p.B, p.M, p.Tout, p.relu, p.len_out, p.len_out_sub, p.len_out_div, p.stats);

    int cc = 0;  // chunks this wavefront has consumed so far: chunk number cc uses buffer cc & 1
    // accumulators: zero here, and again in the epilogue as soon as a tile's values have been handed over
    f32x16 acc[2][NT];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < NT; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

    // ---- work items of this wavefront.  First `full` private tiles: tile k*4G + wave*G + blockIdx
    // (G workgroups), computed by this wavefront alone over every reduction chunk, so they need no
    // exchange between wavefronts; then the shared tiles 4G*full + blockIdx + j*G, whose reduction
    // chunks the four wavefronts split (chunk wave, wave+4, ...) and whose partial sums they add
    // through LDS.  With 1280 tiles on 256 CUs that is one private tile per wavefront and one
    // shared tile per workgroup: four fifths of the work skip the exchange.  Both numberings keep
    // tile mod (channel tiles) = blockIdx mod (channel tiles) when G is a multiple of it, i.e.
    // one slice of the packed weights per XCD.
    const int G = (int)gridDim.x;
    const int nA = KT > 0 ? p.full : 0;
    const int tilesA = nA * kWaves * G;
    auto item_tile = [&](int k) {
        return k < nA ? (k * kWaves + wave) * G + (int)blockIdx.x : tilesA + (int)blockIdx.x + (k - nA) * G;
    };
    auto first_chunk = [&](bool priv) { return priv ? 0 : wave; };
    int item = 0, tile = item_tile(0);
    int tt_unused = 0;
    TileCoords tc_next = tile_coords(tile < p.num_tiles ? tile : 0, tt_unused);
    if (tile < p.num_tiles && p.overlap && (nA > 0 || nmy > 0))
        stage_chunk_now(tc_next.b, first_chunk(nA > 0), tc_next.ws_al, buf_ptr(0));
    if constexpr (KT > 0) {
        if (tile < p.num_tiles && (nA > 0 || nmy > 0)) {
            w_cur = chunk_off(tc_next.mt, first_chunk(nA > 0));
#pragma unroll
            for (int k = 0; k < NS; ++k)
#pragma unroll
                for (int f = 0; f < 4; ++f) wf[k][f] = w_load(w_cur + (uint32_t)k * kTapBytes, f);
#pragma unroll
            for (int e = 0; e < NR; ++e)
#pragma unroll
                for (int f = 0; f < 4; ++f) wf[NS + e][f] = w_load(w_cur + (uint32_t)(NS * NQ + e) * kTapBytes, f);
        }
    }

    for (; tile < p.num_tiles; ++item) {
        const bool priv = item < nA;
        const bool next_priv = item + 1 < nA;
        const int next_tile = item_tile(item + 1);
        const TileCoords tc = tc_next;
        const bool next_ok = p.overlap && next_tile < p.num_tiles;
        tc_next = tile_coords(next_tile < p.num_tiles ? next_tile : tile, tt_unused);
        const TileCoords tn = tc_next;
        tile = next_tile;

        if (!p.overlap && nmy > 0) stage_chunk_now(tc.b, wave, tc.ws_al, buf_ptr(cc));

        if constexpr (KT > 0) {
            // A tile that lies wholly in the padding of its batch item -- every input sample its window covers is at or
            // beyond the valid length (forward), or every output position is at or beyond the output limit (input
            // gradient) -- needs no arithmetic: its accumulators stay zero (the staged window is zero) or its outputs are
            // written as zeros.  It still runs ONE chunk, which keeps the pipeline (staging of the next item's first
            // chunk, weight sets) exactly as it is for a live tile.
            bool dead = false;
            if constexpr (LEN) {
                if (p.len_in) dead = tc.t0 * STRIDE - p.padL >= clipped_len(p.len_in, tc.b, p.Tin);
                if (p.len_out) dead = dead || tc.t0 >= epi.out_limit(tc.b);
            }
            const int n_full = priv ? p.nch : nmy;  // chunks of this item for this wavefront
            const int n_ch = dead ? min(n_full, 1) : n_full;
            auto chunk_of = [&](int i) { return priv ? i : wave + kWaves * i; };
            if (n_ch > 0) {
                // ---- unrolled main loop: one chunk (KT taps, 4*NT*KT MFMAs) is a single straight-line
                // block, so staging loads, staging writes, weight reloads and LDS reads are placed
                // between the MFMAs by the compiler and every wait counts exactly what is in flight.
                // The six staging items of the next chunk are requested one per tap during the
                // first six taps and written one per tap during the last six.
                static_assert(KT == 0 || KT >= 11, "the staging schedule needs eleven taps");
                const int ll = fresh_lane();
                const int lane_off = ((ll & 31) * STRIDE + tc.off0) * kRowBytes + (ll >> 5) * 16;
                const uint32_t lane_lds = (uint32_t)(((ll >> 4) * 8) * kRowBytes + (ll & 15) * 4);
                const uint32_t lane_dump = (uint32_t)(nitems * 32 * kRowBytes + (ll & 15) * 4);
                for (int ci = 0; ci < n_ch; ++ci) {
                    const bool more = ci + 1 < n_ch;
                    const bool has_t = more || next_ok;  // is there a chunk to stage for
                    const int c_nxt = more ? chunk_of(ci + 1) : first_chunk(next_priv);
                    const uint32_t w_nxt = has_t ? chunk_off(more ? tc.mt : tn.mt, c_nxt) : w_cur;
                    StageAddr sa = stage_addr(more ? tc.b : tn.b, c_nxt, more ? tc.ws_al : tn.ws_al);
                    sa.va = has_t ? sa.va : kOutOfRange;
                    sa.vb = has_t ? sa.vb : kOutOfRange;
                    const unsigned char *bbase = buf_ptr(cc) + lane_off;
                    unsigned char *nxt = buf_ptr(cc + 1);
                    bf16x8 b0[NT], b1[NT];
                    auto read_b = [&](bf16x8(&dst)[NT], int k, int ks) {
                        const unsigned char *brow = bbase + (size_t)k * tap_bytes + ks * 32;
#pragma unroll
                        for (int ni = 0; ni < NT; ++ni)
                            dst[ni] = *reinterpret_cast<const bf16x8 *>(brow + ni * 32 * STRIDE * kRowBytes);
                    };
                    auto mma = [&](const bf16x8 &a0, const bf16x8 &a1, const bf16x8(&bf)[NT]) {
#pragma unroll
                        for (int ni = 0; ni < NT; ++ni)
                            acc[0][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, bf[ni], acc[0][ni], 0, 0, 0);
#pragma unroll
                        for (int ni = 0; ni < NT; ++ni)
                            acc[1][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, bf[ni], acc[1][ni], 0, 0, 0);
                    };
                    wave_lds_fence();  // the staged chunk is visible to every lane
                    read_b(b0, 0, 0);
                    auto tap = [&](auto kc) {
                        constexpr int k = decltype(kc)::value;
                        constexpr int set = k < NS * NQ ? k % NS : NS + (k - NS * NQ);
                        // the tap that uses this set next
                        constexpr bool same_chunk = k < NS * NQ && k + NS < NS * NQ;
                        constexpr int next_tap = same_chunk ? k + NS : (k < NS * NQ ? k % NS : k);
                        const uint32_t src = (same_chunk ? w_cur : w_nxt) + (uint32_t)next_tap * kTapBytes;
                        // (a scheduling barrier per k-step keeps every load where it is written: the
                        // compiler would otherwise move the reloads down to their use)
                        read_b(b1, k, 1);
                        mma(wf[set][0], wf[set][1], b0);
                        wf[set][0] = w_load(src, 0);
                        wf[set][1] = w_load(src, 1);
                        __builtin_amdgcn_sched_barrier(0);
                        if constexpr (k + 1 < KT) read_b(b0, k + 1, 0);
                        mma(wf[set][2], wf[set][3], b1);
                        wf[set][2] = w_load(src, 2);
                        wf[set][3] = w_load(src, 3);
                        if constexpr (k < kSlots) stage_load(sa, k, k < nitems, sxa[k], sxb[k]);
                        if constexpr (k >= KT - kSlots) {
                            constexpr int it = k - (KT - kSlots);
                            stage_write_at(nxt, lane_lds, lane_dump, it, has_t && it < nitems, sxa[it], sxb[it]);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    };
                    for_each_index(tap, std::make_integer_sequence<int, (KT > 0 ? KT : 1)>{});
                    if (has_t) clear_padding_rows(nxt, sa.tlen, sa.ws_al);
                    w_cur = w_nxt;
                    ++cc;
                }
            }
        } else if (nmy > 0) {
            // ---- main loop over (chunk, tap pair): 4 k-steps of 16 channels = 8*NT MFMAs per pair
            // (the packed weights pad an odd K with one zero tap).  All MFMAs sit in this loop.
            const int ll = fresh_lane();
            const int lane_off = ((ll & 31) * STRIDE + tc.off0) * kRowBytes + (ll >> 5) * 16;
            int ci_ord = 0, pr = 0;
            // where the staging items of this chunk go: the next chunk of this tile, or the first
            // chunk of the next tile, or nowhere
            bool has_t = nmy > 1 || next_ok;
            const bool async_stage = P > kSlots / 2;  // shorter chunks stage the next one at their end
            int t_b = nmy > 1 ? tc.b : tn.b, t_ws = nmy > 1 ? tc.ws_al : tn.ws_al, t_c = nmy > 1 ? wave + kWaves : wave;
            const unsigned char *bbase = buf_ptr(cc) + lane_off;
            unsigned char *nxt = buf_ptr(cc + 1);
            bf16x8 b0[NT], b1[NT];
            auto read_b = [&](bf16x8(&dst)[NT], int k, int ks) {
                const unsigned char *brow = bbase + (size_t)k * tap_bytes + ks * 32;
#pragma unroll
                for (int ni = 0; ni < NT; ++ni)
                    dst[ni] = *reinterpret_cast<const bf16x8 *>(brow + ni * 32 * STRIDE * kRowBytes);
            };
            auto mma = [&](const bf16x8 &a0, const bf16x8 &a1, const bf16x8(&bf)[NT]) {
#pragma unroll
                for (int ni = 0; ni < NT; ++ni) acc[0][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, bf[ni], acc[0][ni], 0, 0, 0);
#pragma unroll
                for (int ni = 0; ni < NT; ++ni) acc[1][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, bf[ni], acc[1][ni], 0, 0, 0);
            };
            // one tap pair from the register set `af`; `real` is false only for the zero pad pair
            auto do_pair = [&](bf16x8(&af)[8], bool real) {
                // Staging of the next chunk: its items are requested at the first pair of this chunk
                // (static register slots) and written to LDS two at a time at the top of the last
                // three pairs, so the loads have most of a chunk (several microseconds) to arrive.
                // The writes come first in program order and only in pairs after the first, which
                // lets the wait they need leave the latest weight loads in flight.
                if (__builtin_expect(has_t && async_stage && pr >= P - kSlots / 2, 0)) {
#pragma unroll
                    for (int gq = 0; gq < kSlots / 2; ++gq) {
                        if (pr == P - kSlots / 2 + gq) {
#pragma unroll
                            for (int e = 0; e < 2; ++e)
                                if (2 * gq + e < nitems) stage_write(nxt, 2 * gq + e, true, sxa[2 * gq + e], sxb[2 * gq + e]);
                        }
                    }
                }
                if (__builtin_expect(pr == 0 && has_t && async_stage, 0)) {
                    const StageAddr sa = stage_addr(t_b, t_c, t_ws);
#pragma unroll
                    for (int it = 0; it < kSlots; ++it)
                        if (it < nitems) stage_load(sa, it, true, sxa[it], sxb[it]);
                }
                const int k = 2 * pr;
                read_b(b1, k, 1);
                mma(af[0], af[1], b0);
                const uint32_t wn = w_next();
                af[0] = w_load(wn, 0);
                af[1] = w_load(wn, 1);
                read_b(b0, k + 1, 0);
                mma(af[2], af[3], b1);
                af[2] = w_load(wn, 2);
                af[3] = w_load(wn, 3);
                read_b(b1, k + 1, 1);
                mma(af[4], af[5], b0);
                af[4] = w_load(wn, 4);
                af[5] = w_load(wn, 5);
                read_b(b0, min(k + 2, p.Kp - 1), 0);
                mma(af[6], af[7], b1);
                af[6] = w_load(wn, 6);
                af[7] = w_load(wn, 7);
                if (__builtin_expect(real && ++pr == P, 0)) {  // end of a chunk
                    if (has_t) {
                        // windows longer than the register slots, or everything when chunks are short
                        for (int it = async_stage ? kSlots : 0; it < nitems; ++it) {
                            u32x4 ya, yb;
                            const StageAddr sl = stage_addr(t_b, t_c, t_ws);
                            stage_load(sl, it, true, ya, yb);
                            stage_write(nxt, it, true, ya, yb);
                        }
                        clear_padding_rows(nxt, clipped_len(p.len_in, t_b, p.Tin), t_ws);
                    }
                    ++ci_ord;
                    ++cc;
                    pr = 0;
                    has_t = false;
                    if (ci_ord < nmy) {
                        const bool more = ci_ord + 1 < nmy;
                        has_t = more || next_ok;
                        t_b = more ? tc.b : tn.b;
                        t_ws = more ? tc.ws_al : tn.ws_al;
                        t_c = more ? wave + kWaves * (ci_ord + 1) : wave;
                        bbase = buf_ptr(cc) + lane_off;
                        nxt = buf_ptr(cc + 1);
                        wave_lds_fence();
                        read_b(b0, 0, 0);
                    }
                }
            };
            wave_lds_fence();
            read_b(b0, 0, 0);
            for (int g = 0; g < total_pairs; g += 2) {
                do_pair(afA, true);
                do_pair(afB, g + 1 < total_pairs);
            }
        }

        // ---- epilogue (see Epilogue above).  The LDS tile lies in a staging buffer that holds no
        // live data: when the next item's first chunk has been staged into parity cc & 1, the other one.
        const int el = fresh_lane();  // nothing lane-dependent is kept alive across the main loop for this
        const int dead_par = next_ok ? ((cc & 1) ^ 1) : 0;
        float *tp = reinterpret_cast<float *>(smem + ((size_t)dead_par * kWaves + wave) * p.buf_bytes);
        const int tcol = el & 31, thalf = el >> 5;

        if (priv) {
            // A private tile: this wavefront holds all 64 rows.
            epi.template store_private_tile<STATS>(acc, tp, el, tc.b, tc.t0, tc.mt * kTileM, tc.b * p.ntt + tc.t0 / TN);
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int ni = 0; ni < NT; ++ni)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;
        } else {
            // A shared tile.  Wave g finishes accumulator rows [4g, 4g+4) of every 32x32 block: each
            // wave hands the other three quarters over through LDS, one row of blocks (mi) per
            // round; the scratch is the dead-parity staging buffers of all four wavefronts.  The
            // operands of this wave's 16 rows are requested before the sum.
            const auto ld = epi.request_rows(el, tc.b, tc.t0, tc.mt * kTileM + 8 * wave, true);
            f32x4 *red = reinterpret_cast<f32x4 *>(smem + (size_t)dead_par * kWaves * p.buf_bytes);
            __syncthreads();  // every wavefront has left the main loop
            // One copy of the exchange per wave number, so that the accumulator quarters are named
            // statically and nothing has to be merged between the copies.
            auto exchange = [&](auto wave_const) {
                constexpr int Gw = decltype(wave_const)::value;
                f32x4 own[2][NT];
#pragma unroll
                for (int mi = 0; mi < 2; ++mi) {
#pragma unroll
                    for (int g = 0; g < kWaves; ++g) {
                        if (g != Gw) {
                            const int slot = Gw < g ? Gw : Gw - 1;  // position of this wave among the three senders of quarter g
#pragma unroll
                            for (int ni = 0; ni < NT; ++ni) {
                                f32x4 v = {acc[mi][ni][4 * g], acc[mi][ni][4 * g + 1], acc[mi][ni][4 * g + 2],
                                           acc[mi][ni][4 * g + 3]};
                                red[((g * 3 + slot) * NT + ni) * 64 + el] = v;
                            }
                        }
                    }
                    __syncthreads();
#pragma unroll
                    for (int ni = 0; ni < NT; ++ni)
                        own[mi][ni] = f32x4{acc[mi][ni][4 * Gw], acc[mi][ni][4 * Gw + 1], acc[mi][ni][4 * Gw + 2],
                                            acc[mi][ni][4 * Gw + 3]};
#pragma unroll
                    for (int ni = 0; ni < NT; ++ni)  // this row of blocks is done: ready for the next tile
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;
#pragma unroll
                    for (int slot = 0; slot < 3; ++slot) {
#pragma unroll
                        for (int ni = 0; ni < NT; ++ni) own[mi][ni] += red[((Gw * 3 + slot) * NT + ni) * 64 + el];
                    }
                    __syncthreads();  // scratch is reused by the next round / the transpose tile / the next tile's staging
                }
#pragma unroll
                for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int r = mi * 8 + 4 * thalf + j;
#pragma unroll
                        for (int ni = 0; ni < NT; ++ni) tp[r * TN + ni * 32 + tcol] = own[mi][ni][j];
                    }
            };
            switch (wave) {
            case 0: exchange(std::integral_constant<int, 0>{}); break;
            case 1: exchange(std::integral_constant<int, 1>{}); break;
            case 2: exchange(std::integral_constant<int, 2>{}); break;
            default: exchange(std::integral_constant<int, 3>{}); break;
            }
            wave_lds_fence();
            epi.template finish_rows<STATS>(el, tp, ld);
            wave_lds_fence();
            if constexpr (STATS) {  // this wavefront's rows: channels 8*wave .. +7 of both row blocks of the tile
                epi.emit_row_stats(el, tp, tc.mt * kTileM + 8 * wave + (el >> 3) * 32 + (el & 7), tc.b * p.ntt + tc.t0 / TN,
                                   tc.t0);
                wave_lds_fence();
            }
        }
    }
}

// ---- K = 1 (pointwise convolution: a plain GEMM  out[b] = W' . in[b]) ----------------------------
// With one tap an activation element is used for one output row tile only, so the private staging
// of conv_gemm_kernel (each wavefront its own chunk) is staging-bound and reads the activations
// once per 64 output channels.  Here the four wavefronts of a workgroup take four 64-channel row
// tiles of the same 160 time steps and share the staged activations: a workgroup tile is
// 256 channels x 160 steps, the reduction runs in stages of 128 channels ([time][channel] in LDS,
// 272-byte rows, written cooperatively by all 256 lanes with the same transposing scheme), one
// workgroup barrier per stage.  Stages form one stream across the tiles of a workgroup: stage n is
// requested during stage n-2 (two register sets), written to LDS buffer n&1 during stage n-1, and
// each wavefront reloads a weight fragment right after its use with the next stage's.  Every
// wavefront finishes its own rows (no exchange); the LDS tile of that epilogue lies in the buffer
// the tile's last stage has just used.  Packed weights: the layout of prepack_kernel (Kp = 2, tap 0).
// (The figures above are those of the shape (2, 5, 128); PwShape lists the shapes.)
// The shape of a workgroup tile: every wavefront owns MI row blocks (32 channels each) x NT time blocks and the
// reduction runs in stages of SC channels.  (2, 5, 128): 256 channels x 160 steps, 512 LDS bytes read per MFMA;
// (4, 4, 64): 512 channels x 128 steps, all 256 accumulation registers in use, 256 LDS bytes read and half the
// staging work per MFMA -- the faster one wherever its tiles fit the tensor.
template <int MI, int NT, int SC>
struct PwShape {
    static_assert(MI % 2 == 0 && SC % kChunk == 0, "whole 64-row tiles, whole chunks");
    static constexpr int kRowTiles = MI / 2;                 // 64-row tiles of the packed weights per wavefront
    static constexpr int kChunks = SC / kChunk;              // chunks of 32 channels per stage
    static constexpr int kRowBytes = SC * 2 + 16;            // 272 / 144: any 16 consecutive rows cover all banks with 16-byte reads
    static constexpr int kRows = NT * 32;                    // time steps per tile
    static constexpr int kBufBytes = kRows * kRowBytes;
    static constexpr int kPairBlocks = SC / 32;              // blocks of 16 channel pairs
    static constexpr int kItems = NT * kPairBlocks / kWaves; // staging items per lane and stage (blocks of 16 pairs x 4 time groups)
    static_assert(kItems * kWaves == NT * kPairBlocks && kItems <= 2 * kChunks, "one staging item per k-step");
    static constexpr int kEpiBytes = kWaves * 16 * kRows * (int)sizeof(float);  // the four epilogue tiles
    static constexpr bool kEpiInBuf = kEpiBytes <= kBufBytes;  // they fit the buffer the tile's last stage has used
    static constexpr size_t kLds = 2 * (size_t)kBufBytes + (kEpiInBuf ? 0 : kEpiBytes);
};

// LEN: the launch carries input lengths (a staged group may straddle the valid length of its item).
template <bool LEN, int MI, int NT, int SC>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1))) void pointwise_gemm_kernel(const ConvGemmParams p)
{
    using Sh = PwShape<MI, NT, SC>;
    constexpr int TN = NT * 32, RT = Sh::kRowTiles;
    constexpr int kPwStageCh = SC, kPwChunks = Sh::kChunks, kPwRowBytes = Sh::kRowBytes, kPwBufBytes = Sh::kBufBytes;
    constexpr int kPwItems = Sh::kItems, kPB = Sh::kPairBlocks;
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int T = p.Tout;                                  // == p.Tin
    const int nmt4 = (p.nmt + kWaves * RT - 1) / (kWaves * RT);  // workgroup row tiles
    const int nst = (p.R + kPwStageCh - 1) / kPwStageCh;   // stages per tile
    const int ncols = p.ntt * p.B;                         // time tiles of all batch items
    const int ntiles = nmt4 * ncols;
    const int G = (int)gridDim.x;
    // Which tiles a workgroup takes.  Grouped (G a multiple of 8*nmt4): the nmt4 workgroups that need
    // the same activations run on the same XCD at the same time (XCD = blockIdx % 8), so those are
    // fetched into that L2 once: workgroup x = 8*j + c takes row tile j % nmt4 of time tile
    // it*(G/nmt4) + 8*(j/nmt4) + c in its it-th turn.  Otherwise tile x + it*G, row tile fastest.
    const bool grouped = G % (8 * nmt4) == 0;
    const int per_turn = grouped ? G / nmt4 : 0;
    const int col0 = grouped ? 8 * (((int)blockIdx.x >> 3) / nmt4) + ((int)blockIdx.x & 7) : 0;
    const int my_tiles = grouped ? (col0 < ncols ? (ncols - col0 + per_turn - 1) / per_turn : 0)
                                 : ((int)blockIdx.x < ntiles ? (ntiles - (int)blockIdx.x + G - 1) / G : 0);
    const int total = my_tiles * nst;                      // stages in this workgroup's stream
    if (total == 0) return;

    const __amdgpu_buffer_rsrc_t rs_in =
        __builtin_amdgcn_make_buffer_rsrc((void *)p.in, 0, (int)((size_t)p.B * p.R * T * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc((void *)p.wp, 0, (int)p.wp_bytes, 0x00020000);
    Epilogue<NT> epi;
    epi.init(p.out, p.res, p.scale, p.shift, p.B, p.M, p.Tout, p.relu, p.len_out, p.len_out_sub, p.len_out_div);

    // position in the stream: tile coordinates and stage; advanced without divisions except at a tile change
    struct Pos {
        bool valid;
        int tile, mt4, b, t0, s;  // tile: which turn of this workgroup
        int tlen;                 // valid input length of batch item b (T without lengths)
    };
    auto decode = [&](Pos &q) {  // (mt4, b, t0) of turn q.tile; wave-uniform, pinned to scalar registers
        int ntile, mt4;
        if (grouped) {
            ntile = q.tile * per_turn + col0;
            mt4 = ((int)blockIdx.x >> 3) % nmt4;
            q.valid = ntile < ncols;
        } else {
            const int tile = (int)blockIdx.x + q.tile * G;
            q.valid = tile < ntiles;
            ntile = tile / nmt4;
            mt4 = tile - ntile * nmt4;
        }
        ntile = q.valid ? ntile : 0;
        const int b = ntile / p.ntt;
        q.mt4 = __builtin_amdgcn_readfirstlane(mt4);
        q.b = __builtin_amdgcn_readfirstlane(b);
        q.t0 = __builtin_amdgcn_readfirstlane((ntile - b * p.ntt) * TN);
        q.tlen = __builtin_amdgcn_readfirstlane(clipped_len(p.len_in, b, T));
    };
    auto advance = [&](Pos &q) {
        if (++q.s == nst) {
            q.s = 0;
            q.tile += 1;
            decode(q);
        }
    };
    // ---- activations: the stage is SC/2 channel pairs x 4*NT time groups (8 steps each), cut into blocks
    // of 16 pairs x 4 groups; block kItems*wave + it is item `it` of this wavefront: lane = (group, pair), so
    // a load instruction reads 16 rows x 64 contiguous bytes and a write instruction 16 consecutive
    // dwords in each of 4 rows
    u32x4 xa0[kPwItems], xb0[kPwItems], xa1[kPwItems], xb1[kPwItems];
    auto x_load_item = [&](const Pos &q, int it, u32x4 &xa, u32x4 &xb) {
        const uint32_t soff = (uint32_t)(q.b * p.R + q.s * kPwStageCh) * (uint32_t)(T * 2);  // < 2^30: checked by the host
        const int rem = p.R - q.s * kPwStageCh;  // channels left from this stage on
        const int blk = wave * kPwItems + it;
        const int pair = (blk % kPB) * 16 + (lane & 15), tg = (blk / kPB) * 4 + (lane >> 4);
        const int t = q.t0 + 8 * tg;
        const bool ok = q.valid && t < q.tlen;  // groups that start inside the valid length (T % 8 == 0: they end inside the row)
        const uint32_t off = (uint32_t)(((2 * pair) * T + t) * 2);
        xa = __builtin_amdgcn_raw_buffer_load_b128(rs_in, (ok && 2 * pair < rem) ? off : kOutOfRange, soff, 0);
        xb = __builtin_amdgcn_raw_buffer_load_b128(rs_in, (ok && 2 * pair + 1 < rem) ? off + (uint32_t)(T * 2) : kOutOfRange, soff, 0);
    };
    auto x_load = [&](const Pos &q, u32x4(&xa)[kPwItems], u32x4(&xb)[kPwItems]) {
#pragma unroll
        for (int it = 0; it < kPwItems; ++it) x_load_item(q, it, xa[it], xb[it]);
    };
    // (time steps at or beyond the valid length of the stage's batch item are written as zeros)
    auto x_write_item = [&](unsigned char *buf, const Pos &q, int it, const u32x4 &xa, const u32x4 &xb) {
        const int blk = wave * kPwItems + it;
        const int pair = (blk % kPB) * 16 + (lane & 15), tg = (blk / kPB) * 4 + (lane >> 4);
        uint32_t *dst = reinterpret_cast<uint32_t *>(buf + (8 * tg) * kPwRowBytes + pair * 4);
        const int nvalid = q.tlen - (q.t0 + 8 * tg);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if constexpr (LEN) {
                dst[(2 * j) * (kPwRowBytes / 4)] = nvalid > 2 * j ? zip_lo16(xa[j], xb[j]) : 0u;
                dst[(2 * j + 1) * (kPwRowBytes / 4)] = nvalid > 2 * j + 1 ? zip_hi16(xa[j], xb[j]) : 0u;
            } else {  // T % 8 == 0: a group lies wholly inside the row or was loaded as zeros
                dst[(2 * j) * (kPwRowBytes / 4)] = zip_lo16(xa[j], xb[j]);
                dst[(2 * j + 1) * (kPwRowBytes / 4)] = zip_hi16(xa[j], xb[j]);
            }
        }
    };
    // ---- weights of this wavefront's 32*MI rows: [chunk of the stage][ks][mi], reloaded in place
    bf16x8 wf[kPwChunks][2][MI];
    const uint32_t w_lane = (uint32_t)lane * 16;
    const uint32_t chunk_bytes = (uint32_t)p.Kp * 4 * 64 * 16;
    auto w_off = [&](const Pos &q, int j, int rt) {  // byte offset of chunk j of the stage for row tile rt of this wavefront, or out of range
        const int mt = (q.mt4 * kWaves + wave) * RT + rt, c = q.s * kPwChunks + j;
        return (q.valid && mt < p.nmt && c < p.nch) ? (uint32_t)(mt * p.nch + c) * chunk_bytes : kOutOfRange;
    };
    auto w_load = [&](uint32_t off, int f) {
        // an absent chunk: offset beyond the packed tensor (the hardware returns zeros)
        return __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(rs_w, w_lane + (uint32_t)f * 1024u + (off == kOutOfRange ? kOutOfRange : 0u),
                                                                                off == kOutOfRange ? 0u : off, 0));
    };

    f32x16 acc[RT][2][NT];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NT; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi >> 1][mi & 1][ni][r] = 0.f;

    // The accumulators stay in accumulation registers across stages: without these empty statements at
    // every place where the loop-carried value is defined, the allocator moves all of them to vector
    // registers and back at every loop header.
    auto pin_acc = [&]() {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NT; ++ni) asm volatile("" : "+a"(acc[mi >> 1][mi & 1][ni]));
    };
    pin_acc();
    // ---- prologue: stage 0 into buffer 0, stage 1 into the second register set, weights of stage 0
    Pos q0, q1, q2;  // this stage, the next, the one after
    q0.tile = 0;  // turn number
    q0.s = 0;
    decode(q0);
    q1 = q0;
    advance(q1);
    q2 = q1;
    advance(q2);
    {
#pragma unroll
        for (int j = 0; j < kPwChunks; ++j)
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                const uint32_t o = w_off(q0, j, rt);
#pragma unroll
                for (int f = 0; f < 4; ++f) wf[j][f >> 1][2 * rt + (f & 1)] = w_load(o, f);
            }
        x_load(q0, xa0, xb0);
        x_load(q1, xa1, xb1);
#pragma unroll
        for (int it = 0; it < kPwItems; ++it) x_write_item(smem, q0, it, xa0[it], xb0[it]);
        __syncthreads();
    }
    const int lane_off = (lane & 31) * kPwRowBytes + (lane >> 5) * 16;
    // one stage: k even uses buffer 0 / requests into set 0 (whose data, stage k, is in LDS already) and
    // writes set 1 (stage k+1) into buffer 1; k odd the other way round
    auto stage = [&](unsigned char *cur, unsigned char *nxt, u32x4(&xa)[kPwItems], u32x4(&xb)[kPwItems],
                     const u32x4(&xo_a)[kPwItems], const u32x4(&xo_b)[kPwItems]) {
        const Pos q = q0;
        const unsigned char *bbase = cur + lane_off;
        bf16x8 b0[NT], b1[NT];
        pin_acc();
        auto read_b = [&](bf16x8(&dst)[NT], int j, int ks) {
#pragma unroll
            for (int ni = 0; ni < NT; ++ni)
                dst[ni] = *reinterpret_cast<const bf16x8 *>(bbase + ni * 32 * kPwRowBytes + j * 64 + ks * 32);
        };
        read_b(b0, 0, 0);
        // one k-step: MI*NT MFMAs from fragments (j, ks), which are then reloaded with the next stage's
        auto kstep = [&](int j, int ks, const bf16x8(&bc)[NT], const uint32_t(&o)[RT]) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NT; ++ni)
                    acc[mi >> 1][mi & 1][ni] =
                        __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[j][ks][mi], bc[ni], acc[mi >> 1][mi & 1][ni], 0, 0, 0);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) wf[j][ks][mi] = w_load(o[mi >> 1], ks * 2 + (mi & 1));
            // the writes of the next stage ride on the last k-steps (its loads are two stages old)
            constexpr int first = 2 * kPwChunks - kPwItems;
            const int step = 2 * j + ks;
            if (step < kPwItems) x_load_item(q2, step, xa[step], xb[step]);  // the stage after the next, one item per k-step
            if (step >= first) x_write_item(nxt, q1, step - first, xo_a[step - first], xo_b[step - first]);
            __builtin_amdgcn_sched_barrier(0);  // keeps every load where it is written
        };
#pragma unroll
        for (int j = 0; j < kPwChunks; ++j) {
            uint32_t o[RT];
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) o[rt] = w_off(q1, j, rt);
            read_b(b1, j, 1);
            kstep(j, 0, b0, o);
            if (j + 1 < kPwChunks) read_b(b0, j + 1, 0);
            kstep(j, 1, b1, o);
        }
        __syncthreads();  // stage k+1 is complete in LDS; buffer `cur` may be overwritten
        if (q.valid && q.s == nst - 1) {
            // the tile is finished: this wavefront's rows leave through its slice of `cur` (or of the
            // region behind the two buffers where the four slices do not fit one buffer)
            const int el = fresh_lane();
            unsigned char *ebase = Sh::kEpiInBuf ? cur : smem + 2 * kPwBufBytes;
            float *tp = reinterpret_cast<float *>(ebase + (size_t)wave * 16 * TN * sizeof(float));
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
                epi.store_private_tile(acc[rt], tp, el, q.b, q.t0, ((q.mt4 * kWaves + wave) * RT + rt) * kTileM);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NT; ++ni)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[mi >> 1][mi & 1][ni][r] = 0.f;
            if (Sh::kEpiInBuf) __syncthreads();  // before the next stage writes into `cur`
        }
        pin_acc();
        q0 = q1;
        q1 = q2;
        advance(q2);
    };
    for (int k = 0; k < total; k += 2) {
        stage(smem, smem + kPwBufBytes, xa0, xb0, xa1, xb1);
        stage(smem + kPwBufBytes, smem, xa1, xb1, xa0, xb0);
    }
}

// ---- K = 1 with at most 32 reduction channels and no epilogue (the input gradient of a projection onto a few
// channels, 1024 -> 29 in front of the decoder): out[b][m][t] = sum_{r < R} W'[m][r] * in[b][r][t] ------------
// The arithmetic is nothing; the pass is bound by writing `out` once.  A workgroup owns 64 time steps of one
// batch item: the R x 64 strip of `in` is copied to LDS as it lies in memory (one 16-byte load per lane) and
// comes back through the transposing LDS read as the A operand (row = time step, k = reduction channel), the
// packed weights are the B operand straight from L2 (column = output channel), so an accumulator register
// holds four consecutive time steps of one output channel and a block is transposed for the stores with 8-byte
// LDS writes.  The wavefronts of the workgroups of a grid column share out the output channels in blocks of 32.
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
constexpr int kFewStrip = 64;  // time steps per workgroup
constexpr int kFewRowBytes = kFewStrip * 2 + 16;  // 144: 16-byte aligned rows; 16 consecutive lanes write 16 different bank pairs
constexpr int kFewTileBytes = 32 * kFewRowBytes;  // 32 channel rows

__global__ __launch_bounds__(kThreads) void few_channels_gemm_kernel(const ConvGemmParams p)
{
    __shared__ __align__(16) unsigned char strip[4 * 1024];  // block (step s of 16 channels, 32-step half mb): 16 rows x 64 bytes
    __shared__ __align__(16) unsigned char otile[kWaves * 2 * kFewTileBytes];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int T = p.Tout;  // == p.Tin
    const int nstrips = (T + kFewStrip - 1) / kFewStrip;
    const int b = (int)blockIdx.x / nstrips, t0 = ((int)blockIdx.x - b * nstrips) * kFewStrip;
    const __amdgpu_buffer_rsrc_t rs_in =
        __builtin_amdgcn_make_buffer_rsrc((void *)p.in, 0, (int)((size_t)p.B * p.R * T * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc((void *)p.wp, 0, (int)p.wp_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_out =
        __builtin_amdgcn_make_buffer_rsrc((void *)p.out, 0, (int)((size_t)p.B * p.M * T * 2), 0x00020000);
    {   // wavefront w copies block w: lane = (channel row lane/4, time steps 8*(lane%4) .. +7)
        const int s = wave >> 1, mb = wave & 1;
        const int r = s * 16 + (lane >> 2), t = t0 + mb * 32 + 8 * (lane & 3);
        const bool ok = r < p.R && t < T;  // T % 8 == 0: a group lies inside the row or outside
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs_in, ok ? (uint32_t)(((b * p.R + r) * T + t) * 2) : kOutOfRange, 0, 0);
        *reinterpret_cast<u32x4 *>(strip + wave * 1024 + lane * 16) = v;
    }
    __syncthreads();
    // transposing read of a block: the lane receives time step lane%32, channels 8*(lane/32) .. +7 of the step
    const int g4 = lane >> 4, i16 = lane & 15;
    const uint32_t tr_off = (uint32_t)((8 * (g4 >> 1) + (i16 >> 2)) * 64 + (16 * (g4 & 1) + 4 * (i16 & 3)) * 2);
    bf16x8 a[2][2];  // [mb][ks]
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            union {
                s16x4 h[2];
                bf16x8 v;
            } cvt;
            const unsigned char *q = strip + (ks * 2 + mb) * 1024 + tr_off;
            cvt.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(q));
            cvt.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(q + 4 * 64));
            a[mb][ks] = cvt.v;
        }
    // blocks of 32 output channels of this wavefront
    const int nblocks = (p.M + 31) >> 5, nshare = kWaves * (int)gridDim.y, per = (nblocks + nshare - 1) / nshare;
    const int nb0 = ((int)blockIdx.y * kWaves + wave) * per, nb1 = min(nblocks, nb0 + per);
    const uint32_t chunk_bytes = (uint32_t)p.Kp * 4 * 64 * 16;  // one 64-row tile of the packed weights (R <= 32: one chunk)
    auto load_w = [&](int nb, int ks) {  // fragment (ks, mi = nb % 2) of tap 0 of row tile nb / 2; beyond the range: zeros
        const uint32_t off = (uint32_t)(nb >> 1) * chunk_bytes + (uint32_t)(ks * 2 + (nb & 1)) * 1024u;
        return __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(rs_w, nb < nb1 ? (uint32_t)lane * 16 : kOutOfRange,
                                                                                nb < nb1 ? off : 0u, 0));
    };
    // The result block (32 output channels x 64 time steps) goes through a wave-private LDS tile, [channel][time]
    // in bf16 with rows of 144 bytes, so that it leaves in 16-byte stores whose lanes run along the row: a request to L2 per 64 bytes instead of one per
    // 8 (at one request per lane the pass was bound by the request rate, not by the bytes).  Two tiles in turn.
    unsigned char *tiles = otile + wave * 2 * kFewTileBytes;
    const int h = lane >> 5;
    auto block = [&](int nb, const bf16x8(&w)[2], int par) {
        if (nb >= nb1) return;
        unsigned char *tile = tiles + par * kFewTileBytes;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
            f32x16 acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.f;
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mb][0], w[0], acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mb][1], w[1], acc, 0, 0, 0);
            // registers 4j .. 4j+3: time steps 32*mb + 8*j + 4*h .. +3 of output channel lane % 32
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const u32x2 o = {pack_bf16x2(acc[4 * j], acc[4 * j + 1]), pack_bf16x2(acc[4 * j + 2], acc[4 * j + 3])};
                *reinterpret_cast<u32x2 *>(tile + (lane & 31) * kFewRowBytes + (32 * mb + 8 * j + 4 * h) * 2) = o;
            }
        }
        wave_lds_fence();
#pragma unroll
        for (int i = 0; i < 4; ++i) {  // item: (channel row, 8 time steps)
            const int idx = lane + 64 * i, row = idx >> 3, piece = idx & 7;
            const int m = nb * 32 + row, t = t0 + 8 * piece;
            const u32x4 v = *reinterpret_cast<const u32x4 *>(tile + row * kFewRowBytes + piece * 16);
            const bool ok = m < p.M && t < T;  // T % 8 == 0
            __builtin_amdgcn_raw_buffer_store_b128(v, rs_out, ok ? (uint32_t)(((b * p.M + m) * T + t) * 2) : kOutOfRange, 0, 0);
        }
    };
    bf16x8 w0[2] = {load_w(nb0, 0), load_w(nb0, 1)}, w1[2] = {load_w(nb0 + 1, 0), load_w(nb0 + 1, 1)};
    for (int nb = nb0; nb < nb1; nb += 2) {
        block(nb, w0, 0);
        w0[0] = load_w(nb + 2, 0);
        w0[1] = load_w(nb + 2, 1);
        block(nb + 1, w1, 1);
        w1[0] = load_w(nb + 3, 0);
        w1[1] = load_w(nb + 3, 1);
        wave_lds_fence();  // the reads of both tiles are done before the next pair of blocks writes them
    }
}

// Packed weights: [mt][chunk][tap < Kp][ks][mi][lane][8] (Kp = K rounded up to even, the extra
// tap is zero); element (lane, j) of fragment (ks, mi) is
// W'[m = mt*64 + mi*32 + lane%32][r = chunk*32 + ks*16 + 8*(lane/32) + j][tap], zero outside,
// with W'[m][r][k] = w[m][r][k] (forward) or w[r][m][K-1-k] * rscale[r] (input gradient: FLIP; r is the
// block's output channel co, rscale its folded-BatchNorm factor or NULL for 1; the product is rounded to
// bf16, so the input gradient contracts the exact dy*[y>0] with bf16(w*scale)).
// One block packs 16 of the 64 channels of one (mt, chunk): it copies that 16x32xK block of w
// into LDS with coalesced reads (runs of 32*K, resp. 16*K, contiguous elements) and gathers the
// fragments from there.
constexpr int kPackRows = 16;
// elements between consecutive channels m of the LDS tile: 32*K plus one dword of padding, which
// makes the stride an odd number of dwords so that lanes with different m hit different banks
__host__ __device__ constexpr int pack_m_stride(int K) { return kChunk * K + 2; }
template <bool FLIP>
__device__ __forceinline__ void prepack_block(unsigned blk, unsigned char *smem, const bf16_t *__restrict__ w,
                                              u32x4 *__restrict__ wp, int M, int R, int K, int nch,
                                              int ld /* row length of w */, size_t zero_off, int vec /* 16-byte aligned runs */,
                                              const float *__restrict__ rscale = nullptr)
{
    bf16_t *tile = reinterpret_cast<bf16_t *>(smem);  // [16 m][32 r][K] as m*ms + r*K + k
    const int ms = pack_m_stride(K);
    if (blk == 0)  // one tap pair of zero weights after the packed tensor
        for (int i = threadIdx.x; i < 512; i += 256) wp[zero_off + i] = u32x4{0u, 0u, 0u, 0u};
    const int q = blk & 3;                      // which 16 channels of the 64
    const int c = (blk >> 2) % nch, mt = (blk >> 2) / nch;
    const int m0 = mt * kTileM + q * kPackRows, r0 = c * kChunk;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    // Copy the block of w into LDS.  Rows of w that start on a 16-byte boundary (vec != 0) are read
    // with 16-byte buffer loads, four per thread in flight (the copy is latency bound otherwise);
    // elements beyond the tensor read zeros, elements of a neighbouring block are masked.
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void *)w, 0, (int)((size_t)M * R * K * 2), 0x00020000);
    const int nrows = FLIP ? kChunk : kPackRows;            // runs of contiguous elements: one per r, resp. per m
    const int run = (FLIP ? kPackRows : kChunk) * K;        // elements per run (a multiple of 8)
    const int valid = FLIP ? max(0, min(kPackRows, M - m0)) * K : max(0, min(kChunk, R - r0)) * K;
    auto row_ok = [&](int row) { return FLIP ? r0 + row < R : m0 + row < M; };
    auto row_off = [&](int row) {  // element offset of the run in w
        return FLIP ? (size_t)(r0 + row) * ld + (size_t)m0 * K : (size_t)(m0 + row) * ld + (size_t)r0 * K;
    };
    auto row_factor = [&](int row) {  // FLIP only: a run belongs to one reduction channel
        return (FLIP && rscale && r0 + row < R) ? rscale[r0 + row] : 1.f;
    };
    const bool scaled = FLIP && rscale != nullptr;
    auto put = [&](int row, int o, bf16_t v, float f) {  // element o of run `row`
        if (FLIP) {
            const int m = o / K, k = o - m * K;
            tile[m * ms + row * K + (K - 1 - k)] = scaled ? f32_to_bf16(bf16_to_f32(v) * f) : v;
        } else {
            tile[row * ms + o] = v;
        }
    };
    if (vec) {
        const int vpr = run / 8, nvec = nrows * vpr;
        for (int v0 = threadIdx.x; v0 < nvec; v0 += 256 * 4) {
            u32x4 d[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int v = v0 + u * 256;
                const int row = v / vpr, o = (v - row * vpr) * 8;
                const bool ok = v < nvec && row_ok(row) && o < valid;
                d[u] = __builtin_amdgcn_raw_buffer_load_b128(rs, ok ? (uint32_t)((row_off(row) + o) * 2) : 0x80000000u, 0, 0);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int v = v0 + u * 256;
                if (v < nvec) {
                    const int row = v / vpr, o = (v - row * vpr) * 8;
                    const float f = row_factor(row);
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const uint32_t word = d[u][e >> 1];
                        const bf16_t val = (bf16_t)((e & 1) ? word >> 16 : word & 0xffffu);
                        put(row, o + e, (o + e < valid) ? val : (bf16_t)0, f);
                    }
                }
            }
        }
    } else {
        for (int row = wv; row < nrows; row += 4) {
            const bool ok = row_ok(row);
            const bf16_t *src = w + (ok ? row_off(row) : (size_t)0);
            const float f = row_factor(row);
            for (int o = lane; o < run; o += 64) put(row, o, (ok && o < valid) ? src[o] : (bf16_t)0, f);
        }
    }
    __syncthreads();
    const int Kp = (K + 1) & ~1;  // an odd K gets one zero tap
    u32x4 *dst = wp + (size_t)(blk >> 2) * Kp * 256;
    const int mi = q >> 1, lane_lo = (q & 1) * 16;
    for (int idx = threadIdx.x; idx < Kp * 64; idx += 256) {
        const int m16 = idx & 15, half = (idx >> 4) & 1, ks = (idx >> 5) & 1, k = idx >> 6;
        u32x4 out = {0u, 0u, 0u, 0u};
        if (k < K) {
            const bf16_t *src = tile + m16 * ms + (ks * 16 + 8 * half) * K + k;
#pragma unroll
            for (int j = 0; j < 4; ++j) out[j] = (uint32_t)src[(2 * j) * K] | ((uint32_t)src[(2 * j + 1) * K] << 16);
        }
        dst[(k * 4 + ks * 2 + mi) * 64 + half * 32 + lane_lo + m16] = out;
    }
}

template <bool FLIP>
__global__ __launch_bounds__(256) void prepack_kernel(const bf16_t *__restrict__ w, u32x4 *__restrict__ wp, int M,
                                                      int R, int K, int nch, int ld, size_t zero_off, int vec,
                                                      const float *__restrict__ rscale)
{
    extern __shared__ __align__(16) unsigned char smem[];
    prepack_block<FLIP>(blockIdx.x, smem, w, wp, M, R, K, nch, ld, zero_off, vec, rscale);
}

// Everything the input-gradient engine needs, in one launch: the first npack blocks pack the
// flipped weights times the affine factor of their output channel (a latency-bound job), the others
// run the elementwise mask pass g = dy*[y>0] (bandwidth bound), so the two overlap instead of
// following each other.  g is what the engine contracts; it is also the residual gradient, so it
// is written straight into dres when the caller asked for that, into the workspace otherwise.
__global__ __launch_bounds__(256) void dgrad_prepare_kernel(unsigned npack, const bf16_t *__restrict__ w,
                                                            u32x4 *__restrict__ wp, int M, int R, int K, int nch,
                                                            int ld, size_t zero_off, int vec,
                                                            const float *__restrict__ rscale, size_t n8,
                                                            const u32x4 *__restrict__ dy, const u32x4 *__restrict__ y,
                                                            int relu, u32x4 *__restrict__ gout)
{
    extern __shared__ __align__(16) unsigned char smem[];
    if (blockIdx.x < npack) {
        prepack_block<true>(blockIdx.x, smem, w, wp, M, R, K, nch, ld, zero_off, vec, rscale);
    } else {
        const size_t i = (size_t)(blockIdx.x - npack) * 256 + threadIdx.x;
        if (i < n8) gout[i] = relu ? masked_grad8(dy[i], y[i]) : dy[i];
    }
}

// The same for a fused backward call: the elementwise part also writes g in the fragment order
// of the stride-1 weight-gradient kernels (mask_pack_wave), so dy and y are read once for both gradients.
// gplain may be NULL (no ReLU and no residual gradient wanted: the engine then reads dy itself).
__global__ __launch_bounds__(256) void bwd_prepare_kernel(unsigned npack, const bf16_t *__restrict__ w,
                                                          u32x4 *__restrict__ wp, int M, int R, int K, int nch, int ld,
                                                          size_t zero_off, int vec, const float *__restrict__ rscale,
                                                          int B, int Cout, int To, int ncm, int nst,
                                                          const bf16_t *__restrict__ dy, const bf16_t *__restrict__ y,
                                                          int relu, u32x4 *__restrict__ gplain, u32x4 *__restrict__ gf)
{
    extern __shared__ __align__(16) unsigned char smem[];
    if (blockIdx.x < npack) {
        prepack_block<true>(blockIdx.x, smem, w, wp, M, R, K, nch, ld, zero_off, vec, rscale);
        return;
    }
    const unsigned nst4 = (unsigned)(nst + 3) / 4;
    const unsigned item = (blockIdx.x - npack) * 4 + (threadIdx.x >> 6);  // (b, cm, st4), st4 fastest
    if (item >= (unsigned)B * ncm * nst4) return;
    const int st4 = item % nst4, cm = (item / nst4) % ncm, b = item / (nst4 * ncm);
    mask_pack_wave(threadIdx.x & 63, b, cm, st4, Cout, To, ncm, nst, dy, y, relu, gplain, gf);
}

// ---- input gradient of a stride-2 convolution (the encoder's first layer) -------------------------
// dx[ci, s] only receives taps k with s + pad - k even, so the samples of each parity r form a
// stride-1 correlation of dz with every second tap:  dx[ci, 2u+r] = sum_co sum_k' w[co,ci,kp_r+2k'] *
// dz[co, u + c_r - k'],  kp_r = (r+pad) mod 2,  c_r = (r+pad-kp_r)/2.  Each phase runs through the
// stride-1 engine on its own sub-filter; two small kernels cut the sub-filters out of w and
// interleave the two phase outputs into dx.
__global__ __launch_bounds__(256) void tap_subsample_kernel(const bf16_t *__restrict__ w, bf16_t *__restrict__ w0,
                                                            bf16_t *__restrict__ w1, size_t rows, int K, int kp0, int K0,
                                                            int kp1, int K1)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= rows) return;
    const bf16_t *src = w + i * K;
    for (int j = 0; j < K0; ++j) w0[i * K0 + j] = src[kp0 + 2 * j];
    for (int j = 0; j < K1; ++j) w1[i * K1 + j] = src[kp1 + 2 * j];
}

// dx[row][2u] = a0[row][u], dx[row][2u+1] = a1[row][u]; 8 values of u per thread (U % 8 == 0)
__global__ __launch_bounds__(256) void interleave2_kernel(const u32x4 *__restrict__ a0, const u32x4 *__restrict__ a1,
                                                          u32x4 *__restrict__ dx, size_t n8)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n8) return;
    const u32x4 e = a0[i], o = a1[i];
    u32x4 lo, hi;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        lo[2 * j] = zip_lo16(e[j], o[j]);
        lo[2 * j + 1] = zip_hi16(e[j], o[j]);
        hi[2 * j] = zip_lo16(e[2 + j], o[2 + j]);
        hi[2 * j + 1] = zip_hi16(e[2 + j], o[2 + j]);
    }
    dx[2 * i] = lo;
    dx[2 * i + 1] = hi;
}

struct Plan {
    bool ok;
    int nt;       // NT template value (5 or 2)
    int stride;   // 1 or 2
    int nitems;   // staging items per lane; a buffer holds nitems*32 + kDumpRows rows
    int buf_bytes;
    int overlap;  // cross-tile staging possible
    bool unrolled;  // the kernel instance with an unrolled chunk for this K applies
    size_t lds;
};

// Tin, Tout: lengths of the rows that are staged / written; both must be 16-byte aligned (% 8 == 0).
// R: reduction channels (cross-tile staging needs every wavefront to own the same number of chunks).
Plan make_plan(int Tin, int Tout, int R, int K, int stride, int dil)
{
    Plan pl = {};
    pl.stride = stride;
    if (stride != 1 && stride != 2) return pl;
    if (Tin % 8 != 0 || Tout % 8 != 0) return pl;
    if ((size_t)kPackRows * pack_m_stride(K) * sizeof(bf16_t) > (size_t)kMaxLds) return pl;  // weight packing tile
    const int nch = (R + kChunk - 1) / kChunk;
    // candidate 0: the kernel with an unrolled chunk (tap counts it is built for, stride 1, wide tile,
    // equal chunk counts for the four wavefronts); it skips the zero tap of an odd K, so its window
    // counts K taps.  Candidates 1, 2: the tap-pair loop with the wide, then the narrow tile.
    for (int ci = 0; ci < 3; ++ci) {
        const bool unrolled = ci == 0;
        const int nt = ci == 2 ? 2 : 5;
        if (nt == 5 && Tout <= 64) continue;  // short sequences: the narrow tile wastes less
        if (unrolled && !(stride == 1 && unrolled_slots(K) > 0 && nch % kWaves == 0)) continue;
        const long taps = unrolled ? K : (K + 1) & ~1;  // the tap-pair loop also reads the zero tap of an odd K
        const long rows = (long)(nt * 32 - 1) * stride + (taps - 1) * dil + 1 + 7;
        const long nitems = ((rows + 7) / 8 * 16 + 63) / 64;
        if (unrolled && nitems > unrolled_slots(K)) continue;
        const size_t buf = (size_t)(nitems * 32 + kDumpRows) * kRowBytes;
        const size_t stage = (size_t)kWaves * 2 * buf;
        const size_t round_bytes = (size_t)kWaves * 3 * nt * 64 * sizeof(f32x4);  // one row of blocks per round
        // with cross-tile staging the scratch must fit in the buffers of one parity
        const bool overlap = (nch % kWaves == 0) && (kWaves * buf >= round_bytes);
        const size_t lds = stage > round_bytes ? stage : round_bytes;
        if (unrolled && !overlap) continue;
        if (lds <= (size_t)kMaxLds && buf >= (size_t)16 * nt * 32 * sizeof(float)) {  // buf also holds the output transpose tile
            pl.ok = true;
            pl.nt = nt;
            pl.nitems = (int)nitems;
            pl.buf_bytes = (int)buf;
            pl.overlap = overlap ? 1 : 0;
            pl.unrolled = unrolled;
            pl.lds = lds;
            return pl;
        }
    }
    return pl;
}

size_t packed_bytes(int M, int R, int K)
{
    const size_t nmt = (M + kTileM - 1) / kTileM, nch = (R + kChunk - 1) / kChunk;
    const size_t Kp = (size_t)((K + 1) & ~1);
    return align_up((nmt * nch * Kp * 256 + 512) * sizeof(u32x4), 256);  // + one tap pair of zeros
}

constexpr size_t kMaxPacked = (size_t)1 << 31;  // the kernel addresses packed weights with 32-bit offsets
constexpr size_t kMaxInput = (size_t)1 << 30;   // and the activation tensors through buffer descriptors

template <int NT, int STRIDE, int KT, bool LEN = false, bool STATS = false>
hipError_t launch_t(const ConvGemmParams &p, size_t lds, hipStream_t s)
{
    auto kern = conv_gemm_kernel<NT, STRIDE, KT, LEN, STATS>;
    static LdsOptIn opt_in;
    hipError_t e = ensure_dynamic_lds(opt_in, reinterpret_cast<const void *>(kern), kMaxLds);
    if (e != hipSuccess) return e;
    const int cus = current_device_info().cus;
    const int grid = p.num_tiles < cus ? p.num_tiles : cus;
    ConvGemmParams q = p;
    // private tiles per wavefront (unrolled kernels only); a remainder of more than two shared rounds
    // is cheaper as one more private round in which some wavefronts stay idle: no exchange epilogues, and
    // on a chip that runs at its power limit the idle wavefronts' share of the budget raises the clock of
    // the busy ones (256 channels, K=11, B=32: 640 tiles on 1024 wavefronts, step 173 -> 159 us)
    q.full = KT > 0 ? p.num_tiles / (kWaves * grid) + (p.num_tiles % (kWaves * grid) > 2 * grid ? 1 : 0) : 0;
    MainKernelTimer timer(s);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), lds, s, q);
    return hipGetLastError();
}

template <bool LEN, int MI, int NT, int SC>
hipError_t launch_pointwise_shape(const ConvGemmParams &p, hipStream_t s)
{
    using Sh = PwShape<MI, NT, SC>;
    auto kern = pointwise_gemm_kernel<LEN, MI, NT, SC>;
    static LdsOptIn opt_in;
    hipError_t e = ensure_dynamic_lds(opt_in, reinterpret_cast<const void *>(kern), (int)Sh::kLds);
    if (e != hipSuccess) return e;
    ConvGemmParams q = p;
    q.ntt = (p.Tout + NT * 32 - 1) / (NT * 32);
    const int cus = current_device_info().cus;
    const int ntiles = (p.nmt + kWaves * Sh::kRowTiles - 1) / (kWaves * Sh::kRowTiles) * q.ntt * p.B;
    MainKernelTimer timer(s);
    hipLaunchKernelGGL(kern, dim3(ntiles < cus ? ntiles : cus), dim3(kThreads), Sh::kLds, s, q);
    return hipGetLastError();
}

// Padded work of a shape: MFMAs of all its tiles over the MFMAs of the contraction, times the rounds the
// workgroups need over the rounds a perfectly divisible launch would need.
template <int MI, int NT>
double pointwise_waste(const ConvGemmParams &p, int cus)
{
    const int rows = kWaves * MI * 32, cols = NT * 32;
    const long tr = (p.M + rows - 1) / rows, tc = (p.Tout + cols - 1) / cols;
    const long tiles = tr * tc * p.B;
    const double pad = (double)(tr * rows) * (double)(tc * cols) / ((double)p.M * p.Tout);
    const double rounds = (double)((tiles + cus - 1) / cus) * cus / (double)tiles;
    return pad * rounds;
}

hipError_t launch_pointwise(const ConvGemmParams &p, hipStream_t s)
{
    // the 512 x 128 tile does half the LDS and staging work per MFMA and has half as many epilogue rounds per
    // output (measured 1.1 to 1.2 times faster per MFMA issued at 896 <-> 1024 channels); it is taken unless
    // its padding and last-round losses outweigh that
    const int cus = current_device_info().cus;
    const bool big = pointwise_waste<4, 4>(p, cus) <= 1.12 * pointwise_waste<2, 5>(p, cus);
    if (p.len_in)
        return big ? launch_pointwise_shape<true, 4, 4, 64>(p, s) : launch_pointwise_shape<true, 2, 5, 128>(p, s);
    return big ? launch_pointwise_shape<false, 4, 4, 64>(p, s) : launch_pointwise_shape<false, 2, 5, 128>(p, s);
}

hipError_t launch_few_channels(const ConvGemmParams &p, hipStream_t s)
{
    const int nstrips = (p.Tout + kFewStrip - 1) / kFewStrip;
    MainKernelTimer timer(s);
    // the output channels of a strip are shared out among the workgroups of a column of the grid: enough
    // workgroups to give every SIMD several wavefronts (the stores are the work)
    const int cus = current_device_info().cus;
    const int nblocks = (p.M + 31) / 32;
    int split = 1;
    while (split < 8 && p.B * nstrips * split < 4 * cus && nblocks >= 2 * kWaves * split) split *= 2;
    hipLaunchKernelGGL(few_channels_gemm_kernel, dim3(p.B * nstrips, split), dim3(kThreads), 0, s, p);
    return hipGetLastError();
}

hipError_t launch_plan(const Plan &pl, const ConvGemmParams &p, hipStream_t s)
{
    // one tap, at most one chunk of reduction channels, nothing to do after the sums: the store-bound kernel
    if (p.K == 1 && p.R <= kChunk && pl.stride == 1 && p.padL == 0 && p.Tin == p.Tout && p.Tout % 8 == 0 && !p.res &&
        !p.scale && !p.shift && !p.relu && !p.len_in && !p.len_out)
        return launch_few_channels(p, s);
    // one tap, no padding, wide tiles: the GEMM kernel whose wavefronts share the staged activations
    // (worth it from two 64-channel row tiles on: a single one would leave three wavefronts idle)
    if (p.K == 1 && p.nmt >= 2 && pl.nt == 5 && pl.stride == 1 && p.padL == 0 && p.Tin == p.Tout) return launch_pointwise(p, s);
    if (p.stats) {  // (the caller has checked stats_on_engine)
        switch (p.K) {
        case 11: return launch_t<5, 1, 11, false, true>(p, pl.lds, s);
        case 13: return launch_t<5, 1, 13, false, true>(p, pl.lds, s);
        case 21: return launch_t<5, 1, 21, false, true>(p, pl.lds, s);
        case 25: return launch_t<5, 1, 25, false, true>(p, pl.lds, s);
        case 29: return launch_t<5, 1, 29, false, true>(p, pl.lds, s);
        case 17: return launch_t<5, 1, 17, false, true>(p, pl.lds, s);
        default: return hipErrorInvalidValue;
        }
    }
    if (pl.unrolled && (p.len_in || p.len_out)) {
        switch (p.K) {
        case 11: return launch_t<5, 1, 11, true>(p, pl.lds, s);
        case 13: return launch_t<5, 1, 13, true>(p, pl.lds, s);
        case 21: return launch_t<5, 1, 21, true>(p, pl.lds, s);
        case 25: return launch_t<5, 1, 25, true>(p, pl.lds, s);
        case 29: return launch_t<5, 1, 29, true>(p, pl.lds, s);
        case 17: return launch_t<5, 1, 17, true>(p, pl.lds, s);
        default: return hipErrorInvalidValue;
        }
    }
    if (pl.unrolled) {
        switch (p.K) {
        case 11: return launch_t<5, 1, 11>(p, pl.lds, s);
        case 13: return launch_t<5, 1, 13>(p, pl.lds, s);
        case 21: return launch_t<5, 1, 21>(p, pl.lds, s);
        case 25: return launch_t<5, 1, 25>(p, pl.lds, s);
        case 29: return launch_t<5, 1, 29>(p, pl.lds, s);
        case 17: return launch_t<5, 1, 17>(p, pl.lds, s);
        default: return hipErrorInvalidValue;
        }
    }
    if (pl.nt == 5 && pl.stride == 1) return launch_t<5, 1, 0>(p, pl.lds, s);
    if (pl.nt == 2 && pl.stride == 1) return launch_t<2, 1, 0>(p, pl.lds, s);
    if (pl.nt == 5 && pl.stride == 2) return launch_t<5, 2, 0>(p, pl.lds, s);
    if (pl.nt == 2 && pl.stride == 2) return launch_t<2, 2, 0>(p, pl.lds, s);
    return hipErrorInvalidValue;
}

size_t prepack_lds(int K) { return (size_t)kPackRows * pack_m_stride(K) * sizeof(bf16_t); }

// flip == false: W'[m][r][k] = w[m][r][k] (w is [M][R][K]); flip == true: W'[m][r][k] = w[r][m][K-1-k] * rscale[r]
// (w is [R][M][K]; rscale NULL: 1).
struct PackGeom {
    int nmt, nch, vec;
    size_t lds, zero_off;
    unsigned blocks;
};
PackGeom pack_geom(const void *w, int M, int R, int K, bool flip)
{
    PackGeom q;
    q.nmt = (M + kTileM - 1) / kTileM;
    q.nch = (R + kChunk - 1) / kChunk;
    q.lds = prepack_lds(K);
    q.zero_off = (size_t)q.nmt * q.nch * ((K + 1) & ~1) * 256;
    // runs start at multiples of 2*K*(row length) bytes from w: 16-byte aligned when w is and the other
    // channel count is a multiple of 8 (the tensor must also fit a 32-bit byte offset)
    const int other = flip ? M : R;
    q.vec = ((uintptr_t)w % 16 == 0 && other % 8 == 0 && (size_t)M * R * K * 2 < ((size_t)1 << 31)) ? 1 : 0;
    q.blocks = (unsigned)(q.nmt * q.nch * 4);
    return q;
}

hipError_t run_prepack(const void *w, void *wp, int M, int R, int K, bool flip, const float *rscale, hipStream_t s)
{
    const PackGeom q = pack_geom(w, M, R, K, flip);
    hipError_t e;
    if (flip) {
        static LdsOptIn opt_in;
        e = ensure_dynamic_lds(opt_in, reinterpret_cast<const void *>(prepack_kernel<true>), kMaxLds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(prepack_kernel<true>, dim3(q.blocks), dim3(256), q.lds, s, (const bf16_t *)w, (u32x4 *)wp,
                           M, R, K, q.nch, M * K, q.zero_off, q.vec, rscale);
    } else {
        static LdsOptIn opt_in;
        e = ensure_dynamic_lds(opt_in, reinterpret_cast<const void *>(prepack_kernel<false>), kMaxLds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(prepack_kernel<false>, dim3(q.blocks), dim3(256), q.lds, s, (const bf16_t *)w, (u32x4 *)wp,
                           M, R, K, q.nch, R * K, q.zero_off, q.vec, (const float *)nullptr);
    }
    return hipGetLastError();
}

void fill_common(ConvGemmParams &p, const Plan &pl, int B, int M, int R, int Tin, int Tout, int K, int dil, int padL)
{
    p.B = B; p.M = M; p.R = R; p.Tin = Tin; p.Tout = Tout; p.K = K; p.Kp = (K + 1) & ~1; p.dil = dil; p.padL = padL;
    p.nmt = (M + kTileM - 1) / kTileM;
    p.nch = (R + kChunk - 1) / kChunk;
    p.ntt = (Tout + pl.nt * 32 - 1) / (pl.nt * 32);
    p.num_tiles = p.nmt * p.ntt * B;
    p.wp_zero = (size_t)p.nmt * p.nch * p.Kp * 256;
    p.wp_bytes = (p.wp_zero + 512) * sizeof(u32x4);
    p.nitems = pl.nitems;
    p.buf_bytes = pl.buf_bytes;
    p.overlap = pl.overlap;
}

}  // namespace

// ---- forward ---------------------------------------------------------------------------
bool mfma_fwd_supported(const Geom &g)
{
    if ((size_t)g.B * g.Cin * g.T * sizeof(bf16_t) > kMaxInput) return false;
    if ((size_t)g.B * g.Cout * g.To * sizeof(bf16_t) > kMaxInput) return false;
    return packed_bytes(g.Cout, g.Cin, g.K) < kMaxPacked && make_plan(g.T, g.To, g.Cin, g.K, g.stride, g.dil).ok;
}

size_t mfma_fwd_workspace(const Geom &g) { return packed_bytes(g.Cout, g.Cin, g.K); }

// Whether the forward pass of this geometry runs on a kernel instance that can also write the statistics of its
// outputs, and into how many (batch item, time tile) parts: the unrolled engine, wide tile, no lengths.
int mfma_fwd_stats_parts(const Geom &g)
{
    const Plan pl = make_plan(g.T, g.To, g.Cin, g.K, g.stride, g.dil);
    if (!pl.ok || !pl.unrolled || pl.nt != 5 || g.len || !mfma_fwd_supported(g)) return 0;
    if (pl.buf_bytes < Epilogue<5>::kTileBytesWithStats) return 0;
    return g.B * ((g.To + 159) / 160);
}

hipError_t launch_mfma_fwd(const Geom &g, const void *x, const void *w, const float *scale, const float *shift,
                           const void *res, void *y, bool relu, void *ws, hipStream_t s, double *stats)
{
    const Plan pl = make_plan(g.T, g.To, g.Cin, g.K, g.stride, g.dil);
    if (!pl.ok || !mfma_fwd_supported(g)) return hipErrorInvalidValue;
    if (stats && mfma_fwd_stats_parts(g) == 0) return hipErrorInvalidValue;
    // a pointwise layer with a handful of output channels is a stream over x: no packing, no tiles
    if (skinny_fwd_supported(g) && ((uintptr_t)w % 16) == 0) return launch_skinny_fwd(g, x, w, scale, shift, res, y, relu, s);
    hipError_t e = run_prepack(w, ws, g.Cout, g.Cin, g.K, false, nullptr, s);
    if (e != hipSuccess) return e;
    ConvGemmParams p = {};
    fill_common(p, pl, g.B, g.Cout, g.Cin, g.T, g.To, g.K, g.dil, g.pad);
    p.relu = relu ? 1 : 0;
    p.in = (const bf16_t *)x;
    p.len_in = g.len;
    p.wp = (const bf16x8 *)ws;
    p.scale = scale; p.shift = shift; p.res = (const bf16_t *)res;
    p.out = (bf16_t *)y;
    p.stats = stats;
    return launch_plan(pl, p, s);
}

// ---- input gradient (stride 1 only; other strides use the plain kernels) ----------------
// Workspace: packed (flipped, transposed) weights, then dz when it differs from dy.
namespace {
// stride 2 as two stride-1 phases (see tap_subsample_kernel)
struct Phase2 {
    int kp[2], K[2], c[2], U;  // first tap, taps, dz offset of each phase; outputs per phase
    bool ok;
};
Phase2 phases_of_stride2(const Geom &g)
{
    Phase2 ph = {};
    if (g.stride != 2 || g.dil != 1 || g.T % 16 != 0 || g.To % 8 != 0) return ph;
    ph.U = g.T / 2;
    for (int r = 0; r < 2; ++r) {
        ph.kp[r] = (r + g.pad) & 1;
        ph.K[r] = g.K > ph.kp[r] ? (g.K - ph.kp[r] + 1) / 2 : 0;
        ph.c[r] = (r + g.pad - ph.kp[r]) / 2;
        if (ph.K[r] < 1) return ph;
        if (!make_plan(g.To, ph.U, g.Cout, ph.K[r], 1, 1).ok || packed_bytes(g.Cin, g.Cout, ph.K[r]) >= kMaxPacked) return ph;
    }
    ph.ok = true;
    return ph;
}
size_t dz_bytes_of(const Geom &g) { return align_up((size_t)g.B * g.Cout * g.To * sizeof(bf16_t), 256); }
}  // namespace

bool mfma_dgrad_supported(const Geom &g)
{
    if ((size_t)g.B * g.Cout * g.To * sizeof(bf16_t) > kMaxInput) return false;
    if ((size_t)g.B * g.Cin * g.T * sizeof(bf16_t) > kMaxInput) return false;
    if (g.stride == 2) return phases_of_stride2(g).ok;
    if (g.stride != 1 || packed_bytes(g.Cin, g.Cout, g.K) >= kMaxPacked) return false;
    return make_plan(g.To, g.T, g.Cout, g.K, 1, g.dil).ok;
}

size_t mfma_dgrad_workspace(const Geom &g)
{
    if (g.stride == 2) {
        const Phase2 ph = phases_of_stride2(g);
        size_t n = dz_bytes_of(g);
        for (int r = 0; r < 2; ++r)
            n += align_up((size_t)g.Cout * g.Cin * ph.K[r] * sizeof(bf16_t), 256) + packed_bytes(g.Cin, g.Cout, ph.K[r]) +
                 align_up((size_t)g.B * g.Cin * ph.U * sizeof(bf16_t), 256);
        return n;
    }
    return packed_bytes(g.Cin, g.Cout, g.K) + dz_bytes_of(g);
}

namespace {
// The elementwise pass in front of an input gradient whose weights are packed separately: g = dy*[y>0]
// into `gbuf` (when there is a ReLU) and/or `dres`.  Returns the tensor the engine contracts in *g_used.
hipError_t mask_pass(const Geom &g, const void *dy, const void *y, bool relu, void *gbuf, void *dres, const void **g_used,
                     hipStream_t s)
{
    *g_used = dy;
    if (!relu && !dres) return hipSuccess;
    hipError_t e;
    if (dres && ((uintptr_t)dres % 16) == 0) {
        // the residual gradient is g itself: write it once and contract it from there
        e = launch_epilogue_bwd_vec8(g, dy, y, nullptr, relu, nullptr, dres, s);
        if (relu) *g_used = dres;
    } else if (!dres) {
        e = launch_epilogue_bwd_vec8(g, dy, y, nullptr, relu, gbuf, nullptr, s);
        *g_used = gbuf;
    } else {  // a misaligned dres: the 2-byte kernel writes it and an aligned copy for the engine
        e = launch_epilogue_bwd(g, true, dy, y, nullptr, relu, relu ? gbuf : nullptr, dres, s);
        if (relu) *g_used = gbuf;
    }
    return e;
}

hipError_t launch_mfma_dgrad_stride2(const Geom &g, const void *dy, const void *y, const float *scale, const void *w,
                                     void *dx, void *dres, bool relu, void *ws, hipStream_t s)
{
    const Phase2 ph = phases_of_stride2(g);
    if (!ph.ok) return hipErrorInvalidValue;
    unsigned char *cur = (unsigned char *)ws;
    void *gbuf = cur;
    cur += dz_bytes_of(g);
    void *wsub[2], *packed[2], *phase_out[2];
    for (int r = 0; r < 2; ++r) {
        wsub[r] = cur;
        cur += align_up((size_t)g.Cout * g.Cin * ph.K[r] * sizeof(bf16_t), 256);
        packed[r] = cur;
        cur += packed_bytes(g.Cin, g.Cout, ph.K[r]);
        phase_out[r] = cur;
        cur += align_up((size_t)g.B * g.Cin * ph.U * sizeof(bf16_t), 256);
    }
    const void *gin = dy;
    hipError_t e = mask_pass(g, dy, y, relu, gbuf, dres, &gin, s);
    if (e != hipSuccess) return e;
    const size_t rows = (size_t)g.Cout * g.Cin;
    hipLaunchKernelGGL(tap_subsample_kernel, dim3((unsigned)((rows + 255) / 256)), dim3(256), 0, s, (const bf16_t *)w,
                       (bf16_t *)wsub[0], (bf16_t *)wsub[1], rows, g.K, ph.kp[0], ph.K[0], ph.kp[1], ph.K[1]);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    for (int r = 0; r < 2; ++r) {
        const Plan pl = make_plan(g.To, ph.U, g.Cout, ph.K[r], 1, 1);
        e = run_prepack(wsub[r], packed[r], g.Cin, g.Cout, ph.K[r], true, scale, s);
        if (e != hipSuccess) return e;
        ConvGemmParams p = {};
        // out[u] = sum_j W'[j] * g[u - padL + j] with j = K_r-1-k'  ->  padL = K_r - 1 - c_r
        fill_common(p, pl, g.B, g.Cin, g.Cout, g.To, ph.U, ph.K[r], 1, ph.K[r] - 1 - ph.c[r]);
        p.relu = 0;
        p.in = (const bf16_t *)gin;
        p.wp = (const bf16x8 *)packed[r];
        p.out = (bf16_t *)phase_out[r];
        p.len_out = g.len;  // dx[2u+r] is padding from 2u+r >= len on: u >= ceil((len - r) / 2)
        p.len_out_sub = r;
        p.len_out_div = 2;
        e = launch_plan(pl, p, s);  // the first of the two carries the one-shot timer
        if (e != hipSuccess) return e;
    }
    const size_t n8 = (size_t)g.B * g.Cin * ph.U / 8;
    hipLaunchKernelGGL(interleave2_kernel, dim3((unsigned)((n8 + 255) / 256)), dim3(256), 0, s, (const u32x4 *)phase_out[0],
                       (const u32x4 *)phase_out[1], (u32x4 *)dx, n8);
    return hipGetLastError();
}

// parameters of the stride-1 input gradient as a run of the forward engine
void fill_dgrad(ConvGemmParams &p, const Plan &pl, const Geom &g, const void *gin, const void *packed, void *dx, bool accumulate)
{
    fill_common(p, pl, g.B, g.Cin, g.Cout, g.To, g.T, g.K, g.dil, g.dil * (g.K - 1) - g.pad);
    p.relu = 0;
    p.in = (const bf16_t *)gin;
    p.wp = (const bf16x8 *)packed;
    p.out = (bf16_t *)dx;
    p.res = accumulate ? (const bf16_t *)dx : nullptr;  // dx += : every lane reads the 16 bytes it then overwrites
    p.len_out = g.len;
    p.len_out_div = 1;
}
}  // namespace

// accumulate (stride 1 only): dx = bf16(dx + gradient), one rounding.
hipError_t launch_mfma_dgrad(const Geom &g, const void *dy, const void *y, const float *scale, const void *w,
                             void *dx, void *dres, bool relu, bool accumulate, void *ws, hipStream_t s, const void **g_used)
{
    if (g_used) *g_used = nullptr;
    if (g.stride == 2) {
        if (accumulate) return hipErrorInvalidValue;
        return launch_mfma_dgrad_stride2(g, dy, y, scale, w, dx, dres, relu, ws, s);
    }
    const Plan pl = make_plan(g.To, g.T, g.Cout, g.K, 1, g.dil);
    if (!pl.ok || !mfma_dgrad_supported(g)) return hipErrorInvalidValue;
    // g = dy*[y>0] (exact in bf16) comes from one elementwise pass, which shares a launch with the weight
    // packing when it can use 16-byte accesses (To % 8 == 0 on this path; dres aligned); the affine
    // factor scale[co] is folded into the packed weights.
    hipError_t e;
    const void *gin = dy;
    void *gbuf = (unsigned char *)ws + packed_bytes(g.Cin, g.Cout, g.K);
    if (!dres || ((uintptr_t)dres % 16) == 0) {
        const int M = g.Cin, R = g.Cout;  // the engine's roles for this pass
        const PackGeom q = pack_geom(w, M, R, g.K, true);
        void *gout = dres ? dres : (relu ? gbuf : nullptr);
        const size_t n8 = gout ? (size_t)g.B * g.Cout * g.To / 8 : 0;
        static LdsOptIn opt_in;
        e = ensure_dynamic_lds(opt_in, reinterpret_cast<const void *>(dgrad_prepare_kernel), kMaxLds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(dgrad_prepare_kernel, dim3(q.blocks + (unsigned)((n8 + 255) / 256)), dim3(256), q.lds, s, q.blocks,
                           (const bf16_t *)w, (u32x4 *)ws, M, R, g.K, q.nch, M * g.K, q.zero_off, q.vec, scale, n8,
                           (const u32x4 *)dy, (const u32x4 *)y, relu ? 1 : 0, (u32x4 *)gout);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        if (relu) gin = gout;
    } else {
        e = run_prepack(w, ws, g.Cin, g.Cout, g.K, true, scale, s);
        if (e != hipSuccess) return e;
        e = mask_pass(g, dy, y, relu, gbuf, dres, &gin, s);
        if (e != hipSuccess) return e;
    }
    if (g_used) *g_used = gin;
    ConvGemmParams p = {};
    fill_dgrad(p, pl, g, gin, ws, dx, accumulate);
    return launch_plan(pl, p, s);
}

// ---- fused backward -------------------------------------------------------------------------
// Packs the flipped, scaled weights into ws and, in the same launch, forms g = dy*[y>0] in the two
// layouts the gradients read: plain (into dres when the caller wants the residual gradient, else into
// the workspace behind the packed weights; skipped when there is no ReLU and no dres) and in fragment
// order (gf).  *g_plain receives the tensor the input-gradient engine has to contract.
hipError_t launch_bwd_prepare(const Geom &g, const void *dy, const void *y, const float *scale, const void *w,
                              bool relu, void *ws, void *gf, const DzfLayout &layout, void *dres, const void **g_plain,
                              hipStream_t s)
{
    const int M = g.Cin, R = g.Cout;  // the engine's roles for the input gradient
    const PackGeom q = pack_geom(w, M, R, g.K, true);
    const size_t nfrag = (size_t)g.B * layout.ncm * ((layout.nst + 3) / 4);  // items of four fragments, one per wavefront
    void *gbuf = (unsigned char *)ws + packed_bytes(g.Cin, g.Cout, g.K);
    void *gout = dres ? dres : (relu ? gbuf : nullptr);
    *g_plain = gout ? gout : dy;
    static LdsOptIn opt_in;
    hipError_t e = ensure_dynamic_lds(opt_in, reinterpret_cast<const void *>(bwd_prepare_kernel), kMaxLds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(bwd_prepare_kernel, dim3(q.blocks + (unsigned)((nfrag + 3) / 4)), dim3(256), q.lds, s, q.blocks,
                       (const bf16_t *)w, (u32x4 *)ws, M, R, g.K, q.nch, M * g.K, q.zero_off, q.vec, scale, g.B, g.Cout, g.To,
                       layout.ncm, layout.nst, (const bf16_t *)dy, (const bf16_t *)y, relu ? 1 : 0, (u32x4 *)gout, (u32x4 *)gf);
    return hipGetLastError();
}

hipError_t launch_mfma_dgrad_prepared(const Geom &g, const void *g_plain, void *dx, bool accumulate, void *ws, hipStream_t s)
{
    const Plan pl = make_plan(g.To, g.T, g.Cout, g.K, 1, g.dil);
    if (!pl.ok || !mfma_dgrad_supported(g)) return hipErrorInvalidValue;
    ConvGemmParams p = {};
    fill_dgrad(p, pl, g, g_plain, ws, dx, accumulate);
    return launch_plan(pl, p, s);
}

}  // namespace nm
