// Matrix-core weight gradient with a wavefront-level split over time.
//
//   dw[co, ci, k] = sum_b sum_t dz[b, co, t] * x[b, ci, t*stride - pad + k*dil]
//
// is, for each tap k, a GEMM with M = co, N = ci and the reduction over (b, t).  An output
// tile is 64 output channels x 32 input channels x a group of up to KT taps (2*KT 32x32 MFMA
// accumulators per wavefront).  The reduction is cut into units of one batch item x TCH time
// steps; the 4*S wavefronts that share an output tile (4 per workgroup, S workgroups) each
// take every (4*S)-th unit and accumulate privately, so the main loop has no workgroup
// barrier.  The four partial tiles of a workgroup are summed through LDS, the S workgroup
// results go to a float32 scratch laid out [S][K][Cout][Cin] (coalesced along ci) and a small
// kernel adds them in a fixed order and writes dw[co][ci][k]: the result is deterministic.
//
// Operand staging (private to each wavefront, double buffered):
//   * dz rows are copied to LDS as they are ([co][t]); an A fragment (8 consecutive t of one
//     co) is one aligned 16-byte read;
//   * x is written transposed to [time][channel] exactly as in the forward kernel, so a tap is
//     a row offset; a B fragment needs 8 consecutive *time steps* of one channel, i.e. a column
//     of that layout, which the gfx950 transposing LDS read (ds_read_b64_tr_b16: 16 lanes read a
//     4x16 block, lane i receives column i) delivers in two reads.
// The kernels contract g = dy * [y>0] (exact in bf16: a value of dy or zero; materialised once per call
// by a vectorised elementwise kernel) and the affine factor scale[co] multiplies the float32 sums in
// the final reduction, so the operand carries no rounding of its own:
//   dw[co,ci,k] = scale[co] * sum_b sum_t g[b,co,t] * x[b,ci,tau(t,k)].
#include "nm_common.h"

#include <type_traits>

namespace nm {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

constexpr int kWaves = 4;
constexpr int kThreads = 64 * kWaves;
constexpr int kTileCo = 64;
constexpr int kTileCi = 32;
constexpr int kXRowBytes = 80;  // 32 channels * 2 B + 16 B pad
constexpr int kXRowDwords = kXRowBytes / 4;
constexpr int kMaxLds = 160 * 1024;
constexpr int kMaxKT = 6;

struct WgradParams {
    int B, Cin, Cout, T, To, K, stride, dil, pad;
    int ncot, ncit, ntg, KTg;  // tiles per dimension; taps per group
    int S;                     // workgroups sharing one output tile
    int TCH, nchunk, units;    // time steps per unit, units per batch row, total units
    int NRX;                   // rows of the staged x window that are read (multiple of 8)
    int n_dz, n_x, ips;        // staging items per lane (dz, x) and items riding on one MFMA step
    int dz_row_bytes, dz_bytes, x_bytes, buf_bytes;
    int total, per_xcd, CL;    // work-item numbering (CL == 0: plain order)
    const bf16_t *x;           // [B][Cin][T]
    const int *len;            // [B] valid lengths of x (samples beyond read as zero) or NULL
    const bf16_t *dz;          // [B][Cout][To]
    float *part;               // [S][K][Cout][Cin]
    // stride-1, dilation-1 kernel only: dz in MFMA A-fragment order [B][ncm][nst][64 lanes][8]
    const u32x4 *dzf;
    int ncm, nst;              // 32-channel blocks (2 per tile), 16-step blocks per batch row
};

__device__ __forceinline__ void wave_lds_fence()
{
    // LDS operations of one wavefront execute in order; this only keeps the compiler from
    // moving LDS accesses across the point where other lanes' data must be visible.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// 16-byte buffer load: `voff` is the byte offset of the lane inside the tensor, `soff` a
// wave-uniform addend.  A lane whose data lies outside its row passes kOutOfRange, which the
// hardware bounds check turns into zeros: no branch and nothing to fix up after the load.
constexpr uint32_t kOutOfRange = 0xffffffffu;
// An offset beyond every tensor this file addresses through a descriptor (the host keeps them below
// 1 GiB) that stays beyond them when a small immediate or scalar offset is added.
constexpr uint32_t kFar = 0x80000000u;
__device__ __forceinline__ u32x4 buf_load16(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff)
{
    return __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0);
}

// Which (split, tile) a workgroup owns.  Work items are numbered so that the workgroups the
// hardware places on one XCD (blockIdx mod 8) form a contiguous range of items that share the
// T-slice and neighbouring channel tiles.
struct TileCoords {
    int sp, tg, cot, cit;
    bool valid;
};
__device__ __forceinline__ TileCoords decode_tile(const WgradParams &p)
{
    TileCoords tc;
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int v = xcd * p.per_xcd + j;
    tc.valid = !(j >= p.per_xcd || v >= p.total);
    int r = tc.valid ? v : 0;
    if (p.CL < 0) {
        // digits, slowest to fastest: sp, tg, cit, cot (the kernel with shared staging: one XCD then holds
        // all output-channel tiles of a few input-channel tiles, so x is fetched into one L2 only)
        tc.cot = r % p.ncot; r /= p.ncot;
        tc.cit = r % p.ncit; r /= p.ncit;
        tc.tg = r % p.ntg; r /= p.ntg;
        tc.sp = r;
    } else if (p.CL > 0) {
        // digits, slowest to fastest: sp, cot_hi, tg, cot_lo, cit
        tc.cit = r % p.ncit; r /= p.ncit;
        const int cot_lo = r % p.CL; r /= p.CL;
        tc.tg = r % p.ntg; r /= p.ntg;
        const int nhi = p.ncot / p.CL;
        const int cot_hi = r % nhi; r /= nhi;
        tc.sp = r;
        tc.cot = cot_hi * p.CL + cot_lo;
    } else {
        tc.cit = r % p.ncit; r /= p.ncit;
        tc.cot = r % p.ncot; r /= p.ncot;
        tc.tg = r % p.ntg; r /= p.ntg;
        tc.sp = r;
    }
    return tc;
}

// Sum the four wavefronts' partial tiles through LDS (wave g finishes rows [4g,4g+4) of every
// 32x32 block), then write this workgroup's tile to the scratch [S][K][Cout][Cin].
template <int KT>
__device__ __forceinline__ void reduce_and_store(const WgradParams &p, unsigned char *smem, f32x16 (&acc)[2][KT],
                                                 int lane, int wave, int sp, int k0, int kt, int co0, int ci0)
{
    constexpr int kTiles = 2 * KT;
    __syncthreads();
    f32x4 *red = reinterpret_cast<f32x4 *>(smem);
#pragma unroll
    for (int g = 0; g < kWaves; ++g) {
        if (g != wave) {
            const int slot = wave < g ? wave : wave - 1;
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int kk = 0; kk < KT; ++kk) {
                    f32x4 val = {acc[mi][kk][4 * g], acc[mi][kk][4 * g + 1], acc[mi][kk][4 * g + 2],
                                 acc[mi][kk][4 * g + 3]};
                    red[((g * 3 + slot) * kTiles + mi * KT + kk) * 64 + lane] = val;
                }
        }
    }
    __syncthreads();
    f32x4 own[kTiles];
#pragma unroll
    for (int g = 0; g < kWaves; ++g) {
        if (g == wave) {
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int kk = 0; kk < KT; ++kk)
                    own[mi * KT + kk] = f32x4{acc[mi][kk][4 * g], acc[mi][kk][4 * g + 1], acc[mi][kk][4 * g + 2],
                                              acc[mi][kk][4 * g + 3]};
        }
    }
#pragma unroll
    for (int slot = 0; slot < 3; ++slot)
#pragma unroll
        for (int tl = 0; tl < kTiles; ++tl) own[tl] += red[((wave * 3 + slot) * kTiles + tl) * 64 + lane];

    const int ci = ci0 + (lane & 31);
    if (ci < p.Cin) {
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int kk = 0; kk < KT; ++kk) {
                if (kk >= kt) continue;
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    const int co = co0 + mi * 32 + 8 * wave + 4 * (lane >> 5) + jj;
                    if (co < p.Cout)
                        p.part[(((size_t)sp * p.K + k0 + kk) * p.Cout + co) * p.Cin + ci] = own[mi * KT + kk][jj];
                }
            }
    }
}

constexpr int kMaxDzItems = 12;  // staging items per lane and unit the kernel is built for:
constexpr int kMaxXItems = 6;    // dz rows (one 16-byte load each) and x channel pairs (two loads)

// Staging of one unit.
//  dz item q: row = lane/4 + 16*(q&3), time group = lane%4 + 4*(q>>2) (8 steps each); groups
//             past the chunk land in the row's spare columns and are never read.
//  x item q:  channel pair pp = lane & 15, time group = lane/16 + 4*q.
template <int KT>
__global__ __launch_bounds__(kThreads) void wgrad_kernel(const WgradParams p)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    const TileCoords tcd = decode_tile(p);
    if (!tcd.valid) return;
    const int sp = tcd.sp, tg = tcd.tg, cot = tcd.cot, cit = tcd.cit;
    const int k0 = tg * p.KTg;
    const int kt = min(p.KTg, p.K - k0);
    const int co0 = cot * kTileCo, ci0 = cit * kTileCi;

    f32x16 acc[2][KT];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int kk = 0; kk < KT; ++kk)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][kk][r] = 0.f;

    unsigned char *wbuf0 = smem + (size_t)wave * 2 * p.buf_bytes;
    const int nsteps = p.TCH >> 4;
    const int slot_id = sp * kWaves + wave;
    const int slots = p.S * kWaves;
    const __amdgpu_buffer_rsrc_t rs_dz =
        __builtin_amdgcn_make_buffer_rsrc((void *)p.dz, 0, (int)((size_t)p.B * p.Cout * p.To * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_x =
        __builtin_amdgcn_make_buffer_rsrc((void *)p.x, 0, (int)((size_t)p.B * p.Cin * p.T * 2), 0x00020000);

    // per-lane pieces of the staging addresses that do not change with the unit
    const int dz_row = lane >> 2, dz_grp = lane & 3;  // + 16*(q&3), + 4*(q>>2)
    const int x_pp = lane & 15, x_q = lane >> 4;        // time group x_q + 4*q
    const uint32_t dz_lane_off = (uint32_t)(((co0 + dz_row) * p.To + 8 * dz_grp) * 2);
    const uint32_t x_lane_off = (uint32_t)(((ci0 + 2 * x_pp) * p.T + 8 * x_q) * 2);
    uint32_t dz_lds_off = (uint32_t)(dz_row * p.dz_row_bytes + dz_grp * 16);
    uint32_t x_lds_off = (uint32_t)(p.dz_bytes + (x_q * 8) * kXRowBytes + x_pp * 4);

    u32x4 dzr[kMaxDzItems];
    u32x4 xra[kMaxXItems], xrb[kMaxXItems];

    // issue every load of unit (b, tbase, xs_al)
    auto stage_load = [&](int b, int tbase, int xs_al) {
        const uint32_t dz_unit = (uint32_t)(((size_t)b * p.Cout * p.To + tbase) * 2);
#pragma unroll
        for (int q = 0; q < kMaxDzItems; ++q) {
            if (q < p.n_dz) {
                const int row = dz_row + 16 * (q & 3), t = tbase + 8 * (dz_grp + 4 * (q >> 2));
                const bool ok = co0 + row < p.Cout && t + 8 <= p.To;
                const uint32_t so = dz_unit + (uint32_t)((16 * (q & 3) * p.To + 32 * (q >> 2)) * 2);
                dzr[q] = buf_load16(rs_dz, ok ? dz_lane_off : kOutOfRange, so);
            }
        }
        // xs_al may be negative: fold it into the lane offset (wrap-around arithmetic is exact
        // for the lanes that are in range)
        const uint32_t x_unit = (uint32_t)((size_t)b * p.Cin * p.T * 2) + (uint32_t)(xs_al * 2);
#pragma unroll
        for (int q = 0; q < kMaxXItems; ++q) {
            if (q < p.n_x) {
                const int t = xs_al + 8 * (x_q + 4 * q);
                const bool t_ok = t >= 0 && t + 8 <= p.T;
                const bool oka = t_ok && ci0 + 2 * x_pp < p.Cin, okb = t_ok && ci0 + 2 * x_pp + 1 < p.Cin;
                const uint32_t off = x_lane_off + x_unit + (uint32_t)(64 * q);
                xra[q] = buf_load16(rs_x, oka ? off : kOutOfRange, 0);
                xrb[q] = buf_load16(rs_x, okb ? off + (uint32_t)(p.T * 2) : kOutOfRange, 0);
            }
        }
    };
    // write them to the staging buffer `buf`
    auto stage_write = [&](unsigned char *buf) {
#pragma unroll
        for (int q = 0; q < kMaxDzItems; ++q) {
            if (q < p.n_dz)
                *reinterpret_cast<u32x4 *>(buf + dz_lds_off + (16 * (q & 3)) * p.dz_row_bytes + (q >> 2) * 64) = dzr[q];
        }
#pragma unroll
        for (int q = 0; q < kMaxXItems; ++q) {
            if (q < p.n_x) {
                uint32_t *dst = reinterpret_cast<uint32_t *>(buf + x_lds_off + q * 32 * kXRowBytes);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    dst[(2 * e) * kXRowDwords] = zip_lo16(xra[q][e], xrb[q][e]);
                    dst[(2 * e + 1) * kXRowDwords] = zip_hi16(xra[q][e], xrb[q][e]);
                }
            }
        }
    };

    auto unit_coords = [&](int u, int &b, int &tbase, int &xs_al, int &off0) {
        b = u / p.nchunk;
        tbase = (u - b * p.nchunk) * p.TCH;
        const int xs = tbase * p.stride - p.pad + k0 * p.dil;
        xs_al = (xs >> 3) * 8;
        off0 = xs - xs_al;
    };

    // fragment addressing that does not depend on the unit
    const int a_lane_off = (lane & 31) * p.dz_row_bytes + (lane >> 5) * 16;  // row lane%32, t half lane/32
    const int g4 = lane >> 4, i16 = lane & 15;
    const int trow = 8 * (g4 >> 1) + (i16 >> 2);   // time row this lane addresses in a transposing read
    const int tcol = 16 * (g4 & 1) + 4 * (i16 & 3);  // first of the 4 channels it addresses
    const int x_step_bytes = 16 * p.stride * kXRowBytes;
    const int x_half_bytes = 4 * p.stride * kXRowBytes;
    const int x_tap_bytes = p.dil * kXRowBytes;

    int u = slot_id;
    if (u < p.units) {
        int b, tbase, xs_al, off0;
        unit_coords(u, b, tbase, xs_al, off0);
        // first unit of this wavefront: nothing to overlap with
        stage_load(b, tbase, xs_al);
        stage_write(wbuf0);

        int parity = 0;
        for (; u < p.units; u += slots, parity ^= 1) {
            unit_coords(u, b, tbase, xs_al, off0);
            const int un = u + slots;
            const bool has_next = un < p.units;
            const unsigned char *cur = wbuf0 + (size_t)parity * p.buf_bytes;
            unsigned char *nxt = wbuf0 + (size_t)(parity ^ 1) * p.buf_bytes;
            // the whole next unit is requested now and written to LDS after this unit's MFMAs:
            // one unit of MFMA work (about 2000 cycles) hides the memory latency
            if (has_next) {
                int bn, tbn, xsn, offn;
                unit_coords(un, bn, tbn, xsn, offn);
                stage_load(bn, tbn, xsn);
            }
            wave_lds_fence();
            const unsigned char *abase = cur + a_lane_off;
            const unsigned char *xbase = cur + p.dz_bytes + (size_t)(trow * p.stride + off0) * kXRowBytes + tcol * 2;

            auto read_frags = [&](int st, bf16x8(&af)[2], bf16x8(&bfr)[KT]) {
#pragma unroll
                for (int mi = 0; mi < 2; ++mi)
                    af[mi] = *reinterpret_cast<const bf16x8 *>(abase + mi * 32 * p.dz_row_bytes + st * 32);
                const unsigned char *xst = xbase + (size_t)st * x_step_bytes;
#pragma unroll
                for (int kk = 0; kk < KT; ++kk) {
                    // taps past the group read the last valid tap again (never used)
                    const unsigned char *xa = xst + (size_t)min(kk, kt - 1) * x_tap_bytes;
                    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(xa));
                    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(xa + x_half_bytes));
                    union {
                        s16x4 h[2];
                        bf16x8 v;
                    } cvt;
                    cvt.h[0] = lo;
                    cvt.h[1] = hi;
                    bfr[kk] = cvt.v;
                }
            };

            bf16x8 a0[2], a1[2], b0[KT], b1[KT];
            read_frags(0, a0, b0);
            for (int st = 0; st < nsteps; ++st) {
                read_frags(min(st + 1, nsteps - 1), a1, b1);
#pragma unroll
                for (int kk = 0; kk < KT; ++kk) {
                    if (kk < kt) {
#pragma unroll
                        for (int mi = 0; mi < 2; ++mi)
                            acc[mi][kk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[mi], b0[kk], acc[mi][kk], 0, 0, 0);
                    }
                }
#pragma unroll
                for (int mi = 0; mi < 2; ++mi) a0[mi] = a1[mi];
#pragma unroll
                for (int kk = 0; kk < KT; ++kk) b0[kk] = b1[kk];
            }
            if (has_next) stage_write(nxt);
        }
    }

    reduce_and_store<KT>(p, smem, acc, lane, wave, sp, k0, kt, co0, ci0);
}

// ---------------------------------------------------------------------------------------------
// Stride-1 weight gradient for dilation 1 (every block of the Jasper encoder proper) and 2 (its first
// epilog layer).
//
// Same tiling and split over time as wgrad_kernel, with two changes that cut LDS traffic and
// instruction count per MFMA:
//   * dz is produced directly in MFMA A-fragment order by dz_pack_kernel
//     ([b][co/32][t/16][lane][8]: lane l holds co = l%32, t = 8*(l/32)+j), so the A fragments of a
//     whole unit are ten contiguous 1 KiB loads from L2 straight into registers, requested two
//     units ahead; only x goes through LDS;
//   * a unit is 80 time steps = 5 MFMA steps, fully unrolled: the x window is staged transposed in
//     64-byte rows (any 4 consecutive rows cover all 64 banks, so the transposing reads are
//     conflict-free) and every fragment read is `base + immediate`.
// A last tap group that is one tap short skips that tap; shorter ones multiply unused taps.
// valid length of batch item b from an optional device array, clipped to [0, T]
__device__ __forceinline__ int clipped_len(const int *len, int b, int T)
{
    if (!len) return T;
    const int n = len[b];
    return n < 0 ? 0 : (n > T ? T : n);
}
constexpr int kFastTCH = 80;
constexpr int kFastSteps = kFastTCH / 16;
constexpr int kFastXRowBytes = 64;
// x items (32 rows each) of a unit's window: 80 steps + (KT-1)*dilation taps + up to 7 rows of alignment
constexpr int fast_x_items(int dil) { return dil == 1 ? 3 : 4; }  // 92 rows -> 3, 97 rows (dilation 2, 6 taps) -> 4

__global__ __launch_bounds__(256) void dz_pack_kernel(int Cout, int To, int ncm, int nst, const bf16_t *__restrict__ dy,
                                                      const bf16_t *__restrict__ y, int relu, u32x4 *__restrict__ dzf)
{
    const int st4 = blockIdx.x * 4 + (threadIdx.x >> 6);  // four 16-step fragments per wavefront
    if (st4 * 4 >= nst) return;
    mask_pack_wave(threadIdx.x & 63, blockIdx.z, blockIdx.y, st4, Cout, To, ncm, nst, dy, y, relu, nullptr, dzf);
}

// The unit loop of the stride-1 kernel for KA active taps (KA == KT, or KT - 1 for a short last
// group).  Units come in pairs so that two register sets for each operand and the two LDS buffers
// are named statically: the x window of unit i+2 is requested at the start of unit i and written
// to LDS at the end of unit i+1, and the dz fragments of unit i+2 are requested, fragment by
// fragment, right after their last use in unit i: two units of MFMA work for every load.  A wave
// with an odd number of units runs one more on offsets beyond the tensors: both operands read
// zeros and nothing is added.
template <int KT, int KA, int DIL>
__device__ __forceinline__ void fast_units(const WgradParams &p, unsigned char *smem, f32x16 (&acc)[2][KT], int sp,
                                           int k0, int co0, int ci0)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    constexpr int kFastXItems = fast_x_items(DIL);
    constexpr int kRows = kFastXItems * 32;  // rows of one x buffer
    constexpr int kBufBytes = kRows * kFastXRowBytes;
    unsigned char *wbuf0 = smem + (size_t)wave * 2 * kBufBytes;
    const int slot_id = sp * kWaves + wave;
    const int slots = p.S * kWaves;
    const __amdgpu_buffer_rsrc_t rs_x =
        __builtin_amdgcn_make_buffer_rsrc((void *)p.x, 0, (int)((size_t)p.B * p.Cin * p.T * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_dz = __builtin_amdgcn_make_buffer_rsrc(
        (void *)p.dzf, 0, (int)((size_t)p.B * p.ncm * p.nst * 1024), 0x00020000);

    // x staging: lane = channel pair (lane & 15) x time group (lane >> 4) + 4*q, q < 3
    const int x_pp = lane & 15, x_q = lane >> 4;
    const bool ch_a = ci0 + 2 * x_pp < p.Cin, ch_b = ci0 + 2 * x_pp + 1 < p.Cin;
    const uint32_t x_lds_off = (uint32_t)((x_q * 8) * kFastXRowBytes + x_pp * 4);
    // window start of a unit relative to its first output step: -pad + k0, aligned down to 8
    const int xs_rel = k0 * DIL - p.pad;
    const int xs_rel_al = (xs_rel >> 3) * 8;
    const int off0 = xs_rel - xs_rel_al;
    const uint32_t x_lane_a = ch_a ? (uint32_t)(((ci0 + 2 * x_pp) * p.T + 8 * x_q + xs_rel_al) * 2) : kFar;
    const uint32_t x_lane_b = ch_b ? x_lane_a + (uint32_t)(p.T * 2) : kFar;
    const int x_t0 = xs_rel_al + 8 * x_q;

    // unit number -> (batch item, chunk); units past the end get offsets beyond both tensors
    struct UnitAddr {
        uint32_t xs;  // scalar byte offset of the unit's batch item in x
        int tbase;    // first output step
        uint32_t as;  // scalar byte offset of the unit's dz fragments (channel block 0, step 0)
        int tlen;     // valid length of the unit's batch item (T without lengths)
        bool live;
    };
    auto unit_addr = [&](int u) {
        UnitAddr a;
        a.live = u < p.units;
        const int uu = a.live ? u : 0;
        const int b = uu / p.nchunk, chunk = uu - b * p.nchunk;
        a.tbase = chunk * kFastTCH;
        a.xs = (uint32_t)((size_t)b * p.Cin * p.T * 2);
        a.as = (uint32_t)((((size_t)b * p.ncm + (co0 >> 5)) * p.nst + (size_t)chunk * kFastSteps) * 1024);
        a.tlen = p.len ? __builtin_amdgcn_readfirstlane(clipped_len(p.len, b, p.T)) : p.T;
        return a;
    };
    auto x_load_item = [&](const UnitAddr &a, int q, u32x4 &xa, u32x4 &xb) {
        const int t = a.tbase + x_t0 + 32 * q;
        const bool t_ok = a.live && (unsigned)t < (unsigned)a.tlen;  // groups that start inside [0, tlen)
        // the lane offset carries the time (it is negative only where t is, and those lanes are masked)
        xa = buf_load16(rs_x, t_ok ? x_lane_a + (uint32_t)(a.tbase * 2 + 64 * q) : kFar, a.xs);
        xb = buf_load16(rs_x, t_ok ? x_lane_b + (uint32_t)(a.tbase * 2 + 64 * q) : kFar, a.xs);
    };
    auto x_load = [&](const UnitAddr &a, u32x4(&xa)[kFastXItems], u32x4(&xb)[kFastXItems]) {
#pragma unroll
        for (int q = 0; q < kFastXItems; ++q) x_load_item(a, q, xa[q], xb[q]);
    };
    auto x_write_item = [&](unsigned char *buf, int q, const u32x4 &xa, const u32x4 &xb) {
        uint32_t *dst = reinterpret_cast<uint32_t *>(buf + x_lds_off + q * 32 * kFastXRowBytes);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            dst[(2 * e) * (kFastXRowBytes / 4)] = zip_lo16(xa[e], xb[e]);
            dst[(2 * e + 1) * (kFastXRowBytes / 4)] = zip_hi16(xa[e], xb[e]);
        }
    };
    auto x_write = [&](unsigned char *buf, const u32x4(&xa)[kFastXItems], const u32x4(&xb)[kFastXItems]) {
#pragma unroll
        for (int q = 0; q < kFastXItems; ++q) x_write_item(buf, q, xa[q], xb[q]);
    };
    // With lengths the group that contains the first padding sample was staged whole: its rows from the
    // valid length on are cleared after the window has been written.
    const bool masked = p.len != nullptr;
    auto clear_padding_rows = [&](unsigned char *buf, int tlen, int tbase) {
        if (!masked) return;
        const int r0 = tlen - (tbase + xs_rel_al);
        const int nr = ((tlen + 7) & ~7) - tlen;
        if (tlen < p.T && nr > 0 && r0 >= 0 && r0 < kRows) {
            for (int r = lane >> 4; r < nr; r += 4)
                *reinterpret_cast<uint32_t *>(buf + (size_t)(r0 + r) * kFastXRowBytes + (lane & 15) * 4) = 0u;
        }
    };
    // A fragments of one unit: [mi][step], 1 KiB contiguous per wavefront and fragment
    const uint32_t a_lane = (uint32_t)lane * 16;
    const uint32_t a_mi = (uint32_t)p.nst * 1024;  // from channel block mi to mi + 1
    u32x4 afr0[2][kFastSteps], afr1[2][kFastSteps];  // even / odd unit of a pair
    auto a_load = [&](const UnitAddr &a, int mi, int st) {
        return buf_load16(rs_dz, a.live ? a_lane + (uint32_t)(st * 1024) : kFar, a.as + (uint32_t)mi * a_mi);
    };

    // transposing reads: this lane addresses 4 channels 16*((lane/16)&1) + 4*(lane&3) at time row
    // 8*(lane/32) + (lane&15)/4 (+4 for the second read of a fragment)
    const int g4 = lane >> 4, i16 = lane & 15;
    const int trow = 8 * (g4 >> 1) + (i16 >> 2) + off0;
    const int tcol = 16 * (g4 & 1) + 4 * (i16 & 3);
    const unsigned char *xb0 = wbuf0 + trow * kFastXRowBytes + tcol * 2;

    const int my_units = slot_id < p.units ? (p.units - slot_id + slots - 1) / slots : 0;
    if (my_units == 0) return;
    u32x4 xa0[kFastXItems], xb0r[kFastXItems], xa1[kFastXItems], xb1r[kFastXItems];
    int pend_tlen = 0, pend_tbase = 0;  // of the unit whose x window waits in registers for its LDS write
    {
        const UnitAddr a0 = unit_addr(slot_id), a1 = unit_addr(slot_id + slots);
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int st = 0; st < kFastSteps; ++st) {
                afr0[mi][st] = a_load(a0, mi, st);
                afr1[mi][st] = a_load(a1, mi, st);
            }
        x_load(a0, xa0, xb0r);
        x_load(a1, xa1, xb1r);   // written at the end of the first unit
        x_write(wbuf0, xa0, xb0r);
        clear_padding_rows(wbuf0, a0.tlen, a0.tbase);
        pend_tlen = a1.tlen;
        pend_tbase = a1.tbase;
    }
    // one unit: multiply from LDS buffer `par` and the fragment set afr; request the dz fragments and
    // the x window of unit u + 2*slots into afr and (xa, xb) -- the x set that was written before
    // this unit started -- and write the other x set (xo_a, xo_b: unit u + slots) into the other
    // buffer at the end.  Loads complete in order, so both streams run two units ahead: a wait for
    // a fragment also waits for every x load requested before it.
    auto unit = [&](int u, int par, u32x4(&afr)[2][kFastSteps], u32x4(&xa)[kFastXItems], u32x4(&xb)[kFastXItems],
                    const u32x4(&xo_a)[kFastXItems], const u32x4(&xo_b)[kFastXItems]) {
        const UnitAddr an = unit_addr(u + 2 * slots);
        wave_lds_fence();
        const unsigned char *xb_ = xb0 + par * kBufBytes;
        unsigned char *wr = wbuf0 + (par ^ 1) * kBufBytes;
        auto read_b = [&](int st, bf16x8(&bfr)[KA]) {
#pragma unroll
            for (int kk = 0; kk < KA; ++kk) {
                const unsigned char *xp = xb_ + (st * 16 + kk * DIL) * kFastXRowBytes;
                union {
                    s16x4 h[2];
                    bf16x8 v;
                } cvt;
                cvt.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(xp));
                cvt.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(xp + 4 * kFastXRowBytes));
                bfr[kk] = cvt.v;
            }
        };
        bf16x8 bq[2][KA];
        read_b(0, bq[0]);
        __builtin_amdgcn_sched_barrier(0);
        static_assert(kFastXItems <= kFastSteps, "one x item rides on a step: loads on the first steps, writes on the last");
#pragma unroll
        for (int st = 0; st < kFastSteps; ++st) {
            if (st + 1 < kFastSteps) read_b(st + 1, bq[(st + 1) & 1]);
#pragma unroll
            for (int mi = 0; mi < 2; ++mi) {
                union {
                    u32x4 u;
                    bf16x8 v;
                } af;
                af.u = afr[mi][st];
#pragma unroll
                for (int kk = 0; kk < KA; ++kk)
                    acc[mi][kk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af.v, bq[st & 1][kk], acc[mi][kk], 0, 0, 0);
            }
#pragma unroll
            for (int mi = 0; mi < 2; ++mi) afr[mi][st] = a_load(an, mi, st);
            // the x traffic of the unit rides on the steps: one item requested in each of the first
            // steps (the window of unit u + 2*slots), one item of the other set written in each of
            // the last steps (the window of unit u + slots, for the next unit)
            if (st < kFastXItems) x_load_item(an, st, xa[st], xb[st]);
            if (st >= kFastSteps - kFastXItems) {
                const int q = st - (kFastSteps - kFastXItems);
                x_write_item(wr, q, xo_a[q], xo_b[q]);
            }
            // Issue order inside the step: behind every MFMA one LDS read of the next step and a
            // little of the staging work (left alone, the compiler puts the reads after the MFMAs,
            // into the registers these have just freed, and waits for them at the next step).
#pragma unroll
            for (int i = 0; i < 2 * KA; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // LDS read
                __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);  // VALU (addresses, packing)
                if (i % 3 == 2) {
                    __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);  // LDS write
                    __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // VMEM read
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        clear_padding_rows(wr, pend_tlen, pend_tbase);
        pend_tlen = an.tlen;
        pend_tbase = an.tbase;
    };
    const int npairs = (my_units + 1) >> 1;
    int u = slot_id;
    for (int i = 0; i < npairs; ++i, u += 2 * slots) {
        unit(u, 0, afr0, xa0, xb0r, xa1, xb1r);
        unit(u + slots, 1, afr1, xa1, xb1r, xa0, xb0r);
    }
}

template <int KT, int DIL>
__global__ __launch_bounds__(kThreads) void wgrad_fast_kernel(const WgradParams p)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const TileCoords tcd = decode_tile(p);
    if (!tcd.valid) return;
    const int sp = tcd.sp;
    const int k0 = tcd.tg * p.KTg;
    const int kt = min(p.KTg, p.K - k0);
    const int co0 = tcd.cot * kTileCo, ci0 = tcd.cit * kTileCi;

    f32x16 acc[2][KT];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int kk = 0; kk < KT; ++kk)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][kk][r] = 0.f;

    // a last group that is one tap short skips that tap's MFMAs (shorter ones multiply unused taps)
    if (KT > 1 && kt == KT - 1)
        fast_units<KT, (KT > 1 ? KT - 1 : 1), DIL>(p, smem, acc, sp, k0, co0, ci0);
    else
        fast_units<KT, KT, DIL>(p, smem, acc, sp, k0, co0, ci0);
    reduce_and_store<KT>(p, smem, acc, lane, wave, sp, k0, kt, co0, ci0);
}

// ---------------------------------------------------------------------------------------------
// Stride-1 weight gradient with the taps split over the wavefronts.
//
// In wgrad_fast_kernel every wavefront stages its own x window, and a staged element serves only
// 2 x 6 accumulator blocks; the transposing staging (scattered 16-byte loads, 4-byte LDS writes) then
// costs a quarter of the main loop.  Here the four wavefronts of a workgroup walk through the SAME
// units and share one staged window that covers all KG taps of the group (128 rows: each wavefront
// loads and writes one 32-row item, a quarter of the work), and split the 2*KG accumulator blocks
// (tap, 32-channel half of the 64 output channels) among themselves.  A block is owned by one
// wavefront for the whole reduction, so there is no exchange at the end: every wavefront stores its
// blocks to the [S][K][Cout][Cin] scratch.
//
// Which blocks a wavefront owns.  The B fragment of tap t at a step is two transposing LDS reads, of
// rows t*DIL and t*DIL + 4 (relative to the step): taps that are 4/DIL apart share a read.  So the taps
// are dealt out in chains of that stride -- dilation 1: tap t belongs to wavefront t mod 4 (the K mod 4
// taps that are left over are dealt out half by half); dilation 2: even taps form one chain, odd taps
// the other, each cut in two -- and a wavefront reads each row once per step: K = 17 needs 6, 7, 5, 5 reads
// per step in the four wavefronts for 9, 9, 8, 8 blocks, where consecutive taps would need 10 to 12.
//
// Pipeline.  Three window buffers: during unit u (window u in buffer u mod 3) every wavefront writes its
// item of window u+2 (requested one unit earlier) and requests window u+3; the barrier at the end of a
// unit therefore orders things that are a whole unit apart, and the fragments of the next unit's first
// step are read from LDS before it, so the matrix pipe has its operands when the barrier opens.  The
// g = dy*[y>0] fragments stream from L2 straight into registers, two units ahead (all four wavefronts
// read the same ones: L1 hits).
struct TapPlan {
    int nb;                // accumulator blocks of this wavefront
    int tap[16], half[16];
    int nrow;              // distinct rows (relative to the step's first row, in units of DIL-less rows) it reads
    int row[32];
    int lo[16], hi[16];    // per block: positions in row[] of its two reads
};
template <int KG, int DIL>
constexpr int block_owner(int tap, int half)
{
    if (DIL == 1) {
        constexpr int Q4 = (KG / 4) * 4;
        return tap < Q4 ? tap % 4 : (2 * (tap - Q4) + half) % 4;
    }
    const int pos = tap / 2;
    if (tap % 2 == 0) return pos < ((KG + 1) / 2 + 1) / 2 ? 0 : 1;
    return pos < (KG / 2 + 1) / 2 ? 2 : 3;
}
template <int KG, int DIL, int W>
constexpr TapPlan make_tap_plan()
{
    TapPlan q = {};
    for (int tap = 0; tap < KG; ++tap)
        for (int half = 0; half < 2; ++half)
            if (block_owner<KG, DIL>(tap, half) == W) {
                q.tap[q.nb] = tap;
                q.half[q.nb] = half;
                ++q.nb;
            }
    for (int j = 0; j < q.nb; ++j) {
        for (int e = 0; e < 2; ++e) {
            const int r = q.tap[j] * DIL + 4 * e;
            int at = -1;
            for (int i = 0; i < q.nrow; ++i)
                if (q.row[i] == r) at = i;
            if (at < 0) {
                at = q.nrow;
                q.row[q.nrow++] = r;
            }
            (e == 0 ? q.lo[j] : q.hi[j]) = at;
        }
    }
    return q;
}

// LEN: the launch carries valid lengths; the units of an item whose x window lies wholly in the padding
// multiply zeros and are left out of the enumeration (every workgroup walks the same shortened list).
template <int KG, int DIL, int W, bool LEN>
__device__ __forceinline__ void shared_units(const WgradParams &p, unsigned char *smem, int sp, int k0, int kt, int co0,
                                             int ci0)
{
    constexpr TapPlan plan = make_tap_plan<KG, DIL, W>();
    constexpr int NBW = plan.nb, NROW = plan.nrow;
    static_assert(NBW >= 1 && NBW <= 16 && NROW <= 32, "tap plan out of range");
    constexpr int kRows = 128, kBufBytes = kRows * kFastXRowBytes;  // three such windows in LDS
    const int lane = threadIdx.x & 63;
    const int S = p.S;
    const __amdgpu_buffer_rsrc_t rs_x =
        __builtin_amdgcn_make_buffer_rsrc((void *)p.x, 0, (int)((size_t)p.B * p.Cin * p.T * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_dz = __builtin_amdgcn_make_buffer_rsrc(
        (void *)p.dzf, 0, (int)((size_t)p.B * p.ncm * p.nst * 1024), 0x00020000);

    // x staging: this wavefront's item is rows 32*W .. 32*W+31 of the window; lane = channel pair
    // (lane & 15) x time group (lane >> 4)
    const int x_pp = lane & 15, x_q = lane >> 4;
    const bool ch_a = ci0 + 2 * x_pp < p.Cin, ch_b = ci0 + 2 * x_pp + 1 < p.Cin;
    const uint32_t x_lds_off = (uint32_t)((32 * W + x_q * 8) * kFastXRowBytes + x_pp * 4);
    const int xs_rel = k0 * DIL - p.pad;
    const int xs_rel_al = (xs_rel >> 3) * 8;
    const int off0 = xs_rel - xs_rel_al;
    const uint32_t x_lane_a = ch_a ? (uint32_t)(((ci0 + 2 * x_pp) * p.T + 8 * x_q + xs_rel_al + 32 * W) * 2) : kFar;
    const uint32_t x_lane_b = ch_b ? x_lane_a + (uint32_t)(p.T * 2) : kFar;
    const int x_t0 = xs_rel_al + 8 * x_q + 32 * W;

    struct UnitAddr {
        uint32_t xs, as;
        int tbase;
        int tlen;  // valid length of the unit's batch item (T without lengths)
        bool live;
    };
    // units of this workgroup: sp, sp + S, sp + 2S, ...; (batch item, chunk) advance without divisions
    const int step_b = S / p.nchunk, step_c = S - step_b * p.nchunk;
    struct UnitPos {
        int b, c;
    };
    // with lengths: chunks of item b that reach below its valid length (chunk c reads x from c*80 - pad on)
    auto live_chunks_of = [&](int tl) { return tl > 0 ? min(p.nchunk, (tl + p.pad + kFastTCH - 1) / kFastTCH) : 0; };
    auto carry_over = [&](UnitPos &q) {  // c counts live chunks from the start of item b onwards
        while (q.b < p.B) {
            const int n = live_chunks_of(__builtin_amdgcn_readfirstlane(clipped_len(p.len, q.b, p.T)));
            if (q.c < n) break;
            q.c -= n;
            ++q.b;
        }
    };
    auto unit_pos = [&](int u) {
        if constexpr (LEN) {
            UnitPos q{0, u};
            carry_over(q);
            return q;
        } else {
            return UnitPos{u / p.nchunk, u % p.nchunk};
        }
    };
    auto advance = [&](UnitPos &q) {
        if constexpr (LEN) {
            q.c += S;
            carry_over(q);
        } else {
            q.b += step_b;
            q.c += step_c;
            const bool carry = q.c >= p.nchunk;
            q.c -= carry ? p.nchunk : 0;
            q.b += carry ? 1 : 0;
        }
    };
    auto unit_addr = [&](const UnitPos &q) {
        UnitAddr a;
        a.live = q.b < p.B;
        const int b = a.live ? q.b : 0;
        a.tbase = q.c * kFastTCH;
        a.xs = (uint32_t)b * (uint32_t)(p.Cin * p.T * 2);
        a.as = (uint32_t)((b * p.ncm + (co0 >> 5)) * p.nst + q.c * kFastSteps) * 1024u;
        a.tlen = p.len ? __builtin_amdgcn_readfirstlane(clipped_len(p.len, b, p.T)) : p.T;
        return a;
    };
    auto x_load_item = [&](const UnitAddr &a, u32x4 &xa, u32x4 &xb) {
        const int t = a.tbase + x_t0;
        const bool t_ok = a.live && (unsigned)t < (unsigned)a.tlen;  // groups that start inside [0, tlen)
        xa = buf_load16(rs_x, t_ok ? x_lane_a + (uint32_t)(a.tbase * 2) : kFar, a.xs);
        xb = buf_load16(rs_x, t_ok ? x_lane_b + (uint32_t)(a.tbase * 2) : kFar, a.xs);
    };
    auto x_write_item = [&](unsigned char *buf, const u32x4 &xa, const u32x4 &xb) {
        uint32_t *dst = reinterpret_cast<uint32_t *>(buf + x_lds_off);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            dst[(2 * e) * (kFastXRowBytes / 4)] = zip_lo16(xa[e], xb[e]);
            dst[(2 * e + 1) * (kFastXRowBytes / 4)] = zip_hi16(xa[e], xb[e]);
        }
    };
    // With lengths the group that contains the first padding sample was staged whole: the wavefront
    // whose item holds it clears its rows from the valid length on (after its write, before the barrier).
    const bool masked = p.len != nullptr;
    auto clear_padding_rows = [&](unsigned char *buf, int tlen, int tbase) {
        if (!masked) return;
        const int r0 = tlen - (tbase + xs_rel_al);   // first padding row of the window
        const int nr = ((tlen + 7) & ~7) - tlen;
        if (tlen < p.T && nr > 0 && r0 >= 32 * W && r0 < 32 * W + 32) {
            for (int r = lane >> 4; r < nr; r += 4)
                *reinterpret_cast<uint32_t *>(buf + (size_t)(r0 + r) * kFastXRowBytes + (lane & 15) * 4) = 0u;
        }
    };
    const uint32_t a_lane = (uint32_t)lane * 16;
    const uint32_t a_mi = (uint32_t)p.nst * 1024;
    u32x4 afr0[2][kFastSteps], afr1[2][kFastSteps];
    auto a_load = [&](const UnitAddr &a, int mi, int st) {
        return buf_load16(rs_dz, a.live ? a_lane + (uint32_t)(st * 1024) : kFar, a.as + (uint32_t)mi * a_mi);
    };
    // transposing reads: this lane addresses 4 channels 16*((lane/16)&1) + 4*(lane&3) at time row
    // 8*(lane/32) + (lane&15)/4 of the block it reads
    const int g4 = lane >> 4, i16 = lane & 15;
    const int trow = 8 * (g4 >> 1) + (i16 >> 2) + off0;
    const int tcol = 16 * (g4 & 1) + 4 * (i16 & 3);
    const unsigned char *xb0 = smem + trow * kFastXRowBytes + tcol * 2;
    // rows of step st, from the window whose bytes start at xw (a pointer that already carries the lane part)
    auto read_rows = [&](const unsigned char *xw, int st, s16x4(&dst)[NROW]) {
#pragma unroll
        for (int i = 0; i < NROW; ++i)
            dst[i] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(xw + (st * 16 + plan.row[i]) * kFastXRowBytes));
    };

    f32x16 acc[NBW];
#pragma unroll
    for (int j = 0; j < NBW; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;

    int units = p.units;
    if constexpr (LEN) {  // live units of the whole batch: one item per lane, summed over the wavefront
        units = 0;
        for (int b0 = 0; b0 < p.B; b0 += 64) {
            int n = b0 + lane < p.B ? live_chunks_of(clipped_len(p.len, b0 + lane, p.T)) : 0;
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) n += __shfl_xor(n, m, 64);
            units += __builtin_amdgcn_readfirstlane(n);
        }
    }
    const int my_units = sp < units ? (units - sp + S - 1) / S : 0;  // the same for all four wavefronts
    // x items in flight: two register sets; set X(u mod 2) is written to LDS during unit u (it holds this
    // wavefront's item of window u+2), set X((u+1) mod 2) is requested during unit u (window u+3)
    u32x4 xa0, xb0r, xa1, xb1r;
    int tlen0 = 0, tbase0 = 0, tlen1 = 0, tbase1 = 0;  // of the windows waiting in the two sets
    s16x4 rd[2][NROW];                                  // rows of the current / the next step
    UnitPos ahead = unit_pos(sp);                       // the unit whose window is requested next
    UnitPos behind = ahead;                             // with lengths: the unit before `ahead`
    {
        const UnitAddr a0 = unit_addr(ahead);
        advance(ahead);
        const UnitAddr a1 = unit_addr(ahead);
        advance(ahead);
        const UnitAddr a2 = unit_addr(ahead);
        behind = ahead;
        advance(ahead);
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int st = 0; st < kFastSteps; ++st) {
                afr0[mi][st] = a_load(a0, mi, st);
                afr1[mi][st] = a_load(a1, mi, st);
            }
        x_load_item(a0, xa0, xb0r);
        x_load_item(a1, xa1, xb1r);
        x_write_item(smem, xa0, xb0r);
        clear_padding_rows(smem, a0.tlen, a0.tbase);
        x_write_item(smem + kBufBytes, xa1, xb1r);
        clear_padding_rows(smem + kBufBytes, a1.tlen, a1.tbase);
        x_load_item(a2, xa0, xb0r);  // window 2: written during unit 0
        tlen0 = a2.tlen;
        tbase0 = a2.tbase;
        __syncthreads();
        read_rows(xb0, 0, rd[0]);
    }
    // byte offsets of the buffers holding window u, u+1 and the one being written (window u+2)
    int cur = 0, nxt = kBufBytes, wr = 2 * kBufBytes;
    // one unit; PAR: which of rd[] holds its first step (units alternate, a unit has five steps)
    auto unit = [&](auto par_c, u32x4(&afr)[2][kFastSteps], u32x4 &xa, u32x4 &xb, int &tlen_req, int &tbase_req,
                    const u32x4 &xo_a, const u32x4 &xo_b, int tlen_wr, int tbase_wr) {
        constexpr int PAR = decltype(par_c)::value;
        // the dz fragments requested in this unit are those of the unit after the next; the x item is one further
        UnitPos two = ahead;  // `ahead` is three units on
        if constexpr (LEN) {
            two = behind;  // the shortened list has no fixed step to take back
            behind = ahead;
        } else {
            two.b -= step_b;
            two.c -= step_c;
            if (two.c < 0) {
                two.c += p.nchunk;
                two.b -= 1;
            }
        }
        const UnitAddr an2 = unit_addr(two);
        const UnitAddr an3 = unit_addr(ahead);
        advance(ahead);
        const unsigned char *xw = xb0 + cur, *xn = xb0 + nxt;
        unsigned char *wbuf = smem + wr;
#pragma unroll
        for (int st = 0; st < kFastSteps; ++st) {
            constexpr int dummy = 0;
            (void)dummy;
            s16x4(&rc)[NROW] = rd[(PAR + st) & 1];
            s16x4(&rn)[NROW] = rd[(PAR + st + 1) & 1];
            if (st + 1 < kFastSteps)
                read_rows(xw, st + 1, rn);
            else
                read_rows(xn, 0, rn);  // first step of the next unit: its window was complete a barrier ago
#pragma unroll
            for (int j = 0; j < NBW; ++j) {
                union {
                    u32x4 u;
                    bf16x8 v;
                } af;
                af.u = afr[plan.half[j]][st];
                union {
                    s16x4 h[2];
                    bf16x8 v;
                } bf;
                bf.h[0] = rc[plan.lo[j]];
                bf.h[1] = rc[plan.hi[j]];
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af.v, bf.v, acc[j], 0, 0, 0);
            }
#pragma unroll
            for (int mi = 0; mi < 2; ++mi) afr[mi][st] = a_load(an2, mi, st);
            if (st == 0) x_load_item(an3, xa, xb);
            if (st == kFastSteps - 1) x_write_item(wbuf, xo_a, xo_b);
#pragma unroll
            for (int i = 0; i < NBW; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // LDS read
                __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);  // VALU
                if (i % 3 == 2) {
                    __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);  // LDS write
                    __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // VMEM read
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        clear_padding_rows(wbuf, tlen_wr, tbase_wr);
        tlen_req = an3.tlen;
        tbase_req = an3.tbase;
        const int old = cur;
        cur = nxt;
        nxt = wr;
        wr = old;
        __syncthreads();  // window u+2 is complete; window u may be overwritten from the next unit on
    };
    const int npairs = (my_units + 1) >> 1;
    for (int i = 0; i < npairs; ++i) {
        unit(std::integral_constant<int, 0>{}, afr0, xa1, xb1r, tlen1, tbase1, xa0, xb0r, tlen0, tbase0);
        unit(std::integral_constant<int, 1>{}, afr1, xa0, xb0r, tlen0, tbase0, xa1, xb1r, tlen1, tbase1);
    }

    // ---- every block goes straight to the scratch: register r of a block is output channel
    // co0 + 32*half + 8*(r/4) + 4*(lane/32) + r%4, input channel ci0 + lane%32
    const int ci = ci0 + (lane & 31);
    if (ci < p.Cin) {
#pragma unroll
        for (int j = 0; j < NBW; ++j) {
            const int tap = plan.tap[j], half = plan.half[j];
            if (tap >= kt) continue;  // a group shorter than KG
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int co = co0 + 32 * half + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (co < p.Cout) p.part[(((size_t)sp * p.K + k0 + tap) * p.Cout + co) * p.Cin + ci] = acc[j][r];
            }
        }
    }
}

template <int KG, int DIL, bool LEN = false>
__global__ __launch_bounds__(kThreads) void wgrad_shared_kernel(const WgradParams p)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const TileCoords tcd = decode_tile(p);
    if (!tcd.valid) return;
    const int k0 = tcd.tg * p.KTg;
    const int kt = min(p.KTg, p.K - k0);
    const int co0 = tcd.cot * kTileCo, ci0 = tcd.cit * kTileCi;
    switch (wave) {  // one copy per wavefront number: the block lists are static
    case 0: shared_units<KG, DIL, 0, LEN>(p, smem, tcd.sp, k0, kt, co0, ci0); break;
    case 1: shared_units<KG, DIL, 1, LEN>(p, smem, tcd.sp, k0, kt, co0, ci0); break;
    case 2: shared_units<KG, DIL, 2, LEN>(p, smem, tcd.sp, k0, kt, co0, ci0); break;
    default: shared_units<KG, DIL, 3, LEN>(p, smem, tcd.sp, k0, kt, co0, ci0); break;
    }
}

// dw[co][ci][k] = (accumulate ? dw : 0) + scale[co] * sum_s part[s][k][co][ci]; one block per (co, 64 ci).
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const float *__restrict__ part, float *__restrict__ dw,
                                                           const float *__restrict__ scale, int S, int K, int Cout,
                                                           int Cin, int accumulate)
{
    extern __shared__ float tile[];  // [64][K+1]
    const int co = blockIdx.y;
    const int ci0 = blockIdx.x * 64;
    const int l = threadIdx.x & 63, kq = threadIdx.x >> 6;
    const int ci = ci0 + l;
    const size_t plane = (size_t)Cout * Cin;
    const float factor = scale ? scale[co] : 1.f;
    for (int k = kq; k < K; k += 4) {
        float s = 0.f;
        if (ci < Cin) {
            const float *src = part + ((size_t)k * Cout + co) * Cin + ci;
            for (int sp = 0; sp < S; ++sp) s += src[(size_t)sp * K * plane];
        }
        tile[l * (K + 1) + k] = s * factor;
    }
    __syncthreads();
    const int nci = min(64, Cin - ci0);
    const int n = nci * K;
    float *dst = dw + ((size_t)co * Cin + ci0) * K;
    for (int e = threadIdx.x; e < n; e += 256) {
        const int c = e / K, k = e - c * K;
        const float val = tile[c * (K + 1) + k];
        dst[e] = accumulate ? dst[e] + val : val;
    }
}

// The same for Cin % 4 == 0 and 16-byte aligned dw: one block per (co, 256 ci), 16-byte loads along ci
// (a wavefront reads 1 KiB contiguous per partial row) and 16-byte stores of the transposed tile.
constexpr int kReduce4Ci = 256;
__global__ __launch_bounds__(256) void wgrad_reduce4_kernel(const float *__restrict__ part, float *__restrict__ dw,
                                                            const float *__restrict__ scale, int S, int K, int Cout,
                                                            int Cin, int accumulate)
{
    extern __shared__ float tile[];  // [256][K+1]
    const int co = blockIdx.y;
    const int ci0 = blockIdx.x * kReduce4Ci;
    const int l = threadIdx.x & 63, kq = threadIdx.x >> 6;
    const int ci = ci0 + 4 * l;
    const size_t plane = (size_t)Cout * Cin;
    const float factor = scale ? scale[co] : 1.f;
    for (int k = kq; k < K; k += 4) {
        f32x4 sum = {0.f, 0.f, 0.f, 0.f};
        if (ci < Cin) {
            const float *src = part + ((size_t)k * Cout + co) * Cin + ci;
            for (int sp = 0; sp < S; ++sp) sum += *reinterpret_cast<const f32x4 *>(src + (size_t)sp * K * plane);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) tile[(4 * l + e) * (K + 1) + k] = sum[e] * factor;
    }
    __syncthreads();
    const int nci = min(kReduce4Ci, Cin - ci0);
    const int n = nci * K;  // a multiple of 4
    float *dst = dw + ((size_t)co * Cin + ci0) * K;
    for (int e0 = threadIdx.x * 4; e0 < n; e0 += 1024) {
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int c = (e0 + e) / K, k = (e0 + e) - c * K;
            v[e] = tile[c * (K + 1) + k];
        }
        f32x4 *o = reinterpret_cast<f32x4 *>(dst + e0);
        *o = accumulate ? *o + v : v;
    }
}

struct WPlan {
    bool ok;
    int KTg, ntg, TCH, NRX, S;
    int n_dz, n_x, ips;
    int dz_row_bytes, dz_bytes, x_bytes, buf_bytes;
    size_t lds;
};

// Needs 16-byte aligned rows of both operands (T % 8 == 0 and To % 8 == 0).
WPlan make_wplan(const Geom &g)
{
    WPlan w = {};
    if (g.T % 8 != 0 || g.To % 8 != 0) return w;
    const int ntg = (g.K + kMaxKT - 1) / kMaxKT;
    const int KTg = (g.K + ntg - 1) / ntg;
    w.ntg = (g.K + KTg - 1) / KTg;
    w.KTg = KTg;
    const int cands[4] = {80, 64, 48, 32};
    const size_t red = (size_t)kWaves * 3 * (2 * KTg) * 64 * sizeof(f32x4);
    for (int c = 0; c < 4; ++c) {
        const int tch = cands[c];
        if (c < 3 && g.To <= cands[c + 1]) continue;  // do not stage far beyond a short row
        const long rows = (long)(tch - 1) * g.stride + (long)(KTg - 1) * g.dil + 1 + 7;
        const long nrx = (rows + 7) / 8 * 8;
        const long n_x = (nrx / 8 * 16 + 63) / 64;
        const long gpr4 = (tch / 8 + 3) / 4 * 4;       // time groups per dz row, padded to 4
        const long n_dz = gpr4;                         // 4 row blocks x gpr4/4 group blocks
        const long dzrow = gpr4 * 16 + 16;
        const long dzb = kTileCo * dzrow, xb = n_x * 32 * kXRowBytes;
        const long nsteps = tch / 16;
        const long ips = (n_dz + n_x + nsteps - 1) / nsteps;
        const size_t stage = (size_t)kWaves * 2 * (dzb + xb);
        const size_t lds = stage > red ? stage : red;
        if (lds <= (size_t)kMaxLds && n_dz <= kMaxDzItems && n_x <= kMaxXItems) {
            w.ok = true;
            w.TCH = tch; w.NRX = (int)nrx;
            w.n_dz = (int)n_dz; w.n_x = (int)n_x; w.ips = (int)ips;
            w.dz_row_bytes = (int)dzrow; w.dz_bytes = (int)dzb; w.x_bytes = (int)xb; w.buf_bytes = (int)(dzb + xb);
            w.lds = lds;
            break;
        }
    }
    if (!w.ok) return w;
    const int ncot = (g.Cout + kTileCo - 1) / kTileCo, ncit = (g.Cin + kTileCi - 1) / kTileCi;
    const long ntiles = (long)ncot * ncit * w.ntg;
    const long units = (long)g.B * ((g.To + w.TCH - 1) / w.TCH);
    long S = (512 + ntiles - 1) / ntiles;
    if (S > 8) S = 8;
    if (S > units / kWaves) S = units / kWaves;
    if (S < 1) S = 1;
    w.S = (int)S;
    return w;
}

// The stride-1, dilation-1 kernel applies when rows are 16-byte aligned; its split count.
bool fast_ok(const Geom &g)
{
    if (!(g.stride == 1 && (g.dil == 1 || g.dil == 2) && g.T % 8 == 0 && g.To % 8 == 0)) return false;
    // both operands are addressed through buffer descriptors with 32-bit offsets
    const size_t lim = (size_t)1 << 30;
    const size_t nst = (size_t)((g.To + kFastTCH - 1) / kFastTCH) * kFastSteps;
    const size_t ncm = (size_t)((g.Cout + kTileCo - 1) / kTileCo) * 2;
    return (size_t)g.B * g.Cin * g.T * sizeof(bf16_t) <= lim && (size_t)g.B * ncm * nst * 1024 <= lim;
}
struct FastPlan {
    int KTg, ntg, S, nchunk, ncm, nst;
    size_t lds;
    bool shared;  // wgrad_shared_kernel (taps split over the wavefronts) instead of wgrad_fast_kernel
};
// tap-group sizes wgrad_shared_kernel is built for
constexpr bool shared_kernel_built(int KG, int dil) { return dil == 1 ? (KG == 11 || KG == 13 || KG == 17 || KG == 21) : (dil == 2 && KG == 15); }
constexpr int kPlanCUs = 256;  // the planning below aims at this many CUs (a heuristic only: any count works)
FastPlan make_fast_plan(const Geom &g)
{
    FastPlan f = {};
    const int ntg = (g.K + kMaxKT - 1) / kMaxKT;
    f.KTg = (g.K + ntg - 1) / ntg;
    f.ntg = (g.K + f.KTg - 1) / f.KTg;
    f.nchunk = (g.To + kFastTCH - 1) / kFastTCH;
    const int ncot = (g.Cout + kTileCo - 1) / kTileCo, ncit = (g.Cin + kTileCi - 1) / kTileCi;
    f.ncm = ncot * 2;
    f.nst = f.nchunk * kFastSteps;
    const long ntiles = (long)ncot * ncit * f.ntg, units = (long)g.B * f.nchunk;
    long S = (512 + ntiles - 1) / ntiles;
    if (S > 8) S = 8;
    if (S > units / kWaves) S = units / kWaves;
    if (S < 1) S = 1;
    f.S = (int)S;
    const size_t stage = (size_t)kWaves * 2 * fast_x_items(g.dil) * 32 * kFastXRowBytes;
    const size_t red = (size_t)kWaves * 3 * (2 * f.KTg) * 64 * sizeof(f32x4);
    f.lds = stage > red ? stage : red;
    // The kernel with shared staging: up to 24 taps per workgroup (12 accumulator blocks per wavefront);
    // it has no dynamic balancing to speak of (few, long workgroups), so it is taken only when a split
    // count S <= 8 makes the workgroups fill the CUs in whole rounds (>= 95 %).
    {
        const int ntg_s = (g.K + 23) / 24;
        const int KG = (g.K + ntg_s - 1) / ntg_s;
        const long tiles_s = (long)ncot * ncit * ((g.K + KG - 1) / KG);
        if (shared_kernel_built(KG, g.dil) && 18 + 64 + (KG - 1) * g.dil + 4 < 128) {
            for (long Ss = 1; Ss <= 8 && Ss * 2 <= units; ++Ss) {
                const long wgs = tiles_s * Ss, rounds = (wgs + kPlanCUs - 1) / kPlanCUs;
                if (wgs * 100 >= rounds * kPlanCUs * 95) {
                    f.shared = true;
                    f.KTg = KG;
                    f.ntg = (g.K + KG - 1) / KG;
                    f.S = (int)Ss;
                    f.lds = 3 * 128 * kFastXRowBytes;
                    break;
                }
            }
        }
    }
    return f;
}
size_t dzf_bytes(const Geom &g, const FastPlan &f) { return align_up((size_t)g.B * f.ncm * f.nst * 1024, 256); }

size_t part_bytes(const Geom &g, int S) { return align_up((size_t)S * g.K * g.Cout * g.Cin * sizeof(float), 256); }
size_t dz_buf_bytes(const Geom &g) { return align_up((size_t)g.B * g.Cout * g.To * sizeof(bf16_t), 256); }

template <int KT, int DIL>
hipError_t launch_fast_kt(const WgradParams &p, size_t lds, int grid, hipStream_t s)
{
    auto kern = wgrad_fast_kernel<KT, DIL>;
    static LdsOptIn opt_in;
    hipError_t e = ensure_dynamic_lds(opt_in, reinterpret_cast<const void *>(kern), kMaxLds);
    if (e != hipSuccess) return e;
    MainKernelTimer timer(s);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), lds, s, p);
    return hipGetLastError();
}

template <int KG, int DIL>
hipError_t launch_shared(const WgradParams &p, size_t lds, int grid, hipStream_t s)
{
    MainKernelTimer timer(s);
    if (p.len)
        hipLaunchKernelGGL((wgrad_shared_kernel<KG, DIL, true>), dim3(grid), dim3(kThreads), lds, s, p);
    else
        hipLaunchKernelGGL((wgrad_shared_kernel<KG, DIL>), dim3(grid), dim3(kThreads), lds, s, p);
    return hipGetLastError();
}

void number_work_items(WgradParams &p)
{
    p.total = p.ncot * p.ncit * p.ntg * p.S;
    p.per_xcd = (p.total + 7) / 8;
    p.CL = 0;
    if (p.total % 8 == 0) {
        const int denom = p.ntg * p.ncit;
        if (p.per_xcd % denom == 0) {
            const int cl = p.per_xcd / denom;
            if (cl >= 1 && p.ncot % cl == 0) p.CL = cl;
        }
    }
}

template <int KT>
hipError_t launch_kt(const WgradParams &p, size_t lds, int grid, hipStream_t s)
{
    auto kern = wgrad_kernel<KT>;
    static LdsOptIn opt_in;
    hipError_t e = ensure_dynamic_lds(opt_in, reinterpret_cast<const void *>(kern), kMaxLds);
    if (e != hipSuccess) return e;
    MainKernelTimer timer(s);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), lds, s, p);
    return hipGetLastError();
}

// the reduction's LDS tile is [64][K+1] floats: the default 64 KiB limit bounds the tap count
constexpr int kMaxReduceTaps = 64 * 1024 / (64 * (int)sizeof(float)) - 1;  // 255
}  // namespace

hipError_t launch_wgrad_reduce(const Geom &g, const float *part, float *dw, const float *scale, int S, bool accumulate,
                         hipStream_t s)
{
    if (g.Cin % 4 == 0 && ((uintptr_t)dw % 16) == 0 && (size_t)kReduce4Ci * (g.K + 1) * sizeof(float) <= 64 * 1024) {
        dim3 grid4((g.Cin + kReduce4Ci - 1) / kReduce4Ci, g.Cout);
        hipLaunchKernelGGL(wgrad_reduce4_kernel, grid4, dim3(256), kReduce4Ci * (g.K + 1) * sizeof(float), s, part, dw, scale,
                           S, g.K, g.Cout, g.Cin, accumulate ? 1 : 0);
        return hipGetLastError();
    }
    dim3 rgrid((g.Cin + 63) / 64, g.Cout);
    hipLaunchKernelGGL(wgrad_reduce_kernel, rgrid, dim3(256), 64 * (g.K + 1) * sizeof(float), s, part, dw, scale, S, g.K,
                       g.Cout, g.Cin, accumulate ? 1 : 0);
    return hipGetLastError();
}

bool mfma_wgrad_supported(const Geom &g) { return g.K <= kMaxReduceTaps && (fast_ok(g) || make_wplan(g).ok); }

size_t mfma_wgrad_workspace(const Geom &g, bool need_dz)
{
    // (sized without looking at lengths: a call with lengths never takes the pointwise kernel)
    Geom g0 = g;
    g0.len = nullptr;
    if (wgrad_k1_supported(g0)) {
        const FastPlan f = make_fast_plan(g);
        const size_t fast = part_bytes(g, f.S) + dzf_bytes(g, f);
        const size_t k1 = wgrad_k1_part_bytes(g0) + dz_buf_bytes(g);
        return fast > k1 ? fast : k1;
    }
    if (fast_ok(g)) {
        const FastPlan f = make_fast_plan(g);
        return part_bytes(g, f.S) + dzf_bytes(g, f);
    }
    const WPlan w = make_wplan(g);
    if (!w.ok) return 0;
    return part_bytes(g, w.S) + (need_dz ? dz_buf_bytes(g) : 0);
}

// ---- stride-1 kernel with dz already in fragment order (dz_pack_kernel's layout) ----------------
bool mfma_wgrad_fast_supported(const Geom &g) { return fast_ok(g); }

DzfLayout mfma_wgrad_dzf_layout(const Geom &g)
{
    const FastPlan f = make_fast_plan(g);
    DzfLayout l;
    l.ncm = f.ncm;
    l.nst = f.nst;
    l.offset = part_bytes(g, f.S);
    l.bytes = dzf_bytes(g, f);
    return l;
}

hipError_t launch_mfma_wgrad_prepared(const Geom &g, const void *x, const float *scale, float *dw, bool accumulate, void *ws,
                                      hipStream_t s)
{
    const FastPlan f = make_fast_plan(g);
    float *part = (float *)ws;
    const u32x4 *dzf = (const u32x4 *)((unsigned char *)ws + part_bytes(g, f.S));
    WgradParams p = {};
    p.B = g.B; p.Cin = g.Cin; p.Cout = g.Cout; p.T = g.T; p.To = g.To; p.K = g.K;
    p.stride = 1; p.dil = g.dil; p.pad = g.pad;
    p.ncot = (g.Cout + kTileCo - 1) / kTileCo;
    p.ncit = (g.Cin + kTileCi - 1) / kTileCi;
    p.ntg = f.ntg; p.KTg = f.KTg; p.S = f.S;
    p.TCH = kFastTCH; p.nchunk = f.nchunk; p.units = g.B * f.nchunk;
    p.ncm = f.ncm; p.nst = f.nst;
    number_work_items(p);
    if (f.shared) p.CL = -1;
    p.x = (const bf16_t *)x; p.dzf = dzf; p.part = part;
    p.len = g.len;
    const int grid = p.per_xcd * 8;
    hipError_t e;
    if (f.shared) {
        switch (f.KTg * 10 + g.dil) {
        case 111: e = launch_shared<11, 1>(p, f.lds, grid, s); break;
        case 131: e = launch_shared<13, 1>(p, f.lds, grid, s); break;
        case 171: e = launch_shared<17, 1>(p, f.lds, grid, s); break;
        case 211: e = launch_shared<21, 1>(p, f.lds, grid, s); break;
        case 152: e = launch_shared<15, 2>(p, f.lds, grid, s); break;
        default: e = hipErrorInvalidValue; break;
        }
    } else if (g.dil == 1) {
        switch (f.KTg) {
        case 1: e = launch_fast_kt<1, 1>(p, f.lds, grid, s); break;
        case 2: e = launch_fast_kt<2, 1>(p, f.lds, grid, s); break;
        case 3: e = launch_fast_kt<3, 1>(p, f.lds, grid, s); break;
        case 4: e = launch_fast_kt<4, 1>(p, f.lds, grid, s); break;
        case 5: e = launch_fast_kt<5, 1>(p, f.lds, grid, s); break;
        default: e = launch_fast_kt<6, 1>(p, f.lds, grid, s); break;
        }
    } else {
        switch (f.KTg) {
        case 1: e = launch_fast_kt<1, 2>(p, f.lds, grid, s); break;
        case 2: e = launch_fast_kt<2, 2>(p, f.lds, grid, s); break;
        case 3: e = launch_fast_kt<3, 2>(p, f.lds, grid, s); break;
        case 4: e = launch_fast_kt<4, 2>(p, f.lds, grid, s); break;
        case 5: e = launch_fast_kt<5, 2>(p, f.lds, grid, s); break;
        default: e = launch_fast_kt<6, 2>(p, f.lds, grid, s); break;
        }
    }
    if (e != hipSuccess) return e;
    return launch_wgrad_reduce(g, part, dw, scale, f.S, accumulate, s);
}

hipError_t launch_mfma_wgrad(const Geom &g, const void *x, const void *dy, const void *y, const float *scale,
                             float *dw, bool relu, bool accumulate, void *ws, hipStream_t s)
{
    if (wgrad_k1_supported(g)) {
        // pointwise layers: a GEMM over rows as they lie in memory; g = dy*[y>0] only has to be formed with a ReLU
        const void *gplain = dy;
        if (relu) {
            void *gbuf = (unsigned char *)ws + wgrad_k1_part_bytes(g);
            hipError_t e = launch_epilogue_bwd_vec8(g, dy, y, nullptr, relu, gbuf, nullptr, s);
            if (e != hipSuccess) return e;
            gplain = gbuf;
        }
        return launch_wgrad_k1(g, x, gplain, scale, dw, accumulate, ws, s);
    }
    if (fast_ok(g)) {
        const FastPlan f = make_fast_plan(g);
        u32x4 *dzf = (u32x4 *)((unsigned char *)ws + part_bytes(g, f.S));
        hipLaunchKernelGGL(dz_pack_kernel, dim3(((f.nst + 3) / 4 + 3) / 4, f.ncm, g.B), dim3(256), 0, s, g.Cout, g.To, f.ncm,
                           f.nst, (const bf16_t *)dy, (const bf16_t *)y, relu ? 1 : 0, dzf);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        return launch_mfma_wgrad_prepared(g, x, scale, dw, accumulate, ws, s);
    }
    const WPlan w = make_wplan(g);
    if (!w.ok) return hipErrorInvalidValue;
    float *part = (float *)ws;
    const void *dz = dy;
    if (relu) {
        void *dzbuf = (unsigned char *)ws + part_bytes(g, w.S);
        // rows are 16-byte aligned here: To % 8 == 0 and the caller checked the pointers
        hipError_t e = launch_epilogue_bwd_vec8(g, dy, y, nullptr, relu, dzbuf, nullptr, s);
        if (e != hipSuccess) return e;
        dz = dzbuf;
    }
    WgradParams p = {};
    p.B = g.B; p.Cin = g.Cin; p.Cout = g.Cout; p.T = g.T; p.To = g.To; p.K = g.K;
    p.stride = g.stride; p.dil = g.dil; p.pad = g.pad;
    p.ncot = (g.Cout + kTileCo - 1) / kTileCo;
    p.ncit = (g.Cin + kTileCi - 1) / kTileCi;
    p.ntg = w.ntg; p.KTg = w.KTg; p.S = w.S;
    p.TCH = w.TCH; p.nchunk = (g.To + w.TCH - 1) / w.TCH; p.units = g.B * p.nchunk;
    p.NRX = w.NRX;
    p.n_dz = w.n_dz; p.n_x = w.n_x; p.ips = w.ips;
    p.dz_row_bytes = w.dz_row_bytes; p.dz_bytes = w.dz_bytes; p.x_bytes = w.x_bytes; p.buf_bytes = w.buf_bytes;
    number_work_items(p);
    p.x = (const bf16_t *)x; p.dz = (const bf16_t *)dz; p.part = part;
    const int grid = p.per_xcd * 8;
    hipError_t e;
    switch (w.KTg) {
    case 1: e = launch_kt<1>(p, w.lds, grid, s); break;
    case 2: e = launch_kt<2>(p, w.lds, grid, s); break;
    case 3: e = launch_kt<3>(p, w.lds, grid, s); break;
    case 4: e = launch_kt<4>(p, w.lds, grid, s); break;
    case 5: e = launch_kt<5>(p, w.lds, grid, s); break;
    default: e = launch_kt<6>(p, w.lds, grid, s); break;
    }
    if (e != hipSuccess) return e;
    return launch_wgrad_reduce(g, part, dw, scale, w.S, accumulate, s);
}

}  // namespace nm
