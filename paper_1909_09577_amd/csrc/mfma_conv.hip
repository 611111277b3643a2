// Matrix-core implicit-GEMM engine for the forward pass and the input gradient.
//
// Both passes are the same contraction
//     out[b, m, t] = sum_r sum_k  W'[m, r, k] * in[b, r, t*stride - padL + k*dil]
// with (m, r) = (co, ci), W' = w, padL = pad for the forward pass and, for the input gradient
// of a stride-1 convolution, (m, r) = (ci, co), W'[ci,co,k] = w[co,ci,K-1-k],
// padL = dil*(K-1) - pad, in = dz = dy*[y>0]*scale (formed while the tile is staged).
//
// Work decomposition (one workgroup = 4 wavefronts of 64 lanes, one workgroup per CU,
// persistent over output tiles):
//   * an output tile is 64 channels x NT*32 time steps of one batch item;
//   * the four wavefronts split the reduction channels in chunks of 32 (wave w takes chunks
//     w, w+4, ...), each accumulating the whole tile in 2*NT 32x32 MFMA accumulators, so the
//     main loop needs no workgroup barrier; the four partial tiles are summed through LDS
//     at the end of the tile and each wavefront finishes a quarter of the rows;
//   * the activation window of a chunk (32 channels x all time steps the K taps touch) is
//     read from HBM once with 16-byte loads along T and written to the wavefront's private LDS
//     region transposed to [time][channel], so that every tap is a row offset and each MFMA
//     B fragment (8 consecutive channels of one time step) is one aligned 16-byte LDS read;
//   * weights are prepacked once per call into MFMA A-fragment order and stream from L2
//     straight into registers (each lane reads 16 contiguous bytes, a wavefront 1 KiB).
//   * tiles are numbered channel-tile fastest, so the workgroups that the hardware places on
//     one XCD (blockIdx mod 8) keep reusing the same slice of the packed weights in that L2.
#include "nm_common.h"

namespace nm {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWaves = 4;
constexpr int kThreads = 64 * kWaves;
constexpr int kTileM = 64;       // output channels per tile
constexpr int kChunk = 32;       // reduction channels per staged chunk
constexpr int kRowBytes = 80;    // LDS row: 32 channels * 2 B + 16 B pad (bank-conflict-free 16 B reads)
constexpr int kRowDwords = kRowBytes / 4;
constexpr int kMaxLds = 160 * 1024;

enum { MODE_FWD = 0, MODE_DGRAD = 1 };

struct ConvGemmParams {
    int B, M, R, Tin, Tout, K, Kp, dil, padL;  // Kp: K rounded up to even (packed weights)
    int nmt, nch, ntt, num_tiles;
    int NR;          // rows of one staged window that are read (multiple of 8)
    int buf_bytes;   // bytes of one staging buffer: nitems*32 rows of kRowBytes
    int nitems;      // staging items per lane and chunk = ceil(NR/8 * 16 / 64)
    int relu;
    const bf16_t *in;       // [B][R][Tin]
    const bf16_t *ysaved;   // DGRAD: saved forward output (ReLU mask) or NULL
    const float *in_scale;  // DGRAD: per reduction channel scale or NULL
    const bf16x8 *wp;       // packed weights
    const float *scale;     // FWD epilogue (may be NULL)
    const float *shift;     // FWD epilogue (may be NULL)
    const bf16_t *res;      // FWD epilogue (may be NULL)
    bf16_t *out;            // [B][M][Tout]
};

__device__ __forceinline__ int floor_div8(int v) { return v >> 3; }  // arithmetic shift: floor

// Eight consecutive time steps of one 16-byte aligned channel row as 4 packed dwords.  The
// address is clamped to a valid one when the row or the time range lies outside the tensor;
// the caller zeroes such data when it consumes it (not here: a select placed right after the
// load would make the wavefront wait for the load at once).
__device__ __forceinline__ u32x4 load_row8(const bf16_t *base, size_t row_off, int t, bool ok)
{
    return *reinterpret_cast<const u32x4 *>(base + (ok ? row_off + (size_t)t : (size_t)0));
}

__device__ __forceinline__ uint32_t pack2(float lo, float hi)
{
    return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

// dz = dy * [y>0] * scale for 8 packed elements.
__device__ __forceinline__ u32x4 make_dz8(u32x4 dy, u32x4 y, float scale, bool relu)
{
    u32x4 r;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float g0 = __uint_as_float(dy[j] << 16), g1 = __uint_as_float(dy[j] & 0xffff0000u);
        if (relu) {
            const float y0 = __uint_as_float(y[j] << 16), y1 = __uint_as_float(y[j] & 0xffff0000u);
            g0 = (y0 > 0.f) ? g0 : 0.f;
            g1 = (y1 > 0.f) ? g1 : 0.f;
        }
        r[j] = pack2(g0 * scale, g1 * scale);
    }
    return r;
}

// Registers of one staging item in flight: channel rows 2pp and 2pp+1, 8 time steps each.
template <int MODE>
struct StageRegs;
template <>
struct StageRegs<MODE_FWD> {
    u32x4 a, b;
    bool oka, okb;
};
template <>
struct StageRegs<MODE_DGRAD> {
    u32x4 a, b, ya, yb;
    float sa, sb;
    bool oka, okb;
};

// One staging item: channel pair pp = item & 15 of the chunk x time group q = item >> 4.
// stage_load only issues the loads; stage_write consumes them.
template <int MODE>
__device__ __forceinline__ void stage_load(const ConvGemmParams &p, int b, int c, int ws_al, int item,
                                           StageRegs<MODE> &s)
{
    const int pp = item & 15, q = item >> 4;
    const int ch = c * kChunk + 2 * pp;
    const int t = ws_al + 8 * q;
    const size_t row = ((size_t)b * p.R + ch) * p.Tin;
    const bool t_ok = t >= 0 && t + 8 <= p.Tin;
    s.oka = t_ok && ch < p.R;
    s.okb = t_ok && ch + 1 < p.R;
    s.a = load_row8(p.in, row, t, s.oka);
    s.b = load_row8(p.in, row + p.Tin, t, s.okb);
    if constexpr (MODE == MODE_DGRAD) {
        if (p.relu) {
            s.ya = load_row8(p.ysaved, row, t, s.oka);
            s.yb = load_row8(p.ysaved, row + p.Tin, t, s.okb);
        }
        s.sa = 1.f;
        s.sb = 1.f;
        if (p.in_scale) {
            s.sa = p.in_scale[ch < p.R ? ch : 0];
            s.sb = p.in_scale[ch + 1 < p.R ? ch + 1 : 0];
        }
    }
}

// Transposing write: one dword (channel pair) per time step.  The buffer has room for every
// item of every lane, so no bounds test is needed.
template <int MODE>
__device__ __forceinline__ void stage_write(const ConvGemmParams &p, uint32_t *buf, int item, const StageRegs<MODE> &s)
{
    const int pp = item & 15, q = item >> 4;
    uint32_t *dst = buf + (q * 8) * kRowDwords + pp;
    u32x4 a = s.a, b = s.b;
    if constexpr (MODE == MODE_DGRAD) {
        if (p.relu || p.in_scale) {
            a = make_dz8(s.a, s.ya, s.sa, p.relu != 0);
            b = make_dz8(s.b, s.yb, s.sb, p.relu != 0);
        }
    }
    const u32x4 z = {0u, 0u, 0u, 0u};
    a = s.oka ? a : z;
    b = s.okb ? b : z;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        dst[(2 * j) * kRowDwords] = (a[j] & 0xffffu) | (b[j] << 16);
        dst[(2 * j + 1) * kRowDwords] = (a[j] >> 16) | (b[j] & 0xffff0000u);
    }
}

__device__ __forceinline__ void wave_lds_fence()
{
    // LDS operations of one wavefront execute in order; this only stops the compiler from
    // moving LDS accesses across the point where other lanes' data must be visible.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int NT, int STRIDE, int MODE>
__global__ __launch_bounds__(kThreads) void conv_gemm_kernel(const ConvGemmParams p)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    constexpr int kTiles = 2 * NT;
    constexpr int TN = NT * 32;

    unsigned char *wbuf0 = smem + (size_t)wave * 2 * p.buf_bytes;
    const int nitems = p.nitems;                           // staging items per lane and chunk
    const int nmy = (p.nch - wave + kWaves - 1) / kWaves;  // chunks of this wavefront (may be 0)

    for (int tile = blockIdx.x; tile < p.num_tiles; tile += gridDim.x) {
        const int mt = tile % p.nmt;
        const int ntile = tile / p.nmt;
        const int b = ntile / p.ntt;
        const int t0 = (ntile % p.ntt) * TN;
        const int ws = t0 * STRIDE - p.padL;
        const int ws_al = floor_div8(ws) * 8;
        const int off0 = ws - ws_al;

        // ---- first chunk of the tile: nothing to overlap with, so the items are put in flight
        // in batches before any is written (the accumulators are not live yet)
        if (nmy > 0) {
            uint32_t *buf = reinterpret_cast<uint32_t *>(wbuf0);
            constexpr int kBatch = (MODE == MODE_DGRAD) ? 3 : 6;
            for (int it0 = 0; it0 < nitems; it0 += kBatch) {
                StageRegs<MODE> s[kBatch];
#pragma unroll
                for (int q = 0; q < kBatch; ++q)
                    stage_load<MODE>(p, b, wave, ws_al, lane + 64 * min(it0 + q, nitems - 1), s[q]);
#pragma unroll
                for (int q = 0; q < kBatch; ++q)
                    stage_write<MODE>(p, buf, lane + 64 * min(it0 + q, nitems - 1), s[q]);
            }
        }

        f32x16 acc[2][NT];
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int ni = 0; ni < NT; ++ni)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

        if (nmy > 0) {
            // ---- main loop over (chunk, tap pair).  Taps are handled in pairs (the packed
            // weights pad an odd K with one zero tap), 4 k-steps of 16 channels = 8*NT MFMAs per
            // pair.  The weight fragments of a pair are fetched one pair before they are used
            // (the stream runs on over this wave's chunks and, past the end, re-reads the last
            // pair); B fragments are read one k-step ahead; one staging item of the next chunk
            // rides on each pair.  All MFMAs sit in this single loop.
            const int P = p.Kp >> 1;                      // tap pairs per chunk
            const size_t chunk_stride = (size_t)p.Kp * 256;  // bf16x8 per (tile, chunk)
            const bf16x8 *wchunk = p.wp + ((size_t)mt * p.nch + wave) * chunk_stride + lane;
            int pslot = 0, pi = 0;
            bf16x8 afA[8], afB[8];
            auto fetch_pair = [&](bf16x8(&dst)[8]) {
                const bf16x8 *s0 = wchunk + (size_t)pslot * 512;
#pragma unroll
                for (int f = 0; f < 8; ++f) dst[f] = s0[f * 64];
                ++pslot;
                if (pslot == P) {
                    if (pi + 1 < nmy) {
                        ++pi;
                        pslot = 0;
                        wchunk += kWaves * chunk_stride;
                    } else {
                        pslot = P - 1;
                    }
                }
            };
            fetch_pair(afA);

            const int tap_bytes = p.dil * kRowBytes;
            const int lane_off = ((lane & 31) * STRIDE + off0) * kRowBytes + (lane >> 5) * 16;
            int ci_ord = 0, pr = 0;
            bool has_next = nmy > 1;
            int c_next = wave + kWaves;
            const unsigned char *bbase = wbuf0 + lane_off;
            uint32_t *nxt = reinterpret_cast<uint32_t *>(wbuf0 + p.buf_bytes);
            bf16x8 b0[NT], b1[NT];
            auto read_b = [&](bf16x8(&dst)[NT], int k, int ks) {
                const unsigned char *brow = bbase + (size_t)k * tap_bytes + ks * 32;
#pragma unroll
                for (int ni = 0; ni < NT; ++ni)
                    dst[ni] = *reinterpret_cast<const bf16x8 *>(brow + ni * 32 * STRIDE * kRowBytes);
            };
            auto mma = [&](const bf16x8 *af, const bf16x8(&bf)[NT]) {
#pragma unroll
                for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                    for (int ni = 0; ni < NT; ++ni)
                        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], bf[ni], acc[mi][ni], 0, 0, 0);
            };
            wave_lds_fence();
            read_b(b0, 0, 0);
            const int total_pairs = nmy * P;
            for (int g = 0; g < total_pairs; ++g) {
                const bool st = has_next && pr < nitems;  // this pair stages item `pr` of the next chunk
                StageRegs<MODE> sr;
                if (st) stage_load<MODE>(p, b, c_next, ws_al, lane + 64 * pr, sr);
                const int k = 2 * pr;
                fetch_pair(afB);
                read_b(b1, k, 1);
                mma(&afA[0], b0);
                read_b(b0, k + 1, 0);
                mma(&afA[2], b1);
                read_b(b1, k + 1, 1);
                mma(&afA[4], b0);
                read_b(b0, min(k + 2, p.Kp - 1), 0);
                mma(&afA[6], b1);
#pragma unroll
                for (int f = 0; f < 8; ++f) afA[f] = afB[f];
                if (st) stage_write<MODE>(p, nxt, lane + 64 * pr, sr);
                ++pr;
                if (pr == P) {  // end of a chunk
                    if (has_next) {
                        for (int it = P; it < nitems; ++it) {  // more items than tap pairs (short kernels)
                            StageRegs<MODE> s2;
                            stage_load<MODE>(p, b, c_next, ws_al, lane + 64 * it, s2);
                            stage_write<MODE>(p, nxt, lane + 64 * it, s2);
                        }
                    }
                    ++ci_ord;
                    pr = 0;
                    if (ci_ord < nmy) {
                        has_next = ci_ord + 1 < nmy;
                        c_next = wave + kWaves * (ci_ord + 1);
                        bbase = wbuf0 + (size_t)(ci_ord & 1) * p.buf_bytes + lane_off;
                        nxt = reinterpret_cast<uint32_t *>(wbuf0 + (size_t)((ci_ord + 1) & 1) * p.buf_bytes);
                        wave_lds_fence();
                        read_b(b0, 0, 0);
                    }
                }
            }
        }

        // ---- sum the four partial tiles: wave g finishes accumulator rows [4g, 4g+4) of every
        // 32x32 block; every wave hands the other three quarters over through LDS.
        __syncthreads();
        f32x4 *red = reinterpret_cast<f32x4 *>(smem);
#pragma unroll
        for (int g = 0; g < kWaves; ++g) {
            if (g != wave) {
                const int slot = wave < g ? wave : wave - 1;
#pragma unroll
                for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                    for (int ni = 0; ni < NT; ++ni) {
                        f32x4 v = {acc[mi][ni][4 * g], acc[mi][ni][4 * g + 1], acc[mi][ni][4 * g + 2],
                                   acc[mi][ni][4 * g + 3]};
                        red[((g * 3 + slot) * kTiles + mi * NT + ni) * 64 + lane] = v;
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
                    for (int ni = 0; ni < NT; ++ni)
                        own[mi * NT + ni] = f32x4{acc[mi][ni][4 * g], acc[mi][ni][4 * g + 1], acc[mi][ni][4 * g + 2],
                                                  acc[mi][ni][4 * g + 3]};
            }
        }
#pragma unroll
        for (int slot = 0; slot < 3; ++slot)
#pragma unroll
            for (int tl = 0; tl < kTiles; ++tl) own[tl] += red[((wave * 3 + slot) * kTiles + tl) * 64 + lane];
        __syncthreads();  // the staging buffers of the next tile alias `red`

        // ---- epilogue on the rows this wave owns: all residual loads are issued first (with
        // clamped addresses, no branches) so that their latencies overlap
        const int tcol = lane & 31;
        const int m_base = mt * kTileM + 8 * wave + 4 * (lane >> 5);
        uint32_t rv[2][4][NT];
        if (MODE == MODE_FWD && p.res) {
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int m = m_base + mi * 32 + j;
                    const size_t orow = ((size_t)b * p.M + m) * p.Tout;
#pragma unroll
                    for (int ni = 0; ni < NT; ++ni) {
                        const int t = t0 + ni * 32 + tcol;
                        const bool ok = m < p.M && t < p.Tout;
                        rv[mi][j][ni] = p.res[ok ? orow + t : (size_t)0];
                    }
                }
        } else {
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int ni = 0; ni < NT; ++ni) rv[mi][j][ni] = 0u;
        }
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int m = m_base + mi * 32 + j;
                const int mc = m < p.M ? m : 0;
                float sc = 1.f, sh = 0.f;
                if (MODE == MODE_FWD) {
                    if (p.scale) sc = p.scale[mc];
                    if (p.shift) sh = p.shift[mc];
                }
                const size_t orow = ((size_t)b * p.M + m) * p.Tout;
#pragma unroll
                for (int ni = 0; ni < NT; ++ni) {
                    const int t = t0 + ni * 32 + tcol;
                    float v = own[mi * NT + ni][j];
                    if (MODE == MODE_FWD) {
                        v = v * sc + sh + __uint_as_float(rv[mi][j][ni] << 16);
                        if (p.relu) v = v > 0.f ? v : 0.f;
                    }
                    if (m < p.M && t < p.Tout) p.out[orow + t] = f32_to_bf16(v);
                }
            }
        }
    }
}

// Packed weights: [mt][chunk][tap < Kp][ks][mi][lane][8] (Kp = K rounded up to even, the extra
// tap is zero); element (lane, j) of fragment (ks, mi) is
// W'[m = mt*64 + mi*32 + lane%32][r = chunk*32 + ks*16 + 8*(lane/32) + j][tap], zero outside,
// with W'[m][r][k] = w[m][r][k] (forward) or w[r][m][K-1-k] (input gradient: FLIP).
// One block packs 16 of the 64 channels of one (mt, chunk): it copies that 16x32xK block of w
// into LDS with coalesced reads (runs of 32*K, resp. 16*K, contiguous elements) and gathers the
// fragments from there.
constexpr int kPackRows = 16;
template <bool FLIP>
__global__ __launch_bounds__(256) void prepack_kernel(const bf16_t *__restrict__ w, u32x4 *__restrict__ wp, int M,
                                                      int R, int K, int nch, int ld /* row length of w */)
{
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t *tile = reinterpret_cast<bf16_t *>(smem);  // [16 m][32 r][K] as (m*32 + r)*K + k
    const int q = blockIdx.x & 3;                      // which 16 channels of the 64
    const int c = (blockIdx.x >> 2) % nch, mt = (blockIdx.x >> 2) / nch;
    const int m0 = mt * kTileM + q * kPackRows, r0 = c * kChunk;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if (!FLIP) {
        // w[m][r][k]: for each m a run of 32*K elements starting at (m0+m)*ld + r0*K
        const int run = kChunk * K;
        const int rvalid = min(kChunk, R - r0) * K;
        for (int m = wv; m < kPackRows; m += 4) {
            const bool m_ok = m0 + m < M;
            const bf16_t *src = w + (size_t)(m_ok ? m0 + m : 0) * ld + (size_t)r0 * K;
            for (int o = lane; o < run; o += 64) tile[m * run + o] = (m_ok && o < rvalid) ? src[o] : (bf16_t)0;
        }
    } else {
        // w[r][m][k]: for each r a run of 16*K elements starting at (r0+r)*ld + m0*K
        const int run = kPackRows * K;
        const int mvalid = max(0, min(kPackRows, M - m0)) * K;
        for (int r = wv; r < kChunk; r += 4) {
            const bool r_ok = r0 + r < R;
            const bf16_t *src = w + (size_t)(r_ok ? r0 + r : 0) * ld + (size_t)m0 * K;
            for (int o = lane; o < run; o += 64) {
                const int m = o / K, k = o - m * K;
                tile[(m * kChunk + r) * K + (K - 1 - k)] = (r_ok && o < mvalid) ? src[o] : (bf16_t)0;
            }
        }
    }
    __syncthreads();
    const int Kp = (K + 1) & ~1;  // an odd K gets one zero tap
    u32x4 *dst = wp + (size_t)(blockIdx.x >> 2) * Kp * 256;
    const int mi = q >> 1, lane_lo = (q & 1) * 16;
    for (int idx = threadIdx.x; idx < Kp * 64; idx += 256) {
        const int m16 = idx & 15, half = (idx >> 4) & 1, ks = (idx >> 5) & 1, k = idx >> 6;
        u32x4 out = {0u, 0u, 0u, 0u};
        if (k < K) {
            const bf16_t *src = tile + (m16 * kChunk + ks * 16 + 8 * half) * K + k;
#pragma unroll
            for (int j = 0; j < 4; ++j) out[j] = (uint32_t)src[(2 * j) * K] | ((uint32_t)src[(2 * j + 1) * K] << 16);
        }
        dst[(k * 4 + ks * 2 + mi) * 64 + half * 32 + lane_lo + m16] = out;
    }
}

struct Plan {
    bool ok;
    int nt;      // NT template value (5 or 2)
    int stride;  // 1 or 2
    int NR;      // window rows that are read
    int nitems;  // staging items per lane; the buffer holds nitems*32 rows
    size_t lds;
};

// Tin: length of the rows that are staged; they must be 16-byte aligned (Tin % 8 == 0).
Plan make_plan(int Tin, int Tout, int K, int stride, int dil)
{
    Plan pl = {false, 0, stride, 0, 0, 0};
    if (stride != 1 && stride != 2) return pl;
    if (Tin % 8 != 0) return pl;
    if ((size_t)kPackRows * kChunk * K * sizeof(bf16_t) > (size_t)kMaxLds) return pl;  // weight packing tile
    const int cands[2] = {5, 2};
    for (int ci = 0; ci < 2; ++ci) {
        const int nt = cands[ci];
        if (ci == 0 && Tout <= 64) continue;  // short sequences: the narrow tile wastes less
        const long Kp = (K + 1) & ~1;  // the zero tap of an odd K is still read
        const long rows = (long)(nt * 32 - 1) * stride + (Kp - 1) * dil + 1 + 7;
        const long NR = (rows + 7) / 8 * 8;
        const long nitems = (NR / 8 * 16 + 63) / 64;
        const size_t stage = (size_t)kWaves * 2 * (nitems * 32) * kRowBytes;
        const size_t red = (size_t)kWaves * 3 * (2 * nt) * 64 * sizeof(f32x4);
        const size_t lds = stage > red ? stage : red;
        if (lds <= (size_t)kMaxLds) {
            pl.ok = true;
            pl.nt = nt;
            pl.NR = (int)NR;
            pl.nitems = (int)nitems;
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
    return align_up(nmt * nch * Kp * 256 * sizeof(u32x4), 256);
}

template <int NT, int STRIDE, int MODE>
hipError_t launch_t(const ConvGemmParams &p, size_t lds, hipStream_t s)
{
    auto kern = conv_gemm_kernel<NT, STRIDE, MODE>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) cus = v;
    }
    const int grid = p.num_tiles < cus ? p.num_tiles : cus;
    MainKernelTimer timer(s);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), lds, s, p);
    return hipGetLastError();
}

template <int MODE>
hipError_t launch_mode(const Plan &pl, const ConvGemmParams &p, hipStream_t s)
{
    if (pl.nt == 5 && pl.stride == 1) return launch_t<5, 1, MODE>(p, pl.lds, s);
    if (pl.nt == 2 && pl.stride == 1) return launch_t<2, 1, MODE>(p, pl.lds, s);
    if (MODE == MODE_FWD) {
        if (pl.nt == 5 && pl.stride == 2) return launch_t<5, 2, MODE_FWD>(p, pl.lds, s);
        if (pl.nt == 2 && pl.stride == 2) return launch_t<2, 2, MODE_FWD>(p, pl.lds, s);
    }
    return hipErrorInvalidValue;
}

size_t prepack_lds(int K) { return (size_t)kPackRows * kChunk * K * sizeof(bf16_t); }

// flip == false: W'[m][r][k] = w[m][r][k] (w is [M][R][K]); flip == true: W'[m][r][k] = w[r][m][K-1-k]
// (w is [R][M][K]).
hipError_t run_prepack(const void *w, void *wp, int M, int R, int K, bool flip, hipStream_t s)
{
    const int nmt = (M + kTileM - 1) / kTileM, nch = (R + kChunk - 1) / kChunk;
    const size_t lds = prepack_lds(K);
    hipError_t e;
    if (flip) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(prepack_kernel<true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(prepack_kernel<true>, dim3(nmt * nch * 4), dim3(256), lds, s, (const bf16_t *)w, (u32x4 *)wp,
                           M, R, K, nch, M * K);
    } else {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(prepack_kernel<false>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(prepack_kernel<false>, dim3(nmt * nch * 4), dim3(256), lds, s, (const bf16_t *)w, (u32x4 *)wp,
                           M, R, K, nch, R * K);
    }
    return hipGetLastError();
}

void fill_common(ConvGemmParams &p, const Plan &pl, int B, int M, int R, int Tin, int Tout, int K, int dil, int padL,
                 const void *)
{
    p.B = B; p.M = M; p.R = R; p.Tin = Tin; p.Tout = Tout; p.K = K; p.Kp = (K + 1) & ~1; p.dil = dil; p.padL = padL;
    p.nmt = (M + kTileM - 1) / kTileM;
    p.nch = (R + kChunk - 1) / kChunk;
    p.ntt = (Tout + pl.nt * 32 - 1) / (pl.nt * 32);
    p.num_tiles = p.nmt * p.ntt * B;
    p.NR = pl.NR;
    p.nitems = pl.nitems;
    p.buf_bytes = pl.nitems * 32 * kRowBytes;
}

}  // namespace

// ---- forward ---------------------------------------------------------------------------
bool mfma_fwd_supported(const Geom &g) { return make_plan(g.T, g.To, g.K, g.stride, g.dil).ok; }

size_t mfma_fwd_workspace(const Geom &g) { return packed_bytes(g.Cout, g.Cin, g.K); }

hipError_t launch_mfma_fwd(const Geom &g, const void *x, const void *w, const float *scale, const float *shift,
                           const void *res, void *y, bool relu, void *ws, hipStream_t s)
{
    const Plan pl = make_plan(g.T, g.To, g.K, g.stride, g.dil);
    if (!pl.ok) return hipErrorInvalidValue;
    hipError_t e = run_prepack(w, ws, g.Cout, g.Cin, g.K, false, s);
    if (e != hipSuccess) return e;
    ConvGemmParams p = {};
    fill_common(p, pl, g.B, g.Cout, g.Cin, g.T, g.To, g.K, g.dil, g.pad, x);
    p.relu = relu ? 1 : 0;
    p.in = (const bf16_t *)x;
    p.wp = (const bf16x8 *)ws;
    p.scale = scale; p.shift = shift; p.res = (const bf16_t *)res;
    p.out = (bf16_t *)y;
    return launch_mode<MODE_FWD>(pl, p, s);
}

// ---- input gradient (stride 1 only; other strides use the plain kernels) ----------------
bool mfma_dgrad_supported(const Geom &g)
{
    if (g.stride != 1) return false;
    return make_plan(g.To, g.T, g.K, 1, g.dil).ok;
}

size_t mfma_dgrad_workspace(const Geom &g) { return packed_bytes(g.Cin, g.Cout, g.K); }

hipError_t launch_mfma_dgrad(const Geom &g, const void *dy, const void *y, const float *scale, const void *w,
                             void *dx, void *dres, bool relu, void *ws, hipStream_t s)
{
    const Plan pl = make_plan(g.To, g.T, g.K, 1, g.dil);
    if (!pl.ok) return hipErrorInvalidValue;
    hipError_t e = run_prepack(w, ws, g.Cin, g.Cout, g.K, true, s);
    if (e != hipSuccess) return e;
    if (dres) {
        // To % 8 == 0 on this path; dres is written with 2-byte granularity only if misaligned
        if (((uintptr_t)dres % 16) == 0) e = launch_epilogue_bwd_vec8(g, dy, y, nullptr, relu, nullptr, dres, s);
        else e = launch_epilogue_bwd(g, true, dy, y, nullptr, relu, nullptr, dres, s);
        if (e != hipSuccess) return e;
    }
    ConvGemmParams p = {};
    fill_common(p, pl, g.B, g.Cin, g.Cout, g.To, g.T, g.K, g.dil, g.dil * (g.K - 1) - g.pad, dy);
    p.relu = relu ? 1 : 0;
    p.in = (const bf16_t *)dy;
    p.ysaved = (const bf16_t *)y;
    p.in_scale = scale;
    p.wp = (const bf16x8 *)ws;
    p.out = (bf16_t *)dx;
    return launch_mode<MODE_DGRAD>(pl, p, s);
}

}  // namespace nm
