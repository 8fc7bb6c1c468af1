// vmoba_select: mean key blocks (Eq. 2), query x block similarities (Eq. 3), soft-max
// normalisation per query, head-global cumulative threshold (Eq. 4), TopkMask (Eq. 3) as a
// bit mask plus block-major and query-major sparse lists.
//
// The descending-sort-and-accumulate of Eq. 4 is done without sorting: P >= 0, so the order
// of its float bit patterns is the order of its values, and a three-level radix histogram
// (12 + 10 + 10 bits) with per-bin counts and per-bin sums locates the value theta at which
// the descending cumulative sum reaches tau * S.  Per-bin sums are kept as 64-bit integers
// (value * 2^fix_shift, truncated) so the result does not depend on the order of atomics.
#include "common.h"
#include "attn_common.h"

#include <algorithm>
#include <cmath>
#include <mutex>

namespace {

constexpr int HIST_BINS = 1024;
constexpr int QT = 64;          // queries per score tile
constexpr int SCAN_THREADS = 1024;
constexpr int SCAN_ITEMS = 16;

struct HeadState {              // one per (b, h), lives in the workspace
    unsigned long long need;    // fixed-point mass still missing inside the current bin range
    unsigned long long cnt_above;  // pool entries strictly above the current bin range
    unsigned int prefix;        // float bits of theta found so far (high bits)
    unsigned int all;           // 1: threshold never reached -> keep every pair
    unsigned int n_tie;         // entries equal to theta
    unsigned int take;          // how many of them belong to the top k
};

struct SelectWs {               // workspace carve-up (device pointers)
    unsigned int* hist_cnt;         // [3][BH][1024]
    unsigned long long* hist_sum;   // [3][BH][1024]
    HeadState* state;               // [BH]
    int* ties;                      // [BH][S]   per-row count of entries equal to theta
    int* tie_base;                  // [BH][S+1] exclusive scan of ties
    int* wtot;                      // [BH][n_waves]  pairs kept by each group of 64 queries, then its exclusive scan
    int* wcnt;                      // [BH][n_blocks][n_waves]
    int* row_tot;                   // [BH][n_blocks + 1]  totals of the rows of wcnt, then of wtot
    size_t zero_bytes;              // leading bytes (hist + state) cleared on every call
    float2* row_stat;   // [BH * S] {row maximum, row denominator} of the score soft-max (pool soft-max mode)
    float2* pool_stat;  // [BH] {pool maximum, 1 / pool denominator}
    size_t total;
};

SelectWs carve(void* base, int BH, int64_t S, int nb) {
    SelectWs w;
    char* p = (char*)base;
    size_t off = 0;
    w.hist_sum = (unsigned long long*)(p + off);  off += (size_t)3 * BH * HIST_BINS * 8;
    w.hist_cnt = (unsigned int*)(p + off);        off += (size_t)3 * BH * HIST_BINS * 4;
    w.state = (HeadState*)(p + off);              off += align_up((size_t)BH * sizeof(HeadState), 256);
    w.zero_bytes = off;
    w.ties = (int*)(p + off);                     off += align_up((size_t)BH * S * 4, 256);
    w.tie_base = (int*)(p + off);                 off += align_up((size_t)BH * (S + 1) * 4, 256);
    int64_t n_waves = ceil_div64(S, 64);
    w.wtot = (int*)(p + off);                     off += align_up((size_t)BH * n_waves * 4, 256);
    w.wcnt = (int*)(p + off);                     off += align_up((size_t)BH * nb * n_waves * 4, 256);
    w.row_tot = (int*)(p + off);                  off += align_up((size_t)BH * (nb + 1) * 4, 256);
    w.row_stat = (float2*)(p + off);              off += align_up((size_t)BH * S * 8, 256);
    w.pool_stat = (float2*)(p + off);             off += align_up((size_t)BH * 8, 256);
    w.total = off;
    return w;
}

// ---------------------------------------------------------------------------------------------
// Block means, Eq. 2.  One workgroup per (block, b*Hh + h).  Threads are laid out as
// (row group, 16-byte piece of a row); every thread sums its piece over the rows of its group,
// the groups are then added in a fixed order, so the result is reproducible.
// kv_rows: null when K is in block order, else the row of K that holds key position r (keys in place).
template <bool BF16, int D>
__global__ __launch_bounds__(256) void block_mean_kernel(TensorView K, const int* __restrict__ blk_off,
                                                         float* __restrict__ Bmean, int Hh, int nb,
                                                         const int* __restrict__ kv_rows,
                                                         unsigned int* __restrict__ zero_words, unsigned int n_zero) {
    constexpr int EPP = BF16 ? 8 : 4;          // elements per 16-byte piece
    constexpr int PIECES = D / EPP;            // pieces per row
    constexpr int GROUPS = 256 / PIECES;
    const int j = blockIdx.x, bh = blockIdx.y;
    const int b = bh / Hh, h = bh % Hh;
    {   // this workgroup's share of the words that must be zero when the next kernel of the call starts (histograms, state)
        const unsigned int n_wg = gridDim.x * gridDim.y, wg = bh * gridDim.x + j;
        const unsigned int per = (n_zero + n_wg - 1) / n_wg;
        const unsigned int z0 = min(n_zero, wg * per), z1 = min(n_zero, z0 + per);
        for (unsigned int i = z0 + threadIdx.x; i < z1; i += 256) zero_words[i] = 0u;
    }
    const int piece = threadIdx.x % PIECES, grp = threadIdx.x / PIECES;
    const int r0 = blk_off[j], r1 = blk_off[j + 1];
    float acc[EPP];
#pragma unroll
    for (int e = 0; e < EPP; ++e) acc[e] = 0.f;
    const char* base = K.ptr + ((long long)b * K.stride_b + (long long)h * K.stride_h) * (BF16 ? 2 : 4);
    for (int r = r0 + grp; r < r1; r += GROUPS) {
        const int row = kv_rows ? kv_rows[r] : r;
        const char* src = base + (long long)row * K.stride_s * (BF16 ? 2 : 4) + piece * 16;
        u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(src));
        if constexpr (BF16) {
            acc[0] += bf16lo_to_f32(v.x); acc[1] += bf16hi_to_f32(v.x);
            acc[2] += bf16lo_to_f32(v.y); acc[3] += bf16hi_to_f32(v.y);
            acc[4] += bf16lo_to_f32(v.z); acc[5] += bf16hi_to_f32(v.z);
            acc[6] += bf16lo_to_f32(v.w); acc[7] += bf16hi_to_f32(v.w);
        } else {
            acc[0] += __uint_as_float(v.x); acc[1] += __uint_as_float(v.y);
            acc[2] += __uint_as_float(v.z); acc[3] += __uint_as_float(v.w);
        }
    }
    __shared__ float red[GROUPS][D + 4];
#pragma unroll
    for (int e = 0; e < EPP; ++e) red[grp][piece * EPP + e] = acc[e];
    __syncthreads();
    if (threadIdx.x < D) {
        float s = 0.f;
        for (int g = 0; g < GROUPS; ++g) s += red[g][threadIdx.x];
        Bmean[((long long)bh * nb + j) * D + threadIdx.x] = s / (float)(r1 - r0);
    }
}

// p * 2^fix_shift as an integer for a finite p >= 0 below 2^(63 - fix_shift), by a shift of the float's mantissa.
// Exact for every p whose last mantissa bit is worth at least 2^-fix_shift; smaller values (below 2^(-fix_shift + 23),
// at most 2^-14 of the pool's mass all together) count as 0.  Exactness is what lets a bin's sum be formed either value
// by value or as (count * leading bits + sum of trailing bits) << shift: both give the same integer.
__device__ __forceinline__ unsigned long long to_fixed(float p, int fix_shift) {
    const uint32_t b = __float_as_uint(p);
    const int e = (int)(b >> 23);
    const int sh = e - 150 + fix_shift;
    return (e && sh >= 0) ? ((unsigned long long)((b & 0x7fffffu) | 0x800000u) << sh) : 0ull;
}

// Level-0 histogram word in LDS: entries of one bin share sign, exponent and the three leading mantissa bits, so a bin
// needs only how many there are (bits 40..63) and the sum of their 20 trailing mantissa bits (bits 0..39): one 64-bit
// LDS atomic per entry.  Holds up to 2^20 entries per bin and workgroup.
constexpr unsigned long long PK_ONE = 1ull << 40;
// `copies` (a power of two) interleaved replicas of the 1024 words, word = bin * copies + (lane % copies): the entries of
// a row crowd into a few neighbouring bins, and lanes that hit the same word are served one after the other.
__device__ __forceinline__ void packed_hist_add(unsigned long long* sPk, int copy_shift, int copy, float p) {
    const unsigned int u = __float_as_uint(p);
    atomicAdd(&sPk[(min(u >> 20, (unsigned)(HIST_BINS - 1)) << copy_shift) + copy], PK_ONE | (unsigned long long)(u & 0xfffffu));
}
// A workgroup's packed words -> the head's level-0 histogram (count and fixed-point sum per bin).
__device__ __forceinline__ void packed_hist_flush(const unsigned long long* sPk, int copy_shift,
                                                  unsigned int* __restrict__ hist_cnt,
                                                  unsigned long long* __restrict__ hist_sum, long long bh, int fix_shift,
                                                  int tid, int n_threads) {
    for (int i = tid; i < HIST_BINS; i += n_threads) {
        unsigned long long cnt = 0, low = 0;
        for (int c = 0; c < (1 << copy_shift); ++c) {
            const unsigned long long w = sPk[(i << copy_shift) + c];
            cnt += w >> 40;
            low += w & (PK_ONE - 1);
        }
        if (cnt) {
            const int e = i >> 3, sh = e - 150 + fix_shift;
            const unsigned long long lead = 0x800000ull | ((unsigned long long)(i & 7) << 20);
            atomicAdd(&hist_cnt[bh * HIST_BINS + i], (unsigned int)cnt);
            if (e && sh >= 0) atomicAdd(&hist_sum[bh * HIST_BINS + i], (cnt * lead + low) << sh);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Scores (Eq. 3), row soft-max, P write-out and the first radix level, fused, for float32 queries
// (bfloat16 queries take score_mfma_kernel below).  A workgroup owns a tile of QT = 64 queries of
// one head.  The head's block means sit in LDS as float32; thread (q = tid % 64, g = tid / 64)
// keeps its query row in registers and computes the dot products with blocks g, g+4, g+8, ...
template <int D>
__global__ __launch_bounds__(256) void score_kernel(TensorView Q, const float* __restrict__ Bmean,
                                                    float* __restrict__ P, unsigned int* __restrict__ hist_cnt,
                                                    unsigned long long* __restrict__ hist_sum,
                                                    int Hh, int S, int nb, float score_scale, int fix_shift,
                                                    float2* __restrict__ row_stat) {
    extern __shared__ __align__(16) unsigned char smem[];
    float* sB = reinterpret_cast<float*>(smem);                       // [nb][D]
    const int pstride = nb | 1;
    float* sP = sB + (size_t)nb * D;                                  // [QT][pstride]
    unsigned int* sCnt = reinterpret_cast<unsigned int*>(sP + QT * pstride);   // [1024]
    unsigned long long* sSum = reinterpret_cast<unsigned long long*>(sCnt + HIST_BINS);  // [1024]

    const int bh = blockIdx.y;
    const int b = bh / Hh, h = bh % Hh;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;

    for (int i = tid; i < nb * D / 4; i += 256)
        reinterpret_cast<f32x4_t*>(sB)[i] = reinterpret_cast<const f32x4_t*>(Bmean + (long long)bh * nb * D)[i];
    for (int i = tid; i < HIST_BINS; i += 256) { sCnt[i] = 0u; sSum[i] = 0ull; }
    __syncthreads();

    const int n_tiles = (S + QT - 1) / QT;
    for (int tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int q0 = tile * QT;
        const int ql = lane;
        const int q = min(q0 + ql, S - 1);          // tail rows recompute the last query; never stored
        // query row -> registers
        float qr[D];
        {
            const char* src = Q.ptr + ((long long)b * Q.stride_b + (long long)q * Q.stride_s + (long long)h * Q.stride_h) * 4;
#pragma unroll
            for (int i = 0; i < D / 4; ++i) {
                f32x4_t v = reinterpret_cast<const f32x4_t*>(src)[i];
                qr[4 * i + 0] = v.x; qr[4 * i + 1] = v.y; qr[4 * i + 2] = v.z; qr[4 * i + 3] = v.w;
            }
        }
        for (int j = wave; j < nb; j += 4) {
            const f32x4_t* bj = reinterpret_cast<const f32x4_t*>(sB + (size_t)j * D);
            float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
#pragma unroll
            for (int i = 0; i < D / 4; ++i) {
                f32x4_t bv = bj[i];
                a0 = fmaf(qr[4 * i + 0], bv.x, a0);
                a1 = fmaf(qr[4 * i + 1], bv.y, a1);
                a2 = fmaf(qr[4 * i + 2], bv.z, a2);
                a3 = fmaf(qr[4 * i + 3], bv.w, a3);
            }
            sP[ql * pstride + j] = ((a0 + a1) + (a2 + a3)) * score_scale;
        }
        __syncthreads();
        // row maximum and denominator (every one of the 4 threads of a row computes both)
        float m = -INFINITY;
        for (int j = 0; j < nb; ++j) m = fmaxf(m, sP[ql * pstride + j]);
        float den = 0.f;
        for (int j = 0; j < nb; ++j) den += expf(sP[ql * pstride + j] - m);
        if (row_stat && wave == 0 && q0 + ql < S) row_stat[(long long)bh * S + q0 + ql] = make_float2(m, den);
        __syncthreads();
        for (int j = wave; j < nb; j += 4) sP[ql * pstride + j] = expf(sP[ql * pstride + j] - m) / den;
        __syncthreads();
        // coalesced write-out of the [64 x nb] tile + level-0 histogram
        const int rows = min(QT, S - q0);
        for (int r = wave; r < rows; r += 4) {
            float* dst = P + ((long long)bh * S + q0 + r) * nb;
            for (int j = lane; j < nb; j += 64) {
                float p = sP[r * pstride + j];
                dst[j] = p;
                if (hist_cnt) {               // null: the caller takes the first radix level elsewhere (pool soft-max)
                    unsigned int bin = min(__float_as_uint(p) >> 20, (unsigned)(HIST_BINS - 1));
                    atomicAdd(&sCnt[bin], 1u);
                    atomicAdd(&sSum[bin], to_fixed(p, fix_shift));
                }
            }
        }
        __syncthreads();
    }
    for (int i = tid; i < HIST_BINS; i += 256) {
        unsigned int c = sCnt[i];
        if (c) {                               // stays 0 without a histogram
            atomicAdd(&hist_cnt[(long long)bh * HIST_BINS + i], c);
            atomicAdd(&hist_sum[(long long)bh * HIST_BINS + i], sSum[i]);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Scores on the matrix cores for bfloat16 queries (same results as score_kernel to float32
// rounding).  The float32 block means are split exactly into three bfloat16 terms,
// B = Bh + Bm + Bl (8 + 8 + 8 mantissa bits), so that every product with a bfloat16 query is exact
// in float32 and only the accumulation rounds -- a bfloat16 copy of the means alone would move P
// by ~4e-3.  S^T[block, q] = sum over the three terms of Bx[block, :] . Q[q, :], with the query on
// the MFMA column (= lane % 32), so the soft-max over blocks is a reduction over a lane's own
// registers plus one exchange with lane ^ 32.  SCORE_NW wavefronts x 32 queries per tile.
// With more than 128 blocks the three bfloat16 copies no longer fit the LDS; FLY keeps the means there as float32 (row
// stride D + 4) and splits every operand after its fetch: the same three terms from the same operations, so P is the
// same, at the price of vector work per matrix instruction.
// With more than 256 blocks neither the means nor a query's scores fit: the host then launches the kernel once per
// chunk of up to 256 blocks with RAW set -- the launch covers blocks [jb0, jb0 + nb) of nb_total and writes the scaled
// scores themselves into its columns of P -- and softmax_rows_kernel below turns the rows into P afterwards.
// wavefronts per workgroup of the matrix-core score kernel (two per SIMD share one copy of the block means in LDS)
constexpr int SCORE_NW = 8, SCORE_NT = 64 * SCORE_NW, SCORE_QT = 32 * SCORE_NW;
// every value of a lane's rows (N_T tiles of 16) into the packed histogram
template <int N_T>
__device__ __forceinline__ void packed_hist_add_rows(unsigned long long* sPk, int copy_shift, int copy, const f32x16_t (&rows)[N_T], int n_mt) {
#pragma unroll
    for (int mt = 0; mt < N_T; ++mt) {
        if (mt < n_mt) {
#pragma unroll
            for (int v = 0; v < 16; ++v) packed_hist_add(sPk, copy_shift, copy, rows[mt][v]);
        }
    }
}
// Reduction over the 32 lanes of a wavefront half (lanes 0..31 and 32..63 separately): three steps inside rows of 16
// lanes by data-parallel primitives (quad swaps, half-row and row mirror), one across the half's two rows.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ float half32_max(float x) {
    typedef unsigned u2 __attribute__((ext_vector_type(2)));
    x = fmaxf(x, dpp_move<0xB1>(x));      // quad_perm [1, 0, 3, 2]
    x = fmaxf(x, dpp_move<0x4E>(x));      // quad_perm [2, 3, 0, 1]
    x = fmaxf(x, dpp_move<0x141>(x));     // row_half_mirror
    x = fmaxf(x, dpp_move<0x140>(x));     // row_mirror
    const u2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r.x), __uint_as_float(r.y));
}
__device__ __forceinline__ float half32_sum(float x) {
    typedef unsigned u2 __attribute__((ext_vector_type(2)));
    x += dpp_move<0xB1>(x);
    x += dpp_move<0x4E>(x);
    x += dpp_move<0x141>(x);
    x += dpp_move<0x140>(x);
    const u2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r.x) + __uint_as_float(r.y);
}
template <bool FIRST, class T>
__device__ __forceinline__ T& pick_ref(T& a, T& b) {
    if constexpr (FIRST) return a; else return b;
}
// NMT > 0: the number of 32-block tiles is that constant (the launch for up to 128 blocks picks the instantiation), so the
// loops over tiles carry no run-time tests and only the last tile knows padding blocks; NMT = 0: read from nb.
// TR: the accumulators hold S^T (blocks down a lane's registers, the query on the lane: the soft-max of a row is in-lane,
// and a lane stores 16-byte runs of its row of P) -- needs rows of P that start 16-byte aligned (N_b a multiple of 4).
// !TR: they hold S (queries down the registers, the block on the lane): a store instruction then writes 128-byte runs of
// two rows with 4-byte pieces whatever N_b is, and the row maximum and sum take a reduction over 32 lanes.
template <int D, bool FLY, bool RAW, int NMT, bool TR>
__global__ __launch_bounds__(SCORE_NT) void score_mfma_kernel(TensorView Q, const float* __restrict__ Bmean,
                                                         float* __restrict__ P, unsigned int* __restrict__ hist_cnt,
                                                         unsigned long long* __restrict__ hist_sum,
                                                         int BH, int Hh, int S, int nb, int nb_total, int jb0, float score_scale,
                                                         int fix_shift, int copy_shift, float2* __restrict__ row_stat) {
    // LDS rows of the bf16 terms are padded by 16 bytes.  Beyond 128 blocks (NMT > 4) only the nb real rows and one row of
    // zeros are kept -- the lanes of the last tile that stand for padding blocks read the zero row -- which is what lets
    // three terms of up to 189 blocks fit beside the histogram words.
    constexpr bool CLAMP = NMT > 4;
    constexpr int STR = D + 8;                 // LDS row stride in bf16 elements
    constexpr int FSTR = D + 4;                // LDS row stride in float elements (FLY)
    constexpr int KSTEPS = D / 16;
    constexpr int MAX_MT = NMT > 0 ? NMT : (FLY ? 8 : 4);        // up to 256 / 128 blocks
    extern __shared__ __align__(16) unsigned char smem[];
    const int nb_pad = NMT > 0 ? NMT * 32 : ((nb + 31) & ~31);
    const int n_mt = NMT > 0 ? NMT : nb_pad / 32;
    const int n_rows = CLAMP ? nb + 1 : nb_pad;                   // rows of a term in LDS
    auto term_at = [&](int x, int row, int el) { return ((size_t)x * n_rows + row) * STR + el; };
    __bf16* sB = reinterpret_cast<__bf16*>(smem);                                  // [3][n_rows][STR]
    float* sBf = reinterpret_cast<float*>(smem);                                   // FLY: [nb_pad][FSTR]
    unsigned long long* sPk = FLY ? reinterpret_cast<unsigned long long*>(sBf + (size_t)nb_pad * FSTR)
                                  : reinterpret_cast<unsigned long long*>(sB + (size_t)3 * n_rows * STR);   // [1024 << copy_shift]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hf = lane >> 5;
    const int hist_copy = lane & ((1 << copy_shift) - 1);

    // block means of head bh -> LDS, 16 bytes per lane and four loads in flight per lane (the head's means are one
    // contiguous array); clears the histogram words
    auto load_means = [&](int bh) {
        const f32x4_t* src4 = reinterpret_cast<const f32x4_t*>(Bmean + ((long long)bh * nb_total + jb0) * D);
        const int n4 = nb * D / 4, n4_pad = (FLY ? nb_pad : n_rows) * D / 4;      // rows past nb are zeros
        for (int i0 = tid; i0 < n4_pad; i0 += 4 * SCORE_NT) {
            f32x4_t x4[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = i0 + u * SCORE_NT;
                const f32x4_t z = {0.f, 0.f, 0.f, 0.f};
                x4[u] = i < n4 ? src4[i] : z;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = i0 + u * SCORE_NT;
                if (i >= n4_pad) continue;
                const int j = (i * 4) / D, d = (i * 4) % D;
                if constexpr (FLY) {
                    *reinterpret_cast<f32x4_t*>(&sBf[j * FSTR + d]) = x4[u];
                } else {
                    bf16x4_t h4, m4, l4;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float x = x4[u][e];
                        const __bf16 xh = (__bf16)x;
                        const float r1 = x - (float)xh;
                        const __bf16 xm = (__bf16)r1;
                        const float r2 = r1 - (float)xm;
                        h4[e] = xh;
                        m4[e] = xm;
                        l4[e] = (__bf16)r2;
                    }
                    *reinterpret_cast<bf16x4_t*>(&sB[term_at(0, j, d)]) = h4;
                    *reinterpret_cast<bf16x4_t*>(&sB[term_at(1, j, d)]) = m4;
                    *reinterpret_cast<bf16x4_t*>(&sB[term_at(2, j, d)]) = l4;
                }
            }
        }
        for (int i = tid; i < (HIST_BINS << copy_shift); i += SCORE_NT) sPk[i] = 0ull;
    };

    const f32x16_t zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const int n_tiles = (S + SCORE_QT - 1) / SCORE_QT;
    const bool vec_ok = ((nb_total | jb0) & 3) == 0;         // this launch's part of a row of P starts 16-byte aligned
    // The launch's work is the flat list of (head, query tile) pairs; a workgroup takes one contiguous share of it, so
    // all shares are equal to within one tile whatever the number of heads, and reloads the means when its share
    // crosses into the next head.
    const int n_flat = BH * n_tiles;
    const int t0 = (int)((long long)blockIdx.x * n_flat / gridDim.x), t1 = (int)((long long)(blockIdx.x + 1) * n_flat / gridDim.x);
    auto load_q = [&](int flat, bf16x8_t(&dst)[KSTEPS]) {
        const int bh = flat / n_tiles, tile = flat - bh * n_tiles, b = bh / Hh, h = bh - b * Hh;
        const int qc = min(tile * SCORE_QT + wave * 32 + l32, S - 1);     // rows past the end recompute the last query; never stored
        const char* src = Q.ptr + ((long long)b * Q.stride_b + (long long)qc * Q.stride_s + (long long)h * Q.stride_h) * 2;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) dst[ks] = *reinterpret_cast<const bf16x8_t*>(src + (ks * 16 + hf * 8) * 2);
    };
    // Order inside a tile: request the next tile's query rows, matrix phase, soft-max arithmetic, then -- only then --
    // wait for the rows requested a whole tile ago, take them over and store this tile's P.  The stores then drain during
    // the next tile's arithmetic.  The take-over is written as opaque register moves: as a plain assignment the compiler
    // turns it into the loop-carried copy at the bottom of the loop, behind the stores, and its wait for the rows there
    // becomes a wait for every store just issued.
    bf16x8_t qf[KSTEPS], qn[KSTEPS];
    constexpr bool EARLY_ROWS = NMT > 0 && NMT <= 4;                  // see the tile loop
    auto take_next_rows = [&]() {
        if constexpr (!EARLY_ROWS) return;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            const u32x4_t src = __builtin_bit_cast(u32x4_t, qn[ks]);
            unsigned int d0, d1, d2, d3;
            asm volatile("v_mov_b32 %0, %4\n\tv_mov_b32 %1, %5\n\tv_mov_b32 %2, %6\n\tv_mov_b32 %3, %7"
                         : "=&v"(d0), "=&v"(d1), "=&v"(d2), "=&v"(d3)
                         : "v"(src.x), "v"(src.y), "v"(src.z), "v"(src.w));
            const u32x4_t dst = {d0, d1, d2, d3};
            qf[ks] = __builtin_bit_cast(bf16x8_t, dst);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    if (t0 < t1) {                                       // the first tile's rows come the same way (the matrix phase then
        if constexpr (EARLY_ROWS) {                      // never reads a register that a load is still to fill)
            load_q(t0, qn);
            take_next_rows();
        } else {
            load_q(t0, qf);
        }
    }
    int cur_bh = -1, since_flush = 0;
    const int flush_every = max(1, (1 << 20) / (SCORE_QT * nb_pad));   // tiles until a packed histogram word could overflow
    // A tile's P values stay in `outp` until the NEXT tile's matrix phase is over and are entered into the histogram only
    // then.  That keeps them in registers of their own: the matrix phase then writes accumulators that no store still
    // in flight reads (the compiler makes a wavefront wait for such stores before it overwrites their data).
    // (With more than 3 tiles of accumulators there are no registers for a second set: the values stay in the
    // accumulators and are counted right after their stores.)
    constexpr bool DEFER = NMT > 0 && NMT <= 3;
    f32x16_t outp_own[MAX_MT] = {};                                  // never touched unless DEFER
    bool pending = false;                                             // this lane's outp holds a query's row not yet counted
    const bool count = !RAW && hist_cnt != nullptr;
    for (int flat = t0; flat < t1; ++flat) {
        const int bh = flat / n_tiles, tile = flat - bh * n_tiles;
        if (bh != cur_bh || since_flush >= flush_every) {              // same decision in every wavefront
            since_flush = 0;
            if (cur_bh >= 0) {
                if (DEFER && count && pending) packed_hist_add_rows<MAX_MT>(sPk, copy_shift, hist_copy, outp_own, n_mt);
                pending = false;
                __syncthreads();
                if (hist_cnt) packed_hist_flush(sPk, copy_shift, hist_cnt, hist_sum, cur_bh, fix_shift, tid, SCORE_NT);
                __syncthreads();
            }
            load_means(bh);
            __syncthreads();
            cur_bh = bh;
        }
        ++since_flush;
        const int q = tile * SCORE_QT + wave * 32 + l32;
        // the next tile's rows: requested here, a whole tile before their use, where the registers allow (up to four
        // 32-block tiles); else after the matrix phase, which leaves the soft-max arithmetic for them to arrive
        if constexpr (EARLY_ROWS) {
            load_q(min(flat + 1, t1 - 1), qn);
            __builtin_amdgcn_sched_barrier(0);                        // requested here, not after the matrix phase
        }
        f32x16_t acc[MAX_MT];
#pragma unroll
        for (int mt = 0; mt < MAX_MT; ++mt) acc[mt] = zero16;
        // k-step outermost: consecutive matrix instructions go to different accumulators (each accumulator still sums
        // its terms in the order k-step, then high / middle / low part)
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
#pragma unroll
            for (int mt = 0; mt < MAX_MT; ++mt) {
                if (mt < n_mt) {
                    if constexpr (FLY) {
                        const float* src = &sBf[(mt * 32 + l32) * FSTR + ks * 16 + hf * 8];
                        const f32x4_t x0 = *reinterpret_cast<const f32x4_t*>(src), x1 = *reinterpret_cast<const f32x4_t*>(src + 4);
                        bf16x8_t bh8, bm8, bl8;
#pragma unroll
                        for (int i = 0; i < 8; ++i) {
                            const float x = i < 4 ? x0[i] : x1[i - 4];
                            const __bf16 xh = (__bf16)x;
                            const float r1 = x - (float)xh;
                            const __bf16 xm = (__bf16)r1;
                            const float r2 = r1 - (float)xm;
                            bh8[i] = xh;
                            bm8[i] = xm;
                            bl8[i] = (__bf16)r2;
                        }
                        acc[mt] = TR ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(bh8, qf[ks], acc[mt], 0, 0, 0) : __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[ks], bh8, acc[mt], 0, 0, 0);
                        acc[mt] = TR ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(bm8, qf[ks], acc[mt], 0, 0, 0) : __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[ks], bm8, acc[mt], 0, 0, 0);
                        acc[mt] = TR ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(bl8, qf[ks], acc[mt], 0, 0, 0) : __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[ks], bl8, acc[mt], 0, 0, 0);
                    }
                }
            }
            if constexpr (!FLY) {
                // a batch of fragments is requested before its first matrix instruction, so one LDS latency is paid per
                // batch, not per instruction; the whole k-step is one batch where the registers allow it
                constexpr int XB = (NMT > 0 && NMT <= 3) ? 3 : 1;
#pragma unroll
                for (int x0 = 0; x0 < 3; x0 += XB) {
                    bf16x8_t bf[XB][MAX_MT];
#pragma unroll
                    for (int x = 0; x < XB; ++x)
#pragma unroll
                        for (int mt = 0; mt < MAX_MT; ++mt)
                            if (mt < n_mt)
                                bf[x][mt] = *reinterpret_cast<const bf16x8_t*>(
                                    &sB[term_at(x0 + x, (CLAMP && mt == NMT - 1) ? min(mt * 32 + l32, nb) : mt * 32 + l32, ks * 16 + hf * 8)]);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int x = 0; x < XB; ++x)
#pragma unroll
                        for (int mt = 0; mt < MAX_MT; ++mt)
                            if (mt < n_mt) acc[mt] = TR ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[x][mt], qf[ks], acc[mt], 0, 0, 0) : __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[ks], bf[x][mt], acc[mt], 0, 0, 0);
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (!EARLY_ROWS) {                                  // straight into the registers the matrix phase has just freed
            load_q(min(flat + 1, t1 - 1), qf);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (DEFER && count && pending) packed_hist_add_rows<MAX_MT>(sPk, copy_shift, hist_copy, outp_own, n_mt);   // the previous tile's row
        pending = false;
        // accumulator value v of tile mt <-> block 32*mt + 8*(v>>2) + 4*hf + (v&3) = 32*mt + 4*hf + c(v).  A value is a
        // real block (not padding up to the tile) when c(v) < lim, lim = nb - 32*mt - 4*hf; a whole group of four
        // consecutive blocks when c(v) + 3 < lim.  With NMT fixed, every tile but the last is all real blocks.
        auto tile_full = [&](int mt) { return NMT > 0 && mt < NMT - 1; };
        if constexpr (!TR) {
            // accumulator value v of tile mt <-> query row 8*(v>>2) + 4*hf + (v&3) of the wavefront's 32, block 32*mt + l32
            const int q_w = tile * SCORE_QT + wave * 32 + 4 * hf;         // + 8*(v>>2) + (v&3)
            float* prow = P + ((long long)bh * S + q_w) * nb_total + jb0 + l32;
            auto col_ok = [&](int mt) { return tile_full(mt) || mt * 32 + l32 < nb; };
            if constexpr (RAW) {
                take_next_rows();
#pragma unroll
                for (int mt = 0; mt < MAX_MT; ++mt) {
                    if (mt < n_mt && col_ok(mt)) {
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int dq = 8 * (v >> 2) + (v & 3);
                            if (q_w + dq < S) prow[(long long)dq * nb_total + mt * 32] = acc[mt][v] * score_scale;
                        }
                    }
                }
                continue;
            }
            float mrow[16], den[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float t = -INFINITY;
#pragma unroll
                for (int mt = 0; mt < MAX_MT; ++mt) {
                    if (mt < n_mt) {
                        float sv = acc[mt][v] * score_scale;
                        if (!tile_full(mt)) sv = col_ok(mt) ? sv : -INFINITY;
                        acc[mt][v] = sv;
                        t = fmaxf(t, sv);
                    }
                }
                mrow[v] = half32_max(t);
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float d = 0.f;
#pragma unroll
                for (int mt = 0; mt < MAX_MT; ++mt) {
                    if (mt < n_mt) {
                        const float e = __builtin_amdgcn_exp2f((acc[mt][v] - mrow[v]) * 1.44269504088896340736f);
                        acc[mt][v] = e;
                        d += e;
                    }
                }
                den[v] = half32_sum(d);
            }
            take_next_rows();
            auto& outp = pick_ref<DEFER>(outp_own, acc);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int dq = 8 * (v >> 2) + (v & 3);
                const bool live = q_w + dq < S;                   // a row past the end repeats the last query: counted as zeros
                const float inv_den = 1.f / den[v];
                if (row_stat && live && l32 == 0) row_stat[(long long)bh * S + q_w + dq] = make_float2(mrow[v], den[v]);
#pragma unroll
                for (int mt = 0; mt < MAX_MT; ++mt)
                    if (mt < n_mt) outp[mt][v] = live ? acc[mt][v] * inv_den : 0.f;
            }
#pragma unroll
            for (int mt = 0; mt < MAX_MT; ++mt) {
                if (mt < n_mt && col_ok(mt)) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int dq = 8 * (v >> 2) + (v & 3);
                        if (q_w + dq < S) prow[(long long)dq * nb_total + mt * 32] = outp[mt][v];
                    }
                }
            }
            // padding blocks and rows past the end hold P = 0 and land in bin 0 (see below)
            if constexpr (DEFER) pending = true;
            else if (count) packed_hist_add_rows<MAX_MT>(sPk, copy_shift, hist_copy, acc, n_mt);
            continue;
        }
        if constexpr (RAW) {
            take_next_rows();
            if (q < S) {
                float* dst = P + ((long long)bh * S + q) * nb_total + jb0;
#pragma unroll
                for (int mt = 0; mt < MAX_MT; ++mt) {
                    if (mt < n_mt) {
                        const int lim = nb - 32 * mt - 4 * hf;
#pragma unroll
                        for (int g = 0; g < 4; ++g) {
                            const int j0 = mt * 32 + 8 * g + 4 * hf;
                            if (vec_ok && 8 * g + 3 < lim) {
                                const f32x4_t o = {acc[mt][4 * g] * score_scale, acc[mt][4 * g + 1] * score_scale,
                                                   acc[mt][4 * g + 2] * score_scale, acc[mt][4 * g + 3] * score_scale};
                                *reinterpret_cast<f32x4_t*>(dst + j0) = o;
                            } else {
#pragma unroll
                                for (int r = 0; r < 4; ++r) if (8 * g + r < lim) dst[j0 + r] = acc[mt][4 * g + r] * score_scale;
                            }
                        }
                    }
                }
            }
            continue;
        }
        float m = -INFINITY;
#pragma unroll
        for (int mt = 0; mt < MAX_MT; ++mt) {
            if (mt < n_mt) {
                const int lim = nb - 32 * mt - 4 * hf;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    float sv = acc[mt][v] * score_scale;
                    if (!tile_full(mt)) sv = (8 * (v >> 2) + (v & 3) < lim) ? sv : -INFINITY;
                    acc[mt][v] = sv;
                    m = fmaxf(m, sv);
                }
            }
        }
        m = fmaxf(m, __shfl_xor(m, 32, 64));
        // exp(x) for x <= 0 as 2^(x * log2 e): one rounding in the product (relative error of the result below
        // 1e-7 * |x|, i.e. an absolute error below 1e-7 on every P that is not itself negligible) and the hardware's
        // 2^x (1 ulp); exp(-inf) = 0 on padding blocks
        float den = 0.f;
#pragma unroll
        for (int mt = 0; mt < MAX_MT; ++mt) {
            if (mt < n_mt) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float e = __builtin_amdgcn_exp2f((acc[mt][v] - m) * 1.44269504088896340736f);
                    acc[mt][v] = e;
                    den += e;
                }
            }
        }
        den += __shfl_xor(den, 32, 64);
        take_next_rows();
        auto& outp = pick_ref<DEFER>(outp_own, acc);
        {
            const float inv_den = 1.f / den;
#pragma unroll
            for (int mt = 0; mt < MAX_MT; ++mt)
                if (mt < n_mt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) outp[mt][v] = acc[mt][v] * inv_den;
        }
        if (row_stat && q < S && hf == 0) row_stat[(long long)bh * S + q] = make_float2(m, den);
        if (q < S) {
            float* dst = P + ((long long)bh * S + q) * nb_total + jb0;
#pragma unroll
            for (int mt = 0; mt < MAX_MT; ++mt) {
                if (mt < n_mt) {
                    const int lim = nb - 32 * mt - 4 * hf;
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int j0 = mt * 32 + 8 * g + 4 * hf;
                        if (vec_ok && (tile_full(mt) || 8 * g + 3 < lim)) {
                            const f32x4_t o = {outp[mt][4 * g], outp[mt][4 * g + 1], outp[mt][4 * g + 2], outp[mt][4 * g + 3]};
                            *reinterpret_cast<f32x4_t*>(dst + j0) = o;
                        } else {
#pragma unroll
                            for (int r = 0; r < 4; ++r) if (8 * g + r < lim) dst[j0 + r] = outp[mt][4 * g + r];
                        }
                    }
                }
            }
        }
        // first radix level, deferred: padding blocks hold P = 0 and land in bin 0 with the true zeros; that bin has no mass
        // and is the last of the descending scan, so neither a cut by mass nor one by count ever looks at its count.
        if constexpr (DEFER) pending = q < S;
        else if (count && q < S) packed_hist_add_rows<MAX_MT>(sPk, copy_shift, hist_copy, acc, n_mt);
    }
    if (DEFER && count && pending) packed_hist_add_rows<MAX_MT>(sPk, copy_shift, hist_copy, outp_own, n_mt);
    __syncthreads();
    if (hist_cnt && cur_bh >= 0) packed_hist_flush(sPk, copy_shift, hist_cnt, hist_sum, cur_bh, fix_shift, tid, SCORE_NT);
}

// ---------------------------------------------------------------------------------------------
// More than 256 blocks: P holds the scaled scores (score_mfma_kernel with RAW); this kernel turns every row into its
// soft-max in place and takes the first radix level.  One wavefront per row, a lane owns columns lane, lane + 64, ...
__global__ __launch_bounds__(256) void softmax_rows_kernel(float* __restrict__ P, unsigned int* __restrict__ hist_cnt,
                                                           unsigned long long* __restrict__ hist_sum, int S, int nb,
                                                           int fix_shift, float2* __restrict__ row_stat) {
    constexpr int MAXC = VMOBA_MAX_BLOCKS / 64;
    __shared__ unsigned int sCnt[HIST_BINS];
    __shared__ unsigned long long sSum[HIST_BINS];
    const int bh = blockIdx.y;
    for (int i = threadIdx.x; i < HIST_BINS; i += 256) { sCnt[i] = 0u; sSum[i] = 0ull; }
    __syncthreads();
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    for (int q = blockIdx.x * 4 + wv; q < S; q += gridDim.x * 4) {
        float* row = P + ((long long)bh * S + q) * nb;
        float v[MAXC];
        float m = -INFINITY;
#pragma unroll
        for (int c = 0; c < MAXC; ++c) {
            const int j = c * 64 + lane;
            v[c] = j < nb ? row[j] : -INFINITY;
            m = fmaxf(m, v[c]);
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
        float den = 0.f;
#pragma unroll
        for (int c = 0; c < MAXC; ++c) {
            v[c] = expf(v[c] - m);            // exp(-inf) = 0 past the row's end
            den += v[c];
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) den += __shfl_xor(den, off, 64);
        if (row_stat && lane == 0) row_stat[(long long)bh * S + q] = make_float2(m, den);
#pragma unroll
        for (int c = 0; c < MAXC; ++c) {
            const int j = c * 64 + lane;
            if (j < nb) {
                const float p = v[c] / den;
                row[j] = p;
                if (hist_cnt) {
                    const unsigned int bin = min(__float_as_uint(p) >> 20, (unsigned)(HIST_BINS - 1));
                    atomicAdd(&sCnt[bin], 1u);
                    atomicAdd(&sSum[bin], to_fixed(p, fix_shift));
                }
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < HIST_BINS; i += 256) {
        const unsigned int c = sCnt[i];
        if (c) {
            atomicAdd(&hist_cnt[(long long)bh * HIST_BINS + i], c);
            atomicAdd(&hist_sum[(long long)bh * HIST_BINS + i], sSum[i]);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Descending scan of one radix level.  One workgroup of 1024 threads per head; thread t owns
// bin 1023 - t, so an inclusive prefix sum over t is the descending cumulative sum.
// BYCOUNT = false: the cut is where the descending cumulative SUM reaches `target` (threshold selection,
// Eq. 4); BYCOUNT = true: where the descending cumulative COUNT reaches it (a fixed global k).
template <int LEVEL, bool BYCOUNT>
__global__ __launch_bounds__(HIST_BINS) void scan_level_kernel(const unsigned int* __restrict__ hist_cnt,
                                                               const unsigned long long* __restrict__ hist_sum,
                                                               HeadState* __restrict__ state,
                                                               unsigned long long target, int fix_shift,
                                                               long long pool_size, long long* __restrict__ k_out,
                                                               float* __restrict__ theta_out) {
    __shared__ unsigned long long sS[HIST_BINS];
    __shared__ unsigned long long sC[HIST_BINS];
    const int bh = blockIdx.x, t = threadIdx.x;
    const int bin = HIST_BINS - 1 - t;
    HeadState st = state[bh];
    if (LEVEL > 0 && st.all) {
        if (LEVEL == 2 && t == 0) { k_out[bh] = pool_size; theta_out[bh] = 0.f; }
        return;
    }
    const unsigned long long my_s = hist_sum[(long long)bh * HIST_BINS + bin];
    const unsigned long long my_c = hist_cnt[(long long)bh * HIST_BINS + bin];
    sS[t] = my_s;
    sC[t] = my_c;
    __syncthreads();
    for (int off = 1; off < HIST_BINS; off <<= 1) {
        unsigned long long a = 0, c = 0;
        if (t >= off) { a = sS[t - off]; c = sC[t - off]; }
        __syncthreads();
        sS[t] += a;
        sC[t] += c;
        __syncthreads();
    }
    const unsigned long long need = (LEVEL == 0) ? target : st.need;
    const unsigned long long cexcl = sC[t] - my_c;
    const unsigned long long incl = BYCOUNT ? sC[t] : sS[t];
    const unsigned long long excl = BYCOUNT ? cexcl : incl - my_s;
    if (LEVEL == 0 && t == HIST_BINS - 1 && incl < need) {
        // the whole pool does not reach the target (tau >= 1, or rounding): keep everything
        HeadState ns = st;
        ns.all = 1u;
        state[bh] = ns;
    }
    if (excl < need && need <= incl) {
        HeadState ns = st;
        ns.need = need - excl;
        ns.cnt_above = (LEVEL == 0 ? 0ull : st.cnt_above) + cexcl;
        ns.all = 0u;
        if (LEVEL == 0) ns.prefix = ((unsigned)bin) << 20;
        if (LEVEL == 1) ns.prefix = st.prefix | (((unsigned)bin) << 10);
        if (LEVEL == 2) {
            ns.prefix = st.prefix | (unsigned)bin;
            const float theta = __uint_as_float(ns.prefix);
            unsigned long long take;
            if (BYCOUNT) {
                take = ns.need;                                            // entries still missing
            } else {
                const unsigned long long each = to_fixed(theta, fix_shift);   // > 0: this bin has mass
                take = (ns.need + each - 1) / each;
            }
            if (take > my_c) take = my_c;
            if (take < 1) take = 1;
            ns.n_tie = (unsigned)my_c;
            ns.take = (unsigned)take;
            k_out[bh] = (long long)(ns.cnt_above + take);
            theta_out[bh] = theta;
        }
        state[bh] = ns;
    }
}

// ---------------------------------------------------------------------------------------------
// Pool soft-max mode: "normalised" read as ONE soft-max over the head's whole pool of S * N_b scores.
// With the row soft-max P[q, j] = exp(s_qj - m_q) / d_q already written, the pool value is
//   G[q, j] = exp(s_qj - M) / Z = P[q, j] * w_q,   w_q = d_q exp(m_q - M) / Z,
//   M = max_q m_q,   Z = sum_q d_q exp(m_q - M).
// pool_stat_kernel: one workgroup per head, fixed summation order (double), so Z is reproducible.
__global__ __launch_bounds__(1024) void pool_stat_kernel(const float2* __restrict__ row_stat, float2* __restrict__ pool_stat, int S) {
    __shared__ float sM[1024];
    __shared__ double sZ[1024];
    const int bh = blockIdx.x, t = threadIdx.x;
    const float2* rs = row_stat + (long long)bh * S;
    float m = -INFINITY;
    for (int q = t; q < S; q += 1024) m = fmaxf(m, rs[q].x);
    sM[t] = m;
    __syncthreads();
    for (int off = 512; off >= 1; off >>= 1) {
        if (t < off) sM[t] = fmaxf(sM[t], sM[t + off]);
        __syncthreads();
    }
    const float M = sM[0];
    double z = 0.0;
    for (int q = t; q < S; q += 1024) z += (double)rs[q].y * (double)expf(rs[q].x - M);
    sZ[t] = z;
    __syncthreads();
    for (int off = 512; off >= 1; off >>= 1) {
        if (t < off) sZ[t] += sZ[t + off];
        __syncthreads();
    }
    if (t == 0) pool_stat[bh] = make_float2(M, (float)(1.0 / sZ[0]));
}

// P <- G in place, and the first radix level (count + fixed-point sum per bin) of the new values.
__global__ __launch_bounds__(256) void pool_rescale_kernel(float* __restrict__ P, const float2* __restrict__ row_stat,
                                                           const float2* __restrict__ pool_stat,
                                                           unsigned int* __restrict__ hist_cnt,
                                                           unsigned long long* __restrict__ hist_sum,
                                                           int S, int nb, int fix_shift) {
    __shared__ unsigned int sCnt[HIST_BINS];
    __shared__ unsigned long long sSum[HIST_BINS];
    const int bh = blockIdx.y;
    for (int i = threadIdx.x; i < HIST_BINS; i += 256) { sCnt[i] = 0u; sSum[i] = 0ull; }
    __syncthreads();
    const float2 ps = pool_stat[bh];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    for (int q = blockIdx.x * 4 + wv; q < S; q += gridDim.x * 4) {      // one wavefront per row
        const float2 rs = row_stat[(long long)bh * S + q];
        const float w = rs.y * expf(rs.x - ps.x) * ps.y;
        float* row = P + ((long long)bh * S + q) * nb;
        for (int j = lane; j < nb; j += 64) {
            const float g = row[j] * w;
            row[j] = g;
            const unsigned int bin = min(__float_as_uint(g) >> 20, (unsigned)(HIST_BINS - 1));
            atomicAdd(&sCnt[bin], 1u);
            atomicAdd(&sSum[bin], to_fixed(g, fix_shift));
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < HIST_BINS; i += 256) {
        const unsigned int c = sCnt[i];
        if (c) {
            atomicAdd(&hist_cnt[(long long)bh * HIST_BINS + i], c);
            atomicAdd(&hist_sum[(long long)bh * HIST_BINS + i], sSum[i]);
        }
    }
}

// Radix levels 1 and 2: histogram of the next 10 bits over the entries whose higher bits
// equal the prefix found so far.  The entries of one bin share every bit above the level's trailing bits (10 at level 1,
// none at level 2), so a bin needs only their number and the sum of those trailing bits: one packed 64-bit LDS atomic
// per candidate (count in bits 40..63), turned into count and fixed-point sum when the workgroup flushes.
// Few, large workgroups (one per compute unit over all heads): every workgroup ends with up to two device-wide atomics per
// bin, and those, not the pass over P, set the time when thousands of workgroups flush.
constexpr int REFINE_NT = 1024;
template <int LEVEL>
__global__ __launch_bounds__(REFINE_NT) void refine_hist_kernel(const float* __restrict__ P, const HeadState* __restrict__ state,
                                                          unsigned int* __restrict__ hist_cnt,
                                                          unsigned long long* __restrict__ hist_sum,
                                                          long long pool_size, int fix_shift) {
    __shared__ unsigned long long sPk[HIST_BINS];
    const int bh = blockIdx.y;
    const HeadState st = state[bh];
    if (st.all) return;
    for (int i = threadIdx.x; i < HIST_BINS; i += REFINE_NT) sPk[i] = 0ull;
    __syncthreads();
    constexpr int SHIFT_HI = (LEVEL == 1) ? 20 : 10;
    constexpr int SHIFT_LO = (LEVEL == 1) ? 10 : 0;
    constexpr unsigned int LOW_MASK = (1u << SHIFT_LO) - 1u;
    const unsigned int want = st.prefix >> SHIFT_HI;
    auto take = [&](unsigned int u) {
        if ((u >> SHIFT_HI) == want)
            atomicAdd(&sPk[(u >> SHIFT_LO) & (HIST_BINS - 1)], PK_ONE | (unsigned long long)(u & LOW_MASK));
    };
    const u32x4_t* src = reinterpret_cast<const u32x4_t*>(P + (long long)bh * pool_size);
    // 16-byte loads need every head's pool to start on a 16-byte boundary
    const long long n4 = (pool_size % 4 == 0) ? pool_size / 4 : 0;
    // four 16-byte loads in flight per thread: a workgroup takes runs of 4 * REFINE_NT vectors
    for (long long i0 = (long long)blockIdx.x * (4 * REFINE_NT) + threadIdx.x; i0 < n4; i0 += (long long)gridDim.x * (4 * REFINE_NT)) {
        u32x4_t v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const long long i = i0 + REFINE_NT * k;
            const u32x4_t none = {~0u, ~0u, ~0u, ~0u};      // matches no prefix (a NaN pattern; P holds none)
            v[k] = i < n4 ? src[i] : none;
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            take(v[k].x); take(v[k].y); take(v[k].z); take(v[k].w);
        }
    }
    {
        const unsigned int* s1 = reinterpret_cast<const unsigned int*>(P + (long long)bh * pool_size);
        for (long long i = n4 * 4 + (long long)blockIdx.x * REFINE_NT + threadIdx.x; i < pool_size;
             i += (long long)gridDim.x * REFINE_NT)
            take(s1[i]);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < HIST_BINS; i += REFINE_NT) {
        const unsigned long long w = sPk[i];
        if (w) {
            const unsigned long long cnt = w >> 40, low = w & (PK_ONE - 1);
            // every entry of the bin is (lead | its trailing bits) as a float pattern; to_fixed is linear in the
            // mantissa for a fixed exponent, and the exponent lies in the prefix
            const unsigned int lead = (want << SHIFT_HI) | ((unsigned int)i << SHIFT_LO);
            const int e = (int)(lead >> 23), sh = e - 150 + fix_shift;
            atomicAdd(&hist_cnt[(long long)bh * HIST_BINS + i], (unsigned int)cnt);
            if (e && sh >= 0)
                atomicAdd(&hist_sum[(long long)bh * HIST_BINS + i],
                          (cnt * (unsigned long long)((lead & 0x7fffffu) | 0x800000u) + low) << sh);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Per-row count of entries equal to theta.  Only needed when some but not all of them belong
// to the top k; otherwise the kernel returns at once.
__global__ __launch_bounds__(256) void tie_count_kernel(const float* __restrict__ P, const HeadState* __restrict__ state,
                                                        int* __restrict__ ties, int S, int nb) {
    const int bh = blockIdx.y;
    const HeadState st = state[bh];
    if (st.all || st.take == st.n_tie) return;
    const int lane = threadIdx.x & 63;
    const int gw = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int n_gw = gridDim.x * 4;
    for (int q = gw; q < S; q += n_gw) {
        const unsigned int* row = reinterpret_cast<const unsigned int*>(P + ((long long)bh * S + q) * nb);
        int c = 0;
        for (int j0 = 0; j0 < nb; j0 += 64) {
            int j = j0 + lane;
            bool tie = (j < nb) && (row[j] == st.prefix);
            c += __popcll(__ballot(tie));
        }
        if (lane == 0) ties[(long long)bh * S + q] = c;
    }
}

// Exclusive prefix sum of in[bh][0..S) into out[bh][0..S], out[bh][S] = total.  One workgroup
// per head.  `needs_ties` = 1 makes the launch a no-op for heads that do not need tie ranks.
__global__ __launch_bounds__(SCAN_THREADS) void row_scan_kernel(const int* __restrict__ in, int* __restrict__ out,
                                                                const HeadState* __restrict__ state, int needs_ties,
                                                                int S) {
    __shared__ int sW[SCAN_THREADS / 64];
    __shared__ int sCarry;
    // a batch of SCAN_THREADS * SCAN_ITEMS values passes through LDS so that global memory is read and written in whole
    // rows of consecutive lanes while every thread scans SCAN_ITEMS consecutive values; item i sits at i + i / SCAN_ITEMS
    // (a thread's items then start SCAN_ITEMS + 1 words apart: no bank conflicts)
    __shared__ int sBuf[SCAN_THREADS * (SCAN_ITEMS + 1)];
    const int bh = blockIdx.x, t = threadIdx.x;
    if (needs_ties) {
        const HeadState st = state[bh];
        if (st.all || st.take == st.n_tie) return;
    }
    const int* src = in + (long long)bh * S;
    int* dst = out + (long long)bh * (S + 1);
    if (t == 0) sCarry = 0;
    __syncthreads();
    for (int base = 0; base < S; base += SCAN_THREADS * SCAN_ITEMS) {
#pragma unroll
        for (int e = 0; e < SCAN_ITEMS; ++e) {
            const int li = e * SCAN_THREADS + t;
            sBuf[li + li / SCAN_ITEMS] = (base + li < S) ? src[base + li] : 0;
        }
        __syncthreads();
        int v[SCAN_ITEMS];
        int sum = 0;
#pragma unroll
        for (int e = 0; e < SCAN_ITEMS; ++e) {
            v[e] = sBuf[t * (SCAN_ITEMS + 1) + e];
            sum += v[e];
        }
        // inclusive scan of `sum` across the workgroup: wave scan, then scan of wave totals
        int incl = sum;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            int n = __shfl_up(incl, off, 64);
            if ((t & 63) >= off) incl += n;
        }
        if ((t & 63) == 63) sW[t >> 6] = incl;
        __syncthreads();
        int wave_base = 0;
        for (int w = 0; w < (t >> 6); ++w) wave_base += sW[w];
        int run = sCarry + wave_base + incl - sum;
#pragma unroll
        for (int e = 0; e < SCAN_ITEMS; ++e) {
            sBuf[t * (SCAN_ITEMS + 1) + e] = run;
            run += v[e];
        }
        __syncthreads();
        if (t == SCAN_THREADS - 1) sCarry = run;
#pragma unroll
        for (int e = 0; e < SCAN_ITEMS; ++e) {
            const int li = e * SCAN_THREADS + t;
            if (base + li < S) dst[base + li] = sBuf[li + li / SCAN_ITEMS];
        }
        __syncthreads();
    }
    if (t == 0) dst[S] = sCarry;
}

// ---------------------------------------------------------------------------------------------
// TopkMask (Eq. 3): bit (q, j) = P[q, j] is among the k best of the head.  One wavefront per
// 64 consecutive queries.  Also counts, per wavefront, how many of its queries keep each block
// (the raw material of the block-major list).
// Block that holds block-order position q (blk_off ascending, blk_off[0] = 0, blk_off[nb] = S).
__device__ __forceinline__ int block_of_position(const int* __restrict__ blk_off, int nb, int q) {
    int lo = 0, hi = nb;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (blk_off[mid] <= q) lo = mid; else hi = mid;
    }
    return lo;
}

// own_blk_off: null, or blk_off when every query also keeps the block it lies in itself; query_pos: null when query q
// sits at block-order position q, else the position of every query (queries kept in the caller's token order).
__global__ __launch_bounds__(256) void mask_kernel(const float* __restrict__ P, const HeadState* __restrict__ state,
                                                   const int* __restrict__ tie_base, unsigned int* __restrict__ mask,
                                                   int* __restrict__ wtot, int* __restrict__ wcnt,
                                                   int S, int nb, int n_waves, const int* __restrict__ own_blk_off,
                                                   const int* __restrict__ query_pos) {
    __shared__ unsigned int sGt[4][64][VMOBA_MAX_MASK_WORDS + 1];
    __shared__ unsigned int sTie[4][64][VMOBA_MAX_MASK_WORDS + 1];
    const int bh = blockIdx.y;
    const HeadState st = state[bh];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int w = blockIdx.x * 4 + wv;           // global wavefront index = 64-query group
    const bool active = w < n_waves;             // surplus wavefronts only keep the barriers company
    const int q0 = active ? w * 64 : 0;
    const int words = (nb + 31) / 32;
    const int rows = active ? min(64, S - q0) : 0;
    // The wavefront's 64 rows of P are one contiguous run of rows * nb values: it is read flat, 16 bytes per lane and
    // eight loads in flight, and every lane ORs the bits of its four values into the rows' mask words in LDS (a group
    // of four can straddle two words or two rows).
    for (int wd = 0; wd < words; ++wd) { sGt[wv][lane][wd] = 0u; sTie[wv][lane][wd] = 0u; }
    __syncthreads();
    {
        const int n_el = rows * nb;
        const unsigned int* tile = reinterpret_cast<const unsigned int*>(P + ((long long)bh * S + q0) * nb);
        const bool aligned = (reinterpret_cast<uintptr_t>(tile) & 15) == 0;      // wave-uniform
        const int n4 = (aligned && nb >= 4) ? n_el / 4 : 0;                      // whole groups of four (a group spans at most two rows)
        const float inv_nb = 1.f / (float)nb;
        auto put = [&](unsigned int (*arr)[VMOBA_MAX_MASK_WORDS + 1], int row, int col, unsigned int bits, int count) {
            // `count` (1..4) bits for columns col, col + 1, ... of `row`, continuing in the next row past column nb - 1
            const int here = min(count, nb - col);
            const unsigned int b0 = bits & ((1u << here) - 1u);
            if (b0) {
                const unsigned long long v = (unsigned long long)b0 << (col & 31);
                atomicOr(&arr[row][col >> 5], (unsigned int)v);
                if (v >> 32) atomicOr(&arr[row][(col >> 5) + 1], (unsigned int)(v >> 32));
            }
            const unsigned int b1 = bits >> here;
            if (b1) atomicOr(&arr[row + 1][0], b1);
        };
        for (int k0 = 0; k0 < n4; k0 += 64 * 8) {
            u32x4_t x[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i4 = k0 + u * 64 + lane;
                const u32x4_t z = {0u, 0u, 0u, 0u};
                x[u] = i4 < n4 ? reinterpret_cast<const u32x4_t*>(tile)[i4] : z;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i4 = k0 + u * 64 + lane;
                if (i4 >= n4) continue;
                const int e = 4 * i4;
                int row = (int)((float)e * inv_nb);
                if (row * nb > e) --row;
                if ((row + 1) * nb <= e) ++row;
                const int col = e - row * nb;
                unsigned int gt = 0u, ti = 0u;
#pragma unroll
                for (int cidx = 0; cidx < 4; ++cidx) {
                    const unsigned int v = x[u][cidx];
                    if (st.all || v > st.prefix) gt |= 1u << cidx;
                    else if (v == st.prefix) ti |= 1u << cidx;
                }
                put(sGt[wv], row, col, gt, 4);
                if (ti) put(sTie[wv], row, col, ti, 4);
            }
        }
        // what the groups of four did not cover (everything when the run does not start 16-byte aligned)
        for (int e = 4 * n4 + lane; e < n_el; e += 64) {
            int row = (int)((float)e * inv_nb);
            if (row * nb > e) --row;
            if ((row + 1) * nb <= e) ++row;
            const int col = e - row * nb;
            const unsigned int v = tile[e];
            if (st.all || v > st.prefix) put(sGt[wv], row, col, 1u, 1);
            else if (v == st.prefix) put(sTie[wv], row, col, 1u, 1);
        }
    }
    __syncthreads();
    // lane = row
    unsigned int mw[VMOBA_MAX_MASK_WORDS];
    const int q = q0 + lane;
    const bool live = lane < rows;
    if (live) {
        const bool all_ties = (st.take == st.n_tie);
        int rank = all_ties ? 0 : tie_base[(long long)bh * (S + 1) + q];
        const int own = own_blk_off ? block_of_position(own_blk_off, nb, query_pos ? query_pos[q] : q) : -1;
#pragma unroll
        for (int wd = 0; wd < VMOBA_MAX_MASK_WORDS; ++wd) {
            unsigned int g = 0;
            if (wd < words) {
                g = sGt[wv][lane][wd];
                if (wd == (own >> 5)) g |= 1u << (own & 31);       // own = -1: no word matches
                unsigned int t = sTie[wv][lane][wd];
                if (all_ties) {
                    g |= t;
                } else {
                    while (t) {
                        const int bpos = __ffs(t) - 1;
                        t &= t - 1;
                        if ((unsigned)rank < st.take) g |= 1u << bpos;
                        ++rank;
                    }
                }
                mask[((long long)bh * S + q) * words + wd] = g;
            }
            mw[wd] = g;
        }
    } else {
#pragma unroll
        for (int wd = 0; wd < VMOBA_MAX_MASK_WORDS; ++wd) mw[wd] = 0;
    }
    // per-block count over the 64 rows of this wavefront (word by word, so that a word is one register) and their sum,
    // the number of pairs these 64 queries keep
    int kept = 0;
#pragma unroll
    for (int wd = 0; wd < VMOBA_MAX_MASK_WORDS; ++wd) {
        if (wd * 32 < nb) {
            const unsigned int word = mw[wd];
            const int jn = min(32, nb - wd * 32);
            for (int bit = 0; bit < jn; ++bit) {
                const int j = wd * 32 + bit;
                const int c = __popcll(__ballot((word >> bit) & 1u));
                kept += c;
                if (lane == 0 && active) wcnt[((long long)bh * nb + j) * n_waves + w] = c;
            }
        }
    }
    if (lane == 0 && active) wtot[(long long)bh * n_waves + w] = kept;
}

// Per-query ("local") selection, the block-choice variants of the paper's ablation and of its
// training-free runs.  LOCAL_TOPK: a query keeps its `topk` most similar blocks; otherwise it keeps the
// shortest descending prefix of its own row whose sum reaches tau.  Entry j' ranks before j when it is
// larger, or equal with a lower block index.  One wavefront per 64 queries; a row is spread over the
// lanes (up to 4 columns each) and every lane counts, or sums, what ranks before its own entries.
// Same outputs as mask_kernel.
template <bool LOCAL_TOPK>
__global__ __launch_bounds__(256) void local_mask_kernel(const float* __restrict__ P, unsigned int* __restrict__ mask,
                                                         int* __restrict__ wtot, int* __restrict__ wcnt,
                                                         int S, int nb, int n_waves, int topk, float tau,
                                                         const int* __restrict__ own_blk_off, const int* __restrict__ query_pos) {
    constexpr int MAXC = VMOBA_MAX_BLOCKS / 64;
    __shared__ float sRow[4][VMOBA_MAX_BLOCKS];
    __shared__ unsigned int sKeep[4][64][VMOBA_MAX_MASK_WORDS + 1];
    const int bh = blockIdx.y;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int w = blockIdx.x * 4 + wv;
    const bool active = w < n_waves;
    const int q0 = active ? w * 64 : 0;
    const int words = (nb + 31) / 32;
    const int rows = active ? min(64, S - q0) : 0;
    const int ncol = (nb + 63) / 64;
    for (int r = 0; r < 64; ++r) {
        const bool live = r < rows;
        const float* row = P + ((long long)bh * S + q0 + (live ? r : 0)) * nb;
        float v[MAXC];
#pragma unroll
        for (int c = 0; c < MAXC; ++c) {
            const int j = c * 64 + lane;
            v[c] = (c < ncol && j < nb) ? row[j] : -1.f;
            if (c < ncol && j < nb) sRow[wv][j] = v[c];
        }
        __syncthreads();
        float before[MAXC];
#pragma unroll
        for (int c = 0; c < MAXC; ++c) before[c] = 0.f;
        for (int jp = 0; jp < nb; ++jp) {
            const float x = sRow[wv][jp];
#pragma unroll
            for (int c = 0; c < MAXC; ++c) {
                if (c < ncol) {               // uniform: columns past the row's end are not ranked
                    const int j = c * 64 + lane;
                    const bool first = (x > v[c]) || (x == v[c] && jp < j);
                    before[c] += first ? (LOCAL_TOPK ? 1.f : x) : 0.f;
                }
            }
        }
#pragma unroll
        for (int c = 0; c < MAXC; ++c) {
            const int j = c * 64 + lane;
            const bool keep = live && c < ncol && j < nb && (LOCAL_TOPK ? before[c] < (float)topk : (tau >= 1.f || before[c] < tau));
            const unsigned long long bal = __ballot(keep);
            if (lane == 0 && c < ncol) {
                sKeep[wv][r][2 * c] = (unsigned)bal;
                if (2 * c + 1 <= VMOBA_MAX_MASK_WORDS) sKeep[wv][r][2 * c + 1] = (unsigned)(bal >> 32);
            }
        }
        __syncthreads();
    }
    // lane = row
    unsigned int mw[VMOBA_MAX_MASK_WORDS];
    const int q = q0 + lane;
    const bool live = lane < rows;
    const int own = (own_blk_off && live) ? block_of_position(own_blk_off, nb, query_pos ? query_pos[q] : q) : -1;
#pragma unroll
    for (int wd = 0; wd < VMOBA_MAX_MASK_WORDS; ++wd) {
        unsigned int g = 0;
        if (live && wd < words) {
            g = sKeep[wv][lane][wd];
            if (wd == (own >> 5)) g |= 1u << (own & 31);
            mask[((long long)bh * S + q) * words + wd] = g;
        }
        mw[wd] = g;
    }
    int kept = 0;
#pragma unroll
    for (int wd = 0; wd < VMOBA_MAX_MASK_WORDS; ++wd) {
        if (wd * 32 < nb) {
            const unsigned int word = mw[wd];
            const int jn = min(32, nb - wd * 32);
            for (int bit = 0; bit < jn; ++bit) {
                const int j = wd * 32 + bit;
                const int c = __popcll(__ballot((word >> bit) & 1u));
                kept += c;
                if (lane == 0 && active) wcnt[((long long)bh * nb + j) * n_waves + w] = c;
            }
        }
    }
    if (lane == 0 && active) wtot[(long long)bh * n_waves + w] = kept;
}

// Offsets of both list forms, in two small launches.
// wave_scan_kernel, one workgroup per (row, head), rows 0..nb:
//  * row j < nb: wcnt[j][w] (pairs of block j among the 64 queries of wavefront w) -> its exclusive scan over w, in place:
//    where wavefront w's entries of block j start inside the block's list; the total is the block's count;
//  * row nb: wtot[w] (pairs kept by the 64 queries of wavefront w) -> its exclusive scan, in place: where their rows
//    start in the query-major lists; the total is row_ptr[S].
__global__ __launch_bounds__(256) void wave_scan_kernel(int* __restrict__ wcnt, int* __restrict__ wtot,
                                                        int* __restrict__ row_tot, int nb, int n_waves) {
    __shared__ int sW[4];
    __shared__ int sCarry;
    const int j = blockIdx.x, bh = blockIdx.y, t = threadIdx.x;
    int* col = j < nb ? wcnt + ((long long)bh * nb + j) * n_waves : wtot + (long long)bh * n_waves;
    if (t == 0) sCarry = 0;
    __syncthreads();
    for (int base = 0; base < n_waves; base += 256) {
        const int i = base + t;
        const int v = (i < n_waves) ? col[i] : 0;
        int incl = v;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            int n = __shfl_up(incl, off, 64);
            if ((t & 63) >= off) incl += n;
        }
        if ((t & 63) == 63) sW[t >> 6] = incl;
        __syncthreads();
        int wave_base = 0;
        for (int w = 0; w < (t >> 6); ++w) wave_base += sW[w];
        const int excl = sCarry + wave_base + incl - v;
        if (i < n_waves) col[i] = excl;
        __syncthreads();
        if (t == 255) sCarry = excl + v;
        __syncthreads();
    }
    if (t == 0) row_tot[(long long)bh * (nb + 1) + j] = sCarry;
}

// blk_ptr = exclusive scan of the block counts, with the capacity check.  One wavefront per head, a run of blocks per
// lane.  A head that kept more than `cap` pairs gets an all-zero blk_ptr -- to the attention calls it selected nothing,
// so no list entry of it is ever read (the merge kernels recognise the same head by row_ptr[S] > cap) -- and the status
// word is set.  Also row_ptr[S], the head's number of pairs; write_k != 0 (per-query modes, or every query keeps its
// own block: the number of kept pairs is not the k of the cut) copies it to k_out, write_k == 2 also clears theta_out.
__global__ __launch_bounds__(64) void blk_ptr_kernel(const int* __restrict__ row_tot, int* __restrict__ blk_ptr,
                                                     int* __restrict__ row_ptr, long long* __restrict__ k_out,
                                                     float* __restrict__ theta_out, int nb, int S, long long cap,
                                                     int* __restrict__ dev_status, int write_k) {
    const int bh = blockIdx.x, lane = threadIdx.x;
    const int per = (nb + 63) / 64;                  // consecutive blocks per lane
    const int j0 = min(nb, lane * per), j1 = min(nb, j0 + per);
    const int* cnt = row_tot + (long long)bh * (nb + 1);
    int* out = blk_ptr + (long long)bh * (nb + 1);
    int mine = 0;
    for (int j = j0; j < j1; ++j) mine += cnt[j];
    int incl = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(incl, off, 64);
        if (lane >= off) incl += o;
    }
    const long long total = __shfl(incl, 63, 64);
    const bool fits = total <= cap;
    int run = incl - mine;
    for (int j = j0; j < j1; ++j) {
        out[j] = fits ? run : 0;
        run += cnt[j];
    }
    if (lane == 0) {
        out[nb] = fits ? (int)total : 0;
        if (!fits) atomicExch(dev_status, (int)VMOBA_ERR_CAPACITY);
        row_ptr[(long long)bh * (S + 1) + S] = cnt[nb];
        if (write_k) k_out[bh] = cnt[nb];
        if (write_k == 2) theta_out[bh] = 0.f;
    }
}

// Workgroup i of n runs on XCD i % 8; this index makes the workgroups of one XCD neighbours in the work list, so runs
// that different workgroups write into the same cache line meet in one L2.
__device__ __forceinline__ int xcd_contiguous(int i, int n) {
    const int per = n / 8;
    return i < per * 8 ? (i % 8) * per + i / 8 : i;
}

// Fill q_idx (block-major), col_idx and pair_pos (query-major).  One wavefront per 64 queries,
// lane = query; a ballot per block gives every query its rank inside the wavefront.
__global__ __launch_bounds__(256) void fill_lists_kernel(const unsigned int* __restrict__ mask, int* __restrict__ row_ptr,
                                                         const int* __restrict__ wbase,
                                                         const int* __restrict__ blk_ptr, const int* __restrict__ wcnt,
                                                         int* __restrict__ q_idx, int* __restrict__ col_idx,
                                                         int* __restrict__ pair_pos, int S, int nb, int n_waves,
                                                         long long cap) {
    // The query-major entries of a wavefront's 64 rows form one contiguous run of col_idx / pair_pos.  They are collected
    // in LDS, a window of FILL_STAGE entries at a time, and written out as whole runs; a lane writing its own row's
    // entries straight to global memory touches a different cache line in every lane of every store.  A run longer
    // than the window walks the blocks once per window (the walk is a few hundred instructions; the window size sets
    // how many wavefronts a compute unit holds).
    constexpr int FILL_STAGE = 2048;
    __shared__ unsigned short sCol[4][FILL_STAGE];
    __shared__ int sPos[4][FILL_STAGE];
    const int bh = blockIdx.y;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int w = xcd_contiguous(blockIdx.x, gridDim.x) * 4 + wv;
    const bool active = w < n_waves;
    const int words = (nb + 31) / 32;
    // where this wavefront's entries of block j start in the block-major list: lane l keeps it for blocks l, l + 64, ...
    // (the walk below reads it with a lane broadcast: no LDS round trip inside the loop)
    int vbase[VMOBA_MAX_BLOCKS / 64];
#pragma unroll
    for (int i = 0; i < VMOBA_MAX_BLOCKS / 64; ++i) {
        const int j = lane + 64 * i;
        vbase[i] = (active && j < nb) ? blk_ptr[(long long)bh * (nb + 1) + j] + wcnt[((long long)bh * nb + j) * n_waves + w] : 0;
    }
    const int q = w * 64 + lane;
    const bool live = active && q < S;
    unsigned int mw[VMOBA_MAX_MASK_WORDS];
#pragma unroll
    for (int wd = 0; wd < VMOBA_MAX_MASK_WORDS; ++wd)
        mw[wd] = (live && wd < words) ? mask[((long long)bh * S + q) * words + wd] : 0u;
    // row_ptr of the wavefront's rows: where the wavefront's run of the query-major lists starts (wbase, the scan of the
    // wavefronts' totals) plus the pairs of the lanes before; written here, row_ptr[S] by the offsets kernel
    int cnt = 0;
#pragma unroll
    for (int wd = 0; wd < VMOBA_MAX_MASK_WORDS; ++wd) cnt += __popc(mw[wd]);
    int incl = cnt;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(incl, off, 64);
        if (lane >= off) incl += o;
    }
    const long long run0 = active ? wbase[(long long)bh * n_waves + w] : 0;
    const long long run1 = run0 + __shfl(incl, 63, 64);             // the wavefront's run: [run0, run1)
    const long long r0 = run0 + incl - cnt;
    if (live) row_ptr[(long long)bh * (S + 1) + q] = (int)r0;
    const long long seg = (long long)bh * cap;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    const bool staged = run1 <= cap;                                     // wave-uniform; false only for a head that overflowed
    const int n_run = (int)(run1 - run0);
    // window 0 always runs (it also writes q_idx); an overflowed head writes its entries below cap one by one
    for (int win0 = 0; win0 == 0 || (staged && win0 < n_run); win0 += FILL_STAGE) {
        long long r = r0;
        int lr = (int)(r0 - run0) - win0;                                // position inside the window
#pragma unroll
        for (int wd = 0; wd < VMOBA_MAX_MASK_WORDS; ++wd) {          // word by word, so that a word is one register
            if (wd * 32 >= nb) continue;
            const unsigned int word = mw[wd];
            const int jn = min(32, nb - wd * 32);
            for (int b = 0; b < jn; ++b) {
                const int j = wd * 32 + b;
                const bool bit = (word >> b) & 1u;
                const unsigned long long bal = __ballot(bit);
                const int base_j = __builtin_amdgcn_readlane(vbase[wd >> 1], (wd & 1) * 32 + b);
                if (bit) {
                    const long long pos = (long long)base_j + __popcll(bal & lt_mask);
                    if (win0 == 0 && pos < cap) q_idx[seg + pos] = q;
                    if (staged) {
                        if ((unsigned)lr < (unsigned)FILL_STAGE) {
                            sCol[wv][lr] = (unsigned short)j;
                            sPos[wv][lr] = (int)pos;
                        }
                        ++lr;
                    } else {
                        if (r < cap) { col_idx[seg + r] = j; pair_pos[seg + r] = (int)pos; }
                        ++r;
                    }
                }
            }
        }
        if (staged) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            const int n = min(FILL_STAGE, n_run - win0);
            for (int i = lane; i < n; i += 64) {
                col_idx[seg + run0 + win0 + i] = sCol[wv][i];
                pair_pos[seg + run0 + win0 + i] = sPos[wv][i];
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        }
    }
}

size_t score_lds_bytes(int nb, int D) {
    return (size_t)nb * D * 4 + (size_t)QT * (nb | 1) * 4 + HIST_BINS * 4 + HIST_BINS * 8;
}

// The score kernels use more dynamic LDS than the default limit: raise a kernel's limit to the whole 160 KB of a
// compute unit, once per kernel (slot) and device.
int allow_full_lds(const void* kernel, int slot) {
    static std::mutex mu;
    static bool done[40][64] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return VMOBA_ERR_HIP;
    std::lock_guard<std::mutex> lock(mu);
    if (!done[slot][dev]) {
        if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) return VMOBA_ERR_HIP;
        done[slot][dev] = true;
    }
    return VMOBA_OK;
}

int fix_shift_for(int64_t S) {
    int bits = 0;
    while (((int64_t)1 << bits) < S) ++bits;
    return 61 - bits;
}

}  // namespace

size_t vmoba_select_workspace_bytes(int B, int Hh, int64_t S, int nb) {
    return carve(nullptr, B * Hh, S, nb).total;
}

namespace {

// Host-side validation shared by the two entry points; everything that can be rejected without touching the device.
int select_args_ok(int B, int Hh, int64_t S, int D, int32_t n_blocks, const int32_t* blk_off, const vmoba_tensor* Qp,
                   const vmoba_tensor* Kp, float tau, float score_scale, int mode, int32_t topk, const float* Bmean,
                   const float* P, const uint32_t* mask, const int32_t* blk_ptr, const int32_t* q_idx,
                   const int32_t* row_ptr, const int32_t* col_idx, const int32_t* pair_pos, int64_t nnz_capacity,
                   const int64_t* k_out, const float* theta_out, const int32_t* dev_status) {
    if (B <= 0 || Hh <= 0 || S <= 0 || n_blocks <= 0 || nnz_capacity <= 0) return VMOBA_ERR_INVALID_ARG;
    if (!blk_off || !Bmean || !P || !mask || !blk_ptr || !q_idx || !row_ptr || !col_idx || !pair_pos ||
        !k_out || !theta_out || !dev_status)
        return VMOBA_ERR_INVALID_ARG;
    if (!tensor_ok(Qp) || !tensor_ok(Kp)) return VMOBA_ERR_INVALID_ARG;
    if (!std::isfinite(score_scale)) return VMOBA_ERR_INVALID_ARG;
    mode &= ~VMOBA_SELECT_OWN_BLOCK;
    if (mode < VMOBA_GLOBAL_THRESHOLD || mode > VMOBA_POOL_SOFTMAX_THRESHOLD) return VMOBA_ERR_UNSUPPORTED;
    const bool uses_tau = mode == VMOBA_GLOBAL_THRESHOLD || mode == VMOBA_LOCAL_THRESHOLD || mode == VMOBA_POOL_SOFTMAX_THRESHOLD;
    if (uses_tau && (!(tau > 0.f) || !(tau <= 1.f))) return VMOBA_ERR_INVALID_ARG;
    if (!uses_tau && topk < 1) return VMOBA_ERR_INVALID_ARG;
    if (D != 64 && D != 128) return VMOBA_ERR_UNSUPPORTED;
    if (Qp->dtype != Kp->dtype) return VMOBA_ERR_UNSUPPORTED;
    if (n_blocks > VMOBA_MAX_BLOCKS || S > ((int64_t)1 << 30) || S * n_blocks > (int64_t)INT32_MAX)
        return VMOBA_ERR_UNSUPPORTED;
    return VMOBA_OK;
}

// The selection itself; `workspace` is the caller's buffer (vmoba_select) or the library's static one.
int select_impl(int B, int Hh, int64_t S, int D, int32_t n_blocks, const int32_t* blk_off,
                const vmoba_tensor* Qp, const vmoba_tensor* Kp, float tau, float score_scale,
                int mode, int32_t topk, float* Bmean, float* P, uint32_t* mask, int32_t* blk_ptr,
                int32_t* q_idx, int32_t* row_ptr, int32_t* col_idx, int32_t* pair_pos,
                int64_t nnz_capacity, int64_t* k_out, float* theta_out, int32_t* dev_status,
                const int32_t* query_pos, const int32_t* kv_rows, void* workspace, size_t workspace_bytes, void* stream) {
    {
        const int rc = select_args_ok(B, Hh, S, D, n_blocks, blk_off, Qp, Kp, tau, score_scale, mode, topk, Bmean, P, mask,
                                      blk_ptr, q_idx, row_ptr, col_idx, pair_pos, nnz_capacity, k_out, theta_out, dev_status);
        if (rc != VMOBA_OK) return rc;
    }
    if (!workspace) return VMOBA_ERR_INVALID_ARG;
    const bool own_block = (mode & VMOBA_SELECT_OWN_BLOCK) != 0;
    mode &= ~VMOBA_SELECT_OWN_BLOCK;
    const int* own_off = own_block ? blk_off : nullptr;
    const bool pool_softmax = mode == VMOBA_POOL_SOFTMAX_THRESHOLD;
    const bool bf16 = Qp->dtype == VMOBA_BF16;
    // LDS of the score kernel this call launches: bfloat16 queries go to the matrix-core kernel (block means as three
    // bfloat16 terms up to 128 blocks, as float32 beyond), float32 queries to the plain FMA kernel
    constexpr int SCORE_CHUNK = 256;                        // blocks per launch of the score kernel beyond 256 blocks
    const bool chunked = bf16 && n_blocks > SCORE_CHUNK;
    const int nb_pad = chunked ? SCORE_CHUNK : ((n_blocks + 31) & ~31);
    // three bf16 terms of the means in LDS while they fit beside one copy of the histogram words and the accumulators fit
    // the registers (D = 128: up to 189 blocks; D = 64: 192), else the means as float32, split after every fetch
    const size_t lds_terms = (size_t)3 * (nb_pad > 128 ? n_blocks + 1 : nb_pad) * (D + 8) * 2;
    const bool fly = nb_pad > 192 || lds_terms + (size_t)HIST_BINS * 8 > 160 * 1024;
    const size_t lds_means = fly ? (size_t)nb_pad * (D + 4) * 4 : lds_terms;
    // the first radix level of the matrix-core kernel keeps up to 8 replicas of its 8 KB of histogram words, as many as fit
    int copy_shift = 3;
    while (copy_shift > 0 && lds_means + ((size_t)HIST_BINS * 8 << copy_shift) > 160 * 1024) --copy_shift;
    const size_t lds_mfma = lds_means + ((size_t)HIST_BINS * 8 << copy_shift);
    const size_t lds = bf16 ? lds_mfma : score_lds_bytes(n_blocks, D);
    if (lds > 160 * 1024) return VMOBA_ERR_UNSUPPORTED;
    const int BH = B * Hh;
    SelectWs ws = carve(workspace, BH, S, n_blocks);
    if (workspace_bytes < ws.total) return VMOBA_ERR_WORKSPACE;
    if (ws.zero_bytes / 4 > (size_t)UINT32_MAX) return VMOBA_ERR_UNSUPPORTED;       // more than 10^5 heads in one call
    if (((uintptr_t)workspace) & 255) return VMOBA_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    const int n_waves = (int)ceil_div64(S, 64);
    const long long pool = (long long)S * n_blocks;
    // the pool sums to S (row soft-max) or to 1 (pool soft-max); the fixed-point scale leaves headroom for either
    const int fix_shift = pool_softmax ? fix_shift_for(2) : fix_shift_for(S);
    const double pool_total = pool_softmax ? 1.0 : (double)S;
    // target of the head-global cut: mass tau * S in fixed point (rounded up; tau >= 1 asks for more than the
    // pool can hold), or, for a fixed global k, the number of pairs topk * S
    unsigned long long target;
    if (mode == VMOBA_GLOBAL_TOPK) {
        target = (unsigned long long)std::min<long long>((long long)topk * S, pool);
    } else if (tau >= 1.f) {
        target = ~0ull;
    } else {
        target = (unsigned long long)std::ceil((double)tau * pool_total * (double)(1ull << fix_shift));
        if (target == 0) target = 1;
    }
    const TensorView Qv = make_view(Qp), Kv = make_view(Kp);

    // the block-mean kernel also clears the leading words of the workspace (histograms, head state)
#define LAUNCH_MEAN(BF, DD) block_mean_kernel<BF, DD><<<dim3(n_blocks, BH), dim3(256), 0, st>>>(Kv, blk_off, Bmean, Hh, n_blocks, kv_rows, (unsigned int*)workspace, (unsigned int)(ws.zero_bytes / 4))
    if (bf16 && D == 128) LAUNCH_MEAN(true, 128);
    else if (bf16 && D == 64) LAUNCH_MEAN(true, 64);
    else if (D == 128) LAUNCH_MEAN(false, 128);
    else LAUNCH_MEAN(false, 64);
#undef LAUNCH_MEAN
    VMOBA_CHECK_LAUNCH();

    float2* row_stat = pool_softmax ? ws.row_stat : nullptr;
    // pool soft-max: the radix levels run over the pool-normalised values, which only exist after the row statistics
    unsigned int* score_hist = pool_softmax ? nullptr : ws.hist_cnt;
    const int n_tiles = (int)ceil_div64(S, QT);
    const int tiles_per_wg = 4;
    dim3 sgrid((unsigned)ceil_div64(n_tiles, tiles_per_wg), (unsigned)BH);
#define LAUNCH_SCORE(DD)                                                                                  \
    do {                                                                                                  \
        auto kfn = score_kernel<DD>;                                                                      \
        if (allow_full_lds((const void*)kfn, DD == 128 ? 0 : 1) != VMOBA_OK) return VMOBA_ERR_HIP;        \
        kfn<<<sgrid, dim3(256), lds, st>>>(Qv, Bmean, P, score_hist, ws.hist_sum, Hh, (int)S, n_blocks,   \
                                           score_scale, fix_shift, row_stat);                             \
    } while (0)
    if (bf16) {
        // one workgroup per compute unit (the LDS holds one), each with an equal share of all (head, query tile) pairs
        dim3 mgrid((unsigned)std::min<int64_t>((int64_t)BH * ceil_div64(S, SCORE_QT), vmoba_num_cus()));
#define LAUNCH_SCORE_MFMA_T(DD, FL, RW, NM, TRV, NBC, JB0)                                                \
    do {                                                                                                  \
        auto kfn = score_mfma_kernel<DD, FL, RW, NM, TRV>;                                                \
        if (allow_full_lds((const void*)kfn, 2 + (TRV ? 0 : 16) + (DD == 128 ? 0 : 8) + (RW ? 7 : FL ? 6 : NM - 1)) != VMOBA_OK) return VMOBA_ERR_HIP; \
        kfn<<<mgrid, dim3(SCORE_NT), lds, st>>>(Qv, Bmean, P, score_hist, ws.hist_sum, BH, Hh, (int)S, NBC, n_blocks, JB0, \
                                                score_scale, fix_shift, copy_shift, row_stat);            \
    } while (0)
        // rows of P that start 16-byte aligned take the kernel with the query on the lane, others the one with the block there
#define LAUNCH_SCORE_MFMA(DD, FL, RW, NM, NBC, JB0)                                                       \
    do {                                                                                                  \
        /* (193..256 blocks in one launch: eight accumulator tiles leave no registers for the reduction's row values) */ \
        if ((n_blocks & 3) == 0 || (FL && !RW)) LAUNCH_SCORE_MFMA_T(DD, FL, RW, NM, true, NBC, JB0);      \
        else LAUNCH_SCORE_MFMA_T(DD, FL, RW, NM, false, NBC, JB0);                                        \
    } while (0)
        // the bf16 terms fit: one instantiation per number of 32-block tiles
#define LAUNCH_SCORE_TILES(DD)                                                                            \
    do {                                                                                                  \
        switch ((n_blocks + 31) / 32) {                                                                   \
            case 1: LAUNCH_SCORE_MFMA(DD, false, false, 1, n_blocks, 0); break;                           \
            case 2: LAUNCH_SCORE_MFMA(DD, false, false, 2, n_blocks, 0); break;                           \
            case 3: LAUNCH_SCORE_MFMA(DD, false, false, 3, n_blocks, 0); break;                           \
            case 4: LAUNCH_SCORE_MFMA(DD, false, false, 4, n_blocks, 0); break;                           \
            case 5: LAUNCH_SCORE_MFMA(DD, false, false, 5, n_blocks, 0); break;                           \
            default: LAUNCH_SCORE_MFMA(DD, false, false, 6, n_blocks, 0); break;                          \
        }                                                                                                 \
    } while (0)
        if (chunked) {
            // more than 256 blocks: scaled scores chunk by chunk, then the soft-max of the rows and the first radix level
            for (int jb0 = 0; jb0 < n_blocks; jb0 += SCORE_CHUNK) {
                const int nbc = std::min(SCORE_CHUNK, n_blocks - jb0);
                if (D == 128) LAUNCH_SCORE_MFMA(128, true, true, 0, nbc, jb0);
                else LAUNCH_SCORE_MFMA(64, true, true, 0, nbc, jb0);
                VMOBA_CHECK_LAUNCH();
            }
            softmax_rows_kernel<<<dim3((unsigned)std::min<int64_t>(ceil_div64(S, 4 * 8), 2048), (unsigned)BH), dim3(256), 0, st>>>(
                P, score_hist, ws.hist_sum, (int)S, n_blocks, fix_shift, row_stat);
        } else if (D == 128 && fly) LAUNCH_SCORE_MFMA(128, true, false, 0, n_blocks, 0);
        else if (D == 128) LAUNCH_SCORE_TILES(128);
        else if (fly) LAUNCH_SCORE_MFMA(64, true, false, 0, n_blocks, 0);
        else LAUNCH_SCORE_TILES(64);
#undef LAUNCH_SCORE_TILES
#undef LAUNCH_SCORE_MFMA
#undef LAUNCH_SCORE_MFMA_T
    } else if (D == 128) LAUNCH_SCORE(128);
    else LAUNCH_SCORE(64);
#undef LAUNCH_SCORE
    VMOBA_CHECK_LAUNCH();
    if (pool_softmax) {
        // the score kernel took no histogram in this mode: the first radix level is taken over G here
        pool_stat_kernel<<<dim3(BH), dim3(1024), 0, st>>>(ws.row_stat, ws.pool_stat, (int)S);
        VMOBA_CHECK_LAUNCH();
        pool_rescale_kernel<<<dim3((unsigned)std::min<int64_t>(ceil_div64(S, 4 * 8), 1024), (unsigned)BH), dim3(256), 0, st>>>(
            P, ws.row_stat, ws.pool_stat, ws.hist_cnt, ws.hist_sum, (int)S, n_blocks, fix_shift);
        VMOBA_CHECK_LAUNCH();
    }

    unsigned int* hc1 = ws.hist_cnt + (size_t)BH * HIST_BINS;
    unsigned int* hc2 = ws.hist_cnt + (size_t)2 * BH * HIST_BINS;
    unsigned long long* hs1 = ws.hist_sum + (size_t)BH * HIST_BINS;
    unsigned long long* hs2 = ws.hist_sum + (size_t)2 * BH * HIST_BINS;
    // at most 2^20 entries per workgroup (the packed histogram words), else as many workgroups as compute units
    const unsigned refine_gx = (unsigned)std::max<int64_t>(std::max<int64_t>(1, vmoba_num_cus() / BH), ceil_div64(pool, (int64_t)1 << 20));

    const unsigned wave_gx = (unsigned)ceil_div64(n_waves, 4);
    const bool local = mode == VMOBA_LOCAL_TOPK || mode == VMOBA_LOCAL_THRESHOLD;
    if (local) {
        if (mode == VMOBA_LOCAL_TOPK)
            local_mask_kernel<true><<<dim3(wave_gx, BH), dim3(256), 0, st>>>(P, mask, ws.wtot, ws.wcnt, (int)S, n_blocks, n_waves, topk, tau, own_off, query_pos);
        else
            local_mask_kernel<false><<<dim3(wave_gx, BH), dim3(256), 0, st>>>(P, mask, ws.wtot, ws.wcnt, (int)S, n_blocks, n_waves, topk, tau, own_off, query_pos);
        VMOBA_CHECK_LAUNCH();
    } else {
#define SCAN_LEVEL(LV, HC, HS)                                                                                        \
    do {                                                                                                              \
        if (mode == VMOBA_GLOBAL_TOPK)                                                                                \
            scan_level_kernel<LV, true><<<dim3(BH), dim3(HIST_BINS), 0, st>>>(HC, HS, ws.state, target, fix_shift, pool, (long long*)k_out, theta_out); \
        else                                                                                                          \
            scan_level_kernel<LV, false><<<dim3(BH), dim3(HIST_BINS), 0, st>>>(HC, HS, ws.state, target, fix_shift, pool, (long long*)k_out, theta_out); \
    } while (0)
        SCAN_LEVEL(0, ws.hist_cnt, ws.hist_sum);
        VMOBA_CHECK_LAUNCH();
        refine_hist_kernel<1><<<dim3(refine_gx, BH), dim3(REFINE_NT), 0, st>>>(P, ws.state, hc1, hs1, pool, fix_shift);
        VMOBA_CHECK_LAUNCH();
        SCAN_LEVEL(1, hc1, hs1);
        VMOBA_CHECK_LAUNCH();
        refine_hist_kernel<2><<<dim3(refine_gx, BH), dim3(REFINE_NT), 0, st>>>(P, ws.state, hc2, hs2, pool, fix_shift);
        VMOBA_CHECK_LAUNCH();
        SCAN_LEVEL(2, hc2, hs2);
        VMOBA_CHECK_LAUNCH();
#undef SCAN_LEVEL
        const unsigned row_gx = (unsigned)std::min<int64_t>(ceil_div64(S, 4 * 8), 4096);
        tie_count_kernel<<<dim3(row_gx, BH), dim3(256), 0, st>>>(P, ws.state, ws.ties, (int)S, n_blocks);
        VMOBA_CHECK_LAUNCH();
        row_scan_kernel<<<dim3(BH), dim3(SCAN_THREADS), 0, st>>>(ws.ties, ws.tie_base, ws.state, 1, (int)S);
        VMOBA_CHECK_LAUNCH();
        mask_kernel<<<dim3(wave_gx, BH), dim3(256), 0, st>>>(P, ws.state, ws.tie_base, mask, ws.wtot, ws.wcnt,
                                                            (int)S, n_blocks, n_waves, own_off, query_pos);
        VMOBA_CHECK_LAUNCH();
    }
    wave_scan_kernel<<<dim3(n_blocks + 1, BH), dim3(256), 0, st>>>(ws.wcnt, ws.wtot, ws.row_tot, n_blocks, n_waves);
    VMOBA_CHECK_LAUNCH();
    blk_ptr_kernel<<<dim3(BH), dim3(64), 0, st>>>(ws.row_tot, blk_ptr, row_ptr, (long long*)k_out, theta_out, n_blocks, (int)S,
                                                 (long long)nnz_capacity, dev_status, local ? 2 : (own_off ? 1 : 0));
    VMOBA_CHECK_LAUNCH();
    fill_lists_kernel<<<dim3(wave_gx, BH), dim3(256), 0, st>>>(mask, row_ptr, ws.wtot, blk_ptr, ws.wcnt, q_idx, col_idx,
                                                              pair_pos, (int)S, n_blocks, n_waves,
                                                              (long long)nnz_capacity);
    VMOBA_CHECK_LAUNCH();
    return VMOBA_OK;
}

}  // namespace

extern "C" int vmoba_select(int B, int Hh, int64_t S, int D, int32_t n_blocks, const int32_t* blk_off,
                            const vmoba_tensor* Qp, const vmoba_tensor* Kp, float tau, float score_scale,
                            int mode, int32_t topk, float* Bmean, float* P, uint32_t* mask, int32_t* blk_ptr,
                            int32_t* q_idx, int32_t* row_ptr, int32_t* col_idx, int32_t* pair_pos,
                            int64_t nnz_capacity, int64_t* k_out, float* theta_out, int32_t* dev_status,
                            const int32_t* query_pos, const int32_t* kv_rows, void* workspace, size_t workspace_bytes, void* stream) {
    return select_impl(B, Hh, S, D, n_blocks, blk_off, Qp, Kp, tau, score_scale, mode, topk, Bmean, P, mask, blk_ptr, q_idx,
                       row_ptr, col_idx, pair_pos, nnz_capacity, k_out, theta_out, dev_status, query_pos, kv_rows, workspace,
                       workspace_bytes, stream);
}

// ---------------------------------------------------------------------------------------------
// vmoba_select_static: vmoba_select for callers that cannot allocate.  Its scratch memory (histograms, head state,
// tie ranks, row and block counts) is a file-scope device array instead of a caller-provided workspace.  In host code
// the array's name is only a handle for the runtime: the device address is looked up once per device with
// hipGetSymbolAddress and that pointer is what the kernels get, exactly as they get the caller's workspace above.
static __device__ __align__(256) unsigned char scratch[VMOBA_SELECT_STATIC_MAX_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[MAX_DEVICES] = {};          // device address of `scratch` on each device, null until first use

int static_scratch_of_current_device(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return VMOBA_ERR_HIP;
    if (dev < 0 || dev >= MAX_DEVICES) return VMOBA_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return VMOBA_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return VMOBA_OK;
}

}  // namespace

extern "C" int vmoba_select_static(int B, int Hh, int64_t S, int D, int32_t n_blocks, const int32_t* blk_off,
                                   const vmoba_tensor* Qp, const vmoba_tensor* Kp, float tau, float score_scale,
                                   int mode, int32_t topk, float* Bmean, float* P, uint32_t* mask, int32_t* blk_ptr,
                                   int32_t* q_idx, int32_t* row_ptr, int32_t* col_idx, int32_t* pair_pos,
                                   int64_t nnz_capacity, int64_t* k_out, float* theta_out, int32_t* dev_status,
                                   const int32_t* query_pos, const int32_t* kv_rows, void* stream) {
    // everything that can be rejected on the host first, the size limit included
    const int rc = select_args_ok(B, Hh, S, D, n_blocks, blk_off, Qp, Kp, tau, score_scale, mode, topk, Bmean, P, mask,
                                  blk_ptr, q_idx, row_ptr, col_idx, pair_pos, nnz_capacity, k_out, theta_out, dev_status);
    if (rc != VMOBA_OK) return rc;
    if ((int64_t)B * Hh > (1 << 20)) return VMOBA_ERR_WORKSPACE;
    if (carve(nullptr, B * Hh, S, n_blocks).total > VMOBA_SELECT_STATIC_MAX_BYTES) return VMOBA_ERR_WORKSPACE;
    void* ws = nullptr;
    const int rs = static_scratch_of_current_device(&ws);
    if (rs != VMOBA_OK) return rs;
    return select_impl(B, Hh, S, D, n_blocks, blk_off, Qp, Kp, tau, score_scale, mode, topk, Bmean, P, mask, blk_ptr, q_idx,
                       row_ptr, col_idx, pair_pos, nnz_capacity, k_out, theta_out, dev_status, query_pos, kv_rows, ws,
                       VMOBA_SELECT_STATIC_MAX_BYTES, stream);
}
