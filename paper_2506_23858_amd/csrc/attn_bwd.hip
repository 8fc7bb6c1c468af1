// vmoba_attn_bwd: gradient of the block-sparse attention of Sec. 3.1 Step 3 with the selection
// held fixed.  With A the attention weights over the selected keys:
//   delta = rowsum(dO * O),  dV = A^T dO,  dP = dO V^T,  dS = A * (dP - delta),
//   dQ = scale * dS K,       dK = scale * dS^T Q.
//
// Three phases.  (1) delta kernel.  (2) dQ: the forward's decomposition (tile of gathered
// queries x one key block), one partial dQ per (query, block) pair, summed query-major by a
// merge kernel.  (3) dK/dV: a workgroup owns a run of keys of one block and walks the whole
// query list of that block, so dK and dV of its keys stay in registers and are written once --
// no atomics anywhere, results are reproducible.  The attention weights are recomputed from
// Q, K and the forward's LSE in both (2) and (3).
#include "attn_common.h"
#include <type_traits>

#include <algorithm>
#include <cmath>

int64_t vmoba_max_tiles(int64_t cap, int TM);

namespace {

constexpr float LOG2E = 1.4426950408889634f;

// ---------------------------------------------------------------------------------------------
template <bool BF16, int D>
__global__ __launch_bounds__(256) void delta_kernel(TensorView O, TensorView dO, float* __restrict__ delta,
                                                    const int* __restrict__ rows, char* __restrict__ dO_copy, int Hh, int S) {
    constexpr int EPP = BF16 ? 8 : 4;
    constexpr int LPQ = D / EPP;
    constexpr int QPW = 256 / LPQ;
    const int bh = blockIdx.y, b = bh / Hh, h = bh % Hh;
    const int q = blockIdx.x * QPW + threadIdx.x / LPQ;
    const int part = threadIdx.x % LPQ;
    float acc = 0.f;
    if (q < S) {
        // with a row map, O and dO are in the caller's token order and dO is also copied to block order
        const int qs = rows ? rows[q] : q;
        const char* po = O.ptr + ((long long)b * O.stride_b + (long long)qs * O.stride_s + (long long)h * O.stride_h) * (BF16 ? 2 : 4) + part * 16;
        const char* pd = dO.ptr + ((long long)b * dO.stride_b + (long long)qs * dO.stride_s + (long long)h * dO.stride_h) * (BF16 ? 2 : 4) + part * 16;
        const u32x4_t a = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(po));
        const u32x4_t c = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(pd));
        if (rows) *reinterpret_cast<u32x4_t*>(dO_copy + ((long long)bh * S + q) * D * (BF16 ? 2 : 4) + part * 16) = c;
        if constexpr (BF16) {
            acc = bf16lo_to_f32(a.x) * bf16lo_to_f32(c.x) + bf16hi_to_f32(a.x) * bf16hi_to_f32(c.x) +
                  bf16lo_to_f32(a.y) * bf16lo_to_f32(c.y) + bf16hi_to_f32(a.y) * bf16hi_to_f32(c.y) +
                  bf16lo_to_f32(a.z) * bf16lo_to_f32(c.z) + bf16hi_to_f32(a.z) * bf16hi_to_f32(c.z) +
                  bf16lo_to_f32(a.w) * bf16lo_to_f32(c.w) + bf16hi_to_f32(a.w) * bf16hi_to_f32(c.w);
        } else {
            acc = __uint_as_float(a.x) * __uint_as_float(c.x) + __uint_as_float(a.y) * __uint_as_float(c.y) +
                  __uint_as_float(a.z) * __uint_as_float(c.z) + __uint_as_float(a.w) * __uint_as_float(c.w);
        }
    }
#pragma unroll
    for (int off = LPQ / 2; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (q < S && part == 0) delta[(long long)bh * S + q] = acc;
}

// Key-run table of one head.  A "run" is KPW consecutive keys of one block, the share of one dK/dV
// workgroup, and costs time in proportion to the length of the block's query list.  Workgroups are
// dispatched in index order, so the blocks are numbered longest list first (a longest-processing-time
// order: the short ones fill the tail of the launch): kb_order[r] = block at rank r,
// kb_start[r] = number of runs of the blocks at ranks 0..r-1.  One workgroup per head.
// A last run of at most tail_max keys is not counted: the tail kernel takes those keys.
__global__ __launch_bounds__(VMOBA_MAX_BLOCKS) void key_run_order_kernel(const int* __restrict__ blk_off, const int* __restrict__ blk_ptr,
                                                                         int* __restrict__ kb_start, int* __restrict__ kb_order, int nb,
                                                                         int KPW, int tail_max) {
    __shared__ int sCnt[VMOBA_MAX_BLOCKS];
    __shared__ int sRuns[VMOBA_MAX_BLOCKS];
    const int bh = blockIdx.x, j = threadIdx.x;          // one thread per block
    const int* bp = blk_ptr + (long long)bh * (nb + 1);
    const int cnt = j < nb ? bp[j + 1] - bp[j] : -1;
    if (j < nb) sCnt[j] = cnt;
    __syncthreads();
    if (j < nb) {
        int rank = 0;
        for (int i = 0; i < nb; ++i) rank += (sCnt[i] > cnt || (sCnt[i] == cnt && i < j)) ? 1 : 0;
        kb_order[(long long)bh * nb + rank] = j;
        const int L = blk_off[j + 1] - blk_off[j];
        const int tail = L % KPW;
        sRuns[rank] = (tail > 0 && tail <= tail_max) ? L / KPW : (L + KPW - 1) / KPW;
    }
    __syncthreads();
    if (j == 0) {
        int run = 0;
        for (int r = 0; r < nb; ++r) {
            kb_start[(long long)bh * (nb + 1) + r] = run;
            run += sRuns[r];
        }
        kb_start[(long long)bh * (nb + 1) + nb] = run;
    }
}

__device__ __forceinline__ float load_elem(const char* p, int d) { return reinterpret_cast<const float*>(p)[d]; }

// ---------------------------------------------------------------------------------------------
// Plain FMA dQ tile kernel (float32 tensors): one wavefront per 64 gathered queries of one key block, lane = query.
template <int D>
__global__ __launch_bounds__(64) void attn_bwd_dq_simple_kernel(
    TensorView Q, TensorView K, TensorView V, TensorView dO, const float* __restrict__ LSE, const float* __restrict__ delta,
    const int* __restrict__ blk_off, const int* __restrict__ blk_ptr, const int* __restrict__ q_idx,
    const int4* __restrict__ tile_desc, int tiles_per_head, float* __restrict__ dQpart, int Hh, int S, int nb, long long cap, float scale_log2,
    const int* __restrict__ kv_rows) {
    constexpr int KC = 32;
    constexpr int ES = 4;
    __shared__ float sK[KC][D];
    __shared__ float sV[KC][D];
    const int bh = blockIdx.y, b = bh / Hh, h = bh % Hh;
    TileCoord tc;
    if (!find_tile(tile_desc, tiles_per_head, bh, blockIdx.x, tc)) return;
    const int lane = threadIdx.x;
    const long long seg = (long long)bh * cap;
    const int e = min(lane, tc.count - 1);
    const int q = q_idx[seg + tc.list0 + tc.t0 + e];
    float qr[D], dor[D], dq[D];
    {
        const char* sq = Q.ptr + ((long long)b * Q.stride_b + (long long)q * Q.stride_s + (long long)h * Q.stride_h) * ES;
        const char* sd = dO.ptr + ((long long)b * dO.stride_b + (long long)q * dO.stride_s + (long long)h * dO.stride_h) * ES;
#pragma unroll
        for (int d = 0; d < D; ++d) {
            qr[d] = load_elem(sq, d);
            dor[d] = load_elem(sd, d);
            dq[d] = 0.f;
        }
    }
    const float lse2 = LSE[(long long)bh * S + q] * LOG2E;
    const float dl = delta[(long long)bh * S + q];
    const char* kbase = K.ptr + ((long long)b * K.stride_b + (long long)h * K.stride_h) * ES;
    const char* vbase = V.ptr + ((long long)b * V.stride_b + (long long)h * V.stride_h) * ES;
    for (int c0 = 0; c0 < tc.L; c0 += KC) {
        const int kc = min(KC, tc.L - c0);
        __syncthreads();
        for (int i = lane; i < kc * D; i += 64) {
            const int r = i / D, d = i % D;
            const int pos = tc.k0 + c0 + r;
            const long long row = kv_rows ? kv_rows[pos] : pos;       // key position -> row of K and V
            sK[r][d] = load_elem(kbase + row * K.stride_s * ES, d);
            sV[r][d] = load_elem(vbase + row * V.stride_s * ES, d);
        }
        __syncthreads();
        for (int r = 0; r < kc; ++r) {
            float s = 0.f, dp = 0.f;
#pragma unroll
            for (int d = 0; d < D; ++d) {
                s = fmaf(qr[d], sK[r][d], s);
                dp = fmaf(dor[d], sV[r][d], dp);
            }
            const float p = exp2f(s * scale_log2 - lse2);
            const float ds = p * (dp - dl);
#pragma unroll
            for (int d = 0; d < D; ++d) dq[d] = fmaf(ds, sK[r][d], dq[d]);
        }
    }
    if (lane < tc.count) {
        float* dst = dQpart + (seg + tc.list0 + tc.t0 + lane) * D;
#pragma unroll
        for (int d = 0; d < D; ++d) dst[d] = dq[d];
    }
}

// Plain FMA dK/dV kernel (float32 tensors): one wavefront per run of 64 keys of one block, lane = key;
// walks the block's whole query list through LDS.
template <int D>
__global__ __launch_bounds__(64) void attn_bwd_dkv_simple_kernel(
    TensorView Q, TensorView K, TensorView V, TensorView dO, const float* __restrict__ LSE, const float* __restrict__ delta,
    const int* __restrict__ blk_off, const int* __restrict__ blk_ptr, const int* __restrict__ q_idx,
    const int* __restrict__ kb_start, const int* __restrict__ kb_order, TensorView dK, TensorView dV, const int* __restrict__ rows, int Hh, int S, int nb, long long cap,
    float scale_log2, float scale, const int* __restrict__ kv_rows) {
    constexpr int KPW = 64, QC = 16;
    constexpr int ES = 4;
    __shared__ float sQ[QC][D];
    __shared__ float sdO[QC][D];
    __shared__ float sL[QC], sDl[QC];
    const int bh = blockIdx.y, b = bh / Hh, h = bh % Hh;
    const int* ks = kb_start + (long long)bh * (nb + 1);
    if ((int)blockIdx.x >= ks[nb]) return;
    int lo = 0, hi = nb;
    while (hi - lo > 1) { int mid = (lo + hi) >> 1; if (ks[mid] <= (int)blockIdx.x) lo = mid; else hi = mid; }
    const int j = kb_order[(long long)bh * nb + lo];
    const int k0 = blk_off[j], L = blk_off[j + 1] - k0;
    const int kk0 = ((int)blockIdx.x - ks[lo]) * KPW;            // first key of this run inside the block
    const int lane = threadIdx.x;
    const bool live = kk0 + lane < L;
    const int krow = k0 + min(kk0 + lane, L - 1);
    const long long seg = (long long)bh * cap;
    const int list0 = blk_ptr[(long long)bh * (nb + 1) + j];
    const int cnt = blk_ptr[(long long)bh * (nb + 1) + j + 1] - list0;
    float kr[D], vr[D], dk[D], dv[D];
    {
        const long long kin = kv_rows ? kv_rows[krow] : krow;         // row of K and V that holds this key
        const char* sk = K.ptr + ((long long)b * K.stride_b + kin * K.stride_s + (long long)h * K.stride_h) * ES;
        const char* sv = V.ptr + ((long long)b * V.stride_b + kin * V.stride_s + (long long)h * V.stride_h) * ES;
#pragma unroll
        for (int d = 0; d < D; ++d) {
            kr[d] = load_elem(sk, d);
            vr[d] = load_elem(sv, d);
            dk[d] = 0.f;
            dv[d] = 0.f;
        }
    }
    const char* qbase = Q.ptr + ((long long)b * Q.stride_b + (long long)h * Q.stride_h) * ES;
    const char* dobase = dO.ptr + ((long long)b * dO.stride_b + (long long)h * dO.stride_h) * ES;
    for (int c0 = 0; c0 < cnt; c0 += QC) {
        const int qc = min(QC, cnt - c0);
        __syncthreads();
        for (int i = lane; i < qc * D; i += 64) {
            const int r = i / D, d = i % D;
            const long long q = q_idx[seg + list0 + c0 + r];
            sQ[r][d] = load_elem(qbase + q * Q.stride_s * ES, d);
            sdO[r][d] = load_elem(dobase + q * dO.stride_s * ES, d);
        }
        if (lane < qc) {
            const long long q = q_idx[seg + list0 + c0 + lane];
            sL[lane] = LSE[(long long)bh * S + q] * LOG2E;
            sDl[lane] = delta[(long long)bh * S + q];
        }
        __syncthreads();
        for (int r = 0; r < qc; ++r) {
            float s = 0.f, dp = 0.f;
#pragma unroll
            for (int d = 0; d < D; ++d) {
                s = fmaf(sQ[r][d], kr[d], s);
                dp = fmaf(sdO[r][d], vr[d], dp);
            }
            const float p = exp2f(s * scale_log2 - sL[r]);
            const float ds = p * (dp - sDl[r]);
#pragma unroll
            for (int d = 0; d < D; ++d) {
                dv[d] = fmaf(p, sdO[r][d], dv[d]);
                dk[d] = fmaf(ds, sQ[r][d], dk[d]);
            }
        }
    }
    if (live) {
        const int kout = rows ? rows[krow] : krow;
        char* pk = dK.ptr + ((long long)b * dK.stride_b + (long long)kout * dK.stride_s + (long long)h * dK.stride_h) * ES;
        char* pv = dV.ptr + ((long long)b * dV.stride_b + (long long)kout * dV.stride_s + (long long)h * dV.stride_h) * ES;
#pragma unroll
        for (int d = 0; d < D; ++d) {
            reinterpret_cast<float*>(pk)[d] = dk[d] * scale;
            reinterpret_cast<float*>(pv)[d] = dv[d];
        }
    }
}

// Load through a wave-uniform base and a 32-bit byte offset per lane (the address needs no 64-bit vector arithmetic).
template <typename T>
__device__ __forceinline__ T load_at(const void* base, uint32_t byte_off) {
    return *reinterpret_cast<const T*>(reinterpret_cast<const char*>(base) + byte_off);
}

// ---------------------------------------------------------------------------------------------
// bf16 MFMA dQ tile kernel.  Same decomposition and operand orientation as the forward tile
// kernel (query = MFMA column = lane % 32); 4 wavefronts x 32 gathered queries, key chunks of 64:
//   S^T  = K . Q^T                    A = K rows (LDS),  B = Q^T (registers)
//   dP^T = V . dO^T                   A = V rows (LDS),  B = dO^T (registers)
//   dS^T = P^T * (dP^T - delta)       in registers, packed to bf16 as the next B operand
//   dQ^T += K^T . dS^T                A = K^T by transpose reads of the same K tile
template <int D>
__global__ __launch_bounds__(256, 2) void attn_bwd_dq_mfma_kernel(
    TensorView Q, TensorView K, TensorView V, TensorView dO, const float* __restrict__ LSE, const float* __restrict__ delta,
    const int* __restrict__ blk_off, const int* __restrict__ blk_ptr, const int* __restrict__ q_idx,
    const int4* __restrict__ flat_desc, const int* __restrict__ head_base, int BH, float* __restrict__ dQpart, int Hh, int S, int nb,
    long long cap, float scale_log2, const int* __restrict__ kv_rows) {
    constexpr int TM = 128, KC = 64;
    constexpr int STR = D + 8;
    constexpr int KSTEPS = D / 16, DT = D / 32;
    constexpr int LOADS = KC * D * 2 / 16 / 256;
    __shared__ __align__(1024) char sKV[2 * KC * STR * 2];                     // the K tile, then the V tile
    __bf16* const sK = reinterpret_cast<__bf16*>(sKV);
    __bf16* const sV = reinterpret_cast<__bf16*>(sKV + KC * STR * 2);
    // a wavefront's 32 partial rows on their way out: written as the accumulators hold them, read back as whole rows
    constexpr int OPITCH = D * 2 + 16;
    __shared__ __align__(1024) char sOut[4 * 32 * OPITCH];
    static_assert(4 * 32 * D * 2 <= 2 * KC * STR * 2, "the gathered Q rows of the four wavefronts fit the K/V tiles");

    // One workgroup per tile of the flat list (all heads).  Workgroup ids go round the 8 XCDs, so XCD x = id % 8 takes the
    // x-th eighth of the list: a key block's tiles then share one L2 instead of eight (gridDim.x is a multiple of 8).
    const int total = head_base[BH];
    const int per_xcd = (total + 7) >> 3;
    const int slot = (int)(blockIdx.x >> 3);
    const int f = (int)(blockIdx.x & 7) * per_xcd + slot;
    if (slot >= per_xcd || f >= total) return;
    TileCoord tc;
    const int4 fd = flat_desc[f];               // {first list entry, count | head << 10, first key, block length}
    tc.list0 = fd.x;
    tc.t0 = 0;
    tc.count = fd.y & 1023;
    tc.k0 = fd.z;
    tc.L = fd.w;
    const int bh = fd.y >> 10, b = bh / Hh, h = bh % Hh;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hf = lane >> 5;
    const long long seg = (long long)bh * cap;

    const int ent = wave * 32 + l32;
    const int e = min(ent, tc.count - 1);
    const int q = q_idx[seg + tc.list0 + tc.t0 + e];
    // The wavefront's 32 gathered rows of Q' and of dO go straight to LDS, a whole row per 16 (8) lanes -- one request
    // covers 4 (8) rows instead of a 32-byte piece of 32 rows -- into the K/V tiles (Q') and the output staging (dO),
    // both idle at this point; piece p of row r sits at slot p ^ (r % pieces), which keeps the fragment reads below
    // free of bank conflicts.  Each wavefront reads back only what it wrote.
    constexpr int RB = D * 2, PPR = RB / 16, RPI = 64 / PPR;     // row bytes, 16-byte pieces per row, rows per request
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const uint32_t gq0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)sKV + (uint32_t)wave_u * 32 * RB;
    const uint32_t gd0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)sOut + (uint32_t)wave_u * 32 * OPITCH;
    {
        const char* qb = Q.ptr + ((long long)b * Q.stride_b + (long long)h * Q.stride_h) * 2;
        const char* db = dO.ptr + ((long long)b * dO.stride_b + (long long)h * dO.stride_h) * 2;
        const uint32_t qss = (uint32_t)(Q.stride_s * 2), doss = (uint32_t)(dO.stride_s * 2);     // host-checked: 24-bit
#pragma unroll
        for (int k = 0; k < 32 / RPI; ++k) {
            const int r = k * RPI + lane / PPR;
            const uint32_t qr = (uint32_t)__shfl(q, r, 64);
            const uint32_t pc = (uint32_t)(((lane % PPR) ^ (r & (PPR - 1))) * 16);
            dma16(qb, __umul24(qr, qss) + pc, gq0 + k * 1024);
            dma16(db, __umul24(qr, doss) + pc, gd0 + k * 1024);
        }
    }
    const float lse2 = LSE[(long long)bh * S + q] * LOG2E;
    const float dl = delta[(long long)bh * S + q];

    f32x16_t dqacc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) dqacc[dt][i] = 0.f;

    const char* kbase = K.ptr + ((long long)b * K.stride_b + (long long)h * K.stride_h) * 2;
    const char* vbase = V.ptr + ((long long)b * V.stride_b + (long long)h * V.stride_h) * 2;
    // row strides in bytes: below 2^24 and rows below 2^24, so a row's offset is one 24-bit multiply (host-checked)
    const uint32_t kss = (uint32_t)(K.stride_s * 2), vss = (uint32_t)(V.stride_s * 2);
    const int n_chunks = (tc.L + KC - 1) / KC;

    u32x4_t kreg[LOADS], vreg[LOADS];
    // rows of K and V that hold the keys of the chunk to be fetched next: the key positions themselves, or, with keys in
    // place, what kv_rows says -- looked up one chunk before the rows are fetched, so that two dependent loads never
    // sit in one chunk's shadow
    uint32_t krow_n[LOADS];
    auto lookup_rows = [&](int c) {
        const int c0 = c * KC;
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            const int r = (tid + 256 * i) / (D / 8);
            const uint32_t pos = (uint32_t)(tc.k0 + min(c0 + r, tc.L - 1));
            krow_n[i] = kv_rows ? (uint32_t)kv_rows[pos] : pos;
        }
    };
    auto prefetch = [&](int c) {
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            const int pc = (tid + 256 * i) % (D / 8);
            kreg[i] = load_at<u32x4_t>(kbase, __umul24(krow_n[i], kss) + pc * 16);
            vreg[i] = load_at<u32x4_t>(vbase, __umul24(krow_n[i], vss) + pc * 16);
        }
        lookup_rows(c + 1);
    };
    auto stage = [&]() {
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            const int piece = tid + 256 * i;
            const int r = piece / (D / 8), pc = piece % (D / 8);
            *reinterpret_cast<u32x4_t*>(&sK[r * STR + pc * 8]) = kreg[i];
            *reinterpret_cast<u32x4_t*>(&sV[r * STR + pc * 8]) = vreg[i];
        }
    };
    const __bf16* sK_lane = sK + rho(l32) * STR + hf * 8;
    const __bf16* sV_lane = sV + rho(l32) * STR + hf * 8;
    const __bf16* sKt_lane = sK + tr_lane_offset<STR>(lane);

    // A 32-key group is a sequence of 2 * KSTEPS + NU matrix instructions: S^T over the k-steps, dP^T over the k-steps
    // (with P = exp(S - LSE) computed between them), then the third product, first over the keys whose dS is ready
    // (with the rest of dS computed between them).  Their LDS operands pass through one ring of AHEAD + 1 registers,
    // fetched AHEAD instructions before use, across the phases and into the next group; fences keep that order, so no
    // matrix instruction waits a full LDS round trip.
    constexpr int NU = 2 * DT;                  // matrix instructions of the third product per 32-key group
    constexpr int NSEQ = 2 * KSTEPS + NU;
    constexpr int AHEAD = 3, RING = AHEAD + 1;
    static_assert(NSEQ % RING == 0, "the second group continues the ring where the first one left it");
    auto fetch = [&](int mt, int n) -> bf16x8_t {     // operand of instruction n of group mt (n past the end: next group)
        if (n >= NSEQ) { mt += 1; n -= NSEQ; }
        if (n < KSTEPS) return *reinterpret_cast<const bf16x8_t*>(sK_lane + mt * 32 * STR + n * 16);
        if (n < 2 * KSTEPS) return *reinterpret_cast<const bf16x8_t*>(sV_lane + mt * 32 * STR + (n - KSTEPS) * 16);
        const int u = n - 2 * KSTEPS;
        return tr_operand<STR>(sKt_lane, mt * 32, u / DT, (u % DT) * 32);
    };
    lookup_rows(0);
    prefetch(0);
    bf16x8_t qf[KSTEPS], dof[KSTEPS];
    VMOBA_WAIT_VMCNT(0);                       // the gathered rows have landed (and the first key chunk with them)
    asm volatile("" ::: "memory");
    {
        const char* gq = sKV + wave_u * 32 * RB + l32 * RB;
        const char* gd = sOut + wave_u * 32 * OPITCH + l32 * RB;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            const int slot = (2 * ks + hf) ^ (l32 & (PPR - 1));
            qf[ks] = *reinterpret_cast<const bf16x8_t*>(gq + slot * 16);
            dof[ks] = *reinterpret_cast<const bf16x8_t*>(gd + slot * 16);
        }
    }
    for (int c = 0; c < n_chunks; ++c) {
        __syncthreads();
        stage();
        __syncthreads();
        if (c + 1 < n_chunks) prefetch(c + 1);
        const int valid = tc.L - c * KC;
        const int n_mt = valid > 32 ? 2 : 1;
        bf16x8_t op[RING];
#pragma unroll
        for (int n = 0; n < RING; ++n) op[n] = fetch(0, n < AHEAD ? n : 0);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            if (mt < n_mt) {
                f32x16_t sacc, dpacc;
#pragma unroll
                for (int i = 0; i < 16; ++i) { sacc[i] = 0.f; dpacc[i] = 0.f; }
                float ds[16];
                bf16x8_t dsf;
                auto p_value = [&](int i) {           // S^T value -> P^T value, in place
                    sacc[i] = exp2_raw(fmaf(sacc[i], scale_log2, -lse2));
                };
                auto ds_value = [&](int i) {
                    ds[i] = sacc[i] * (dpacc[i] - dl);
                    asm volatile("" : "+v"(ds[i]));
                };
#pragma unroll
                for (int n = 0; n < NSEQ; ++n) {
                    // the operand AHEAD instructions on (the group after the second one waits for the next chunk)
                    if (n + AHEAD < NSEQ || mt == 0) op[(n + AHEAD) % RING] = fetch(mt, n + AHEAD);
                    if (n < KSTEPS) {
                        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[n % RING], qf[n], sacc, 0, 0, 0);
                    } else if (n < 2 * KSTEPS) {
                        const int ks = n - KSTEPS;
                        dpacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[n % RING], dof[ks], dpacc, 0, 0, 0);
                        __builtin_amdgcn_sched_barrier(0);
                        if (ks == 0 && valid < KC) {      // last chunk (uniform branch): keys past the block get weight 0
                            const int vh = valid - mt * 32 - hf;
#pragma unroll
                            for (int i = 0; i < 16; ++i)
                                if (acc_row(i, 0) >= vh) sacc[i] = -INFINITY;
                        }
#pragma unroll
                        for (int v = 0; v < 16 / KSTEPS; ++v) p_value(ks * (16 / KSTEPS) + v);
                    } else {
                        const int u = n - 2 * KSTEPS;
                        if (u == 0) {
#pragma unroll
                            for (int i = 0; i < 8; ++i) ds_value(i);
                            dsf = pack8(&ds[0]);
                        }
                        if (u == DT) dsf = pack8(&ds[8]);
                        dqacc[u % DT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[n % RING], dsf, dqacc[u % DT], 0, 0, 0);
                        if (u < DT) {
#pragma unroll
                            for (int v = 0; v < 8 / DT; ++v) ds_value(8 + u * (8 / DT) + v);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    }
    {
        // the tile's partials are consecutive rows of dQpart (bfloat16): stores of 1 KB runs instead of 16-byte pieces
        char* mine = sOut + wave * 32 * OPITCH;                               // this wavefront's rows only: no barrier
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                u32x2_t v;
                v.x = pack_bf16x2(dqacc[dt][4 * g + 0], dqacc[dt][4 * g + 1]);
                v.y = pack_bf16x2(dqacc[dt][4 * g + 2], dqacc[dt][4 * g + 3]);
                *reinterpret_cast<u32x2_t*>(mine + l32 * OPITCH + (dt * 32 + g * 8 + hf * 4) * 2) = v;
            }
        char* dst = reinterpret_cast<char*>(dQpart) + (seg + tc.list0 + tc.t0) * (long long)(D * 2);
        constexpr int LPR = D * 2 / 16;                                       // lanes per row
#pragma unroll
        for (int k = 0; k < 32 * LPR / 64; ++k) {
            const int row = k * (64 / LPR) + lane / LPR, piece = lane % LPR;
            const u32x4_t x = *reinterpret_cast<const u32x4_t*>(mine + row * OPITCH + piece * 16);
            const int e2 = wave * 32 + row;
            if (e2 < tc.count) *reinterpret_cast<u32x4_t*>(dst + (long long)e2 * (D * 2) + piece * 16) = x;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// bf16 MFMA dK/dV kernel.  A workgroup owns 128 consecutive keys of one block (key = MFMA column
// = lane % 32) and walks the block's query list in chunks of 64 gathered queries (two half-chunks
// of 32), which pass through a ring of four LDS buffers; the gathered rows are prefetched into
// registers one chunk ahead of the ring and their indices one more chunk ahead.
//   S   = Q . K^T      A = Q rows (LDS),   B = K^T (registers, loaded once)
//   dP  = dO . V^T     A = dO rows (LDS),  B = V^T (registers, loaded once)
//   dV^T += dO^T . P   A = dO^T by transpose reads of the dO tile,  B = P packed from S
//   dK^T += Q^T . dS   A = Q^T  by transpose reads of the Q tile,   B = dS
// What limits such a kernel is the LDS issue rate (one operand fetch per matrix instruction, two
// for a transposed operand), not the matrix pipe.  So the 128 keys are held by two PAIRS of
// wavefronts with 64 keys (two 32-key groups) each, and the two wavefronts of a pair split the products:
//   wavefront 0 of the pair:  S  = Q  . K^T  ->  P = exp(S - LSE)  ->  dV^T += dO^T . P
//   wavefront 1 of the pair:  dP = dO . V^T  ->  dS = P * (dP - delta)  ->  dK^T += Q^T . dS
// so every operand fetched from LDS feeds two matrix instructions (one per key group), and each
// wavefront keeps only one set of fragments (K or V) and one accumulator tile (dV^T or dK^T).
// P travels from wavefront 0 to wavefront 1 as packed bf16 through a small LDS buffer (same lane,
// same accumulator layout on both sides); wavefront 1 therefore runs the same pipeline one
// half-chunk later, and the steps are separated by one workgroup barrier per half-chunk.
// Step hc of the workgroup, local step t = hc - (wavefront % 2), all interleaved:
//   matrix:  S or dP of half-chunk t + 1,  dV or dK of half-chunk t - 1      vector: P or dS of t
//   memory (even hc): rows of chunk hc/2 + 2 from registers into the ring, loads of chunk hc/2 + 3.
// The ring buffer written during steps 2c, 2c + 1 was last read in step 2c - 1 and is first read in 2c + 3.
// A wavefront issues in order and a matrix instruction occupies the matrix pipe for 32 cycles, so the step is cut
// into units of one matrix instruction followed by an equal share of the vector, LDS and memory instructions,
// with scheduling fences between them (two matrix instructions back to back would stall the second one while
// the vector unit idles).  S / dP of even and odd half-chunks live in two register sets that swap roles, so
// no accumulator is ever copied.
// LDS bytes of the pair body: a ring of four 64-row tiles of Q and of dO, their LSE / delta, the packed-P hand-over
template <int D>
constexpr int dkv_pair_lds_bytes() { return 2 * 4 * 64 * (D + 8) * 2 + 2 * 4 * 64 * 4 + 2 * 2 * 4 * 64 * 16; }

template <int D>
__device__ __forceinline__ void dkv_pair_body(
    char* smem, int bh, int run_id, const TensorView& Q, const TensorView& K, const TensorView& V, const TensorView& dO, const float* __restrict__ LSE,
    const float* __restrict__ delta, const int* __restrict__ blk_off, const int* __restrict__ blk_ptr, const int* __restrict__ q_idx,
    const int* __restrict__ kb_start, const int* __restrict__ kb_order, const TensorView& dK, const TensorView& dV, const int* __restrict__ rows,
    const int* __restrict__ kv_rows, int Hh, int S, int nb, long long cap, float scale_log2, float scale) {
    constexpr int NT = 256;
    constexpr int QC = 64;
    constexpr int STR = D + 8;
    constexpr int KSTEPS = D / 16, DT = D / 32;
    constexpr int LOADS = QC * D * 2 / 16 / NT;
    constexpr int NBUF = 4;
    constexpr int NST = KSTEPS;
    static_assert(NST == 2 * DT && NST == 2 * LOADS, "one row piece, one k-step and one (s, dt) step per step");
    constexpr int VP = 8 / NST;               // value pairs per key group and step
    __bf16(*sQ)[QC * STR] = reinterpret_cast<__bf16(*)[QC * STR]>(smem);
    __bf16(*sdO)[QC * STR] = reinterpret_cast<__bf16(*)[QC * STR]>(smem + NBUF * QC * STR * 2);
    float(*sL)[QC] = reinterpret_cast<float(*)[QC]>(smem + 2 * NBUF * QC * STR * 2);
    float(*sDl)[QC] = reinterpret_cast<float(*)[QC]>(smem + 2 * NBUF * QC * STR * 2 + NBUF * QC * 4);
    // [pair][step parity][kg * 2 + s][lane]: packed P
    u32x4_t(*sX)[2][4][64] = reinterpret_cast<u32x4_t(*)[2][4][64]>(smem + 2 * NBUF * QC * STR * 2 + 2 * NBUF * QC * 4);
    static_assert(dkv_pair_lds_bytes<D>() == 2 * NBUF * QC * STR * 2 + 2 * NBUF * QC * 4 + 2 * 2 * 4 * 64 * 16, "LDS carve");

    const int b = bh / Hh, h = bh % Hh;
    const int* ks = kb_start + (long long)bh * (nb + 1);
    int lo = 0, hi = nb;
    while (hi - lo > 1) { int mid = (lo + hi) >> 1; if (ks[mid] <= run_id) lo = mid; else hi = mid; }
    const int j = kb_order[(long long)bh * nb + lo], run = run_id - ks[lo];
    const int k0 = blk_off[j], L = blk_off[j + 1] - k0;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int pair = wave >> 1, role = wave & 1;
    const int l32 = lane & 31, hf = lane >> 5;
    const int kbase = run * 128 + pair * 64;            // first key of the pair inside the block
    const bool pair_live = kbase < L;
    const long long seg = (long long)bh * cap;
    const int list0 = blk_ptr[(long long)bh * (nb + 1) + j];
    const int cnt = blk_ptr[(long long)bh * (nb + 1) + j + 1] - list0;

    // fragments of the pair's keys: K rows for wavefront 0, V rows for wavefront 1 (B operands, key = lane % 32)
    bf16x8_t frag[2][KSTEPS];
    int krow[2];
    bool key_live[2];
    {
        const TensorView& src = role == 0 ? K : V;
#pragma unroll
        for (int kg = 0; kg < 2; ++kg) {
            const int kk = kbase + kg * 32 + l32;
            key_live[kg] = kk < L;
            krow[kg] = k0 + min(kk, L - 1);
            const long long kin = kv_rows ? kv_rows[krow[kg]] : krow[kg];     // row of K / V that holds this key
            const char* sp = src.ptr + ((long long)b * src.stride_b + kin * src.stride_s + (long long)h * src.stride_h) * 2;
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) frag[kg][ks] = *reinterpret_cast<const bf16x8_t*>(sp + (ks * 16 + hf * 8) * 2);
        }
    }
    f32x16_t acc[2][DT];                       // dV^T (wavefront 0) or dK^T (wavefront 1), [key group][channel tile]
#pragma unroll
    for (int kg = 0; kg < 2; ++kg)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[kg][dt][i] = 0.f;

    if (cnt > 0) {
        const char* qbase = Q.ptr + ((long long)b * Q.stride_b + (long long)h * Q.stride_h) * 2;
        const char* dobase = dO.ptr + ((long long)b * dO.stride_b + (long long)h * dO.stride_h) * 2;
        // row strides in bytes: below 2^24 and rows below 2^24, so a row's offset is one 24-bit multiply (host-checked)
        const uint32_t qss = (uint32_t)(Q.stride_s * 2), doss = (uint32_t)(dO.stride_s * 2);
        const int* list = q_idx + seg + list0;
        const float* lse_h = LSE + (long long)bh * S;
        const float* dl_h = delta + (long long)bh * S;
        const int n_chunks = (cnt + QC - 1) / QC;
        const int H = 2 * n_chunks;

        u32x4_t qreg[LOADS], doreg[LOADS];
        float lreg = 0.f;
        uint32_t qn[LOADS], ql = 0;
        const int ld_row = (wave >> 1) * 32 + (lane & 31);      // the chunk row whose LSE or delta this lane moves
        bool ql_live = false, rows_live = false;
        auto prefetch_idx_piece = [&](int c, int i) {       // chunks past the list: indices clamp, rows count as dead
            const int c0 = c * QC;
            if (i < LOADS) {
                const int r = (tid + NT * i) / (D / 8);
                qn[i] = load_at<uint32_t>(list, (uint32_t)min(c0 + r, cnt - 1) << 2);
            } else {
                ql = load_at<uint32_t>(list, (uint32_t)min(c0 + ld_row, cnt - 1) << 2);
                ql_live = c0 + ld_row < cnt;
            }
        };
        auto prefetch_idx = [&](int c) {
#pragma unroll
            for (int i = 0; i <= LOADS; ++i) prefetch_idx_piece(c, i);
        };
        auto load_piece = [&](int i) {
            if (i < LOADS) {
                const uint32_t pc = (tid + NT * i) % (D / 8);
                qreg[i] = load_at<u32x4_t>(qbase, __umul24(qn[i], qss) + pc * 16);
            } else {
                const int k = i - LOADS;
                const uint32_t pc = (tid + NT * k) % (D / 8);
                doreg[k] = load_at<u32x4_t>(dobase, __umul24(qn[k], doss) + pc * 16);
            }
        };
        // LSE and delta of the chunk's 64 rows: even wavefronts fetch and store LSE values, odd ones delta values, the
        // first pair those of rows 0..31 and the second pair those of rows 32..63 (both halves of a wavefront the same
        // 32) -- free of branches inside the pipelined loop, and a request touches 32 scattered words, not 2 x 64
        const float* ld_src = (wave & 1) ? dl_h : lse_h;
        const float ld_mul = (wave & 1) ? 1.f : LOG2E, ld_dead = (wave & 1) ? 0.f : INFINITY;
        auto load_ld_regs = [&]() {
            lreg = load_at<float>(ld_src, ql << 2);
            rows_live = ql_live;
        };
        auto stage_piece = [&](int buf, int i) {
            const int k = i < LOADS ? i : i - LOADS;
            const int piece = tid + NT * k;
            const int r = piece / (D / 8), pc = piece % (D / 8);
            if (i < LOADS) *reinterpret_cast<u32x4_t*>(&sQ[buf][r * STR + pc * 8]) = qreg[k];
            else *reinterpret_cast<u32x4_t*>(&sdO[buf][r * STR + pc * 8]) = doreg[k];
        };
        // accumulator order: the 16 values a lane half needs per 32-query group are contiguous
        const int ld_pos = (ld_row & 32) + ((ld_row & 1) << 4) + (((ld_row & 31) >> 4) << 3) + (((ld_row >> 1) & 1) << 2) + ((ld_row >> 2) & 3);
        float* const ld_dst = (wave & 1) ? &sDl[0][0] : &sL[0][0];
        auto stage_ld = [&](int buf) {         // rows past the end of the list: LSE = +inf (weight 0), delta = 0
            ld_dst[buf * QC + ld_pos] = rows_live ? lreg * ld_mul : ld_dead;
        };
        auto load_all = [&]() {
#pragma unroll
            for (int i = 0; i < 2 * LOADS; ++i) load_piece(i);
            load_ld_regs();
        };
        auto stage_all = [&](int buf) {
#pragma unroll
            for (int i = 0; i < 2 * LOADS; ++i) stage_piece(buf, i);
            stage_ld(buf);
        };
        // prologue: chunks 0 and 1 staged, rows of chunk 2 in flight, indices of chunk 3 in flight
        prefetch_idx(0);
        load_all();
        prefetch_idx(1);
        stage_all(0);
        load_all();
        prefetch_idx(2);
        stage_all(1);
        load_all();
        prefetch_idx(3);

        const f32x16_t zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        // row operands come from the Q tile for wavefront 0 (S) and from the dO tile for wavefront 1 (dP);
        // transposed operands from the dO tile for wavefront 0 (dV) and from the Q tile for wavefront 1 (dK)
        const __bf16* rows_tile = role == 0 ? &sQ[0][0] : &sdO[0][0];
        const __bf16* tr_tile = role == 0 ? &sdO[0][0] : &sQ[0][0];
        const float* ld_tile = role == 0 ? &sL[0][0] : &sDl[0][0];
        const int row_lane = rho(l32) * STR + hf * 8;
        const int tr_lane = tr_lane_offset<STR>(lane);
        auto half_off = [&](int half) { return ((half >> 1) & (NBUF - 1)) * (QC * STR) + (half & 1) * 32 * STR; };
        auto read_rows = [&](int half, int ks) {
            return *reinterpret_cast<const bf16x8_t*>(rows_tile + half_off(half) + row_lane + ks * 16);
        };
        auto read_tr = [&](int half, int step) {
            return tr_operand<STR>(tr_tile + half_off(half) + tr_lane, 0, step / DT, (step % DT) * 32);
        };
        auto read_tr_half = [&](int half, int step, int part) {     // the two 8-byte transpose reads of read_tr, one at a time
            const __bf16* pp = tr_tile + half_off(half) + tr_lane + (16 * (step / DT) + 2 * part) * STR + (step % DT) * 32;
            return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_t*)(pp));
        };

        if (pair_live) {
            f32x16_t xa[2] = {zero16, zero16}, xb[2] = {zero16, zero16};    // S or dP of the even / odd local half-chunks
            bf16x8_t w_prev[2][2];                          // packed P or dS of local half-chunk t - 1, [kg][s]
            {
                const f32x4_t z4 = {0.f, 0.f, 0.f, 0.f};
                const bf16x4_t zb = __builtin_convertvector(z4, bf16x4_t);
                const bf16x8_t z8 = __builtin_shufflevector(zb, zb, 0, 1, 2, 3, 4, 5, 6, 7);
                w_prev[0][0] = w_prev[0][1] = w_prev[1][0] = w_prev[1][1] = z8;
            }
            __syncthreads();
            // S / dP of half-chunk 0
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) {
                const bf16x8_t a = read_rows(0, ks);
#pragma unroll
                for (int kg = 0; kg < 2; ++kg)
                    xa[kg] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, frag[kg][ks], ks == 0 ? zero16 : xa[kg], 0, 0, 0);
            }
            bf16x8_t rcur = read_rows(1, 0);
            bf16x8_t tcur = read_tr(0, 0);                  // local step 0 multiplies it by zeros
            u32x4_t* xbuf = &sX[pair][0][0][lane];          // + parity * 256 + slot * 64

            // one local step; ROLE and EVEN (parity of the workgroup step hc = t + ROLE) are compile-time
            // (x_cur holds S or dP of half-chunk t, x_nxt receives that of t + 1: the two sets swap roles every step)
            auto local_step = [&](int t, auto role_tag, auto even_tag, f32x16_t(&x_cur)[2], f32x16_t(&x_nxt)[2]) {
                constexpr int ROLE = decltype(role_tag)::value;
                constexpr bool EVEN = decltype(even_tag)::value;
                const int hc = t + ROLE;
                const int wbuf = ((hc >> 1) + 2) & (NBUF - 1);
                float ld[16];
                {
                    const float* lp = ld_tile + ((t >> 1) & (NBUF - 1)) * QC + (t & 1) * 32 + hf * 16;
#pragma unroll
                    for (int g4 = 0; g4 < 4; ++g4) {
                        const f32x4_t a4 = *reinterpret_cast<const f32x4_t*>(lp + g4 * 4);
#pragma unroll
                        for (int u = 0; u < 4; ++u) ld[g4 * 4 + u] = a4[u];
                    }
                }
                u32x4_t pin[4];
                if constexpr (ROLE == 1) {
#pragma unroll
                    for (int sl = 0; sl < 4; ++sl) pin[sl] = xbuf[(t & 1) * 256 + sl * 64];
                }
                float w[2][16];
                const int th = t > 0 ? t - 1 : 0;
#pragma unroll
                for (int st = 0; st < NST; ++st) {
                    // four units per k-step, each one matrix instruction plus a quarter of everything else, fenced so
                    // that the matrix instructions stay evenly spaced in the (in-order) instruction stream
                    bf16x8_t rn;
                    bf16x4_t tlo, thi;
                    const bool last_st = st + 1 == NST;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int kg = q >> 1;
                        if (q == 0) rn = last_st ? read_rows(t + 2, 0) : read_rows(t + 1, st + 1);
                        if (q == 1) tlo = last_st ? read_tr_half(t, 0, 0) : read_tr_half(th, st + 1, 0);
                        if (q == 2) thi = last_st ? read_tr_half(t, 0, 1) : read_tr_half(th, st + 1, 1);
                        if ((q & 1) == 0)
                            x_nxt[kg] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rcur, frag[kg][st], st == 0 ? zero16 : x_nxt[kg], 0, 0, 0);
                        else
                            acc[kg][st % DT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tcur, w_prev[kg][st / DT], acc[kg][st % DT], 0, 0, 0);
                        __builtin_amdgcn_sched_barrier(0);          // the matrix instruction leads its unit
                        // the unit's VP values of P or dS: second half of this k-step's values when q is odd, key group kg
#pragma unroll
                        for (int u = 0; u < VP; ++u) {
                            const int i = 2 * VP * st + VP * (q & 1) + u;
                            if constexpr (ROLE == 0) {
                                w[kg][i] = exp2_raw(fmaf(x_cur[kg][i], scale_log2, -ld[i]));
                            } else {
                                const u32x4_t pk = pin[kg * 2 + i / 8];
                                const uint32_t word = (i % 8) / 2 == 0 ? pk.x : (i % 8) / 2 == 1 ? pk.y : (i % 8) / 2 == 2 ? pk.z : pk.w;
                                const float pval = (i & 1) ? bf16hi_to_f32(word) : bf16lo_to_f32(word);
                                w[kg][i] = pval * (x_cur[kg][i] - ld[i]);
                            }
                            asm volatile("" : "+v"(w[kg][i]));
                        }
                        // packed operands are replaced as soon as their last reader of this step has issued
                        if (q == 3 && (st == NST / 2 - 1 || last_st)) {
                            const int sidx = last_st ? 1 : 0;
#pragma unroll
                            for (int k2 = 0; k2 < 2; ++k2) {
                                w_prev[k2][sidx] = pack8(&w[k2][8 * sidx]);
                                if constexpr (ROLE == 0) {
                                    u32x4_t o;
                                    __builtin_memcpy(&o, &w_prev[k2][sidx], 16);
                                    xbuf[(t & 1) * 256 + (k2 * 2 + sidx) * 64] = o;
                                }
                            }
                        }
                        if constexpr (EVEN) {
                            if (q == 2) stage_piece(wbuf, st);
                            if (q == 3) load_piece(st);
                            if (st == 0 && q == 1) { stage_ld(wbuf); load_ld_regs(); }
                        } else {
                            if (4 * st + q <= LOADS) prefetch_idx_piece((hc >> 1) + 4, 4 * st + q);     // one index load per unit
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    rcur = rn;
                    tcur = __builtin_shufflevector(tlo, thi, 0, 1, 2, 3, 4, 5, 6, 7);
                }
            };
            // a step in which this wavefront has no local step (hc = 0 for wavefront 1, hc = H + 1 for
            // wavefront 0) still moves its share of the rows
            auto idle_step = [&](int hc, auto even_tag) {
                constexpr bool EVEN = decltype(even_tag)::value;
                if constexpr (EVEN) {
                    stage_all(((hc >> 1) + 2) & (NBUF - 1));
                    load_all();
                } else {
                    prefetch_idx((hc >> 1) + 4);
                }
            };
            if (role == 0) {
                for (int c = 0; c < n_chunks; ++c) {
                    if (c > 0) __syncthreads();
                    local_step(2 * c, std::integral_constant<int, 0>{}, std::true_type{}, xa, xb);
                    __syncthreads();
                    local_step(2 * c + 1, std::integral_constant<int, 0>{}, std::false_type{}, xb, xa);
                }
                __syncthreads();
                local_step(H, std::integral_constant<int, 0>{}, std::true_type{}, xa, xb);       // drain: dV of the last half-chunk
                __syncthreads();
                idle_step(H + 1, std::false_type{});
            } else {
                idle_step(0, std::true_type{});
                for (int c = 0; c < n_chunks; ++c) {
                    __syncthreads();
                    local_step(2 * c, std::integral_constant<int, 1>{}, std::false_type{}, xa, xb);
                    __syncthreads();
                    local_step(2 * c + 1, std::integral_constant<int, 1>{}, std::true_type{}, xb, xa);
                }
                __syncthreads();
                local_step(H, std::integral_constant<int, 1>{}, std::false_type{}, xa, xb);      // drain: dK of the last half-chunk
            }
        } else {
            // a pair whose keys lie past the end of the block only helps to move rows
            __syncthreads();
            for (int c = 0; c <= n_chunks; ++c) {
                if (c > 0) __syncthreads();
                stage_all((c + 2) & (NBUF - 1));
                load_all();
                __syncthreads();
                prefetch_idx(c + 4);
            }
        }
    }
    {
        const TensorView& dst = role == 0 ? dV : dK;
        const float f = role == 0 ? 1.f : scale;
#pragma unroll
        for (int kg = 0; kg < 2; ++kg) {
            if (pair_live && key_live[kg]) {
                const int kout = rows ? rows[krow[kg]] : krow[kg];
                char* pd = dst.ptr + ((long long)b * dst.stride_b + (long long)kout * dst.stride_s + (long long)h * dst.stride_h) * 2;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int d = dt * 32 + g * 8 + hf * 4;
                        u32x2_t wv;
                        wv.x = pack_bf16x2(acc[kg][dt][4 * g + 0] * f, acc[kg][dt][4 * g + 1] * f);
                        wv.y = pack_bf16x2(acc[kg][dt][4 * g + 2] * f, acc[kg][dt][4 * g + 3] * f);
                        *reinterpret_cast<u32x2_t*>(pd + d * 2) = wv;
                    }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// bf16 MFMA dK/dV kernel for a block's last L % 128 keys when they are at most 32.  The pair kernel above
// spends a whole walk of the block's query list on every 128-key run, however few of its keys exist; here
// the cost follows the keys: one workgroup per (head, block), its four wavefronts hold the same <= 32 keys
// and split the query list (wavefront w takes the 32-query chunks w, w + 4, ...), each computing all four
// products for its chunks (same operand orientation as above, key = MFMA column) from its own LDS tiles,
// without workgroup barriers; the four partial dK^T / dV^T are added through LDS at the end.
template <int D>
__device__ __forceinline__ void dkv_tail_body(
    char* smem, int bh, int rank, const TensorView& Q, const TensorView& K, const TensorView& V, const TensorView& dO, const float* __restrict__ LSE,
    const float* __restrict__ delta, const int* __restrict__ blk_off, const int* __restrict__ blk_ptr, const int* __restrict__ q_idx,
    const int* __restrict__ kb_order, const TensorView& dK, const TensorView& dV, const int* __restrict__ rows,
    const int* __restrict__ kv_rows, int Hh, int S, int nb, long long cap, float scale_log2, float scale) {
    constexpr int QC = 32;                       // queries per chunk
    constexpr int STR = D + 8;
    constexpr int KSTEPS = D / 16, DT = D / 32;
    constexpr int LOADS = QC * (D / 8) / 64;     // 16-byte pieces per lane per chunk and tensor
    // Q tiles, then dO tiles, one of each per wavefront; then LSE and delta
    __bf16(*sT)[4][QC * STR] = reinterpret_cast<__bf16(*)[4][QC * STR]>(smem);
    float(*sL)[QC] = reinterpret_cast<float(*)[QC]>(smem + 2 * 4 * QC * STR * 2);
    float(*sDl)[QC] = reinterpret_cast<float(*)[QC]>(smem + 2 * 4 * QC * STR * 2 + 4 * QC * 4);
    static_assert(2 * 4 * QC * STR * 2 + 2 * 4 * QC * 4 <= dkv_pair_lds_bytes<D>(), "the tail body fits the pair body's LDS");
    const int b = bh / Hh, h = bh % Hh;
    const int j = kb_order[(long long)bh * nb + rank];            // longest query list first
    const int k0 = blk_off[j], L = blk_off[j + 1] - k0;
    const int tail = L % 128;
    if (tail == 0 || tail > 32) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hf = lane >> 5;
    const long long seg = (long long)bh * cap;
    const int list0 = blk_ptr[(long long)bh * (nb + 1) + j];
    const int cnt = blk_ptr[(long long)bh * (nb + 1) + j + 1] - list0;
    const int* list = q_idx + seg + list0;
    const float* lse_h = LSE + (long long)bh * S;
    const float* dl_h = delta + (long long)bh * S;

    // the tail keys: B operands (key = lane % 32); columns past the tail repeat the block's last key and are not written
    const bool key_live = l32 < tail;
    const int krow = k0 + min(L - tail + l32, L - 1);
    bf16x8_t kf[KSTEPS], vf[KSTEPS];
    {
        const long long kin = kv_rows ? kv_rows[krow] : krow;         // row of K and V that holds this key
        const char* pk = K.ptr + ((long long)b * K.stride_b + kin * K.stride_s + (long long)h * K.stride_h) * 2;
        const char* pv = V.ptr + ((long long)b * V.stride_b + kin * V.stride_s + (long long)h * V.stride_h) * 2;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            kf[ks] = *reinterpret_cast<const bf16x8_t*>(pk + (ks * 16 + hf * 8) * 2);
            vf[ks] = *reinterpret_cast<const bf16x8_t*>(pv + (ks * 16 + hf * 8) * 2);
        }
    }
    const f32x16_t zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f32x16_t dvacc[DT], dkacc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) { dvacc[dt] = zero16; dkacc[dt] = zero16; }

    const char* qbase = Q.ptr + ((long long)b * Q.stride_b + (long long)h * Q.stride_h) * 2;
    const char* dobase = dO.ptr + ((long long)b * dO.stride_b + (long long)h * dO.stride_h) * 2;
    const long long qss = Q.stride_s * 2, doss = dO.stride_s * 2;
    const int n_chunks = (cnt + QC - 1) / QC;
    __bf16* tQ = &sT[0][wave][0];
    __bf16* tdO = &sT[1][wave][0];
    float* tL = &sL[wave][0];
    float* tDl = &sDl[wave][0];
    // LSE / delta of row r are stored at the place where the accumulator layout wants them: a lane half reads its 16 rows
    // (acc_row(i, hf), i = 0..15) as 16 consecutive floats
    const int ld_pos = ((l32 & 1) << 4) + ((l32 >> 4) << 3) + (((l32 >> 1) & 1) << 2) + ((l32 >> 2) & 3);
    const int row_lane = rho(l32) * STR + hf * 8;
    const int tr_lane = tr_lane_offset<STR>(lane);

    // Gathered rows travel list index -> row address -> registers -> LDS; a wavefront keeps the rows of its next two
    // chunks in flight (register sets 0 / 1 by chunk parity) and the list indices of the one after.
    struct RowSet {
        u32x4_t q[LOADS], d[LOADS];
        float l, dl;
        bool live;
    };
    RowSet rs[2];
    int qn[LOADS], ql = 0;
    bool ql_live = false;
    auto fetch_idx = [&](int c) {                // list entries of chunk c (entries past the list repeat its last one)
        const int c0 = c * QC;
#pragma unroll
        for (int i = 0; i < LOADS; ++i) qn[i] = list[max(min(c0 + (lane + 64 * i) / (D / 8), cnt - 1), 0)];
        ql = list[max(min(c0 + l32, cnt - 1), 0)];
        ql_live = c0 + l32 < cnt;
    };
    auto fetch_rows = [&](RowSet& r) {           // rows of the chunk whose indices were fetched last
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            const int pc = (lane + 64 * i) % (D / 8);
            r.q[i] = *reinterpret_cast<const u32x4_t*>(qbase + (long long)qn[i] * qss + pc * 16);
            r.d[i] = *reinterpret_cast<const u32x4_t*>(dobase + (long long)qn[i] * doss + pc * 16);
        }
        r.l = lse_h[ql];
        r.dl = dl_h[ql];
        r.live = ql_live;
    };
    auto stage = [&](const RowSet& r) {
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            const int piece = lane + 64 * i;
            const int row = piece / (D / 8), pc = piece % (D / 8);
            *reinterpret_cast<u32x4_t*>(&tQ[row * STR + pc * 8]) = r.q[i];
            *reinterpret_cast<u32x4_t*>(&tdO[row * STR + pc * 8]) = r.d[i];
        }
        if (hf == 0) {                           // rows past the end of the list: LSE = +inf (weight 0), delta = 0
            tL[ld_pos] = r.live ? r.l * LOG2E : INFINITY;
            tDl[ld_pos] = r.live ? r.dl : 0.f;
        }
    };
    // the wavefront's k-th chunk is chunk wave + 4 k
    const int my_chunks = n_chunks > wave ? (n_chunks - wave + 3) / 4 : 0;
    if (my_chunks > 0) {
        fetch_idx(wave);
        fetch_rows(rs[0]);
        fetch_idx(wave + 4);
        fetch_rows(rs[1]);
        fetch_idx(wave + 8);
    }
    auto one_chunk = [&](int k, RowSet& r) {
        stage(r);
        fetch_rows(r);                           // chunk k + 2 (indices are already here)
        fetch_idx(wave + 4 * (k + 3));
        // S = Q . K^T and dP = dO . V^T
        f32x16_t sacc = zero16, dpacc = zero16;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            const bf16x8_t qa = *reinterpret_cast<const bf16x8_t*>(tQ + row_lane + ks * 16);
            const bf16x8_t da = *reinterpret_cast<const bf16x8_t*>(tdO + row_lane + ks * 16);
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa, kf[ks], sacc, 0, 0, 0);
            dpacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(da, vf[ks], dpacc, 0, 0, 0);
        }
        float ld[16], dl[16];
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            const f32x4_t a4 = *reinterpret_cast<const f32x4_t*>(tL + hf * 16 + g4 * 4);
            const f32x4_t d4 = *reinterpret_cast<const f32x4_t*>(tDl + hf * 16 + g4 * 4);
#pragma unroll
            for (int u = 0; u < 4; ++u) { ld[g4 * 4 + u] = a4[u]; dl[g4 * 4 + u] = d4[u]; }
        }
        float pw[16], dsw[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            pw[i] = exp2_raw(fmaf(sacc[i], scale_log2, -ld[i]));
            dsw[i] = pw[i] * (dpacc[i] - dl[i]);
        }
        // dV^T += dO^T . P and dK^T += Q^T . dS
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            const bf16x8_t pb = pack8(&pw[8 * s2]);
            const bf16x8_t db = pack8(&dsw[8 * s2]);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                const bf16x8_t dot = tr_operand<STR>(tdO + tr_lane, 0, s2, dt * 32);
                const bf16x8_t qt = tr_operand<STR>(tQ + tr_lane, 0, s2, dt * 32);
                dvacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dot, pb, dvacc[dt], 0, 0, 0);
                dkacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qt, db, dkacc[dt], 0, 0, 0);
            }
        }
    };
    for (int k = 0; k < my_chunks; k += 2) {
        one_chunk(k, rs[0]);
        if (k + 1 < my_chunks) one_chunk(k + 1, rs[1]);
    }
    // ---- add the four wavefronts' partial sums (the row tiles are free now) and write the tail's rows
    static_assert(2 * 4 * QC * STR * 2 >= 3 * 64 * DT * 16 * sizeof(float), "reduction buffer fits the row tiles");
    float* red = reinterpret_cast<float*>(&sT[0][0][0]);       // [3][DT * 16][64]
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        f32x16_t* acc = pass == 0 ? dvacc : dkacc;
        __syncthreads();
        if (wave > 0) {
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int i = 0; i < 16; ++i) red[((wave - 1) * DT * 16 + dt * 16 + i) * 64 + lane] = acc[dt][i];
        }
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int w = 0; w < 3; ++w)
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[dt][i] += red[(w * DT * 16 + dt * 16 + i) * 64 + lane];
            if (key_live) {
                const TensorView& dst = pass == 0 ? dV : dK;
                const float fsc = pass == 0 ? 1.f : scale;
                const int kout = rows ? rows[krow] : krow;
                char* pd = dst.ptr + ((long long)b * dst.stride_b + (long long)kout * dst.stride_s + (long long)h * dst.stride_h) * 2;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        u32x2_t wv;
                        wv.x = pack_bf16x2(acc[dt][4 * g + 0] * fsc, acc[dt][4 * g + 1] * fsc);
                        wv.y = pack_bf16x2(acc[dt][4 * g + 2] * fsc, acc[dt][4 * g + 3] * fsc);
                        *reinterpret_cast<u32x2_t*>(pd + (dt * 32 + g * 8 + hf * 4) * 2) = wv;
                    }
            }
        }
    }
}

// The dK/dV launch.  Every head has `slots` slots: slots [0, runs of the head) run the pair body on one 128-key run each
// (longest query list first); the next n_blocks slots run the tail body on one block each; the rest do nothing.  Slots
// are handed out slot group first, head second (see the kernel): the order is longest-first over the whole launch
// rather than per head, and the short tail workgroups fill its end, where the long runs finish unevenly.
template <int D>
__global__ __launch_bounds__(256) void attn_bwd_dkv_kernel(
    TensorView Q, TensorView K, TensorView V, TensorView dO, const float* __restrict__ LSE, const float* __restrict__ delta,
    const int* __restrict__ blk_off, const int* __restrict__ blk_ptr, const int* __restrict__ q_idx,
    const int* __restrict__ kb_start, const int* __restrict__ kb_order, TensorView dK, TensorView dV, const int* __restrict__ rows, int Hh, int S, int nb, long long cap,
    float scale_log2, float scale, const int* __restrict__ kv_rows, int BH, int slots, int group) {
    __shared__ __align__(16) char smem[dkv_pair_lds_bytes<D>()];
    // One-dimensional grid.  Workgroup i runs on XCD i % 8 as that XCD's workgroup number i / 8.  A head's slots are cut
    // into groups of `group` consecutive slots (the runs of one key block, when the blocks are equally long); groups are
    // numbered slot group first, head second -- longest query lists first over the whole launch -- and dealt to the XCDs
    // in turn, each XCD taking the slots of a group one after the other: the runs of one block, which all walk the same
    // query list, run at the same time on the same XCD and share its L2.
    const int xcd = (int)blockIdx.x & 7, n = (int)blockIdx.x >> 3;
    const int G = (n / group) * 8 + xcd;
    if (G >= BH * (slots / group)) return;
    const int bh = G % BH;
    const int id = (G / BH) * group + n % group;
    const int runs = kb_start[(long long)bh * (nb + 1) + nb];
    if (id < runs)
        dkv_pair_body<D>(smem, bh, id, Q, K, V, dO, LSE, delta, blk_off, blk_ptr, q_idx, kb_start, kb_order, dK, dV, rows, kv_rows, Hh, S, nb, cap, scale_log2, scale);
    else if (id - runs < nb)
        dkv_tail_body<D>(smem, bh, id - runs, Q, K, V, dO, LSE, delta, blk_off, blk_ptr, q_idx, kb_order, dK, dV, rows, kv_rows, Hh, S, nb, cap, scale_log2, scale);
}

// dQ[q] = scale * sum over the query's pairs of dQpart[pair]; the partials have the tensors' type.  A head whose
// selection did not fit the lists (row_ptr[S] > cap, see vmoba_select) counts as having selected nothing.
template <bool BF16, int D>
__global__ __launch_bounds__(256) void dq_merge_kernel(const float* __restrict__ dQpart, const int* __restrict__ row_ptr,
                                                       const int* __restrict__ pair_pos, TensorView dQ, const int* __restrict__ rows, int Hh, int S,
                                                       long long cap, float scale) {
    constexpr int CH = BF16 ? 8 : 4;
    constexpr int LPQ = D / CH;
    constexpr int QPW = 256 / LPQ;
    const int bh = blockIdx.y, b = bh / Hh, h = bh % Hh;
    const int q = blockIdx.x * QPW + threadIdx.x / LPQ;
    const int part = threadIdx.x % LPQ;
    if (q >= S) return;
    const bool fits = row_ptr[(long long)bh * (S + 1) + S] <= cap;
    const int r0 = row_ptr[(long long)bh * (S + 1) + q];
    const int r1 = fits ? row_ptr[(long long)bh * (S + 1) + q + 1] : r0;
    const long long seg = (long long)bh * cap;
    float acc[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) acc[c] = 0.f;
    constexpr int MB = 8;                            // partial rows in flight per lane
    for (int r = r0; r < r1; r += MB) {
        long long pair[MB];
#pragma unroll
        for (int u = 0; u < MB; ++u) pair[u] = seg + pair_pos[seg + min(r + u, r1 - 1)];
#pragma unroll
        for (int u = 0; u < MB; ++u) {
            const float keep = (r + u < r1) ? 1.f : 0.f;
            if constexpr (BF16) {
                // (read once: non-temporal, as in the forward merge)
                const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(reinterpret_cast<const uint16_t*>(dQpart) + pair[u] * D + part * 8));
                acc[0] += keep * bf16lo_to_f32(v.x); acc[1] += keep * bf16hi_to_f32(v.x);
                acc[2] += keep * bf16lo_to_f32(v.y); acc[3] += keep * bf16hi_to_f32(v.y);
                acc[4] += keep * bf16lo_to_f32(v.z); acc[5] += keep * bf16hi_to_f32(v.z);
                acc[6] += keep * bf16lo_to_f32(v.w); acc[7] += keep * bf16hi_to_f32(v.w);
            } else {
                const f32x4_t v = *reinterpret_cast<const f32x4_t*>(dQpart + pair[u] * D + part * 4);
                acc[0] += keep * v.x; acc[1] += keep * v.y; acc[2] += keep * v.z; acc[3] += keep * v.w;
            }
        }
    }
#pragma unroll
    for (int c = 0; c < CH; ++c) acc[c] *= scale;
    const int qo = rows ? rows[q] : q;
    char* dst = dQ.ptr + ((long long)b * dQ.stride_b + (long long)qo * dQ.stride_s + (long long)h * dQ.stride_h) * (BF16 ? 2 : 4);
    if constexpr (BF16) {
        const u32x4_t o = {pack_bf16x2(acc[0], acc[1]), pack_bf16x2(acc[2], acc[3]), pack_bf16x2(acc[4], acc[5]),
                           pack_bf16x2(acc[6], acc[7])};
        *reinterpret_cast<u32x4_t*>(dst + part * 16) = o;
    } else {
#pragma unroll
        for (int c = 0; c < CH; c += 4) {
            f32x4_t o = {acc[c], acc[c + 1], acc[c + 2], acc[c + 3]};
            *reinterpret_cast<f32x4_t*>(dst + (part * CH + c) * 4) = o;
        }
    }
}

struct BwdWs {
    float* dQpart;     // [BH * cap][D], in the tensors' type
    float* delta;      // [BH][S]
    int* tile_start;   // [BH][257]
    int4* tile_desc;   // [BH][tiles_per_head], or the flat list of all heads' tiles
    int* head_base;    // [BH + 1]
    int* kb_start;     // [BH][257]
    int* kb_order;     // [BH][256]
    char* dO_copy;     // [BH, S, D] block-order copy of dO (used with a row map)
    size_t total;
};

BwdWs carve_bwd(void* base, int BH, int64_t S, int D, int64_t cap, int es) {
    BwdWs w;
    char* p = (char*)base;
    size_t off = 0;
    w.dQpart = (float*)(p + off);    off += align_up((size_t)BH * cap * D * es, 256);
    w.delta = (float*)(p + off);     off += align_up((size_t)BH * S * 4, 256);
    w.tile_start = (int*)(p + off);  off += align_up((size_t)BH * (VMOBA_MAX_BLOCKS + 1) * 4, 256);
    w.tile_desc = (int4*)(p + off);  off += align_up((size_t)BH * vmoba_max_tiles(cap, 64) * 16, 256);
    w.head_base = (int*)(p + off);   off += align_up((size_t)(BH + 1) * 4, 256);
    w.kb_start = (int*)(p + off);    off += align_up((size_t)BH * (VMOBA_MAX_BLOCKS + 1) * 4, 256);
    w.kb_order = (int*)(p + off);    off += align_up((size_t)BH * VMOBA_MAX_BLOCKS * 4, 256);
    w.dO_copy = p + off;             off += align_up((size_t)BH * S * D * es, 256);
    w.total = off;
    return w;
}

}  // namespace

size_t vmoba_attn_bwd_workspace_bytes(int B, int Hh, int64_t S, int D, int64_t cap, int dtype) {
    return carve_bwd(nullptr, B * Hh, S, D, cap, dtype == VMOBA_BF16 ? 2 : 4).total;
}

extern "C" int vmoba_attn_bwd(int B, int Hh, int64_t S, int D, int32_t n_blocks, const int32_t* blk_off,
                              const vmoba_tensor* Qp, const vmoba_tensor* Kp, const vmoba_tensor* Vp,
                              const vmoba_tensor* O, const float* LSE, const vmoba_tensor* dO,
                              const int32_t* blk_ptr, const int32_t* q_idx, const int32_t* row_ptr,
                              const int32_t* pair_pos, int64_t nnz_capacity, float softmax_scale,
                              const vmoba_tensor* dQ, const vmoba_tensor* dK, const vmoba_tensor* dV,
                              const int32_t* rows, const int32_t* key_rows, const int32_t* kv_rows, void* workspace,
                              size_t workspace_bytes, void* stream) {
    if (B <= 0 || Hh <= 0 || S <= 0 || n_blocks <= 0 || nnz_capacity <= 0) return VMOBA_ERR_INVALID_ARG;
    if (!blk_off || !blk_ptr || !q_idx || !row_ptr || !pair_pos || !LSE || !workspace) return VMOBA_ERR_INVALID_ARG;
    if (!tensor_ok(Qp) || !tensor_ok(Kp) || !tensor_ok(Vp) || !tensor_ok(O) || !tensor_ok(dO) || !tensor_ok(dQ) ||
        !tensor_ok(dK) || !tensor_ok(dV))
        return VMOBA_ERR_INVALID_ARG;
    if (!std::isfinite(softmax_scale)) return VMOBA_ERR_INVALID_ARG;
    if (D != 64 && D != 128) return VMOBA_ERR_UNSUPPORTED;
    if (n_blocks > VMOBA_MAX_BLOCKS) return VMOBA_ERR_UNSUPPORTED;
    const int dt = Qp->dtype;
    if (Kp->dtype != dt || Vp->dtype != dt || O->dtype != dt || dO->dtype != dt || dQ->dtype != dt ||
        dK->dtype != dt || dV->dtype != dt)
        return VMOBA_ERR_UNSUPPORTED;
    const int BH = B * Hh;
    if (nnz_capacity > INT32_MAX) return VMOBA_ERR_UNSUPPORTED;
    BwdWs ws = carve_bwd(workspace, BH, S, D, nnz_capacity, dt == VMOBA_BF16 ? 2 : 4);
    if (workspace_bytes < ws.total) return VMOBA_ERR_WORKSPACE;
    if (((uintptr_t)workspace) & 255) return VMOBA_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    const bool bf16 = dt == VMOBA_BF16;
    const TensorView Qv = make_view(Qp), Kv = make_view(Kp), Vv = make_view(Vp), Ov = make_view(O);
    const TensorView dQv = make_view(dQ), dKv = make_view(dK), dVv = make_view(dV);
    TensorView dOv = make_view(dO);
    const float scale_log2 = softmax_scale * LOG2E;
    const bool simple = !bf16;              // float32 tensors take the plain FMA kernels
    // the tile kernels form the byte offset of a row of Q', K', V' or dO with one 24-bit multiply and 32-bit adds
    if (!simple) {
        const int64_t do_stride = rows ? D : dO->stride_s;          // dO is read from its block-order copy when `rows` is given
        const int64_t strides[4] = {Qp->stride_s, Kp->stride_s, Vp->stride_s, do_stride};
        if (S >= (1 << 24)) return VMOBA_ERR_UNSUPPORTED;
        for (int64_t ss : strides)
            if (ss <= 0 || ss * 2 >= (1 << 24) || (uint64_t)S * (uint64_t)ss * 2 >= ((uint64_t)1 << 32)) return VMOBA_ERR_UNSUPPORTED;
    }

    {   // delta
        const int epp = bf16 ? 8 : 4;
        const int qpw = 256 / (D / epp);
        dim3 grid((unsigned)ceil_div64(S, qpw), (unsigned)BH);
        if (bf16 && D == 128) delta_kernel<true, 128><<<grid, dim3(256), 0, st>>>(Ov, dOv, ws.delta, rows, ws.dO_copy, Hh, (int)S);
        else if (bf16) delta_kernel<true, 64><<<grid, dim3(256), 0, st>>>(Ov, dOv, ws.delta, rows, ws.dO_copy, Hh, (int)S);
        else if (D == 128) delta_kernel<false, 128><<<grid, dim3(256), 0, st>>>(Ov, dOv, ws.delta, rows, ws.dO_copy, Hh, (int)S);
        else delta_kernel<false, 64><<<grid, dim3(256), 0, st>>>(Ov, dOv, ws.delta, rows, ws.dO_copy, Hh, (int)S);
        VMOBA_CHECK_LAUNCH();
    }
    if (rows) {   // from here on dO is the block-order copy [B, Hh, S, D] the delta kernel wrote
        dOv.ptr = ws.dO_copy;
        dOv.stride_b = (int64_t)Hh * S * D;
        dOv.stride_h = S * D;
        dOv.stride_s = D;
    }
    // ---- dQ
    const int TM = simple ? 64 : 128;
    tile_plan_kernel<<<dim3(1), dim3(1024), 0, st>>>(blk_ptr, ws.tile_start, ws.head_base, BH, n_blocks, TM);
    VMOBA_CHECK_LAUNCH();
    const int64_t max_tiles = std::min<int64_t>(vmoba_max_tiles(nnz_capacity, TM), (nnz_capacity / TM + n_blocks + 7) / 8 * 8);
    if (simple) {
        tile_desc_kernel<<<dim3((unsigned)ceil_div64(max_tiles, 256), (unsigned)BH), dim3(256), 0, st>>>(
            ws.tile_start, blk_ptr, blk_off, ws.tile_desc, n_blocks, TM, (int)max_tiles);
    } else {
        flat_tile_desc_kernel<<<dim3((unsigned)ceil_div64(max_tiles, 256), (unsigned)BH), dim3(256), 0, st>>>(
            ws.tile_start, blk_ptr, blk_off, ws.tile_desc, n_blocks, TM, (int)max_tiles);
    }
    VMOBA_CHECK_LAUNCH();
    {
        VMOBA_PROFILE_BEGIN(1, st);
        if (simple) {
            dim3 grid((unsigned)max_tiles, (unsigned)BH);
#define DQ_ARGS Qv, Kv, Vv, dOv, LSE, ws.delta, blk_off, blk_ptr, q_idx, ws.tile_desc, (int)max_tiles, ws.dQpart, Hh, (int)S, n_blocks, (long long)nnz_capacity, scale_log2, kv_rows
            if (D == 128) attn_bwd_dq_simple_kernel<128><<<grid, dim3(64), 0, st>>>(DQ_ARGS);
            else attn_bwd_dq_simple_kernel<64><<<grid, dim3(64), 0, st>>>(DQ_ARGS);
#undef DQ_ARGS
        } else {
            // one workgroup per entry of the flat tile list; the bound on the list length is a multiple of 8
            const dim3 grid((unsigned)std::min<int64_t>((int64_t)BH * max_tiles, ((nnz_capacity / TM + n_blocks) * (int64_t)BH + 15) / 8 * 8));
#define DQ_ARGS Qv, Kv, Vv, dOv, LSE, ws.delta, blk_off, blk_ptr, q_idx, ws.tile_desc, ws.head_base, BH, ws.dQpart, Hh, (int)S, n_blocks, (long long)nnz_capacity, scale_log2, kv_rows
            if (D == 128) attn_bwd_dq_mfma_kernel<128><<<grid, dim3(256), 0, st>>>(DQ_ARGS);
            else attn_bwd_dq_mfma_kernel<64><<<grid, dim3(256), 0, st>>>(DQ_ARGS);
#undef DQ_ARGS
        }
        VMOBA_PROFILE_END(1, st);
        VMOBA_CHECK_LAUNCH();
        const int qpw = 256 / (D / (bf16 ? 8 : 4));     // partials: bfloat16 from the MFMA tile kernel, float32 otherwise
        dim3 mgrid((unsigned)ceil_div64(S, qpw), (unsigned)BH);
#define MG_ARGS ws.dQpart, row_ptr, pair_pos, dQv, rows, Hh, (int)S, (long long)nnz_capacity, softmax_scale
        if (bf16 && D == 128) dq_merge_kernel<true, 128><<<mgrid, dim3(256), 0, st>>>(MG_ARGS);
        else if (bf16) dq_merge_kernel<true, 64><<<mgrid, dim3(256), 0, st>>>(MG_ARGS);
        else if (D == 128) dq_merge_kernel<false, 128><<<mgrid, dim3(256), 0, st>>>(MG_ARGS);
        else dq_merge_kernel<false, 64><<<mgrid, dim3(256), 0, st>>>(MG_ARGS);
#undef MG_ARGS
        VMOBA_CHECK_LAUNCH();
    }
    // ---- dK, dV
    {
        const int KPW = simple ? 64 : 128;      // keys per workgroup
        key_run_order_kernel<<<dim3(BH), dim3(VMOBA_MAX_BLOCKS), 0, st>>>(blk_off, blk_ptr, ws.kb_start, ws.kb_order, n_blocks, KPW, simple ? 0 : 32);
        VMOBA_CHECK_LAUNCH();
        // a multiple of 8 so that (workgroup id % 8) is the same for every head; + 8 for the per-XCD rounding
        dim3 grid((unsigned)((S / KPW + n_blocks + 7) / 8 * 8 + 8 + (simple ? 0 : n_blocks)), (unsigned)BH);
        // slots of the matrix-core kernel in groups of one block's runs (the usual block: S / n_blocks keys, a last run of at
        // most 32 keys goes to the tail workgroups)
        const int64_t usual = S / n_blocks;
        const int group = (int)std::max<int64_t>(1, (usual % KPW > 0 && usual % KPW <= 32) ? usual / KPW : ceil_div64(usual, KPW));
        const int slots = (int)ceil_div64(grid.x, group) * group;
        VMOBA_PROFILE_BEGIN(2, st);
        const int32_t* krows = key_rows ? key_rows : rows;      // row map of dK and dV
#define DKV_ARGS Qv, Kv, Vv, dOv, LSE, ws.delta, blk_off, blk_ptr, q_idx, ws.kb_start, ws.kb_order, dKv, dVv, krows, Hh, (int)S, n_blocks, (long long)nnz_capacity, scale_log2, softmax_scale, kv_rows
        if (simple) {
            if (D == 128) attn_bwd_dkv_simple_kernel<128><<<grid, dim3(64), 0, st>>>(DKV_ARGS);
            else attn_bwd_dkv_simple_kernel<64><<<grid, dim3(64), 0, st>>>(DKV_ARGS);
        } else {
            const dim3 hgrid((unsigned)(ceil_div64((int64_t)BH * slots, 8) * 8 + 7 * group));   // see the kernel
            if (D == 128) attn_bwd_dkv_kernel<128><<<hgrid, dim3(256), 0, st>>>(DKV_ARGS, BH, slots, group);
            else attn_bwd_dkv_kernel<64><<<hgrid, dim3(256), 0, st>>>(DKV_ARGS, BH, slots, group);
        }
#undef DKV_ARGS
        VMOBA_PROFILE_END(2, st);
        VMOBA_CHECK_LAUNCH();
    }
    return VMOBA_OK;
}
