// vmoba_attn_fwd: Step 3 of Sec. 3.1 -- every query attends to the keys/values of its selected
// blocks only.
//
// Two phases.  (1) Tile kernel, block-major: a workgroup takes TM gathered queries of one key
// block j and runs flash-attention (online soft-max) over the L_j keys of that block alone,
// writing a normalised partial output and its log-sum-exp per (query, block) pair.  (2) Merge
// kernel, query-major: the partials of a query's selected blocks are combined with weights
// exp(lse_pair - LSE).  bfloat16 inputs use the 32x32x16 bf16 MFMA; float32 inputs use a plain
// FMA kernel of the same structure.
#include "attn_common.h"

#include <algorithm>
#include <cmath>

__global__ __launch_bounds__(64) void tile_start_kernel(const int* __restrict__ blk_ptr, int* __restrict__ tile_start,
                                                        int BH, int nb, int TM) {
    const int bh = blockIdx.x * 64 + threadIdx.x;
    if (bh >= BH) return;
    const int* bp = blk_ptr + (long long)bh * (nb + 1);
    int* ts = tile_start + (long long)bh * (nb + 1);
    int run = 0;
    for (int j = 0; j < nb; ++j) {
        ts[j] = run;
        run += (bp[j + 1] - bp[j] + TM - 1) / TM;
    }
    ts[nb] = run;
}

__global__ __launch_bounds__(256) void tile_desc_kernel(const int* __restrict__ tile_start, const int* __restrict__ blk_ptr,
                                                        const int* __restrict__ blk_off, int4* __restrict__ tile_desc,
                                                        int nb, int TM, int tiles_per_head) {
    const int bh = blockIdx.y;
    const int tile = blockIdx.x * 256 + threadIdx.x;
    if (tile >= tiles_per_head) return;
    const int* ts = tile_start + (long long)bh * (nb + 1);
    int4 d = {0, 0, 0, 0};
    if (tile < ts[nb]) {
        int lo = 0, hi = nb;           // largest j with ts[j] <= tile
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (ts[mid] <= tile) lo = mid; else hi = mid;
        }
        const int* bp = blk_ptr + (long long)bh * (nb + 1);
        const int t0 = (tile - ts[lo]) * TM;
        d.x = bp[lo] + t0;
        d.y = min(TM, bp[lo + 1] - bp[lo] - t0);
        d.z = blk_off[lo];
        d.w = blk_off[lo + 1] - blk_off[lo];
    }
    tile_desc[(long long)bh * tiles_per_head + tile] = d;
}

namespace {

constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

// ---------------------------------------------------------------------------------------------
// Plain FMA tile kernel (float32 or bfloat16 inputs, float32 arithmetic).  One wavefront per
// tile of 64 gathered queries, lane = query.  Keys and values of the block pass through LDS in
// chunks of KC rows.
template <bool BF16, int D>
__global__ __launch_bounds__(64) void attn_fwd_tile_simple_kernel(
    TensorView Q, TensorView K, TensorView V, const int* __restrict__ blk_off, const int* __restrict__ blk_ptr,
    const int* __restrict__ q_idx, const int4* __restrict__ tile_desc, int tiles_per_head, float* __restrict__ Opart,
    float* __restrict__ lse_part, int Hh, int nb, long long cap, float scale_log2) {
    constexpr int TM = 64, KC = 32;
    constexpr int ES = BF16 ? 2 : 4;
    __shared__ float sK[KC][D];
    __shared__ float sV[KC][D];
    const int bh = blockIdx.y, b = bh / Hh, h = bh % Hh;
    TileCoord tc;
    if (!find_tile(tile_desc, tiles_per_head, bh, blockIdx.x, tc)) return;
    const int lane = threadIdx.x;
    const long long seg = (long long)bh * cap;
    const int e = min(lane, tc.count - 1);
    const int q = q_idx[seg + tc.list0 + tc.t0 + e];
    float qr[D], o[D];
    {
        const char* src = Q.ptr + ((long long)b * Q.stride_b + (long long)q * Q.stride_s + (long long)h * Q.stride_h) * ES;
#pragma unroll
        for (int d = 0; d < D; ++d) {
            qr[d] = BF16 ? bf16_bits_to_f32(reinterpret_cast<const uint16_t*>(src)[d])
                         : reinterpret_cast<const float*>(src)[d];
            o[d] = 0.f;
        }
    }
    float m = -INFINITY, l = 0.f;
    const char* kbase = K.ptr + ((long long)b * K.stride_b + (long long)h * K.stride_h) * ES;
    const char* vbase = V.ptr + ((long long)b * V.stride_b + (long long)h * V.stride_h) * ES;
    for (int c0 = 0; c0 < tc.L; c0 += KC) {
        const int kc = min(KC, tc.L - c0);
        __syncthreads();
        for (int i = lane; i < kc * D; i += 64) {
            const int r = i / D, d = i % D;
            const long long row = tc.k0 + c0 + r;
            const char* ks = kbase + row * K.stride_s * ES;
            const char* vs = vbase + row * V.stride_s * ES;
            sK[r][d] = BF16 ? bf16_bits_to_f32(reinterpret_cast<const uint16_t*>(ks)[d]) : reinterpret_cast<const float*>(ks)[d];
            sV[r][d] = BF16 ? bf16_bits_to_f32(reinterpret_cast<const uint16_t*>(vs)[d]) : reinterpret_cast<const float*>(vs)[d];
        }
        __syncthreads();
        for (int r = 0; r < kc; ++r) {
            float a = 0.f;
#pragma unroll
            for (int d = 0; d < D; ++d) a = fmaf(qr[d], sK[r][d], a);
            a *= scale_log2;
            const float mc = fmaxf(m, a);
            const float alpha = exp2f(m - mc);
            const float p = exp2f(a - mc);
            l = l * alpha + p;
#pragma unroll
            for (int d = 0; d < D; ++d) o[d] = fmaf(p, sV[r][d], o[d] * alpha);
            m = mc;
        }
    }
    if (lane < tc.count) {
        const long long pair = seg + tc.list0 + tc.t0 + lane;
        const float inv = 1.f / l;
        float* dst = Opart + pair * D;
#pragma unroll
        for (int d = 0; d < D; ++d) dst[d] = o[d] * inv;
        lse_part[pair] = (m + log2f(l)) * LN2;
    }
}

// ---------------------------------------------------------------------------------------------
// bf16 MFMA tile kernel.  4 wavefronts; wavefront w owns NQ groups of 32 gathered queries
// (TM = 128 * NQ per workgroup) and walks the block's keys in chunks of 64.
//
// All products are computed transposed so that the query index is the MFMA column (= lane % 32):
//   S^T[key, q] = K[key, :] . Q[q, :]          A = K rows from LDS, B = Q^T held in registers
//   O^T[d, q]  += V^T[d, key] . P^T[key, q]    A = V^T by transpose reads, B = P^T packed from S^T
// With the query on the lane, the row maximum and row sum of the online soft-max are reductions
// over a lane's own registers plus one exchange with lane ^ 32.  The running maximum is only
// raised when a chunk exceeds it by more than 2^8 (the probabilities then stay below 2^8, well
// inside float32/bf16 range), so the accumulator rescale is rare; the final division by the row
// sum makes the result independent of which maximum was used.
template <int D, int NQ>
__global__ __launch_bounds__(256, (NQ == 1 ? 2 : 1)) void attn_fwd_tile_mfma_kernel(
    TensorView Q, TensorView K, TensorView V, const int* __restrict__ blk_off, const int* __restrict__ blk_ptr,
    const int* __restrict__ q_idx, const int4* __restrict__ tile_desc, int tiles_per_head, float* __restrict__ Opart,
    float* __restrict__ lse_part, int Hh, int nb, long long cap, float scale_log2) {
    constexpr int TM = 128 * NQ;
    constexpr int KC = 64;                  // keys per chunk
    constexpr int STR = D + 8;              // LDS row stride (bf16 elements)
    constexpr int KSTEPS = D / 16;          // MFMA k-steps of the first product
    constexpr int DT = D / 32;              // 32-row tiles of O^T
    constexpr int LOADS = KC * D * 2 / 16 / 256;   // 16-byte pieces per thread per chunk and tensor
    constexpr float LAZY = 8.f;
    __shared__ __align__(16) __bf16 sK[KC * STR];
    __shared__ __align__(16) __bf16 sV[KC * STR];

    const int bh = blockIdx.y, b = bh / Hh, h = bh % Hh;
    TileCoord tc;
    if (!find_tile(tile_desc, tiles_per_head, bh, blockIdx.x, tc)) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hf = lane >> 5;
    const long long seg = (long long)bh * cap;

    // ---- Q^T operand: lane holds, for each of its NQ queries, 8 channels per k-step
    bf16x8_t qf[NQ][KSTEPS];
    int my_entry[NQ];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        const int ent = (wave * NQ + nq) * 32 + l32;          // entry inside the tile
        my_entry[nq] = ent;
        const int e = min(ent, tc.count - 1);                 // surplus rows repeat the last query
        const int q = q_idx[seg + tc.list0 + tc.t0 + e];
        const char* src = Q.ptr + ((long long)b * Q.stride_b + (long long)q * Q.stride_s + (long long)h * Q.stride_h) * 2;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks)
            qf[nq][ks] = *reinterpret_cast<const bf16x8_t*>(src + (ks * 16 + hf * 8) * 2);
    }

    f32x16_t oacc[NQ][DT];
    float m_run[NQ], l_run[NQ];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        m_run[nq] = -INFINITY;
        l_run[nq] = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[nq][dt][i] = 0.f;
    }

    const char* kbase = K.ptr + ((long long)b * K.stride_b + (long long)h * K.stride_h) * 2;
    const char* vbase = V.ptr + ((long long)b * V.stride_b + (long long)h * V.stride_h) * 2;
    const long long kss = K.stride_s * 2, vss = V.stride_s * 2;
    const int n_chunks = (tc.L + KC - 1) / KC;

    u32x4_t kreg[LOADS], vreg[LOADS];
    auto prefetch = [&](int c) {
        const int c0 = c * KC;
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            const int piece = tid + 256 * i;
            const int r = piece / (D / 8), pc = piece % (D / 8);
            const long long row = tc.k0 + min(c0 + r, tc.L - 1);   // rows past the block repeat its last key
            kreg[i] = *reinterpret_cast<const u32x4_t*>(kbase + row * kss + pc * 16);
            vreg[i] = *reinterpret_cast<const u32x4_t*>(vbase + row * vss + pc * 16);
        }
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
    const __bf16* sV_lane = sV + tr_lane_offset<STR>(lane);

    prefetch(0);
    for (int c = 0; c < n_chunks; ++c) {
        __syncthreads();                      // everyone is done reading the previous chunk
        stage();
        __syncthreads();
        if (c + 1 < n_chunks) prefetch(c + 1);

        const int valid = tc.L - c * KC;      // keys of this chunk inside the block (may exceed KC)
        const int n_mt = valid > 32 ? 2 : 1;  // 32-key groups with at least one valid key

        // ---- S^T = K . Q^T
        f32x16_t sacc[NQ][2];
        const f32x16_t zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            if (mt < n_mt) {
#pragma unroll
                for (int ks = 0; ks < KSTEPS; ++ks) {
                    const bf16x8_t kf = *reinterpret_cast<const bf16x8_t*>(sK_lane + mt * 32 * STR + ks * 16);
#pragma unroll
                    for (int nq = 0; nq < NQ; ++nq)
                        sacc[nq][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[nq][ks], ks == 0 ? zero16 : sacc[nq][mt], 0, 0, 0);
                }
            } else {
#pragma unroll
                for (int nq = 0; nq < NQ; ++nq) sacc[nq][mt] = zero16;   // masked to -inf below
            }
        }
        __builtin_amdgcn_s_setprio(0);
        if (valid < KC) {                     // last chunk: keys past the block get -inf
#pragma unroll
            for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        if (mt * 32 + acc_row(i, hf) >= valid) sacc[nq][mt][i] = -INFINITY;
        }
        // ---- online soft-max (per lane = per query), in base-2 units
        bf16x8_t pf[NQ][2][2];
        bool need_rescale = false;
        float alpha[NQ];
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq) {
            float mx = sacc[nq][0][0];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[nq][mt][i]);
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * scale_log2;       // scale_log2 > 0
            const bool raise = mx > m_run[nq] + LAZY;
            const float m_new = raise ? mx : m_run[nq];
            alpha[nq] = raise ? exp2_raw(m_run[nq] - m_new) : 1.f;
            need_rescale |= raise;
            m_run[nq] = m_new;
            float rs = 0.f;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                float p[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    p[i] = exp2_raw(fmaf(sacc[nq][mt][i], scale_log2, -m_new));
                    rs += p[i];
                }
                pf[nq][mt][0] = pack8(&p[0]);
                pf[nq][mt][1] = pack8(&p[8]);
            }
            rs += __shfl_xor(rs, 32, 64);
            l_run[nq] = l_run[nq] * alpha[nq] + rs;
        }
        if (__any(need_rescale)) {
#pragma unroll
            for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int i = 0; i < 16; ++i) oacc[nq][dt][i] *= alpha[nq];
        }
        // ---- O^T += V^T . P^T
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            if (mt < n_mt) {
#pragma unroll
                for (int s = 0; s < 2; ++s) {
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt) {
                        const bf16x8_t vf = tr_operand<STR>(sV_lane, mt * 32, s, dt * 32);
#pragma unroll
                        for (int nq = 0; nq < NQ; ++nq)
                            oacc[nq][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[nq][mt][s], oacc[nq][dt], 0, 0, 0);
                    }
                }
            }
        }
        __builtin_amdgcn_s_setprio(0);
    }

    // ---- partial output: O^T value i of tile dt <-> channel 32*dt + 8*(i>>2) + 4*hf + (i&3)
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        if (my_entry[nq] < tc.count) {
            const long long pair = seg + tc.list0 + tc.t0 + my_entry[nq];
            const float inv = 1.f / l_run[nq];
            uint16_t* dst = reinterpret_cast<uint16_t*>(Opart) + pair * D;      // bf16 partials
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    u32x2_t v;
                    v.x = pack_bf16x2(oacc[nq][dt][4 * g + 0] * inv, oacc[nq][dt][4 * g + 1] * inv);
                    v.y = pack_bf16x2(oacc[nq][dt][4 * g + 2] * inv, oacc[nq][dt][4 * g + 3] * inv);
                    *reinterpret_cast<u32x2_t*>(dst + dt * 32 + g * 8 + hf * 4) = v;
                }
            if (hf == 0) lse_part[pair] = (m_run[nq] + log2f(l_run[nq])) * LN2;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// bf16 MFMA tile kernel, two-group variant.  8 wavefronts = 2 groups of 4; each group owns 128 of
// the tile's 256 gathered queries (32 per wavefront) and both walk the same 64-key chunks, so a
// chunk is staged once for 256 queries.  Time is cut into slots separated by workgroup barriers;
// in every slot one group runs its matrix phase (S^T of chunk i, O^T += V^T P^T of chunk i-1) while
// the other runs its soft-max phase, then they swap.  Each SIMD hosts one wavefront of either
// group, so its matrix pipe and its vector ALU are busy at the same time by construction.
//   group g: matrix phase of chunk i in slot 2i+g, soft-max of chunk i in slot 2i+g+1.
// LDS: K and V chunks double-buffered.  K(i) is read in slots 2i, 2i+1 and V(i) in slots 2i+2, 2i+3;
// at the start of every even slot 2m all threads store K(m+1) and V(m) (fetched two slots earlier
// into registers) and issue the global loads of K(m+2) and V(m+1).
template <int D>
__global__ __launch_bounds__(512, 2) void attn_fwd_tile_pp_kernel(
    TensorView Q, TensorView K, TensorView V, const int* __restrict__ blk_off, const int* __restrict__ blk_ptr,
    const int* __restrict__ q_idx, const int4* __restrict__ tile_desc, int tiles_per_head, float* __restrict__ Opart,
    float* __restrict__ lse_part, int Hh, int nb, long long cap, float scale_log2) {
    constexpr int TM = 256, KC = 64, STR = D + 8;
    constexpr int KSTEPS = D / 16, DT = D / 32;
    constexpr int LOADS = KC * D * 2 / 16 / 512;      // 16-byte pieces per thread per chunk and tensor
    constexpr float LAZY = 8.f;
    __shared__ __align__(16) __bf16 sK[2][KC * STR];
    __shared__ __align__(16) __bf16 sV[2][KC * STR];

    const int bh = blockIdx.y, b = bh / Hh, h = bh % Hh;
    TileCoord tc;
    if (!find_tile(tile_desc, tiles_per_head, bh, blockIdx.x, tc)) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int grp = wave >> 2;
    const int l32 = lane & 31, hf = lane >> 5;
    const long long seg = (long long)bh * cap;

    const int ent = grp * 128 + (wave & 3) * 32 + l32;
    bf16x8_t qf[KSTEPS];
    {
        const int e = min(ent, tc.count - 1);
        const int q = q_idx[seg + tc.list0 + tc.t0 + e];
        const char* src = Q.ptr + ((long long)b * Q.stride_b + (long long)q * Q.stride_s + (long long)h * Q.stride_h) * 2;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8_t*>(src + (ks * 16 + hf * 8) * 2);
    }
    f32x16_t oacc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[dt][i] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    const char* kbase = K.ptr + ((long long)b * K.stride_b + (long long)h * K.stride_h) * 2;
    const char* vbase = V.ptr + ((long long)b * V.stride_b + (long long)h * V.stride_h) * 2;
    const long long kss = K.stride_s * 2, vss = V.stride_s * 2;
    const int n = (tc.L + KC - 1) / KC;

    u32x4_t kreg[LOADS], vreg[LOADS];
    auto load_k = [&](int c) {       // chunk index may run past the block: rows are clamped to its last key
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            const int piece = tid + 512 * i;
            const int r = piece / (D / 8), pc = piece % (D / 8);
            const long long row = tc.k0 + min(c * KC + r, tc.L - 1);
            kreg[i] = *reinterpret_cast<const u32x4_t*>(kbase + row * kss + pc * 16);
        }
    };
    auto load_v = [&](int c) {
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            const int piece = tid + 512 * i;
            const int r = piece / (D / 8), pc = piece % (D / 8);
            const long long row = tc.k0 + min(c * KC + r, tc.L - 1);
            vreg[i] = *reinterpret_cast<const u32x4_t*>(vbase + row * vss + pc * 16);
        }
    };
    auto store_k = [&](int buf) {
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            const int piece = tid + 512 * i;
            const int r = piece / (D / 8), pc = piece % (D / 8);
            *reinterpret_cast<u32x4_t*>(&sK[buf][r * STR + pc * 8]) = kreg[i];
        }
    };
    auto store_v = [&](int buf) {
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            const int piece = tid + 512 * i;
            const int r = piece / (D / 8), pc = piece % (D / 8);
            *reinterpret_cast<u32x4_t*>(&sV[buf][r * STR + pc * 8]) = vreg[i];
        }
    };
    const int k_lane = rho(l32) * STR + hf * 8;
    const int v_lane = tr_lane_offset<STR>(lane);

    // prologue: K(0) in place, K(1) and V(0) in flight
    load_k(0);
    store_k(0);
    load_k(1);
    load_v(0);
    __syncthreads();

    f32x16_t sacc[2];
    bf16x8_t pf[2][2];
    const f32x16_t zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const int n_slots = 2 * n + 2;
    for (int sigma = 0; sigma < n_slots; ++sigma) {
        if ((sigma & 1) == 0) {
            const int m = sigma >> 1;
            store_k((m + 1) & 1);       // K(m+1)
            store_v(m & 1);             // V(m)
            load_k(m + 2);
            load_v(m + 1);
        }
        const int phase = sigma - grp;
        const int i = phase >> 1;
        if (phase >= 0 && (phase & 1) == 0) {
            // ---- matrix phase: S^T(i) = K(i) . Q^T ;  O^T += V(i-1)^T . P(i-1)^T
            __builtin_amdgcn_s_setprio(1);
            if (i < n) {
                const __bf16* kt = &sK[i & 1][0] + k_lane;
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int ks = 0; ks < KSTEPS; ++ks) {
                        const bf16x8_t kf = *reinterpret_cast<const bf16x8_t*>(kt + mt * 32 * STR + ks * 16);
                        sacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], ks == 0 ? zero16 : sacc[mt], 0, 0, 0);
                    }
            }
            if (i >= 1) {
                const __bf16* vt = &sV[(i - 1) & 1][0] + v_lane;
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int s = 0; s < 2; ++s)
#pragma unroll
                        for (int dt = 0; dt < DT; ++dt) {
                            const bf16x8_t vf = tr_operand<STR>(vt, mt * 32, s, dt * 32);
                            oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[mt][s], oacc[dt], 0, 0, 0);
                        }
            }
            __builtin_amdgcn_s_setprio(0);
        } else if (phase >= 0 && i < n) {
            // ---- soft-max phase of chunk i (per lane = per query), base-2 units
            const int valid = tc.L - i * KC;
            if (valid < KC) {
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        if (mt * 32 + acc_row(v, hf) >= valid) sacc[mt][v] = -INFINITY;
            }
            float mx = sacc[0][0];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int v = 0; v < 16; ++v) mx = fmaxf(mx, sacc[mt][v]);
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * scale_log2;
            const bool raise = mx > m_run + LAZY;
            const float m_new = raise ? mx : m_run;
            const float alpha = raise ? exp2_raw(m_run - m_new) : 1.f;
            m_run = m_new;
            float rs = 0.f;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                float p[16];
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    p[v] = exp2_raw(fmaf(sacc[mt][v], scale_log2, -m_new));
                    rs += p[v];
                }
                pf[mt][0] = pack8(&p[0]);
                pf[mt][1] = pack8(&p[8]);
            }
            rs += __shfl_xor(rs, 32, 64);
            l_run = l_run * alpha + rs;
            if (__any(raise)) {
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) oacc[dt][v] *= alpha;
            }
        }
        __syncthreads();
    }

    if (ent < tc.count) {
        const long long pair = seg + tc.list0 + tc.t0 + ent;
        const float inv = 1.f / l_run;
        uint16_t* dst = reinterpret_cast<uint16_t*>(Opart) + pair * D;      // bf16 partials
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                u32x2_t v;
                v.x = pack_bf16x2(oacc[dt][4 * g + 0] * inv, oacc[dt][4 * g + 1] * inv);
                v.y = pack_bf16x2(oacc[dt][4 * g + 2] * inv, oacc[dt][4 * g + 3] * inv);
                *reinterpret_cast<u32x2_t*>(dst + dt * 32 + g * 8 + hf * 4) = v;
            }
        if (hf == 0) lse_part[pair] = (m_run + log2f(l_run)) * LN2;
    }
}

// ---------------------------------------------------------------------------------------------
// Merge: O[q] = sum_pairs exp(lse_pair - LSE[q]) * Opart[pair], LSE[q] = logsumexp(lse_pair).
// A group of lanes per query, each owning CH consecutive channels (one 16-byte load per partial).
// Partials are bfloat16 when the MFMA tile kernels wrote them (PBF16), float32 otherwise.
template <bool BF16, bool PBF16, int D>
__global__ __launch_bounds__(256) void attn_fwd_merge_kernel(const float* __restrict__ Opart, const float* __restrict__ lse_part,
                                                             const int* __restrict__ row_ptr, const int* __restrict__ pair_pos,
                                                             TensorView O, float* __restrict__ LSE,
                                                             const int* __restrict__ out_rows, int Hh, int S, long long cap) {
    constexpr int CH = PBF16 ? 8 : 4;
    constexpr int LPQ = D / CH;              // lanes per query
    constexpr int QPW = 256 / LPQ;           // queries per workgroup
    const int bh = blockIdx.y, b = bh / Hh, h = bh % Hh;
    const int q = blockIdx.x * QPW + threadIdx.x / LPQ;
    const int part = threadIdx.x % LPQ;
    if (q >= S) return;
    const int r0 = row_ptr[(long long)bh * (S + 1) + q], r1 = row_ptr[(long long)bh * (S + 1) + q + 1];
    const long long seg = (long long)bh * cap;
    // one pass with a running maximum; four partials in flight per step (index -> lse and row loads)
    float mx = -INFINITY;
    float acc[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) acc[c] = 0.f;
    float wsum = 0.f;
    for (int r = r0; r < r1; r += 4) {
        long long pair[4];
        float l[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) pair[u] = seg + pair_pos[seg + min(r + u, r1 - 1)];
#pragma unroll
        for (int u = 0; u < 4; ++u) l[u] = (r + u < r1) ? lse_part[pair[u]] : -INFINITY;
        float v[4][CH];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if constexpr (PBF16) {
                const u32x4_t x = *reinterpret_cast<const u32x4_t*>(reinterpret_cast<const uint16_t*>(Opart) + pair[u] * D + part * 8);
                v[u][0] = bf16lo_to_f32(x.x); v[u][1] = bf16hi_to_f32(x.x); v[u][2] = bf16lo_to_f32(x.y); v[u][3] = bf16hi_to_f32(x.y);
                v[u][4 % CH] = bf16lo_to_f32(x.z); v[u][5 % CH] = bf16hi_to_f32(x.z);
                v[u][6 % CH] = bf16lo_to_f32(x.w); v[u][7 % CH] = bf16hi_to_f32(x.w);
            } else {
                const f32x4_t x = *reinterpret_cast<const f32x4_t*>(Opart + pair[u] * D + part * 4);
                v[u][0] = x.x; v[u][1] = x.y; v[u][2] = x.z; v[u][3] = x.w;
            }
        }
        const float m_new = fmaxf(fmaxf(mx, fmaxf(l[0], l[1])), fmaxf(l[2], l[3]));
        const float alpha = expf(mx - m_new);          // exp(-inf) = 0 on the first step (m_new is finite: l[0] is)
        wsum *= alpha;
#pragma unroll
        for (int c = 0; c < CH; ++c) acc[c] *= alpha;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float w = expf(l[u] - m_new);        // 0 for the padding entries
            wsum += w;
#pragma unroll
            for (int c = 0; c < CH; ++c) acc[c] += w * v[u][c];
        }
        mx = m_new;
    }
    float lse = -INFINITY;
    if (r1 > r0) {
        const float inv = 1.f / wsum;
#pragma unroll
        for (int c = 0; c < CH; ++c) acc[c] *= inv;
        lse = mx + logf(wsum);
    }
    const int qo = out_rows ? out_rows[q] : q;       // row of O that block-order row q is written to
    char* dst = O.ptr + ((long long)b * O.stride_b + (long long)qo * O.stride_s + (long long)h * O.stride_h) * (BF16 ? 2 : 4);
    if constexpr (BF16) {
        uint32_t w[CH / 2];
#pragma unroll
        for (int c = 0; c < CH / 2; ++c) w[c] = pack_bf16x2(acc[2 * c], acc[2 * c + 1]);
        if constexpr (CH == 8) {
            u32x4_t o = {w[0], w[1], w[2], w[3]};
            *reinterpret_cast<u32x4_t*>(dst + part * 16) = o;
        } else {
            u32x2_t o = {w[0], w[1]};
            *reinterpret_cast<u32x2_t*>(dst + part * 8) = o;
        }
    } else {
#pragma unroll
        for (int c = 0; c < CH; c += 4) {
            f32x4_t o = {acc[c], acc[c + 1], acc[c + 2], acc[c + 3]};
            *reinterpret_cast<f32x4_t*>(dst + (part * CH + c) * 4) = o;
        }
    }
    if (part == 0) LSE[(long long)bh * S + q] = lse;
}

struct FwdWs {
    float* Opart;      // [BH * cap][D]
    float* lse_part;   // [BH * cap]
    int* tile_start;   // [BH][nb + 1]
    int4* tile_desc;   // [BH][tiles_per_head]
    size_t total;
};

}  // namespace
// Grid width (tiles per head) for tiles of TM list entries: a host-side bound on sum_j ceil(cnt_j / TM).
int64_t vmoba_max_tiles(int64_t cap, int TM) { return (cap / TM + VMOBA_MAX_BLOCKS + 7) / 8 * 8; }
namespace {

FwdWs carve_fwd(void* base, int BH, int D, int64_t cap, int nb) {
    FwdWs w;
    char* p = (char*)base;
    size_t off = 0;
    w.Opart = (float*)(p + off);     off += align_up((size_t)BH * cap * D * 4, 256);
    w.lse_part = (float*)(p + off);  off += align_up((size_t)BH * cap * 4, 256);
    w.tile_start = (int*)(p + off);  off += align_up((size_t)BH * (VMOBA_MAX_BLOCKS + 1) * 4, 256);
    w.tile_desc = (int4*)(p + off);  off += align_up((size_t)BH * vmoba_max_tiles(cap, 64) * 16, 256);
    (void)nb;
    w.total = off;
    return w;
}

}  // namespace

size_t vmoba_attn_fwd_workspace_bytes(int B, int Hh, int64_t S, int D, int64_t cap, int dtype) {
    (void)S; (void)dtype;
    return carve_fwd(nullptr, B * Hh, D, cap, 0).total;
}

// Which MFMA tile width the bf16 path uses (queries per workgroup = 128 * NQ).
int vmoba_fwd_nq() {
    const char* e = getenv("VMOBA_FWD_NQ");
    int v = e ? atoi(e) : 1;      // 1: two workgroups per CU (measured faster); 2: wider tile, one per CU
    return (v == 2) ? 2 : 1;
}

extern "C" int vmoba_attn_fwd(int B, int Hh, int64_t S, int D, int32_t n_blocks, const int32_t* blk_off,
                              const vmoba_tensor* Qp, const vmoba_tensor* Kp, const vmoba_tensor* Vp,
                              const int32_t* blk_ptr, const int32_t* q_idx, const int32_t* row_ptr,
                              const int32_t* pair_pos, int64_t nnz_capacity, float softmax_scale,
                              const vmoba_tensor* O, float* LSE, const int32_t* out_rows, void* workspace,
                              size_t workspace_bytes, void* stream) {
    if (B <= 0 || Hh <= 0 || S <= 0 || n_blocks <= 0 || nnz_capacity <= 0) return VMOBA_ERR_INVALID_ARG;
    if (!blk_off || !blk_ptr || !q_idx || !row_ptr || !pair_pos || !LSE || !workspace) return VMOBA_ERR_INVALID_ARG;
    if (!tensor_ok(Qp) || !tensor_ok(Kp) || !tensor_ok(Vp) || !tensor_ok(O)) return VMOBA_ERR_INVALID_ARG;
    if (!std::isfinite(softmax_scale)) return VMOBA_ERR_INVALID_ARG;
    if (D != 64 && D != 128) return VMOBA_ERR_UNSUPPORTED;
    if (n_blocks > VMOBA_MAX_BLOCKS) return VMOBA_ERR_UNSUPPORTED;
    const int dt = Qp->dtype;
    if (Kp->dtype != dt || Vp->dtype != dt || O->dtype != dt) return VMOBA_ERR_UNSUPPORTED;
    const int BH = B * Hh;
    if (nnz_capacity > INT32_MAX || (int64_t)BH * nnz_capacity * D > ((int64_t)1 << 40)) return VMOBA_ERR_UNSUPPORTED;
    FwdWs ws = carve_fwd(workspace, BH, D, nnz_capacity, n_blocks);
    if (workspace_bytes < ws.total) return VMOBA_ERR_WORKSPACE;
    if (((uintptr_t)workspace) & 255) return VMOBA_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    const bool bf16 = dt == VMOBA_BF16;
    const TensorView Qv = make_view(Qp), Kv = make_view(Kp), Vv = make_view(Vp), Ov = make_view(O);
    const float scale_log2 = softmax_scale * LOG2E;
    const bool simple = !bf16 || getenv("VMOBA_FORCE_SIMPLE") != nullptr;
    const int nq = vmoba_fwd_nq();
    const char* ppe = getenv("VMOBA_FWD_PP");
    const bool two_group = ppe ? atoi(ppe) != 0 : false;
    const int TM = simple ? 64 : (two_group ? 256 : 128 * nq);
    tile_start_kernel<<<dim3((BH + 63) / 64), dim3(64), 0, st>>>(blk_ptr, ws.tile_start, BH, n_blocks, TM);
    VMOBA_CHECK_LAUNCH();
    const int64_t max_tiles = std::min<int64_t>(vmoba_max_tiles(nnz_capacity, TM), (nnz_capacity / TM + n_blocks + 7) / 8 * 8);
    tile_desc_kernel<<<dim3((unsigned)ceil_div64(max_tiles, 256), (unsigned)BH), dim3(256), 0, st>>>(
        ws.tile_start, blk_ptr, blk_off, ws.tile_desc, n_blocks, TM, (int)max_tiles);
    VMOBA_CHECK_LAUNCH();
    dim3 grid((unsigned)max_tiles, (unsigned)BH);
    VMOBA_PROFILE_BEGIN(0, st);
#define TILE_ARGS Qv, Kv, Vv, blk_off, blk_ptr, q_idx, ws.tile_desc, (int)max_tiles, ws.Opart, ws.lse_part, Hh, n_blocks, (long long)nnz_capacity, scale_log2
    if (simple) {
        if (bf16 && D == 128) attn_fwd_tile_simple_kernel<true, 128><<<grid, dim3(64), 0, st>>>(TILE_ARGS);
        else if (bf16) attn_fwd_tile_simple_kernel<true, 64><<<grid, dim3(64), 0, st>>>(TILE_ARGS);
        else if (D == 128) attn_fwd_tile_simple_kernel<false, 128><<<grid, dim3(64), 0, st>>>(TILE_ARGS);
        else attn_fwd_tile_simple_kernel<false, 64><<<grid, dim3(64), 0, st>>>(TILE_ARGS);
    } else if (two_group) {
        if (D == 128) attn_fwd_tile_pp_kernel<128><<<grid, dim3(512), 0, st>>>(TILE_ARGS);
        else attn_fwd_tile_pp_kernel<64><<<grid, dim3(512), 0, st>>>(TILE_ARGS);
    } else {
        if (D == 128 && nq == 2) attn_fwd_tile_mfma_kernel<128, 2><<<grid, dim3(256), 0, st>>>(TILE_ARGS);
        else if (D == 128) attn_fwd_tile_mfma_kernel<128, 1><<<grid, dim3(256), 0, st>>>(TILE_ARGS);
        else if (nq == 2) attn_fwd_tile_mfma_kernel<64, 2><<<grid, dim3(256), 0, st>>>(TILE_ARGS);
        else attn_fwd_tile_mfma_kernel<64, 1><<<grid, dim3(256), 0, st>>>(TILE_ARGS);
    }
#undef TILE_ARGS
    VMOBA_PROFILE_END(0, st);
    VMOBA_CHECK_LAUNCH();
    const bool pbf16 = !simple;               // the MFMA tile kernels write bfloat16 partials
    const int qpw = 256 / (D / (pbf16 ? 8 : 4));
    dim3 mgrid((unsigned)ceil_div64(S, qpw), (unsigned)BH);
#define MERGE_ARGS ws.Opart, ws.lse_part, row_ptr, pair_pos, Ov, LSE, out_rows, Hh, (int)S, (long long)nnz_capacity
    if (pbf16 && D == 128) attn_fwd_merge_kernel<true, true, 128><<<mgrid, dim3(256), 0, st>>>(MERGE_ARGS);
    else if (pbf16) attn_fwd_merge_kernel<true, true, 64><<<mgrid, dim3(256), 0, st>>>(MERGE_ARGS);
    else if (bf16 && D == 128) attn_fwd_merge_kernel<true, false, 128><<<mgrid, dim3(256), 0, st>>>(MERGE_ARGS);
    else if (bf16) attn_fwd_merge_kernel<true, false, 64><<<mgrid, dim3(256), 0, st>>>(MERGE_ARGS);
    else if (D == 128) attn_fwd_merge_kernel<false, false, 128><<<mgrid, dim3(256), 0, st>>>(MERGE_ARGS);
    else attn_fwd_merge_kernel<false, false, 64><<<mgrid, dim3(256), 0, st>>>(MERGE_ARGS);
#undef MERGE_ARGS
    VMOBA_CHECK_LAUNCH();
    return VMOBA_OK;
}
