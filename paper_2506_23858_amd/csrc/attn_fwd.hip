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
#include <type_traits>

// Tile plan of a call: tile_start[bh][j] = number of tiles (of TM list entries) in all (head, block) pairs before
// (bh, j), counted over the whole flat list of the call -- heads in order, blocks in order -- tile_start[bh][nb] = the
// same for the first pair of the next head, and head_base[bh] = tile_start[bh][0], head_base[BH] = total.  One
// workgroup; a scan over the BH * nb tile counts in batches of 1024.
__global__ __launch_bounds__(1024) void tile_plan_kernel(const int* __restrict__ blk_ptr, int* __restrict__ tile_start,
                                                         int* __restrict__ head_base, int BH, int nb, int TM) {
    __shared__ int sW[16];
    __shared__ int sCarry;
    const int t = threadIdx.x, n = BH * nb;
    if (t == 0) sCarry = 0;
    __syncthreads();
    for (int base = 0; base < n; base += 1024) {
        const int i = base + t;
        int v = 0, bh = 0, j = 0;
        if (i < n) {
            bh = i / nb;
            j = i - bh * nb;
            const int* bp = blk_ptr + (long long)bh * (nb + 1);
            v = (bp[j + 1] - bp[j] + TM - 1) / TM;
        }
        int incl = v;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int o = __shfl_up(incl, off, 64);
            if ((t & 63) >= off) incl += o;
        }
        if ((t & 63) == 63) sW[t >> 6] = incl;
        __syncthreads();
        int wave_base = 0;
        for (int w = 0; w < (t >> 6); ++w) wave_base += sW[w];
        const int excl = sCarry + wave_base + incl - v;
        if (i < n) {
            tile_start[(long long)bh * (nb + 1) + j] = excl;
            if (j == 0) {
                head_base[bh] = excl;
                if (bh > 0) tile_start[(long long)(bh - 1) * (nb + 1) + nb] = excl;
            }
        }
        __syncthreads();
        if (t == 1023) sCarry = excl + v;
        __syncthreads();
    }
    if (t == 0) {
        tile_start[(long long)(BH - 1) * (nb + 1) + nb] = sCarry;
        head_base[BH] = sCarry;
    }
}

// Per-head tile descriptors of the float32 path (grid: tile id x head; ids past the head's last tile get count 0).
__global__ __launch_bounds__(256) void tile_desc_kernel(const int* __restrict__ tile_start, const int* __restrict__ blk_ptr,
                                                        const int* __restrict__ blk_off, int4* __restrict__ tile_desc,
                                                        int nb, int TM, int tiles_per_head) {
    const int bh = blockIdx.y;
    const int tile = blockIdx.x * 256 + threadIdx.x;
    if (tile >= tiles_per_head) return;
    const int* ts = tile_start + (long long)bh * (nb + 1);
    const int first = ts[0];
    int4 d = {0, 0, 0, 0};
    if (tile < ts[nb] - first) {
        int lo = 0, hi = nb;           // largest j with ts[j] - first <= tile
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (ts[mid] - first <= tile) lo = mid; else hi = mid;
        }
        const int* bp = blk_ptr + (long long)bh * (nb + 1);
        const int t0 = (tile - (ts[lo] - first)) * TM;
        d.x = bp[lo] + t0;
        d.y = min(TM, bp[lo + 1] - bp[lo] - t0);
        d.z = blk_off[lo];
        d.w = blk_off[lo + 1] - blk_off[lo];
    }
    tile_desc[(long long)bh * tiles_per_head + tile] = d;
}

// Flat tile list over all heads for the MFMA tile kernels: flat_desc[tile_start[bh][0] + tile] = {first list entry,
// count | bh << 10, first key, block length}; one thread per (head, tile id below tiles_per_head).
__global__ __launch_bounds__(256) void flat_tile_desc_kernel(const int* __restrict__ tile_start, const int* __restrict__ blk_ptr,
                                                             const int* __restrict__ blk_off, int4* __restrict__ flat_desc,
                                                             int nb, int TM, int tiles_per_head) {
    const int bh = blockIdx.y;
    const int tile = blockIdx.x * 256 + threadIdx.x;
    const int* ts = tile_start + (long long)bh * (nb + 1);
    const int first = ts[0];
    if (tile >= tiles_per_head || tile >= ts[nb] - first) return;
    int lo = 0, hi = nb;           // largest j with ts[j] - first <= tile
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (ts[mid] - first <= tile) lo = mid; else hi = mid;
    }
    const int* bp = blk_ptr + (long long)bh * (nb + 1);
    const int t0 = (tile - (ts[lo] - first)) * TM;
    int4 d;
    d.x = bp[lo] + t0;
    d.y = min(TM, bp[lo + 1] - bp[lo] - t0) | (bh << 10);
    d.z = blk_off[lo];
    d.w = blk_off[lo + 1] - blk_off[lo];
    flat_desc[first + tile] = d;
}

namespace {

constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

// ---------------------------------------------------------------------------------------------
// Plain FMA tile kernel for float32 inputs.  One wavefront per tile of 64 gathered queries,
// lane = query.  Keys and values of the block pass through LDS in chunks of KC rows.
template <int D>
__global__ __launch_bounds__(64) void attn_fwd_tile_simple_kernel(
    TensorView Q, TensorView K, TensorView V, const int* __restrict__ blk_off, const int* __restrict__ blk_ptr,
    const int* __restrict__ q_idx, const int4* __restrict__ tile_desc, int tiles_per_head, float* __restrict__ Opart,
    float* __restrict__ lse_part, int Hh, int nb, long long cap, float scale_log2, const int* __restrict__ kv_rows) {
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
    float qr[D], o[D];
    {
        const char* src = Q.ptr + ((long long)b * Q.stride_b + (long long)q * Q.stride_s + (long long)h * Q.stride_h) * ES;
#pragma unroll
        for (int d = 0; d < D; ++d) {
            qr[d] = reinterpret_cast<const float*>(src)[d];
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
            const int pos = tc.k0 + c0 + r;
            const long long row = kv_rows ? kv_rows[pos] : pos;       // key position -> row of K and V
            const char* ks = kbase + row * K.stride_s * ES;
            const char* vs = vbase + row * V.stride_s * ES;
            sK[r][d] = reinterpret_cast<const float*>(ks)[d];
            sV[r][d] = reinterpret_cast<const float*>(vs)[d];
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
// bf16 MFMA tile kernel.  NW wavefronts; wavefront w owns 32 gathered queries (a tile is 32 * NW list
// entries of one key block) and the block's keys are walked in groups of 32.
//
// Operand orientation.  All products are computed transposed so that the query index is the MFMA
// column (= lane % 32):
//   S^T[key, q] = K[key, :] . Q[q, :]          A = K rows from LDS, B = Q^T held in registers
//   O^T[d, q]  += V^T[d, key] . P^T[key, q]    A = V^T by transpose reads, B = P^T packed from S^T
// With the query on the lane, the row maximum and row sum of the online soft-max are reductions
// over a lane's own registers plus one exchange between the lane halves (v_permlane32_swap).  The
// running maximum is only raised when a group exceeds it by more than 2^8 (the probabilities then
// stay below 2^8, well inside float32 / bf16 range), so the accumulator rescale is rare; the final
// division by the row sum makes the result independent of which maximum was used.  The row sum is
// kept per lane half and the halves are added once at the end (they always agree on the maximum).
//
// Pipeline.  A wavefront's instruction stream is a three-stage software pipeline: step g issues
//     S^T(g+1) = K(g+1) . Q^T               (matrix)
//     P(g)     = soft-max piece of S^T(g)   (vector)
//     O^T     += V(g-1)^T . P(g-1)^T        (matrix)
// interleaved unit by unit (unit u = k-step u of the first product and (s, dt) = (u / DT, u % DT)
// of the second), with the LDS operands of unit u + 2 fetched during unit u, so neither LDS
// latency nor the soft-max sits between dependent matrix instructions.  S^T and P live in two
// register sets that swap roles every step.
//
// Rows.  K and V groups are loaded straight from global memory into rings of four LDS slots each
// (global_load_lds_dwordx4: 64 lanes x 16 bytes land in 1024 consecutive LDS bytes), so no
// registers hold rows in flight and a group is requested two steps before it is first read.  A
// slot is 32 rows of 2*D bytes without padding; 16-byte piece p of row r is stored at piece
// position p ^ f(r), f(r) = (r >> SH) & (pieces per row - 1), which keeps both the row reads of
// the first product and the transposed reads of the second free of bank conflicts (D = 128; for
// D = 64 the transposed reads take two-way conflicts).  The swizzle is applied on the global side
// (the lane that fills piece position p' fetches piece p' ^ f(r)) and undone on the read side
// with one XOR of the per-lane address.  Rows past the end of the block repeat its last key; the
// surplus keys of the last group are masked to -inf in the soft-max.
//
// Ordering.  The loads are issued by inline assembly, so their waits are written by hand: every
// step that requests rows starts with s_waitcnt vmcnt(loads of one step) -- the wavefront's own
// loads of two steps ago have landed -- followed by the workgroup barrier, which makes every
// wavefront's loads of two steps ago visible.  Step g requests K(g+4) into the slot of K(g) (last
// read in step g-1) and V(g+2) into the slot of V(g-2) (last read in step g-1); K(g+2) and V(g)
// are first read at the end of step g.
//
// Persistence.  A workgroup strides through its XCD's share of the flat tile list (all heads, see
// flat_tile_desc_kernel) and overlaps the start of its next tile with the end of the current one:
// the next descriptor and the next tile's query index are fetched at the start of the tile, and its
// query rows (into the Q^T registers, the first product is done by then) and K(0..3), V(0..1)
// during the last soft-max step, into slots nobody reads any more (the rings are indexed by
// running group counters, so the next tile's first V slots differ from the slots of the two groups
// the last two steps read).
//
// Output.  A wavefront writes its 32 partial rows to LDS as the accumulators hold them (8 bytes
// per lane and channel group) and reads them back as whole rows: the tile's partials are
// consecutive rows of Opart, so each store request is a 1 KB run instead of 16-byte pieces of 32
// rows (the address unit needs about as long for one such request as for eight full-row ones).
//
// Keys in place (KVR).  K and V may stay where the caller has them: key position p of the block order is then row
// kv_rows[p] of both.  A tile's slice of that map, kv_rows[k0 .. k0 + L), is copied into LDS (global_load_lds_dword,
// 64 entries per instruction) one tile ahead -- two tables that alternate, filled for the next tile at the start of
// the current one -- and a row request reads its row number there instead of advancing an offset.  Blocks longer
// than a table (TOKMAX keys) look their rows up in global memory, which is correct but waits for the lookup.
template <int D, int NW, bool KVR>
__global__ __launch_bounds__(64 * NW, 8 / NW) void attn_fwd_tile_mfma_kernel(
    TensorView Q, TensorView K, TensorView V, const int* __restrict__ q_idx, const int4* __restrict__ flat_desc,
    const int* __restrict__ head_base, int BH, float* __restrict__ Opart, float* __restrict__ lse_part, int Hh,
    long long cap, float scale_log2, const int* __restrict__ kv_rows) {
    constexpr int G = 32;                   // keys per group
    constexpr int RB = 2 * D;               // bytes per LDS row
    constexpr int PPR = D / 8;              // 16-byte pieces per row
    constexpr int SH = PPR == 16 ? 0 : 1;   // swizzle f(r) = (r >> SH) & (PPR - 1)
    constexpr int SLOT = G * RB;            // bytes per ring slot
    constexpr int NR = 4;                   // ring slots per tensor
    constexpr int KSTEPS = D / 16, DT = D / 32, UNITS = KSTEPS;
    constexpr int IPW = SLOT / 1024 / NW;   // load instructions per wavefront per group
    constexpr int RPI = 1024 / RB;          // rows per load instruction
    constexpr int NDMA = 2 * IPW;           // loads a wavefront issues per step (one K group, one V group)
    constexpr float LAZY = 8.f;
    static_assert(UNITS % 4 == 0 && UNITS == 2 * DT && IPW >= 1 && IPW * NW * 1024 == SLOT && (D == 64 || D == 128), "unit bookkeeping");
    __shared__ __align__(1024) char sK[NR * SLOT];
    __shared__ __align__(1024) char sV[NR * SLOT];
    // a wavefront's 32 partial rows on their way out: written as the accumulators hold them (8 bytes per lane and
    // channel group), read back as whole rows, so that the global stores are 1 KB runs instead of 16-byte pieces
    constexpr int OPITCH = D * 2 + 16;
    __shared__ __align__(16) char sOut[NW * 32 * OPITCH];
    constexpr int TOKMAX = 3584;            // entries per row-number table (two of them fill what is left of the 160 KB)
    __shared__ __align__(256) int sTok[KVR ? 2 * TOKMAX : 4];

    // Workgroup ids go round the 8 XCDs (each with its own L2), so XCD x = id % 8 takes the x-th eighth of the tile
    // list and its workgroups stride through it: a key block's tiles then share one L2 instead of eight.
    const int total = head_base[BH];
    const bool by_xcd = (gridDim.x & 7) == 0;
    const int xcd = by_xcd ? (int)(blockIdx.x & 7) : 0;
    const int f_step = by_xcd ? (int)(gridDim.x >> 3) : (int)gridDim.x;
    const int per_xcd = by_xcd ? (total + 7) >> 3 : total;
    const int f_end = min(total, (xcd + 1) * per_xcd);
    int f = xcd * per_xcd + (by_xcd ? (int)(blockIdx.x >> 3) : (int)blockIdx.x);
    if (f >= f_end) return;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, hf = lane >> 5;
    const int ent = wave * 32 + l32;
    const uint32_t sK0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)sK;
    const uint32_t sV0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)sV;
    const uint32_t sTok0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) int*)sTok;

    // ---- per-tile state.  Descriptor: {first list entry, count | head << 10, first key, block length}
    struct Tile {
        int list0, count, bh, k0, L;
        const char* kbase;
        const char* vbase;
        long long seg;
    };
    auto decode = [&](const int4 d) {
        Tile t;
        t.list0 = d.x;
        t.count = d.y & 1023;
        t.bh = d.y >> 10;
        t.k0 = d.z;
        t.L = d.w;
        const int b = t.bh / Hh, h = t.bh % Hh;
        t.kbase = K.ptr + ((long long)b * K.stride_b + (long long)h * K.stride_h) * 2;
        t.vbase = V.ptr + ((long long)b * V.stride_b + (long long)h * V.stride_h) * 2;
        t.seg = (long long)t.bh * cap;
        return t;
    };
    auto query_of = [&](const Tile& t) {                          // surplus rows repeat the tile's last query
        return q_idx[t.seg + t.list0 + min(ent, t.count - 1)];
    };
    bf16x8_t qf[KSTEPS];
    auto load_q = [&](const Tile& t, int q) {
        const int b = t.bh / Hh, h = t.bh % Hh;
        const char* src = Q.ptr + ((long long)b * Q.stride_b + (long long)q * Q.stride_s + (long long)h * Q.stride_h) * 2;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8_t*>(src + (ks * 16 + hf * 8) * 2);
    };
    const uint32_t kss = (uint32_t)(K.stride_s * 2), vss = (uint32_t)(V.stride_s * 2);
    const uint32_t k_adv = G * kss, v_adv = G * vss;

    // Load instruction i of this wavefront fills LDS bytes [(wave * IPW + i) * 1024, + 1024) of a slot: lane -> row
    // dr[i] of the group, piece position lane % PPR, i.e. piece (lane % PPR) ^ f(dr[i]) of the global row.  Byte offsets
    // from the head's base are 32-bit (checked on the host); an offset past the block's last row is clamped to it.
    uint32_t k_off[IPW], v_off[IPW], k_last[IPW], v_last[IPW];
    auto first_offsets = [&](const Tile& t) {
#pragma unroll
        for (int i = 0; i < IPW; ++i) {
            const int dr = (wave * IPW + i) * RPI + lane / PPR;
            const uint32_t pc16 = (uint32_t)((lane % PPR) ^ ((dr >> SH) & (PPR - 1))) * 16;
            k_off[i] = (uint32_t)(t.k0 + dr) * kss + pc16;
            v_off[i] = (uint32_t)(t.k0 + dr) * vss + pc16;
            k_last[i] = (uint32_t)(t.k0 + t.L - 1) * kss + pc16;
            v_last[i] = (uint32_t)(t.k0 + t.L - 1) * vss + pc16;
        }
    };
    // request the next group of a tensor into ring slot `slot`; every call advances the offsets by one group
    auto request = [&](const char* base, uint32_t* off, const uint32_t* last, uint32_t adv, uint32_t ring0, int slot) {
#pragma unroll
        for (int i = 0; i < IPW; ++i) {
            dma16(base, min(off[i], last[i]), ring0 + (uint32_t)(slot & (NR - 1)) * SLOT + (uint32_t)(wave * IPW + i) * 1024);
            off[i] += adv;
        }
    };
    // KVR: the row-number table of tile t into table `tb`; the instructions are dealt round the wavefronts, entries
    // past the block's end repeat its last key
    auto dma_tokens = [&](const Tile& t, int tb) {
        if (t.L > TOKMAX) return;
        const int n_instr = (t.L + 63) >> 6;
        for (int i = wave; i < n_instr; i += NW) {
            const int e = min(i * 64 + lane, t.L - 1);
            dma4(reinterpret_cast<const char*>(kv_rows), (uint32_t)(t.k0 + e) << 2, sTok0 + (uint32_t)(tb * TOKMAX + i * 64) * 4);
        }
    };
    // KVR: request group `grp` of tile t (whose row numbers are in table `tb`) into ring slot `slot`
    auto request_rows = [&](const Tile& t, const char* base, uint32_t stride, int grp, uint32_t ring0, int slot, int tb) {
#pragma unroll
        for (int i = 0; i < IPW; ++i) {
            const int dr = (wave * IPW + i) * RPI + lane / PPR;
            const uint32_t pc16 = (uint32_t)((lane % PPR) ^ ((dr >> SH) & (PPR - 1))) * 16;
            const int idx = min(grp * G + dr, t.L - 1);
            const uint32_t row = t.L <= TOKMAX ? (uint32_t)sTok[tb * TOKMAX + idx] : (uint32_t)kv_rows[t.k0 + idx];
            dma16(base, __umul24(row, stride) + pc16, ring0 + (uint32_t)(slot & (NR - 1)) * SLOT + (uint32_t)(wave * IPW + i) * 1024);
        }
    };
    int kb = 0, vb = 0;                    // running group counters: group x of the current tile uses slot (kb + x) & 3 / (vb + x) & 3
    int tp = 0;                            // KVR: table that holds the current tile's row numbers
    auto request_first_groups = [&](const Tile& t, int kb_t, int vb_t, int tb) {     // K(0..3), V(0..1) of tile t
        if constexpr (KVR) {
#pragma unroll
            for (int x = 0; x < 4; ++x) request_rows(t, t.kbase, kss, x, sK0, kb_t + x, tb);
#pragma unroll
            for (int x = 0; x < 2; ++x) request_rows(t, t.vbase, vss, x, sV0, vb_t + x, tb);
        } else {
            first_offsets(t);
#pragma unroll
            for (int x = 0; x < 4; ++x) request(t.kbase, k_off, k_last, k_adv, sK0, kb_t + x);
#pragma unroll
            for (int x = 0; x < 2; ++x) request(t.vbase, v_off, v_last, v_adv, sV0, vb_t + x);
        }
    };

    // read side: per-lane byte offsets inside a slot, completed by XOR with the k-step / channel-tile bits
    const int kr = rho(l32);
    const uint32_t a_lane = (uint32_t)kr * RB + (uint32_t)((hf ^ (kr >> SH)) & (PPR - 1)) * 16;
    uint32_t c_lane[2];
    {
        const int g4 = lane >> 4, e = (lane >> 2) & 3, a = lane & 3;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int r = 4 * e + hf + 2 * t;
            const int p0 = 2 * (g4 & 1) + (a >> 1);
            c_lane[t] = (uint32_t)r * RB + (uint32_t)((p0 ^ (r >> SH)) & (PPR - 1)) * 16 + (a & 1) * 8;
        }
    }
    auto readK = [&](int x, int ks) {
        const uint32_t off = (a_lane ^ (uint32_t)(ks << 5)) + (uint32_t)((kb + x) & (NR - 1)) * SLOT;
        return *reinterpret_cast<const bf16x8_t*>(sK + off);
    };
    auto readV = [&](int x, int u) {       // transposed operand: channel tile dt = u % DT, 16-row step s = u / DT
        const uint32_t sl = (uint32_t)((vb + x) & (NR - 1)) * SLOT + (uint32_t)(u / DT) * 16 * RB;
        const uint32_t x6 = (uint32_t)(u % DT) << 6;
        const bf16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_t*)(sV + ((c_lane[0] ^ x6) + sl)));
        const bf16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_t*)(sV + ((c_lane[1] ^ x6) + sl)));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };
    const f32x16_t zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    Tile cur = decode(flat_desc[f]);
    load_q(cur, query_of(cur));
    if constexpr (KVR) {                   // the first tile's row numbers: nothing to overlap them with
        dma_tokens(cur, 0);
        VMOBA_WAIT_VMCNT(0);
        __syncthreads();
    }
    request_first_groups(cur, kb, vb, 0);

    for (;;) {
        const int fn = f + f_step;
        const bool has_next = fn < f_end;
        const int4 nd = flat_desc[has_next ? fn : f];   // without a next tile the look-ahead repeats this one (loads only)
        const int L = cur.L;
        const int Gt = (L + G - 1) / G;
        // A tile has Ge >= 2 steps with a soft-max (a block of one group gets a second, fully masked one) and
        // Ge - 2 of them are "middle" steps.  The two register sets swap roles every step; the set that starts is
        // chosen so that the last soft-max step always finds S^T in sB and P(g-1) in pA.
        const int Ge = max(Gt, 2);
        const int n_mid = Ge - 2;
        const bool odd = n_mid & 1;

        f32x16_t oacc[DT];
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) oacc[dt] = zero16;
        float m_run = -INFINITY, l_run = 0.f;      // l_run: this lane half's share of the row sum
        bf16x8_t opK[4], opV[4];                    // operands of units u .. u + 2, slot = unit % 4
        f32x16_t sA = zero16, sB = zero16;
        bf16x8_t pA[2], pB[2];

        VMOBA_WAIT_VMCNT(0);                       // this wavefront's K(0..3), V(0..1) (and Q rows) have landed
        __syncthreads();                           // ... and everybody else's
        // S^T(0), and the operands of the first two units of step 0
        if (odd) {
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) sB = __builtin_amdgcn_mfma_f32_32x32x16_bf16(readK(0, ks), qf[ks], sB, 0, 0, 0);
        } else {
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) sA = __builtin_amdgcn_mfma_f32_32x32x16_bf16(readK(0, ks), qf[ks], sA, 0, 0, 0);
        }
        opK[0] = readK(1, 0);
        opK[1] = readK(1, 1);
        opV[0] = opK[0];
        opV[1] = opK[1];
        const Tile nxt = decode(nd);
        const int nq = query_of(nxt);              // needed a tile later: the load has the whole tile to land

        // one pipeline step; the flags are compile-time: QK / PV = the step has a first / second product, SM = it has a
        // soft-max (MASK: with the keys past the block's end masked), NEXTPV = the next step has a second product,
        // STAGE = it requests rows
        auto step = [&](int g, auto qk_t, auto pv_t, auto sm_t, auto mask_t, auto nextpv_t, auto stage_t, f32x16_t& s_cur,
                        f32x16_t& s_nxt, bf16x8_t(&p_new)[2], bf16x8_t(&p_prev)[2]) {
            constexpr bool QK = decltype(qk_t)::value, PV = decltype(pv_t)::value, SM = decltype(sm_t)::value;
            constexpr bool MASK = decltype(mask_t)::value, NEXTPV = decltype(nextpv_t)::value, STAGE = decltype(stage_t)::value;
            constexpr bool LAST_SM = SM && !QK;       // the first product is complete: Q^T may be replaced
            if constexpr (STAGE) { VMOBA_WAIT_VMCNT(NDMA); __syncthreads(); }
            if constexpr (LAST_SM) { VMOBA_WAIT_VMCNT(0); __syncthreads(); }
            uint32_t w[8];                            // P of this step as packed bf16 pairs (accumulator values 2j, 2j + 1)
            float m_new = m_run, alpha = 1.f;
            bool raise = false;
#pragma unroll
            for (int u = 0; u < UNITS; ++u) {
                const int u2 = u + 2;
                bf16x8_t nk = opK[u2 & 3], nv = opV[u2 & 3];
                if (u2 < UNITS) {
                    if constexpr (QK) nk = readK(g + 1, u2);
                    if constexpr (PV) nv = readV(g - 1, u2);
                } else {
                    if constexpr (QK) nk = readK(g + 2, u2 - UNITS);
                    if constexpr (NEXTPV) nv = readV(g, u2 - UNITS);
                }
                if constexpr (QK) s_nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(opK[u & 3], qf[u], u == 0 ? zero16 : s_nxt, 0, 0, 0);
                if constexpr (PV) oacc[u % DT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(opV[u & 3], p_prev[u / DT], oacc[u % DT], 0, 0, 0);
                if constexpr (SM) {
                    if (u == 0) {
                        if constexpr (MASK) {
                            const int vh = L - g * G - hf;          // accumulator value i is key row acc_row(i, 0) + hf
#pragma unroll
                            for (int i = 0; i < 16; ++i)
                                if (acc_row(i, 0) >= vh) s_cur[i] = -INFINITY;
                        }
                        float mx = fmaxf(s_cur[0], s_cur[1]);
#pragma unroll
                        for (int i = 2; i < 16; i += 2) mx = fmaxf(fmaxf(mx, s_cur[i]), s_cur[i + 1]);
                        mx = swap_halves_max(mx * scale_log2);            // scale_log2 > 0
                        raise = mx > m_run + LAZY;
                        m_new = raise ? mx : m_run;
                        alpha = raise ? exp2_raw(m_run - m_new) : 1.f;
                        m_run = m_new;
                        l_run *= alpha;
                    } else {
                        // the 8 value pairs are spread over units 1 .. UNITS - 1; a pair is packed as soon as it exists
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            if (1 + (j * (UNITS - 1)) / 8 == u) {
                                const float p0 = exp2_raw(fmaf(s_cur[2 * j], scale_log2, -m_new));
                                const float p1 = exp2_raw(fmaf(s_cur[2 * j + 1], scale_log2, -m_new));
                                l_run += p0 + p1;
                                w[j] = pack_bf16x2(p0, p1);
                                asm volatile("" : "+v"(w[j]));     // keeps the pair in this unit (it is only read a step later)
                            }
                        }
                        asm volatile("" : "+v"(l_run));
                        if (u == UNITS - 1) {
                            const u32x4_t lo = {w[0], w[1], w[2], w[3]}, hi = {w[4], w[5], w[6], w[7]};
                            __builtin_memcpy(&p_new[0], &lo, 16);
                            __builtin_memcpy(&p_new[1], &hi, 16);
                        }
                    }
                }
                if constexpr (STAGE) {
                    if (u == 1) {
                        if constexpr (KVR) {
                            // the next tile's row numbers go first: they are then older than this step's row requests and
                            // have landed when the next step's wait lets only those stay in flight
                            if (g == 0) dma_tokens(nxt, tp ^ 1);
                            request_rows(cur, cur.kbase, kss, g + 4, sK0, kb + g + 4, tp);
                            request_rows(cur, cur.vbase, vss, g + 2, sV0, vb + g + 2, tp);
                        } else {
                            request(cur.kbase, k_off, k_last, k_adv, sK0, kb + g + 4);
                            request(cur.vbase, v_off, v_last, v_adv, sV0, vb + g + 2);
                        }
                    }
                }
                if constexpr (LAST_SM) {
                    // the next tile's query rows (Q^T is free: the first product is complete) and its first key groups (all K
                    // slots are free, the two V slots after the current tile's last two as well): two steps ahead of their use
                    if (u == 1) {
                        load_q(nxt, nq);
                        request_first_groups(nxt, kb + g + 1, vb + g + 1, tp ^ 1);
                    }
                }
                opK[u2 & 3] = nk;
                opV[u2 & 3] = nv;
                __builtin_amdgcn_sched_barrier(0);
            }
            if constexpr (PV && SM) {                 // the accumulator holds groups <= g - 1, all relative to the old maximum
                if (__builtin_amdgcn_ballot_w64(raise)) {
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                        for (int i = 0; i < 16; ++i) oacc[dt][i] *= alpha;
                }
            }
        };
        using T = std::true_type;
        using F = std::false_type;
        //   (g,  QK,  PV,  SM,  MASK, NEXTPV, STAGE, S^T(g), S^T(g+1), P(g), P(g-1))
        int g = 1;
        if (odd) {
            step(0, T{}, F{}, T{}, T{}, T{}, T{}, sB, sA, pB, pA);
            step(1, T{}, T{}, T{}, F{}, T{}, T{}, sA, sB, pA, pB);
            g = 2;
        } else {
            step(0, T{}, F{}, T{}, T{}, T{}, T{}, sA, sB, pA, pB);
        }
        for (int it = 0; it < (n_mid >> 1); ++it) {
            step(g, T{}, T{}, T{}, F{}, T{}, T{}, sB, sA, pB, pA);
            step(g + 1, T{}, T{}, T{}, F{}, T{}, T{}, sA, sB, pA, pB);
            g += 2;
        }
        step(g, F{}, T{}, T{}, T{}, T{}, F{}, sB, sA, pB, pA);          // g = Ge - 1: last soft-max
        step(g + 1, F{}, T{}, F{}, F{}, F{}, F{}, sA, sB, pA, pB);      // final step (g + 1 = Ge): second product of group Ge - 1

        // ---- partial output: O^T value i of tile dt <-> channel 32*dt + 8*(i>>2) + 4*hf + (i&3)
        const float l_tot = swap_halves_sum(l_run);
        {
            const float inv = 1.f / l_tot;
            char* mine = sOut + wave * 32 * OPITCH;                               // this wavefront's rows only: no barrier
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    u32x2_t v;
                    v.x = pack_bf16x2(oacc[dt][4 * gq + 0] * inv, oacc[dt][4 * gq + 1] * inv);
                    v.y = pack_bf16x2(oacc[dt][4 * gq + 2] * inv, oacc[dt][4 * gq + 3] * inv);
                    *reinterpret_cast<u32x2_t*>(mine + l32 * OPITCH + (dt * 32 + gq * 8 + hf * 4) * 2) = v;
                }
            // the tile's partials are consecutive rows of Opart (bfloat16): row = first pair of the tile + entry
            char* dst = reinterpret_cast<char*>(Opart) + (cur.seg + cur.list0) * (long long)(D * 2);
            constexpr int LPR = D * 2 / 16;                                       // lanes per row
#pragma unroll
            for (int k = 0; k < 32 * LPR / 64; ++k) {
                const int row = k * (64 / LPR) + lane / LPR, piece = lane % LPR;
                const u32x4_t x = *reinterpret_cast<const u32x4_t*>(mine + row * OPITCH + piece * 16);
                const int e = wave * 32 + row;
                if (e < cur.count) *reinterpret_cast<u32x4_t*>(dst + (long long)e * (D * 2) + piece * 16) = x;
            }
            if (ent < cur.count && hf == 0) lse_part[cur.seg + cur.list0 + ent] = (m_run + log2f(l_tot)) * LN2;
        }
        if (!has_next) break;
        f = fn;
        cur = nxt;
        kb += Ge;
        vb += Ge;
        tp ^= 1;
    }
}

// ---------------------------------------------------------------------------------------------
// Merge: O[q] = sum_pairs exp(lse_pair - LSE[q]) * Opart[pair], LSE[q] = logsumexp(lse_pair).
// A group of lanes per query, each owning CH consecutive channels (one 16-byte load per partial).
// Partials have the tensors' type: bfloat16 from the MFMA tile kernel, float32 from the FMA one.
// A head whose selection did not fit the lists (row_ptr[S] > cap, see vmoba_select) counts as having selected nothing.
template <bool BF16, int D>
__global__ __launch_bounds__(256) void attn_fwd_merge_kernel(const float* __restrict__ Opart, const float* __restrict__ lse_part,
                                                             const int* __restrict__ row_ptr, const int* __restrict__ pair_pos,
                                                             TensorView O, float* __restrict__ LSE,
                                                             const int* __restrict__ out_rows, int Hh, int S, long long cap) {
    constexpr int CH = BF16 ? 8 : 4;
    constexpr int MB = 8;                    // partial rows in flight per lane
    constexpr int LPQ = D / CH;              // lanes per query
    constexpr int QPW = 256 / LPQ;           // queries per workgroup
    const int bh = blockIdx.y, b = bh / Hh, h = bh % Hh;
    const int q = blockIdx.x * QPW + threadIdx.x / LPQ;
    const int part = threadIdx.x % LPQ;
    if (q >= S) return;
    const bool fits = row_ptr[(long long)bh * (S + 1) + S] <= cap;
    const int r0 = row_ptr[(long long)bh * (S + 1) + q];
    const int r1 = fits ? row_ptr[(long long)bh * (S + 1) + q + 1] : r0;
    const long long seg = (long long)bh * cap;
    // one pass with a running maximum; MB partials in flight per step (index -> lse and row loads)
    float mx = -INFINITY;
    float acc[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) acc[c] = 0.f;
    float wsum = 0.f;
    for (int r = r0; r < r1; r += MB) {
        long long pair[MB];
        float l[MB];
#pragma unroll
        for (int u = 0; u < MB; ++u) pair[u] = seg + pair_pos[seg + min(r + u, r1 - 1)];
#pragma unroll
        for (int u = 0; u < MB; ++u) l[u] = (r + u < r1) ? lse_part[pair[u]] : -INFINITY;
        float v[MB][CH];
#pragma unroll
        for (int u = 0; u < MB; ++u) {
            if constexpr (BF16) {
                // (read once: a non-temporal load, so the rows do not displace what the L2 holds; -7 % kernel time)
                const u32x4_t x = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(reinterpret_cast<const uint16_t*>(Opart) + pair[u] * D + part * 8));
                v[u][0] = bf16lo_to_f32(x.x); v[u][1] = bf16hi_to_f32(x.x); v[u][2] = bf16lo_to_f32(x.y); v[u][3] = bf16hi_to_f32(x.y);
                v[u][4] = bf16lo_to_f32(x.z); v[u][5] = bf16hi_to_f32(x.z); v[u][6] = bf16lo_to_f32(x.w); v[u][7] = bf16hi_to_f32(x.w);
            } else {
                const f32x4_t x = *reinterpret_cast<const f32x4_t*>(Opart + pair[u] * D + part * 4);
                v[u][0] = x.x; v[u][1] = x.y; v[u][2] = x.z; v[u][3] = x.w;
            }
        }
        float m_new = mx;
#pragma unroll
        for (int u = 0; u < MB; ++u) m_new = fmaxf(m_new, l[u]);
        const float alpha = expf(mx - m_new);          // exp(-inf) = 0 on the first step (m_new is finite: l[0] is)
        wsum *= alpha;
#pragma unroll
        for (int c = 0; c < CH; ++c) acc[c] *= alpha;
#pragma unroll
        for (int u = 0; u < MB; ++u) {
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
    if (part == 0) LSE[(long long)bh * S + q] = lse;
}

struct FwdWs {
    float* Opart;      // [BH * cap][D], in the tensors' type
    float* lse_part;   // [BH * cap]
    int* tile_start;   // [BH][nb + 1]
    int4* tile_desc;   // [BH][tiles_per_head], or the flat list of all heads' tiles
    int* head_base;    // [BH + 1]
    size_t total;
};

}  // namespace
// Grid width (tiles per head) for tiles of TM list entries: a host-side bound on sum_j ceil(cnt_j / TM).
int64_t vmoba_max_tiles(int64_t cap, int TM) { return (cap / TM + VMOBA_MAX_BLOCKS + 7) / 8 * 8; }
namespace {

FwdWs carve_fwd(void* base, int BH, int D, int64_t cap, int es) {       // es: bytes per element of the partial rows
    FwdWs w;
    char* p = (char*)base;
    size_t off = 0;
    w.Opart = (float*)(p + off);     off += align_up((size_t)BH * cap * D * es, 256);
    w.lse_part = (float*)(p + off);  off += align_up((size_t)BH * cap * 4, 256);
    w.tile_start = (int*)(p + off);  off += align_up((size_t)BH * (VMOBA_MAX_BLOCKS + 1) * 4, 256);
    w.tile_desc = (int4*)(p + off);  off += align_up((size_t)BH * vmoba_max_tiles(cap, 64) * 16, 256);
    w.head_base = (int*)(p + off);   off += align_up((size_t)(BH + 1) * 4, 256);
    w.total = off;
    return w;
}

}  // namespace

size_t vmoba_attn_fwd_workspace_bytes(int B, int Hh, int64_t S, int D, int64_t cap, int dtype) {
    (void)S;
    return carve_fwd(nullptr, B * Hh, D, cap, dtype == VMOBA_BF16 ? 2 : 4).total;
}

// Compute units of the current device (queried once).
int vmoba_num_cus() {
    static int n = 0;
    if (n == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            n = v;
        else
            n = 256;
    }
    return n;
}

extern "C" int vmoba_attn_fwd(int B, int Hh, int64_t S, int D, int32_t n_blocks, const int32_t* blk_off,
                              const vmoba_tensor* Qp, const vmoba_tensor* Kp, const vmoba_tensor* Vp,
                              const int32_t* blk_ptr, const int32_t* q_idx, const int32_t* row_ptr,
                              const int32_t* pair_pos, int64_t nnz_capacity, float softmax_scale,
                              const vmoba_tensor* O, float* LSE, const int32_t* out_rows, const int32_t* kv_rows,
                              void* workspace, size_t workspace_bytes, void* stream) {
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
    FwdWs ws = carve_fwd(workspace, BH, D, nnz_capacity, dt == VMOBA_BF16 ? 2 : 4);
    if (workspace_bytes < ws.total) return VMOBA_ERR_WORKSPACE;
    if (((uintptr_t)workspace) & 255) return VMOBA_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    const bool bf16 = dt == VMOBA_BF16;
    const TensorView Qv = make_view(Qp), Kv = make_view(Kp), Vv = make_view(Vp), Ov = make_view(O);
    const float scale_log2 = softmax_scale * LOG2E;
    const bool simple = !bf16;              // float32 tensors take the plain FMA kernels
    // the MFMA kernel addresses the rows of one (batch, head) slice of K and V with 32-bit byte offsets
    if (!simple && (Kp->stride_s <= 0 || Vp->stride_s <= 0 ||
                    (uint64_t)(S + 256) * (uint64_t)Kp->stride_s * 2 >= ((uint64_t)1 << 32) ||
                    (uint64_t)(S + 256) * (uint64_t)Vp->stride_s * 2 >= ((uint64_t)1 << 32)))
        return VMOBA_ERR_UNSUPPORTED;
    // with keys in place a row's byte offset is one 24-bit multiply of its row number and the row stride
    if (!simple && kv_rows && (S >= (1 << 24) || Kp->stride_s * 2 >= (1 << 24) || Vp->stride_s * 2 >= (1 << 24)))
        return VMOBA_ERR_UNSUPPORTED;
    // bf16, D = 128: 256-query tiles, one persistent workgroup of 8 wavefronts per compute unit (a tile's K and V
    // rows are fetched once per 256 queries); D = 64: 128-query tiles, two workgroups of 4 wavefronts per compute unit
    const bool wide = !simple && D == 128;
    const int TM = simple ? 64 : (wide ? 256 : 128);
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
    VMOBA_PROFILE_BEGIN(0, st);
    if (simple) {
        dim3 grid((unsigned)max_tiles, (unsigned)BH);
#define TILE_ARGS Qv, Kv, Vv, blk_off, blk_ptr, q_idx, ws.tile_desc, (int)max_tiles, ws.Opart, ws.lse_part, Hh, n_blocks, (long long)nnz_capacity, scale_log2, kv_rows
        if (D == 128) attn_fwd_tile_simple_kernel<128><<<grid, dim3(64), 0, st>>>(TILE_ARGS);
        else attn_fwd_tile_simple_kernel<64><<<grid, dim3(64), 0, st>>>(TILE_ARGS);
#undef TILE_ARGS
    } else {
        const dim3 pgrid((unsigned)std::min<int64_t>((wide ? 1 : 2) * (int64_t)vmoba_num_cus(), (int64_t)BH * max_tiles));
#define MFMA_ARGS Qv, Kv, Vv, q_idx, ws.tile_desc, ws.head_base, BH, ws.Opart, ws.lse_part, Hh, (long long)nnz_capacity, scale_log2, kv_rows
        if (wide && kv_rows) attn_fwd_tile_mfma_kernel<128, 8, true><<<pgrid, dim3(512), 0, st>>>(MFMA_ARGS);
        else if (wide) attn_fwd_tile_mfma_kernel<128, 8, false><<<pgrid, dim3(512), 0, st>>>(MFMA_ARGS);
        else if (kv_rows) attn_fwd_tile_mfma_kernel<64, 4, true><<<pgrid, dim3(256), 0, st>>>(MFMA_ARGS);
        else attn_fwd_tile_mfma_kernel<64, 4, false><<<pgrid, dim3(256), 0, st>>>(MFMA_ARGS);
#undef MFMA_ARGS
    }
    VMOBA_PROFILE_END(0, st);
    VMOBA_CHECK_LAUNCH();
    const int qpw = 256 / (D / (bf16 ? 8 : 4));     // partials: bfloat16 from the MFMA tile kernel, float32 otherwise
    dim3 mgrid((unsigned)ceil_div64(S, qpw), (unsigned)BH);
#define MERGE_ARGS ws.Opart, ws.lse_part, row_ptr, pair_pos, Ov, LSE, out_rows, Hh, (int)S, (long long)nnz_capacity
    if (bf16 && D == 128) attn_fwd_merge_kernel<true, 128><<<mgrid, dim3(256), 0, st>>>(MERGE_ARGS);
    else if (bf16) attn_fwd_merge_kernel<true, 64><<<mgrid, dim3(256), 0, st>>>(MERGE_ARGS);
    else if (D == 128) attn_fwd_merge_kernel<false, 128><<<mgrid, dim3(256), 0, st>>>(MERGE_ARGS);
    else attn_fwd_merge_kernel<false, 64><<<mgrid, dim3(256), 0, st>>>(MERGE_ARGS);
#undef MERGE_ARGS
    VMOBA_CHECK_LAUNCH();
    return VMOBA_OK;
}
