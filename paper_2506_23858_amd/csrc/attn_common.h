// Pieces shared by the forward and backward block-sparse attention kernels.
//
// Work decomposition (both directions).  The selection mask is kept block-major, the
// orientation M_i in (N_b, s) of Eq. 3: for key block j, q_idx[blk_ptr[j] .. blk_ptr[j+1]) lists
// the queries that keep it.  A "tile" is TM consecutive entries of one such list, i.e. TM gathered
// queries that all attend to the same key block.  tile_start[bh][j] = number of tiles before block
// j of head bh, written on the device from blk_ptr, so the host never learns the data-dependent counts;
// the grid is sized from nnz_capacity and surplus workgroups leave at once.
//
// MFMA operand plumbing (v_mfma_f32_32x32x16_bf16; lane = 32*hf + l32):
//   A operand: lane holds row l32, 8 consecutive k at 8*hf;   B operand: column l32, same k.
//   C/D:       lane holds column l32, rows 8*i + 4*hf + r as value 4*i + r (i, r = 0..3).
// LDS tiles are row-major [row][D].  The backward kernels pad every row by 8 bf16 (row stride D + 8, 16 bytes); the
// forward kernel's K/V rings are unpadded and swizzled instead (16-byte piece p of row r sits at piece p ^ f(r), see
// attn_fwd.hip), because its rows arrive by direct global-to-LDS loads that fill 1024 consecutive bytes.
//   * An operand that contracts over the channels of a row is a 16-byte row read.
//   * An operand that contracts over the ROWS (the transposed tile) is two ds_read_b64_tr_b16:
//     in each group of 16 lanes, lane 4*e + a supplies the address of 4 consecutive channels of
//     one row and receives, for channel 4*a' + c of the group (lane = 4*a' + c), the values of
//     the 4 rows supplied by lanes a', a'+4, a'+8, a'+12.
//   * Rows are fed to the first MFMA through the bit permutation rho below.  With it the 8
//     accumulator values a lane holds per 16-row step belong to rows {16*s + 4*e + 2*t + hf},
//     e = 0..3, t = 0..1: they pack straight into the next MFMA's B operand (no shuffle), the
//     matching transposed A operand is exactly what the two transpose reads (t = 0, 1) deliver,
//     and both kinds of LDS access are bank-conflict free with either layout.
#pragma once
#include "common.h"

// MFMA row m (0..31) of a 32-row group is fed tile row rho(m):
//   rho = 16*m[4] + 4*m[1:0] + 2*m[3] + m[2]
__device__ __forceinline__ int rho(int m) {
    return (m & 16) | ((m & 3) << 2) | ((m & 8) >> 2) | ((m & 4) >> 2);
}
// Tile row (0..31) that accumulator value v (0..15) of lane half hf belongs to.
__device__ __forceinline__ int acc_row(int v, int hf) {
    return ((v >> 3) << 4) | ((v & 3) << 2) | (((v >> 2) & 1) << 1) | hf;
}

typedef __bf16 __attribute__((address_space(3))) lds_bf16_t;
typedef bf16x4_t __attribute__((address_space(3))) lds_bf16x4_t;

// Per-lane element offset of the transposed-operand reads inside a tile of row stride STR:
// row 4*e + hf, channel 16*(g&1) + 4*a, with lane = 16*g + 4*e + a.
template <int STR>
__device__ __forceinline__ int tr_lane_offset(int lane) {
    const int g = lane >> 4, e = (lane >> 2) & 3, a = lane & 3, hf = lane >> 5;
    return (4 * e + hf) * STR + 16 * (g & 1) + 4 * a;
}

// Transposed A operand: m = channel col0 + l32, k-slots = rows {row0 + 16*s + 4*e + 2*t + hf}.
// `tile_lane` = tile base + tr_lane_offset (per lane); row0 = 32 * (row group), s = 16-row step.
template <int STR>
__device__ __forceinline__ bf16x8_t tr_operand(const __bf16* tile_lane, int row0, int s, int col0) {
    const __bf16* p = tile_lane + (row0 + 16 * s) * STR + col0;
    const bf16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_t*)(p));
    const bf16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_t*)(p + 2 * STR));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

__device__ __forceinline__ bf16x8_t pack8(const float* p) {
    f32x4_t lo = {p[0], p[1], p[2], p[3]};
    f32x4_t hi = {p[4], p[5], p[6], p[7]};
    bf16x4_t blo = __builtin_convertvector(lo, bf16x4_t);
    bf16x4_t bhi = __builtin_convertvector(hi, bf16x4_t);
    return __builtin_shufflevector(blo, bhi, 0, 1, 2, 3, 4, 5, 6, 7);
}

struct TileCoord {
    int count;    // valid entries in the tile (1..TM)
    int list0;    // first list entry of the tile, relative to the head's segment
    int t0;       // always 0 (the tile's offset is folded into list0)
    int k0, L;    // first key position and number of keys of the tile's key block
};

// Tile descriptors: one int4 {first list entry, count, k0, L} per (head, tile), written by
// tile_desc_kernel so that a tile kernel learns its work with a single 16-byte load instead of a
// binary search over dependent loads.  count = 0 marks a tile that does not exist.
__device__ __forceinline__ bool find_tile(const int4* __restrict__ tile_desc, int tiles_per_head, int bh, int tile,
                                          TileCoord& tc) {
    const int4 d = tile_desc[(long long)bh * tiles_per_head + tile];
    if (d.y <= 0) return false;
    tc.list0 = d.x;
    tc.t0 = 0;
    tc.count = d.y;
    tc.k0 = d.z;
    tc.L = d.w;
    return true;
}

// Tile plan (defined in attn_fwd.hip): tile_start[bh][j] = tiles of all (head, block) pairs before (bh, j) in the call's
// flat list, tile_start[bh][nb] = first tile of the next head, head_base[bh] = tile_start[bh][0], head_base[BH] = total.
__global__ __launch_bounds__(1024) void tile_plan_kernel(const int* __restrict__ blk_ptr, int* __restrict__ tile_start,
                                                         int* __restrict__ head_base, int BH, int nb, int TM);
// Descriptor of every tile id below tiles_per_head of a head (one thread per id; ids past the head's last tile get count 0).
__global__ __launch_bounds__(256) void tile_desc_kernel(const int* __restrict__ tile_start, const int* __restrict__ blk_ptr,
                                                        const int* __restrict__ blk_off, int4* __restrict__ tile_desc,
                                                        int nb, int TM, int tiles_per_head);

inline __device__ float exp2_raw(float x) { return __builtin_amdgcn_exp2f(x); }

// Flat tile list over all heads for the MFMA tile kernels.
__global__ __launch_bounds__(256) void flat_tile_desc_kernel(const int* __restrict__ tile_start, const int* __restrict__ blk_ptr,
                                                             const int* __restrict__ blk_off, int4* __restrict__ flat_desc,
                                                             int nb, int TM, int tiles_per_head);
// Compute units of the current device (queried once).
int vmoba_num_cus();

// Exchange between the two halves of a wavefront (lane i <-> lane i ^ 32), reduced with max / sum.
__device__ __forceinline__ float swap_halves_max(float x) {
    typedef unsigned u2 __attribute__((ext_vector_type(2)));
    const u2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r.x), __uint_as_float(r.y));
}
__device__ __forceinline__ float swap_halves_sum(float x) {
    typedef unsigned u2 __attribute__((ext_vector_type(2)));
    const u2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r.x) + __uint_as_float(r.y);
}
// 64 lanes x 16 bytes from base + byte_off (per lane) to LDS: lane i writes lds_addr + 16 * i (lds_addr is
// wave-uniform).  Counts in vmcnt like any vector load; the compiler does not know about it.
__device__ __forceinline__ void dma16(const char* base, uint32_t byte_off, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(byte_off), "s"(base), "s"(lds_addr)
                 : "memory", "m0");
}
// The same with 4 bytes per lane: lane i writes lds_addr + 4 * i.
__device__ __forceinline__ void dma4(const char* base, uint32_t byte_off, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" ::"v"(byte_off), "s"(base), "s"(lds_addr)
                 : "memory", "m0");
}
#define VMOBA_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))

