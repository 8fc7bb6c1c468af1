// Pieces shared by the forward and backward block-sparse attention kernels.
//
// Work decomposition (both directions).  The selection mask is kept block-major, the
// orientation M_i in (N_b, s) of Eq. 3: for key block j, q_idx[blk_ptr[j] .. blk_ptr[j+1]) lists
// the queries that keep it.  A "tile" is TM consecutive entries of one such list, i.e. TM gathered
// queries that all attend to the same key block.  tile_start[bh][j] = number of tiles of blocks
// 0..j-1, written on the device from blk_ptr, so the host never learns the data-dependent counts;
// the grid is sized from nnz_capacity and surplus workgroups leave at once.
#pragma once
#include "common.h"

// bits 2 and 3 of a 5-bit row index exchanged.  Feeding MFMA row m with key (or query)
// swap23(m) makes the accumulator registers of a lane hold 8 *consecutive* keys per 16-key
// step, so they can be packed straight into the next MFMA's operand without a shuffle.
__device__ __forceinline__ int swap23(int m) { return (m & 0x13) | ((m & 4) << 1) | ((m & 8) >> 1); }

struct TileCoord {
    int j;        // key block
    int t0;       // first list entry of the tile, relative to blk_ptr[j]
    int count;    // valid entries in the tile (1..TM)
    int list0;    // blk_ptr[j]: first list entry of the block, relative to the head's segment
    int k0, L;    // first key position and number of keys of block j
};

// Locate tile `tile` of head `bh`.  Returns false if the tile does not exist.
__device__ __forceinline__ bool find_tile(const int* __restrict__ tile_start, const int* __restrict__ blk_ptr,
                                          const int* __restrict__ blk_off, int bh, int nb, int tile, int TM,
                                          TileCoord& tc) {
    const int* ts = tile_start + (long long)bh * (nb + 1);
    if (tile >= ts[nb]) return false;
    int lo = 0, hi = nb;           // largest j with ts[j] <= tile
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (ts[mid] <= tile) lo = mid; else hi = mid;
    }
    const int* bp = blk_ptr + (long long)bh * (nb + 1);
    tc.j = lo;
    tc.list0 = bp[lo];
    const int cnt = bp[lo + 1] - bp[lo];
    tc.t0 = (tile - ts[lo]) * TM;
    tc.count = min(TM, cnt - tc.t0);
    tc.k0 = blk_off[lo];
    tc.L = blk_off[lo + 1] - blk_off[lo];
    return true;
}

// tile_start for all heads.  One thread per head (n_blocks <= 256).
__global__ __launch_bounds__(64) void tile_start_kernel(const int* __restrict__ blk_ptr, int* __restrict__ tile_start,
                                                        int BH, int nb, int TM);

inline __device__ float exp2_raw(float x) { return __builtin_amdgcn_exp2f(x); }
