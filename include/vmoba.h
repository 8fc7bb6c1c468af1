/*
 * libvmoba -- VMoBA block-sparse attention for AMD MI355X (gfx950), C ABI.
 *
 * One attention layer of "VMoBA: Mixture-of-Block Attention for Video Diffusion Models"
 * (arxiv 2506.23858) is four calls, in this order:
 *
 *     vmoba_partition  ->  vmoba_select  ->  vmoba_attn_fwd  ( ->  vmoba_attn_bwd )
 *
 * followed by vmoba_partition(inverse = 1) to bring O (and dQ, dK, dV) back to the
 * caller's token order.
 *
 * General conventions
 *  - Every data pointer is a DEVICE pointer unless it says "host".  The library never
 *    allocates or frees device memory and keeps no state between calls; the caller owns
 *    every buffer, including workspaces (size them with vmoba_workspace_bytes).
 *  - `stream` is a hipStream_t passed as void*.  Calls only enqueue work on it and return;
 *    nothing on this path waits for the device.  Sizes that depend on the data (k, nnz)
 *    stay on the device.
 *  - Return value: VMOBA_OK or a negative vmoba_status.  Arguments are validated on the
 *    host before anything is launched: a call that fails validation launches nothing.
 *    (VMOBA_ERR_HIP reports a failed launch or runtime call; kernels enqueued before it stay
 *    enqueued.)  No C++ exception crosses this boundary.
 *  - "Block order" is the token order produced by the partition (Eq. 1 of the paper):
 *    the tokens of key block 0 first, then block 1, ...  All index arrays (mask, CSR lists)
 *    are in block-order positions.
 *  - Tensors are described by vmoba_tensor: element (b, s, h, d) lives at
 *    ptr + (b*stride_b + s*stride_s + h*stride_h + d) elements; the D channels of one
 *    (token, head) are contiguous and 16-byte aligned.
 *  - Supported: head dimension D in {64, 128}; dtype float32 or bfloat16 (all tensors of a
 *    call share one dtype); 1 <= n_blocks <= 512 (float32: as long as the score kernel's tile of block means
 *    fits the LDS, n_blocks * (D + 64) * 4 + 12 KB <= 160 KB); bidirectional attention (no causal mask).
 */
#ifndef VMOBA_H
#define VMOBA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    VMOBA_OK = 0,
    VMOBA_ERR_INVALID_ARG = -1, /* null pointer, non-positive extent, tau outside (0, 1], ... */
    VMOBA_ERR_UNSUPPORTED = -2, /* D, dtype or n_blocks outside the supported set            */
    VMOBA_ERR_WORKSPACE = -3,   /* workspace_bytes smaller than vmoba_workspace_bytes(...)    */
    VMOBA_ERR_CAPACITY = -4,    /* (device status word) a head selected more than nnz_capacity */
    VMOBA_ERR_HIP = -5          /* a HIP launch reported an error                             */
} vmoba_status;

typedef enum { VMOBA_F32 = 0, VMOBA_BF16 = 1 } vmoba_dtype;

/* Operations that need a workspace (argument `op` of vmoba_workspace_bytes). */
typedef enum { VMOBA_OP_SELECT = 1, VMOBA_OP_ATTN_FWD = 2, VMOBA_OP_ATTN_BWD = 3 } vmoba_op;

/* Block-choice designs (argument `mode` of vmoba_select).  Sec. 3.3-3.4 define global + threshold, the
 * paper's training setting; the other three are the variants of its block-choice ablation (Sec. 4.3) --
 * local + top-k, the option of the original MoBA, is what its training-free runs use (App. A). */
typedef enum {
    VMOBA_GLOBAL_THRESHOLD = 0, /* head's whole pool, descending cumulative similarity until tau * S (Eq. 4) */
    VMOBA_LOCAL_TOPK = 1,       /* every query keeps its `topk` most similar blocks                          */
    VMOBA_LOCAL_THRESHOLD = 2,  /* every query keeps the shortest descending prefix of its row reaching tau  */
    VMOBA_GLOBAL_TOPK = 3,      /* head's whole pool, the topk * S most similar pairs (Eq. 3 with a fixed k)  */
    /* The other reading of "normalised similarity" in Sec. 3.4: ONE soft-max over the head's whole pool of
     * S * n_blocks scores instead of one per query.  The pool then sums to 1, the cut is the shortest
     * descending prefix that reaches tau, and P holds the pool-normalised values (its rows no longer sum to 1). */
    VMOBA_POOL_SOFTMAX_THRESHOLD = 4,
    /* Flag, OR-ed into any of the above: every query also keeps the block it lies in itself, so no query is
     * left without keys (under global selection some are, Sec. 3.3; the original MoBA always keeps the
     * current chunk).  The cut (k of the pool, theta) is taken as without the flag; k_out then reports the
     * number of kept pairs, which can exceed it by up to S. */
    VMOBA_SELECT_OWN_BLOCK = 0x100
} vmoba_select_mode;

/* Latent grid and key-block shape (Sec. 3.2, Eq. 1).  A block is a box of bt x bh x bw
 * latent positions: the paper's 1D partition is (s^T, H, W), its 2D partition (T, s^H, s^W),
 * its 3D partition (s^T, s^H, s^W).  If chunk > 0 the box is ignored and a block is `chunk`
 * consecutive tokens of the row-major (t, h, w) order.  Extents that do not divide the grid
 * leave truncated blocks at the far edges. */
typedef struct {
    int32_t T, H, W;
    int32_t bt, bh, bw;
    int64_t chunk;
} vmoba_grid;

typedef struct {
    void* ptr;        /* device */
    int32_t dtype;    /* vmoba_dtype */
    int64_t stride_b; /* elements */
    int64_t stride_s;
    int64_t stride_h;
} vmoba_tensor;

/* Host helpers (no GPU work). */

/* Partition kind of transformer layer `layer` (0-based): 0 = 1D, 1 = 2D, 2 = 3D.
 * (Sec. 3.2, Eq. 1: the case is chosen by l mod 3.) */
int vmoba_layer_kind(int layer);

/* Token count S = T*H*W and block count N_b of a partition (Eq. 1-2).  Host pointers. */
int vmoba_partition_dims(const vmoba_grid* g, int64_t* S, int32_t* n_blocks);

/* Bytes of workspace `op` needs for this geometry.  nnz_capacity is per (batch, head). */
size_t vmoba_workspace_bytes(int op, int B, int Hh, int64_t S, int D, int32_t n_blocks,
                             int64_t nnz_capacity, int dtype);

const char* vmoba_status_string(int status);

/*
 * vmoba_partition -- the rearrangement K' = rearrange(K) of Sec. 3.2, Eq. 1, applied to
 * n_tensors tensors at once (the library also keeps Q and V in block order), or its inverse.
 *
 *  inverse = 0:  out[i](b, p, h, :) = in[i](b, perm[p], h, :)      caller order -> block order
 *  inverse = 1:  out[i](b, perm[p], h, :) = in[i](b, p, h, :)      block order -> caller order
 *
 *  perm     [S]   int32, perm[p] = row-major token index (t*H + h)*W + w at block-order position p
 *  inv_perm [S]   int32, inverse permutation
 *  blk_off  [n_blocks + 1] int32, first position of every block, blk_off[n_blocks] = S
 *  With inverse = 0 and inv_perm, blk_off non-null the three arrays are WRITTEN (rebuilt from
 *  `g`); with inverse = 0 and both null, or with inverse = 1, perm is READ as an earlier call
 *  wrote it and the other two are not touched.
 *  in / out: host arrays of n_tensors descriptors (1..8); a pair must have equal dtype, except
 *  that a float32 input may be written to a bfloat16 output (round to nearest even).
 *  Pure data movement: results are bit-exact.
 */
int vmoba_partition(const vmoba_grid* g, int inverse, int B, int Hh, int D, int n_tensors,
                    const vmoba_tensor* in, const vmoba_tensor* out, int32_t* perm,
                    int32_t* inv_perm, int32_t* blk_off, void* stream);

/*
 * vmoba_select -- Steps 1-2 of Sec. 3.1: mean key blocks (Eq. 2), query x block similarity
 * (Eq. 3), soft-max normalisation over the blocks of each query, head-global descending
 * cumulative-sum threshold (Eq. 4) and the TopkMask of Eq. 3, returned as a bit mask and as
 * two sparse lists.
 *
 *  Qp, Kp      tensors (b, s, h, d) with the strides given.  Row k of Kp is key position k in BLOCK order (keys are
 *              what Eq. 1 rearranges).  Row q of Qp is "query q" in every output -- the rows of P and mask, row_ptr,
 *              the entries of q_idx, later LSE: pass the block-order Q' (query ids are then block-order positions),
 *              or the caller's Q as it is (query ids are then token ids; the paper rearranges K only and the
 *              selection treats every query on its own, so Q never has to move)
 *  tau         threshold in (0, 1]; tau >= 1 keeps every pair
 *  score_scale factor applied to <q, b> before the soft-max (1/sqrt(D) by convention)
 *  mode        a vmoba_select_mode, optionally | VMOBA_SELECT_OWN_BLOCK (then allow S more pairs in
 *              nnz_capacity); tau is used by the threshold modes, topk (>= 1) by the top-k modes.
 *              Ties rank by ascending block index (local modes) or ascending (query, block) (global modes).
 *              In the local modes k_out is the number of kept pairs and theta_out is 0
 *  Bmean  out  [B, Hh, n_blocks, D] float32 block means
 *  P      out  [B, Hh, S, n_blocks] float32 normalised similarities (each row sums to 1)
 *  mask   out  [B, Hh, S, ceil(n_blocks/32)] uint32, bit j of a row = query keeps block j
 *  Per (b, h) the pool of S*n_blocks values is cut after the k best, k = the shortest
 *  descending prefix whose sum reaches tau*S; equal values at the cut are taken in ascending
 *  (query id, block) order.  k_out [B*Hh] int64 and theta_out [B*Hh] float (the k-th value; 0 when
 *  every pair is kept).
 *  Sparse lists, every (b, h) owning a segment of nnz_capacity entries starting at
 *  (b*Hh + h)*nnz_capacity:
 *    blk_ptr  [B*Hh, n_blocks + 1] int32  offsets (relative to the segment) of block j's queries
 *    q_idx    [B*Hh * nnz_capacity] int32 queries (ascending) that keep block j
 *    row_ptr  [B*Hh, S + 1]        int32  offsets of query q's blocks
 *    col_idx  [B*Hh * nnz_capacity] int32 blocks (ascending) kept by query q
 *    pair_pos [B*Hh * nnz_capacity] int32 for each (q, block) in query-major order, its offset
 *                                         in the block-major list
 *  In mode 0, k <= ceil(tau*S*n_blocks) holds in exact arithmetic (the k - 1 best of a pool of N values that sum to
 *  S carry at least (k - 1)/N of it), so nnz_capacity = min(S*n_blocks, ceil(tau*S*n_blocks)) plus a few entries for
 *  the rounding of P suffices; the top-k modes keep exactly min(topk, n_blocks)*S pairs; the local threshold mode
 *  can keep up to S*n_blocks.  If a head would still exceed it, nothing is written out of bounds, *dev_status is set
 *  to VMOBA_ERR_CAPACITY (dev_status is a device int32 the caller zeroes and reads after its own synchronisation),
 *  and that head's blk_ptr is all zero: vmoba_attn_fwd / vmoba_attn_bwd called with these lists treat the head as
 *  having selected nothing (O = 0, LSE = -inf, zero gradients) and read none of its incomplete list entries.
 *  mask, k_out, theta_out and row_ptr are complete either way.
 *  query_pos   optional int32 [S]: block-order position of query q (the partition's inv_perm).  Only read with
 *              VMOBA_SELECT_OWN_BLOCK, to find the block a query lies in; null = query q sits at position q.
 *  kv_rows     optional int32 [S]: keys in place.  Null: Kp is in block order.  Otherwise key position k is row
 *              kv_rows[k] of Kp -- pass the partition's perm and the caller's K: nothing is rearranged in memory,
 *              the blocks of Eq. 1 are addressed where they lie.
 */
int vmoba_select(int B, int Hh, int64_t S, int D, int32_t n_blocks, const int32_t* blk_off,
                 const vmoba_tensor* Qp, const vmoba_tensor* Kp, float tau, float score_scale,
                 int mode, int32_t topk, float* Bmean, float* P, uint32_t* mask, int32_t* blk_ptr,
                 int32_t* q_idx, int32_t* row_ptr, int32_t* col_idx, int32_t* pair_pos,
                 int64_t nnz_capacity, int64_t* k_out, float* theta_out, int32_t* dev_status,
                 const int32_t* query_pos, const int32_t* kv_rows, void* workspace, size_t workspace_bytes,
                 void* stream);

/*
 * vmoba_select_static -- vmoba_select for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels
 * and bit-identical results; the scratch memory vmoba_select takes as `workspace` is a static device array inside
 * the library instead (VMOBA_SELECT_STATIC_MAX_BYTES, held on every GPU the library runs on until the process
 * ends).  The call allocates and frees nothing.  Its first call on a device looks up the array's device address
 * (hipGetSymbolAddress): make that call outside any capture.
 * Limit: geometries with vmoba_workspace_bytes(VMOBA_OP_SELECT, ...) > VMOBA_SELECT_STATIC_MAX_BYTES return
 * VMOBA_ERR_WORKSPACE before anything is launched (32 MiB covers 12 heads at 480p and at 720p).
 * Every call on a GPU uses that GPU's one array: calls that overlap on one GPU (two streams, two threads) race --
 * serialise them.  The array keeps the previous call's contents; the call clears what it needs zeroed itself.
 */
#define VMOBA_SELECT_STATIC_MAX_BYTES ((size_t)32 << 20)
int vmoba_select_static(int B, int Hh, int64_t S, int D, int32_t n_blocks, const int32_t* blk_off,
                        const vmoba_tensor* Qp, const vmoba_tensor* Kp, float tau, float score_scale,
                        int mode, int32_t topk, float* Bmean, float* P, uint32_t* mask, int32_t* blk_ptr,
                        int32_t* q_idx, int32_t* row_ptr, int32_t* col_idx, int32_t* pair_pos,
                        int64_t nnz_capacity, int64_t* k_out, float* theta_out, int32_t* dev_status,
                        const int32_t* query_pos, const int32_t* kv_rows, void* stream);

/*
 * vmoba_attn_fwd -- Step 3 of Sec. 3.1: every query attends to the keys/values of its selected
 * blocks only.  O(q) = sum_n softmax_n(softmax_scale * <Q'(q), K'(n)>) V'(n) over the keys n of
 * the selected blocks; LSE [B, Hh, S] float32 is the natural-log-sum-exp of the scaled scores.
 * A query that selected nothing gets O = 0 and LSE = -inf.
 * Inputs: Q as vmoba_select saw it (block-order Q', or the caller's Q with token ids as query ids), block-order
 * K', V', blk_off, and the lists written by vmoba_select with the same nnz_capacity.  O and LSE are indexed
 * by query id.  Accumulation and soft-max are float32; bfloat16 inputs are multiplied on the
 * matrix cores.
 *  out_rows  optional int32 [S].  Null: O is written in block order.  Otherwise block-order row q
 *            goes to row out_rows[q] of O: pass the partition's perm and a tensor in the caller's
 *            token order to skip the inverse partition of O.  LSE stays in block order either way.
 *  kv_rows   optional int32 [S]: keys in place, as in vmoba_select -- key position k is row kv_rows[k] of Kp and Vp.
 *            (bfloat16: the tile kernel keeps the row numbers of a key block in LDS, up to 3584 keys per block;
 *            longer blocks are looked up in global memory, which is correct but slower.)
 *  Limit (bfloat16): one (batch, head) slice of K' and of V' must span less than 4 GiB, i.e.
 *  (S + 256) * stride_s * 2 < 2^32 with a positive stride_s; with kv_rows also S < 2^24 and stride_s * 2 < 2^24;
 *  otherwise VMOBA_ERR_UNSUPPORTED.
 */
int vmoba_attn_fwd(int B, int Hh, int64_t S, int D, int32_t n_blocks, const int32_t* blk_off,
                   const vmoba_tensor* Qp, const vmoba_tensor* Kp, const vmoba_tensor* Vp,
                   const int32_t* blk_ptr, const int32_t* q_idx, const int32_t* row_ptr,
                   const int32_t* pair_pos, int64_t nnz_capacity, float softmax_scale,
                   const vmoba_tensor* O, float* LSE, const int32_t* out_rows, const int32_t* kv_rows,
                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * vmoba_attn_bwd -- gradient of vmoba_attn_fwd with the selection held fixed (the paper trains
 * through Step 3; the hard selection of Step 2 passes no gradient).  With A the attention
 * weights over the selected keys: delta = rowsum(dO * O), dV = A^T dO, dP = dO V^T,
 * dS = A * (dP - delta), dQ = softmax_scale * dS K, dK = softmax_scale * dS^T Q.
 * O and LSE are the forward results; dQ, dK, dV are written (not accumulated into).  Rows that
 * selected nothing get dQ = 0 and contribute nothing.
 *  rows  optional int32 [S].  Null: O, dO, dQ are indexed by query id and dK, dV by key position like Q and K', V'.
 *        Otherwise O, dO, dQ, dK and dV (not Q, K', V', LSE) are addressed through it -- row r is row rows[r] of
 *        each: with block-order Q', pass the partition's perm and tensors in the caller's token order to skip the
 *        partition of dO and the inverse partition of the three gradients.
 *  key_rows  optional int32 [S]: row map of dK and dV alone (key position k -> row key_rows[k]); overrides `rows`
 *        for them.  With the caller's Q as it is (query ids = token ids): rows = null, key_rows = perm.
 *  kv_rows   optional int32 [S]: keys in place, as in vmoba_select -- key position k is row kv_rows[k] of Kp and Vp.
 *  Limit (bfloat16): S < 2^24, and for Q', K', V' and dO a positive stride_s with stride_s * 2 < 2^24 and
 *  S * stride_s * 2 < 2^32 (one (batch, head) slice spans less than 4 GiB); otherwise
 *  VMOBA_ERR_UNSUPPORTED.
 */
int vmoba_attn_bwd(int B, int Hh, int64_t S, int D, int32_t n_blocks, const int32_t* blk_off,
                   const vmoba_tensor* Qp, const vmoba_tensor* Kp, const vmoba_tensor* Vp,
                   const vmoba_tensor* O, const float* LSE, const vmoba_tensor* dO,
                   const int32_t* blk_ptr, const int32_t* q_idx, const int32_t* row_ptr,
                   const int32_t* pair_pos, int64_t nnz_capacity, float softmax_scale,
                   const vmoba_tensor* dQ, const vmoba_tensor* dK, const vmoba_tensor* dV,
                   const int32_t* rows, const int32_t* key_rows, const int32_t* kv_rows, void* workspace,
                   size_t workspace_bytes, void* stream);

/*
 * vmoba_profile_events -- measurement aid, not part of the method.  Asks the library to record
 * the caller's two hipEvent_t (passed as void*) on the call's stream immediately before and after
 * the launch of one of its compute kernels, so a benchmark can time that kernel alone:
 *   slot 0: forward tile kernel (vmoba_attn_fwd)      slot 1: dQ tile kernel (vmoba_attn_bwd)
 *   slot 2: dK/dV kernel (vmoba_attn_bwd)             slot 3: row copy kernel (vmoba_partition)
 * Pass null events to switch a slot off (the default).  Process-wide, not thread-safe.
 */
int vmoba_profile_events(int slot, void* start_event, void* stop_event);

/*
 * vmoba_probe_mfma -- measurement aid, not part of the method.  Launches `workgroups` workgroups of four
 * wavefronts that each issue iters x 4 independent v_mfma_f32_32x32x16_bf16 and nothing else; *flop_out (host)
 * receives the FLOP count of the launch.  Timed by the caller, it gives the bfloat16 matrix rate the GPU
 * sustains under matrix load (its clock drops below the nominal one there), next to the published peak.
 * sink: device float the kernel never writes in practice (it keeps the loop from being optimised away).
 */
int vmoba_probe_mfma(int64_t iters, int workgroups, float* sink, double* flop_out, void* stream);

/*
 * vmoba_probe_atomic_rows -- measurement aid, not part of the method.  Launches only the atomic traffic of a
 * backward pass that would add dQ from inside the dK/dV kernel (the design this library does not use): `runs` x `heads`
 * workgroups, each walking one of n_lists ascending query lists of cnt rows (lists: device int32 [n_lists][cnt], rows
 * in [0, S)) and adding a row of 128 floats per entry into dq (device float32 [heads][S][128], which the caller
 * zeroes) with hardware float atomics.  bench.py --probe-atomics times it against the dQ path it would replace.
 */
int vmoba_probe_atomic_rows(float* dq, const int32_t* lists, int n_lists, int cnt, int64_t S, int runs, int heads,
                            void* stream);

#ifdef __cplusplus
}
#endif
#endif /* VMOBA_H */
