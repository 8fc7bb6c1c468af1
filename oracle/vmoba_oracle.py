"""CPU oracle for the VMoBA attention layer (arxiv 2506.23858).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain reference that the HIP
library is checked against.  Nothing in the product path may import it; only the
tests, the smoke check and the benchmark's CPU-baseline leg do.  It shares no code
with the HIP path and imports nothing from it.

What it follows, step by step (paper section / equation in brackets):

  1. block partition of the T x H x W latent grid into 1D / 2D / 3D blocks,
     chosen by layer index modulo 3                       [Sec. 3.2, Eq. 1]
  2. mean of every key block                              [Sec. 3.1 Step 1, Eq. 2]
  3. query x block-key similarity matrix, one per head    [Sec. 3.3, Eq. 3]
  4. normalisation of the similarities                    [Sec. 3.4, text before Eq. 4]
  5. descending sort of the head's whole pool, cumulative
     sum, k = first prefix length reaching tau            [Sec. 3.4, Eq. 4]
  6. TopkMask: the k best (query, block) pairs            [Sec. 3.3, Eq. 3]
  7. attention of every query over the keys/values of its
     selected blocks only                                 [Sec. 3.1 Step 3]
  8. the gradient of step 7 for training                  [Sec. 3.1 Step 3; the paper
     trains through this layer, Sec. 4.1]

Step 7 given the mask is exactly dense soft-max attention under an explicit mask
(the paper states its implementation is equivalent to the conceptual procedure), so
steps 7-8 are the textbook definition written out in float64.  Steps 2-6 decide an
integer result (which pairs are kept); the method runs them in single precision and
so does this oracle: block means and scores are accumulated in float64 and rounded
once to float32, the soft-max is evaluated in float32, the cumulative sum in float64.

Query rows are processed in independent batches of rows so the S x S matrix is never
held at once; every row is still computed by the plain definition, nothing is fused.

Readings taken where the paper leaves the computation open (listed with reasons in
the design document of this repository):
  * "normalised similarity" = soft-max over the blocks of one query (each query's
    similarities sum to one, the head's pool sums to S, the threshold is tau * S);
  * similarities are scaled by 1/sqrt(D) before that soft-max (an argument);
  * Eq. 4's ">=" decides the cut, ties are ordered by ascending (query, block);
  * a query that keeps no block outputs zero, has LSE = -inf and receives/sends no gradient;
  * grids that do not divide evenly get truncated edge blocks, means over real sizes;
  * no gradient flows through steps 2-6 (hard selection);
  * layer index is 0-based: layer 0 -> 1D, 1 -> 2D, 2 -> 3D.

Parity status: every function below is pinned by tests/test_oracle_*.py against
closed forms, brute force, library routines or a hand-worked example.  Agreement of the
whole method with the authors' own numbers is "parity unpinned": the paper prints no
worked numeric example and no code or weights are available.
"""
from __future__ import annotations

import math

import numpy as np

__all__ = [
    "layer_kind", "partition_dims", "partition_index", "gather_rows", "scatter_rows",
    "block_means", "block_scores", "normalise_rows", "threshold_topk", "select_blocks",
    "local_topk", "local_threshold", "global_topk",
    "csr_from_mask", "masked_attention_fwd", "masked_attention_bwd", "vmoba_layer",
]


# --------------------------------------------------------------------------- step 1
def layer_kind(layer: int) -> int:
    """Partition kind of layer `layer`: 0 = temporal (1D), 1 = spatial (2D),
    2 = spatio-temporal (3D).  [Sec. 3.2, Eq. 1: the case is picked by l mod 3.]"""
    return int(layer) % 3


def _ceil_div(a: int, b: int) -> int:
    return -(-a // b)


def partition_dims(T, H, W, bt, bh, bw, chunk=0):
    """Number of tokens S and number of key blocks N_b.  [Sec. 3.2, Eq. 1-2.]

    A block is a box of bt x bh x bw latent positions (1D of the paper: bh=H, bw=W;
    2D: bt=T; 3D: all three smaller), or, when chunk > 0, `chunk` consecutive tokens of
    the row-major (t, h, w) order.  Sizes that do not divide leave truncated edge blocks.
    """
    S = T * H * W
    if chunk > 0:
        return S, _ceil_div(S, chunk)
    return S, _ceil_div(T, bt) * _ceil_div(H, bh) * _ceil_div(W, bw)


def partition_index(T, H, W, bt, bh, bw, chunk=0):
    """The rearrangement of Eq. 1 as index arrays.  [Sec. 3.2, Eq. 1.]

    Returns (perm, inv_perm, blk_off), all int32:
      perm[p]      token (row-major index (t*H+h)*W+w) that sits at block-ordered position p
      inv_perm[n]  block-ordered position of token n
      blk_off[j]   first position of block j; blk_off[N_b] = S
    Block ids run row-major over (N^T, N^H, N^W) -- W fastest, as the grouping
    "(N^T N^H N^W)" of Eq. 1 reads -- and tokens inside a block run row-major over
    (s^T, s^H, s^W) restricted to the block's real extent.
    """
    S, nb = partition_dims(T, H, W, bt, bh, bw, chunk)
    perm = np.empty(S, dtype=np.int32)
    blk_off = np.zeros(nb + 1, dtype=np.int32)
    if chunk > 0:
        perm[:] = np.arange(S, dtype=np.int32)
        for j in range(nb):
            blk_off[j + 1] = min(S, (j + 1) * chunk)
    else:
        nT, nH, nW = _ceil_div(T, bt), _ceil_div(H, bh), _ceil_div(W, bw)
        p = 0
        j = 0
        for it in range(nT):
            for ih in range(nH):
                for iw in range(nW):
                    t0, h0, w0 = it * bt, ih * bh, iw * bw
                    t1, h1, w1 = min(T, t0 + bt), min(H, h0 + bh), min(W, w0 + bw)
                    tt, hh, ww = np.meshgrid(np.arange(t0, t1), np.arange(h0, h1),
                                             np.arange(w0, w1), indexing="ij")
                    tok = ((tt * H + hh) * W + ww).reshape(-1)
                    perm[p:p + tok.size] = tok
                    p += tok.size
                    j += 1
                    blk_off[j] = p
        assert p == S
    inv_perm = np.empty(S, dtype=np.int32)
    inv_perm[perm] = np.arange(S, dtype=np.int32)
    return perm, inv_perm, blk_off


def gather_rows(X, perm):
    """X' = rearrange(X): caller layout [B, S, Hh, D] -> block order [B, Hh, S, D].  [Eq. 1]"""
    return np.ascontiguousarray(np.transpose(X[:, perm, :, :], (0, 2, 1, 3)))


def scatter_rows(Xp, perm):
    """Inverse of gather_rows: block order [B, Hh, S, D] -> caller layout [B, S, Hh, D]."""
    B, Hh, S, D = Xp.shape
    X = np.empty((B, S, Hh, D), dtype=Xp.dtype)
    X[:, perm, :, :] = np.transpose(Xp, (0, 2, 1, 3))
    return X


# --------------------------------------------------------------------------- step 2
def block_means(Kp, blk_off):
    """B[j] = mean of the keys of block j (one head; Kp is [S, D] in block order).
    Float64 accumulation, one rounding to float32, divisor = the block's real size.
    [Sec. 3.1 Step 1, Eq. 2.]"""
    nb = len(blk_off) - 1
    out = np.empty((nb, Kp.shape[1]), dtype=np.float32)
    K64 = Kp.astype(np.float64)
    for j in range(nb):
        a, b = int(blk_off[j]), int(blk_off[j + 1])
        out[j] = (K64[a:b].sum(axis=0) / float(b - a)).astype(np.float32)
    return out


# --------------------------------------------------------------------------- step 3
def block_scores(Qp, Bm, score_scale):
    """S_hat[q, j] = score_scale * <Q'[q], B[j]> (one head).  Float64 accumulation,
    one rounding to float32.  [Sec. 3.3, Eq. 3: the matrix q_i b_i^T.]"""
    s = Qp.astype(np.float64) @ Bm.astype(np.float64).T
    return (s * float(score_scale)).astype(np.float32)


# --------------------------------------------------------------------------- step 4
def normalise_rows(S_hat):
    """P[q, :] = soft-max over blocks of S_hat[q, :], in float32 with the row maximum
    subtracted.  This is the reading of "normalised similarity scores".  [Sec. 3.4.]"""
    S_hat = S_hat.astype(np.float32)
    m = S_hat.max(axis=1, keepdims=True)
    e = np.exp(S_hat - m, dtype=np.float32)
    den = e.sum(axis=1, keepdims=True, dtype=np.float32)
    return (e / den).astype(np.float32)


def normalise_pool(S_hat):
    """The other reading of "normalised": ONE soft-max over the head's whole pool,
    G[q, j] = exp(S_hat[q, j] - max) / sum over all (q, j), accumulated in float64 and rounded
    once to float32.  The pool then sums to 1.  [Sec. 3.4, text before Eq. 4.]"""
    x = S_hat.astype(np.float64)
    e = np.exp(x - x.max())
    return (e / e.sum()).astype(np.float32)


# --------------------------------------------------------------------------- steps 5-6
def threshold_topk(P, tau, total=None):
    """Head-global threshold selection.  [Sec. 3.4, Eq. 4 and Sec. 3.3, Eq. 3.]

    The pool is every entry of P (shape [S, N_b], rows sum to one, so the pool sums
    to S).  Sort it descending (equal values: ascending (q, j)), accumulate in float64,
    k = the first prefix length whose sum is >= tau * S; the k best pairs form the mask.
    tau is taken in single precision (that is how it crosses the library boundary).
    total: what the pool sums to when it is not S (1 for the pool soft-max of normalise_pool).
    Returns (k, theta, mask) with theta = the k-th largest value and mask bool [S, N_b].
    """
    S, nb = P.shape
    N = S * nb
    flat = P.astype(np.float32).reshape(-1)
    order = np.argsort(-flat, kind="stable")
    sorted_vals = flat[order]
    tau32 = float(np.float32(tau))
    if tau32 >= 1.0:
        k = N
    else:
        csum = np.cumsum(sorted_vals.astype(np.float64))
        target = tau32 * (float(S) if total is None else float(total))
        k = int(np.searchsorted(csum, target, side="left")) + 1
        if k > N:            # rounding kept the total just below tau * S
            k = N
    theta = np.float32(sorted_vals[k - 1])
    mask = np.zeros(N, dtype=bool)
    mask[order[:k]] = True
    return k, theta, mask.reshape(S, nb)


# Selection variants of the paper's ablation ("block choice design": top-k or threshold, chosen
# per query -- "local" -- or from the head's whole pool -- "global"; the training-free runs use
# local + top-k, the option of the original MoBA).  Ties are ordered by ascending block / (q, j).
MODE_GLOBAL_THRESHOLD, MODE_LOCAL_TOPK, MODE_LOCAL_THRESHOLD, MODE_GLOBAL_TOPK, MODE_POOL_SOFTMAX = 0, 1, 2, 3, 4
MODE_OWN_BLOCK = 0x100      # flag: every query also keeps the block it lies in


def local_topk(P, topk):
    """Every query keeps its `topk` most similar blocks (all of them if topk >= N_b).
    [App. A, "Local + TopK"; Sec. 4.3 block choice ablation.]"""
    S, nb = P.shape
    k = min(int(topk), nb)
    order = np.argsort(-P.astype(np.float32), axis=1, kind="stable")
    mask = np.zeros((S, nb), dtype=bool)
    np.put_along_axis(mask, order[:, :k], True, axis=1)
    return mask


def local_threshold(P, tau):
    """Every query keeps the shortest descending prefix of its own blocks whose normalised
    similarities sum to >= tau (float64 running sum; tau in single precision).
    [Sec. 4.3 block choice ablation, "threshold + local": Eq. 4 applied per query.]"""
    S, nb = P.shape
    P32 = P.astype(np.float32)
    order = np.argsort(-P32, axis=1, kind="stable")
    sorted_vals = np.take_along_axis(P32, order, axis=1).astype(np.float64)
    before = np.cumsum(sorted_vals, axis=1) - sorted_vals        # mass ranked strictly before each entry
    tau32 = float(np.float32(tau))
    keep_sorted = before < tau32 if tau32 < 1.0 else np.ones_like(before, dtype=bool)
    mask = np.zeros((S, nb), dtype=bool)
    np.put_along_axis(mask, order, keep_sorted, axis=1)
    return mask


def global_topk(P, k_total):
    """The k_total most similar (query, block) pairs of the head's pool.
    [Sec. 3.3, Eq. 3 with a fixed k: "topk + global" of the ablation.]"""
    S, nb = P.shape
    k = max(1, min(int(k_total), S * nb))
    flat = P.astype(np.float32).reshape(-1)
    order = np.argsort(-flat, kind="stable")
    mask = np.zeros(S * nb, dtype=bool)
    mask[order[:k]] = True
    return k, np.float32(flat[order[k - 1]]), mask.reshape(S, nb)


def select_blocks(Qp, Kp, blk_off, tau, score_scale, mode=MODE_GLOBAL_THRESHOLD, topk=0):
    """Steps 2-6 for one head.  Returns dict(Bmean, S_hat, P, k, theta, mask).
    mode may carry MODE_OWN_BLOCK: after the selection every query also keeps the block that
    holds its own position (no query is left without keys; the cut itself, theta, is unchanged
    and k becomes the number of kept pairs).  [Sec. 3.3 leaves queries without blocks possible;
    keeping the current block is the original MoBA's rule.]"""
    own = bool(mode & MODE_OWN_BLOCK)
    mode &= ~MODE_OWN_BLOCK
    Bm = block_means(Kp, blk_off)
    S_hat = block_scores(Qp, Bm, score_scale)
    P = normalise_rows(S_hat)
    if mode == MODE_GLOBAL_THRESHOLD:
        k, theta, mask = threshold_topk(P, tau)
    elif mode == MODE_LOCAL_TOPK:
        mask = local_topk(P, topk)
        k, theta = int(mask.sum()), np.float32(0)
    elif mode == MODE_LOCAL_THRESHOLD:
        mask = local_threshold(P, tau)
        k, theta = int(mask.sum()), np.float32(0)
    elif mode == MODE_GLOBAL_TOPK:
        k, theta, mask = global_topk(P, topk * P.shape[0])
    elif mode == MODE_POOL_SOFTMAX:
        P = normalise_pool(S_hat)
        k, theta, mask = threshold_topk(P, tau, total=1.0)
    else:
        raise ValueError(mode)
    if own:
        sizes = np.diff(np.asarray(blk_off, dtype=np.int64))
        mask = mask.copy()
        mask[np.arange(P.shape[0]), np.repeat(np.arange(len(sizes)), sizes)] = True
        k = int(mask.sum())
    return dict(Bmean=Bm, S_hat=S_hat, P=P, k=k, theta=theta, mask=mask)


def csr_from_mask(mask):
    """The two sparse views of one head's mask [S, N_b] that the library returns:
    block-major (blk_ptr [N_b+1], q_idx ascending inside each block) -- the (N_b, s)
    orientation of Eq. 3 -- and query-major (row_ptr [S+1], col_idx ascending)."""
    S, nb = mask.shape
    cnt_b = mask.sum(axis=0).astype(np.int64)
    blk_ptr = np.concatenate([[0], np.cumsum(cnt_b)]).astype(np.int64)
    q_idx = np.concatenate([np.nonzero(mask[:, j])[0] for j in range(nb)]).astype(np.int32) \
        if nb else np.zeros(0, np.int32)
    cnt_q = mask.sum(axis=1).astype(np.int64)
    row_ptr = np.concatenate([[0], np.cumsum(cnt_q)]).astype(np.int64)
    col_idx = np.nonzero(mask)[1].astype(np.int32)
    return blk_ptr, q_idx, row_ptr, col_idx


# --------------------------------------------------------------------------- step 7
def _token_mask_rows(mask_rows, blk_off):
    """Expand block-level mask rows [r, N_b] to key-token level [r, S]."""
    sizes = np.diff(np.asarray(blk_off, dtype=np.int64))
    blk_of_pos = np.repeat(np.arange(len(sizes)), sizes)
    return mask_rows[:, blk_of_pos]


def masked_attention_fwd(Qp, Kp, Vp, mask, blk_off, softmax_scale, rows_per_batch=1024):
    """O[q] = sum_n softmax_n(scale * <Q'[q], K'[n]>) V'[n] over the keys n of the blocks
    query q selected; LSE[q] = log-sum-exp of the allowed scaled scores.  One head,
    float64.  A query with no selected block gets O = 0 and LSE = -inf.
    [Sec. 3.1 Step 3.]"""
    S, D = Qp.shape
    Q = Qp.astype(np.float64)
    K = Kp.astype(np.float64)
    V = Vp.astype(np.float64)
    O = np.zeros((S, V.shape[1]), dtype=np.float64)
    LSE = np.full(S, -np.inf, dtype=np.float64)
    for r0 in range(0, S, rows_per_batch):
        r1 = min(S, r0 + rows_per_batch)
        allow = _token_mask_rows(mask[r0:r1], blk_off)
        s = (Q[r0:r1] @ K.T) * float(softmax_scale)
        s = np.where(allow, s, -np.inf)
        m = s.max(axis=1)
        live = np.isfinite(m)
        m_safe = np.where(live, m, 0.0)
        e = np.exp(s - m_safe[:, None])           # exp(-inf) = 0 on masked entries
        den = e.sum(axis=1)
        den_safe = np.where(live, den, 1.0)
        A = e / den_safe[:, None]
        O[r0:r1] = np.where(live[:, None], A @ V, 0.0)
        LSE[r0:r1] = np.where(live, m_safe + np.log(den_safe), -np.inf)
    return O, LSE


# --------------------------------------------------------------------------- step 8
def masked_attention_bwd(Qp, Kp, Vp, mask, blk_off, softmax_scale, dO, rows_per_batch=1024):
    """Gradient of masked_attention_fwd with the mask held fixed.  One head, float64.
    With A the attention weights: delta = rowsum(dO * O), dV = A^T dO, dP = dO V^T,
    dS = A * (dP - delta), dQ = scale * dS K, dK = scale * dS^T Q.  Rows with no
    selected block contribute nothing.  Returns (dQ, dK, dV)."""
    S, D = Qp.shape
    Q = Qp.astype(np.float64)
    K = Kp.astype(np.float64)
    V = Vp.astype(np.float64)
    dO = dO.astype(np.float64)
    scale = float(softmax_scale)
    dQ = np.zeros_like(Q)
    dK = np.zeros_like(K)
    dV = np.zeros_like(V)
    for r0 in range(0, S, rows_per_batch):
        r1 = min(S, r0 + rows_per_batch)
        allow = _token_mask_rows(mask[r0:r1], blk_off)
        s = (Q[r0:r1] @ K.T) * scale
        s = np.where(allow, s, -np.inf)
        m = s.max(axis=1)
        live = np.isfinite(m)
        m_safe = np.where(live, m, 0.0)
        e = np.exp(s - m_safe[:, None])
        den = np.where(live, e.sum(axis=1), 1.0)
        A = e / den[:, None]
        A[~live] = 0.0
        O_rows = A @ V
        delta = (dO[r0:r1] * O_rows).sum(axis=1)
        dV += A.T @ dO[r0:r1]
        dP = dO[r0:r1] @ V.T
        dS = A * (dP - delta[:, None])
        dQ[r0:r1] = scale * (dS @ K)
        dK += scale * (dS.T @ Q[r0:r1])
    return dQ, dK, dV


# --------------------------------------------------------------------------- whole layer
def vmoba_layer(Q, K, V, grid, block, tau, dO=None, score_scale=None, softmax_scale=None,
                chunk=0, mode=MODE_GLOBAL_THRESHOLD, topk=0):
    """One VMoBA attention layer on caller-layout tensors [B, S, Hh, D].  [Sec. 3.1-3.4.]

    grid = (T, H, W); block = (bt, bh, bw) (ignored when chunk > 0).
    Returns a dict with O (caller layout, float64), LSE [B, Hh, S] in block order, the
    per-head selection results, and dQ, dK, dV (caller layout) when dO is given.
    """
    B, S, Hh, D = Q.shape
    T, H, W = grid
    bt, bh, bw = block
    if score_scale is None:
        score_scale = 1.0 / math.sqrt(D)
    if softmax_scale is None:
        softmax_scale = 1.0 / math.sqrt(D)
    perm, inv_perm, blk_off = partition_index(T, H, W, bt, bh, bw, chunk)
    Qp, Kp, Vp = gather_rows(Q, perm), gather_rows(K, perm), gather_rows(V, perm)
    nb = len(blk_off) - 1
    Op = np.zeros((B, Hh, S, D), dtype=np.float64)
    LSE = np.zeros((B, Hh, S), dtype=np.float64)
    masks = np.zeros((B, Hh, S, nb), dtype=bool)
    ks = np.zeros((B, Hh), dtype=np.int64)
    thetas = np.zeros((B, Hh), dtype=np.float32)
    Ps = np.zeros((B, Hh, S, nb), dtype=np.float32)
    Bms = np.zeros((B, Hh, nb, D), dtype=np.float32)
    grads = None
    if dO is not None:
        dOp = gather_rows(dO, perm)
        grads = [np.zeros((B, Hh, S, D), dtype=np.float64) for _ in range(3)]
    for b in range(B):
        for h in range(Hh):
            sel = select_blocks(Qp[b, h], Kp[b, h], blk_off, tau, score_scale, mode, topk)
            masks[b, h], ks[b, h], thetas[b, h] = sel["mask"], sel["k"], sel["theta"]
            Ps[b, h], Bms[b, h] = sel["P"], sel["Bmean"]
            Op[b, h], LSE[b, h] = masked_attention_fwd(Qp[b, h], Kp[b, h], Vp[b, h],
                                                      sel["mask"], blk_off, softmax_scale)
            if dO is not None:
                g = masked_attention_bwd(Qp[b, h], Kp[b, h], Vp[b, h], sel["mask"], blk_off,
                                         softmax_scale, dOp[b, h])
                for dst, src in zip(grads, g):
                    dst[b, h] = src
    out = dict(O=scatter_rows(Op, perm), Op=Op, LSE=LSE, mask=masks, k=ks, theta=thetas,
               P=Ps, Bmean=Bms, perm=perm, inv_perm=inv_perm, blk_off=blk_off)
    if dO is not None:
        out["dQ"], out["dK"], out["dV"] = (scatter_rows(g, perm) for g in grads)
        out["dQp"], out["dKp"], out["dVp"] = grads
    return out
