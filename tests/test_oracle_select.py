"""Pins for the oracle's scores, normalisation and threshold selection (Sec. 3.3-3.4, Eq. 3-4)."""
import json
import math
import os

import numpy as np
import pytest

from oracle import vmoba_oracle as vo

GOLD = os.path.join(os.path.dirname(__file__), "golden", "two_block_example.json")


def test_scores_are_scaled_dot_products():
    rng = np.random.default_rng(2)
    Q = rng.standard_normal((11, 6)).astype(np.float32)
    Bm = rng.standard_normal((4, 6)).astype(np.float32)
    S_hat = vo.block_scores(Q, Bm, 0.5)
    assert S_hat.shape == (11, 4) and S_hat.dtype == np.float32
    for q in range(11):
        for j in range(4):
            ref = 0.5 * math.fsum(float(Q[q, d]) * float(Bm[j, d]) for d in range(6))
            assert abs(S_hat[q, j] - ref) <= 1e-6 * max(1.0, abs(ref))
    # a transposed operand or a dropped scale would break this asymmetric case
    Q1 = np.array([[1.0, 2.0]], dtype=np.float32)
    B1 = np.array([[3.0, 0.0], [0.0, 5.0], [1.0, 1.0]], dtype=np.float32)
    assert np.allclose(vo.block_scores(Q1, B1, 2.0), [[6.0, 20.0, 6.0]])


def test_rows_of_P_sum_to_one_and_zero_query_is_uniform():
    rng = np.random.default_rng(3)
    S_hat = (rng.standard_normal((200, 13)) * 5).astype(np.float32)
    P = vo.normalise_rows(S_hat)
    assert P.dtype == np.float32 and np.all(P >= 0)
    np.testing.assert_allclose(P.sum(1, dtype=np.float64), 1.0, atol=1e-6)
    # soft-max definition against float64 exp
    ref = np.exp(S_hat.astype(np.float64))
    ref /= ref.sum(1, keepdims=True)
    np.testing.assert_allclose(P, ref, rtol=2e-6, atol=1e-9)
    # shift invariance and no overflow for large logits
    P2 = vo.normalise_rows(S_hat + np.float32(1000.0))
    assert np.all(np.isfinite(P2))
    P0 = vo.normalise_rows(np.zeros((5, 8), dtype=np.float32))
    assert np.all(P0 == np.float32(1.0 / 8))


def _brute_k(P, tau):
    """Enumerate every prefix length of the descending pool with exact rational-ish sums."""
    vals = sorted((float(v) for v in P.reshape(-1)), reverse=True)
    target = float(np.float32(tau)) * P.shape[0]
    for kk in range(1, len(vals) + 1):
        if math.fsum(vals[:kk]) >= target:
            return kk
    return len(vals)


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("tau", [0.1, 0.25, 0.5, 0.9])
def test_threshold_k_brute_force(seed, tau):
    rng = np.random.default_rng(100 + seed)
    S, nb = int(rng.integers(3, 9)), int(rng.integers(2, 6))
    P = vo.normalise_rows((rng.standard_normal((S, nb)) * 2).astype(np.float32))
    k, theta, mask = vo.threshold_topk(P, tau)
    assert k == _brute_k(P, tau)
    assert mask.sum() == k
    # the mask holds the k largest values: nothing unselected exceeds anything selected
    assert P[mask].min() >= P[~mask].max() if k < P.size else True
    assert theta == P[mask].min()
    # minimality: one pair fewer does not reach the threshold
    top = np.sort(P.reshape(-1).astype(np.float64))[::-1]
    assert top[:k].sum() >= np.float32(tau) * S - 1e-9
    assert k == 1 or top[:k - 1].sum() < np.float32(tau) * S + 1e-9


def test_threshold_invariants():
    rng = np.random.default_rng(7)
    P = vo.normalise_rows((rng.standard_normal((300, 24)) * 3).astype(np.float32))
    N = P.size
    prev = 0
    for tau in [0.05, 0.15, 0.25, 0.35, 0.5, 0.75, 0.95]:
        k, theta, mask = vo.threshold_topk(P, tau)
        # Sec. 4.1: the kept fraction is always smaller than tau -> k <= ceil(tau * N)
        assert k <= math.ceil(np.float32(tau) * N)
        assert k >= prev                       # monotone in tau (cf. the tau ablation)
        prev = k
    k, theta, mask = vo.threshold_topk(P, 1.0)
    assert k == N and mask.all()


def test_uniform_pool_and_tie_order():
    P = np.full((16, 8), 1.0 / 8, dtype=np.float32)
    for tau in [0.25, 0.3, 0.5]:
        k, theta, mask = vo.threshold_topk(P, tau)
        assert k == math.ceil(float(np.float32(tau)) * 128 - 1e-9)
        # equal values are taken in ascending (q, j) order: the mask is a prefix of the
        # row-major flattening
        flat = mask.reshape(-1)
        assert flat[:k].all() and not flat[k:].any()


def test_hand_worked_two_block_example():
    g = json.load(open(GOLD))
    K = np.array(g["keys"], dtype=np.float32)[:, None]
    q = np.array([0.5 * math.log(3), 0.5 * math.log(1.5), -math.log(2),
                  -0.5 * math.log(7 / 3)], dtype=np.float32)[:, None]
    off = np.array(g["blk_off"])
    Bm = vo.block_means(K, off)
    assert Bm.reshape(-1).tolist() == [1.0, -1.0]
    P = vo.normalise_rows(vo.block_scores(q, Bm, 1.0))
    np.testing.assert_allclose(P, np.array(g["P"]), atol=2e-7)
    order = np.argsort(-P.reshape(-1), kind="stable")
    assert [[int(i // 2), int(i % 2)] for i in order] == g["sorted_pairs_q_b"]
    np.testing.assert_allclose(np.cumsum(P.reshape(-1)[order].astype(np.float64)) / 4,
                               g["cumsum_over_S"], atol=1e-6)
    for tau, k_ref in g["k_by_tau"].items():
        k, theta, mask = vo.threshold_topk(P, float(tau))
        assert k == k_ref
        sel = {(int(a), int(b)) for a, b in zip(*np.nonzero(mask))}
        assert sel == {tuple(p) for p in g["sorted_pairs_q_b"][:k_ref]}
    # attention on top of it: keys are constant inside a block, so a query that keeps one
    # block outputs that block's mean value; q1 keeps nothing at tau = 0.5
    V = np.array(g["values"], dtype=np.float64)
    k, theta, mask = vo.threshold_topk(P, 0.5)
    O, LSE = vo.masked_attention_fwd(q, K, V, mask, off, 1.0)
    for qi, ref in g["O_tau_0.5"].items():
        np.testing.assert_allclose(O[int(qi)], ref, atol=1e-12)
    assert LSE[1] == -np.inf and np.all(np.isfinite(LSE[[0, 2, 3]]))
    k, theta, mask = vo.threshold_topk(P, 0.75)
    O, LSE = vo.masked_attention_fwd(q, K, V, mask, off, 1.0)
    np.testing.assert_allclose(O[1], g["O_tau_0.75_q1"], atol=1e-6)


def test_csr_views_are_consistent():
    rng = np.random.default_rng(9)
    mask = rng.random((50, 7)) < 0.3
    mask[5] = False
    blk_ptr, q_idx, row_ptr, col_idx = vo.csr_from_mask(mask)
    assert blk_ptr[-1] == row_ptr[-1] == mask.sum()
    rebuilt = np.zeros_like(mask)
    for j in range(7):
        qs = q_idx[blk_ptr[j]:blk_ptr[j + 1]]
        assert np.all(np.diff(qs) > 0)
        rebuilt[qs, j] = True
    assert np.array_equal(rebuilt, mask)
    rebuilt2 = np.zeros_like(mask)
    for q in range(50):
        cs = col_idx[row_ptr[q]:row_ptr[q + 1]]
        assert np.all(np.diff(cs) > 0)
        rebuilt2[q, cs] = True
    assert np.array_equal(rebuilt2, mask)
    assert row_ptr[5] == row_ptr[6]


# ----------------------------------------------------------------- selection variants (ablation)
def _rank_before(row, j):
    """Brute force: entries of `row` ranked before entry j (larger value, or equal and lower index)."""
    return [i for i in range(len(row)) if row[i] > row[j] or (row[i] == row[j] and i < j)]


@pytest.mark.parametrize("seed", range(4))
def test_local_topk_brute_force(seed):
    rng = np.random.default_rng(200 + seed)
    S, nb, k = 9, 7, int(rng.integers(1, 7))
    P = vo.normalise_rows((rng.standard_normal((S, nb)) * 2).astype(np.float32))
    P[3] = np.float32(1.0 / nb)                       # a row of ties: lowest block indices win
    mask = vo.local_topk(P, k)
    assert np.all(mask.sum(1) == k)
    for q in range(S):
        for j in range(nb):
            assert mask[q, j] == (len(_rank_before(P[q], j)) < k)
    assert mask[3, :k].all() and not mask[3, k:].any()
    assert vo.local_topk(P, nb + 5).all()


@pytest.mark.parametrize("tau", [0.2, 0.5, 0.9])
def test_local_threshold_brute_force(tau):
    rng = np.random.default_rng(300)
    P = vo.normalise_rows((rng.standard_normal((12, 6)) * 2).astype(np.float32))
    mask = vo.local_threshold(P, tau)
    t32 = float(np.float32(tau))
    for q in range(12):
        for j in range(6):
            before = math.fsum(float(P[q, i]) for i in _rank_before(P[q], j))
            if abs(before - t32) > 1e-9:
                assert mask[q, j] == (before < t32)
        # the kept mass reaches tau, and dropping the weakest kept block would fall short
        kept = np.sort(P[q][mask[q]].astype(np.float64))[::-1]
        assert kept.sum() >= t32 - 1e-7 and kept[:-1].sum() < t32 + 1e-7
    assert np.all(mask.sum(1) >= 1)
    assert vo.local_threshold(P, 1.0).all()


def test_global_topk_matches_threshold_machinery():
    rng = np.random.default_rng(301)
    P = vo.normalise_rows((rng.standard_normal((20, 5)) * 2).astype(np.float32))
    k, theta, mask = vo.global_topk(P, 37)
    assert k == 37 and mask.sum() == 37
    flat = np.sort(P.reshape(-1))[::-1]
    assert theta == flat[36] and P[mask].min() >= P[~mask].max()
    # the threshold rule with the mass of those 37 pairs as tau picks the same set
    tau = float(flat[:37].astype(np.float64).sum() / 20)
    k2, _, mask2 = vo.threshold_topk(P, np.nextafter(np.float32(tau), np.float32(0)))
    assert k2 == 37 and np.array_equal(mask2, mask)
    k_all, _, m_all = vo.global_topk(P, 10 ** 6)
    assert k_all == 100 and m_all.all()


def test_select_blocks_modes_feed_the_layer():
    from paper_2506_23858_amd import synth
    Q, K, V, dO = synth.make_qkv("tiny")
    out = vo.vmoba_layer(Q, K, V, (4, 8, 16), (2, 4, 4), tau=0.25, mode=vo.MODE_LOCAL_TOPK, topk=3)
    assert np.all(out["mask"].sum(-1) == 3)
    out = vo.vmoba_layer(Q, K, V, (4, 8, 16), (2, 4, 4), tau=0.25, mode=vo.MODE_GLOBAL_TOPK, topk=3)
    assert np.all(out["mask"].sum((-1, -2)) == 3 * 512)


def test_own_block_flag_adds_exactly_the_diagonal_blocks():
    """MODE_OWN_BLOCK: the mask is the plain selection OR the (query, own block) pairs -- brute force over
    positions -- so no row is empty, the cut (theta) is unchanged and k counts the kept pairs.  On the
    hand-worked example at tau = 0.5 the query that kept nothing (q1, block 0) gets its own block."""
    rng = np.random.default_rng(31)
    blk_off = np.array([0, 5, 6, 14, 20])
    S, D = 20, 8
    Q, K = rng.standard_normal((S, D)).astype(np.float32), rng.standard_normal((S, D)).astype(np.float32)
    for mode, topk in ((vo.MODE_GLOBAL_THRESHOLD, 0), (vo.MODE_LOCAL_TOPK, 1), (vo.MODE_GLOBAL_TOPK, 1)):
        plain = vo.select_blocks(Q, K, blk_off, 0.2, 0.35, mode, topk)
        own = vo.select_blocks(Q, K, blk_off, 0.2, 0.35, mode | vo.MODE_OWN_BLOCK, topk)
        expect = plain["mask"].copy()
        for q in range(S):
            j = max(j for j in range(4) if blk_off[j] <= q)
            expect[q, j] = True
        assert np.array_equal(own["mask"], expect)
        assert own["mask"].any(axis=1).all()
        assert own["k"] == expect.sum() and own["theta"] == plain["theta"]
    # the golden two-block example: q1 is empty at tau = 0.5 without the flag
    keys = np.array([[1.0], [1.0], [-1.0], [-1.0]], dtype=np.float32)
    qs = np.array([[0.5 * np.log(3)], [0.5 * np.log(1.5)], [-np.log(2)], [-0.5 * np.log(7 / 3)]], dtype=np.float32)
    off = np.array([0, 2, 4])
    plain = vo.select_blocks(qs, keys, off, 0.5, 1.0)
    own = vo.select_blocks(qs, keys, off, 0.5, 1.0, vo.MODE_OWN_BLOCK)
    assert not plain["mask"][1].any()
    assert own["mask"].tolist() == [[True, False], [True, False], [False, True], [False, True]]
    assert own["k"] == 4


def test_pool_softmax_reading():
    """normalise_pool / MODE_POOL_SOFTMAX: closed forms and the relation to the per-query soft-max."""
    # worked by hand: scores [[ln 4, 0], [0, 0]] -> exp = [[4, 1], [1, 1]], sum 7
    s = np.array([[np.log(4.0), 0.0], [0.0, 0.0]], dtype=np.float32)
    G = vo.normalise_pool(s)
    np.testing.assert_allclose(G, np.array([[4, 1], [1, 1]]) / 7.0, rtol=1e-6)
    assert vo.threshold_topk(G, 0.5, total=1.0)[0] == 1                     # 4/7 >= 0.5
    k, theta, mask = vo.threshold_topk(G, 0.6, total=1.0)                   # 5/7: ties enter in (q, j) order
    assert k == 2 and mask.tolist() == [[True, True], [False, False]]
    assert vo.threshold_topk(G, 0.75, total=1.0)[0] == 3                    # 6/7
    assert vo.threshold_topk(G, 0.9, total=1.0)[0] == 4
    # invariants on random scores: sums to one, shift invariance, rows renormalise to the row soft-max
    rng = np.random.default_rng(8)
    x = (3 * rng.standard_normal((40, 7))).astype(np.float32)
    G = vo.normalise_pool(x)
    assert abs(G.sum(dtype=np.float64) - 1.0) < 1e-6
    np.testing.assert_allclose(vo.normalise_pool(x + np.float32(2.5)), G, rtol=2e-6)
    np.testing.assert_allclose(G / G.sum(1, keepdims=True), vo.normalise_rows(x), rtol=2e-6)
    # brute force of the cut
    flat = np.sort(G.astype(np.float64).reshape(-1))[::-1]
    for tau in (0.1, 0.37, 0.8):
        k = vo.threshold_topk(G, tau, total=1.0)[0]
        kk = next(i + 1 for i in range(flat.size) if flat[:i + 1].sum() >= float(np.float32(tau)))
        assert k == kk
    # the two readings differ: a query with one large score takes the pool's mass
    Q = np.array([[10.0], [0.0]], dtype=np.float32)
    K = np.array([[1.0], [0.0]], dtype=np.float32)
    off = np.array([0, 1, 2])
    pool = vo.select_blocks(Q, K, off, 0.5, 1.0, vo.MODE_POOL_SOFTMAX)
    rows = vo.select_blocks(Q, K, off, 0.5, 1.0)
    assert pool["mask"].tolist() == [[True, False], [False, False]] and pool["k"] == 1
    assert rows["k"] == 2 and rows["mask"][1].any()
