"""GPU parity tests: the HIP path, called through the C ABI, against the CPU oracle, element by
element, on the same seeded inputs.  Integer results (permutation, block offsets, mask, lists)
must match bit-exactly (mask pairs within 1e-6 of the threshold are exempt); outputs and
gradients within max-abs 1e-4 (float32) / 2e-2 (bfloat16)."""
import json
import math
import os

import numpy as np
import pytest
import torch

from oracle import vmoba_oracle as vo
from paper_2506_23858_amd import binding as vb, synth
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

TOL = {torch.float32: 1e-4, torch.bfloat16: 2e-2}
# relative Frobenius-norm bound checked next to the max-abs one, so that small-magnitude
# gradients are not waved through by the absolute tolerance alone
REL = {torch.float32: 2e-5, torch.bfloat16: 1.5e-2}


def rel_err(a, b):
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30))


def oracle_with_gpu_mask(g, Q, K, V, dO, softmax_scale):
    """Oracle attention (fwd + bwd) under the mask the GPU produced, per head, block order."""
    B, S, Hh, D = Q.shape
    perm, blk_off = g["perm"], g["blk_off"]
    Qp, Kp, Vp = (vo.gather_rows(x, perm) for x in (Q, K, V))
    dOp = vo.gather_rows(dO, perm) if dO is not None else None
    res = dict(Op=np.zeros((B, Hh, S, D)), LSE=np.zeros((B, Hh, S)),
               dQp=np.zeros((B, Hh, S, D)), dKp=np.zeros((B, Hh, S, D)), dVp=np.zeros((B, Hh, S, D)))
    for b in range(B):
        for h in range(Hh):
            m = g["mask"][b, h]
            res["Op"][b, h], res["LSE"][b, h] = vo.masked_attention_fwd(Qp[b, h], Kp[b, h], Vp[b, h], m, blk_off, softmax_scale)
            if dO is not None:
                res["dQp"][b, h], res["dKp"][b, h], res["dVp"][b, h] = vo.masked_attention_bwd(
                    Qp[b, h], Kp[b, h], Vp[b, h], m, blk_off, softmax_scale, dOp[b, h])
    return res


def compare_layer(Q, K, V, dO, grid, block, chunk, tau, dtype, label="", mode=0, topk=0, fused_io=False):
    B, S, Hh, D = Q.shape
    print(f"[parity] {label} S={S} Hh={Hh} D={D} grid={grid} block={block} chunk={chunk} tau={tau} {dtype}", flush=True)
    g = gu.run_gpu(Q, K, V, dO, grid, block, chunk, tau, dtype, mode=mode, topk=topk, fused_io=fused_io)
    o = vo.vmoba_layer(Q, K, V, grid, block, tau, dO=None, chunk=chunk, mode=mode, topk=topk)   # selection + its own attention
    # --- partition: bit exact
    assert np.array_equal(g["perm"], o["perm"])
    assert np.array_equal(g["inv_perm"], o["inv_perm"])
    assert np.array_equal(g["blk_off"], o["blk_off"])
    assert np.array_equal(g["Qp"], vo.gather_rows(Q, o["perm"]))
    assert np.array_equal(g["Kp"], vo.gather_rows(K, o["perm"]))
    assert np.array_equal(g["Vp"], vo.gather_rows(V, o["perm"]))
    # --- selection
    np.testing.assert_allclose(g["Bmean"], o["Bmean"], rtol=0, atol=2e-6)
    if (mode & 0xff) == 4:        # pool soft-max: the head's pool sums to one
        np.testing.assert_allclose(g["P"], o["P"], rtol=1e-5, atol=1e-12)
        np.testing.assert_allclose(g["P"].sum((-1, -2), dtype=np.float64), 1.0, atol=5e-6)
    else:
        np.testing.assert_allclose(g["P"], o["P"], rtol=0, atol=5e-7)
        np.testing.assert_allclose(g["P"].sum(-1, dtype=np.float64), 1.0, atol=2e-6)
    for b in range(B):
        for h in range(Hh):
            nband, ndiff = gu.check_selection(g, o, b, h, mode=mode, tau=tau, topk=topk)
            gu.check_lists(g, b, h)
            if (mode & 0xff) in (1, 2):
                assert g["theta"][b, h] == 0
            elif int(g["k"][b, h]) < S * g["nb"]:      # theta is reported as 0 when every pair is kept
                np.testing.assert_allclose(g["theta"][b, h], o["theta"][b, h], atol=1e-6, rtol=2e-5)
            print(f"   head {h}: k_gpu={g['k'][b, h]} k_oracle={o['k'][b, h]} band={nband} flipped={ndiff}", flush=True)
    # --- attention under the GPU's own mask
    ref = oracle_with_gpu_mask(g, Q, K, V, dO, 1.0 / math.sqrt(D))
    tol, rtol = TOL[dtype], REL[dtype]
    o_err, o_mag = np.abs(g["Op"] - ref["Op"]).max(), np.abs(ref["Op"]).max()
    print(f"   Op: max-abs {o_err:.3e} rel {rel_err(g['Op'], ref['Op']):.3e} max|ref| {o_mag:.3e}", flush=True)
    assert o_err <= tol * max(1.0, o_mag), (o_err, o_mag)      # same range-scaled bound as for the gradients
    assert rel_err(g["Op"], ref["Op"]) <= rtol
    assert np.array_equal(g["O"][:, o["perm"]].transpose(0, 2, 1, 3), g["Op"])      # inverse permutation is exact
    live = np.isfinite(ref["LSE"])
    assert np.array_equal(np.isfinite(g["LSE"]), live)
    assert np.all(g["LSE"][~live] == -np.inf) and np.all(g["Op"][~live] == 0)
    np.testing.assert_allclose(g["LSE"][live], ref["LSE"][live], atol=(1e-4 if dtype == torch.float32 else 1e-2))
    if dO is not None:
        for name in ("dQp", "dKp", "dVp"):
            err = np.abs(g[name] - ref[name]).max()
            rel = rel_err(g[name], ref[name])
            mag = np.abs(ref[name]).max()
            print(f"   {name}: max-abs {err:.3e} rel {rel:.3e} max|ref| {mag:.3e}", flush=True)
            # the absolute tolerance is for O(1) values; a bfloat16 result of magnitude x carries a
            # rounding error of up to x * 2^-9 on its own, so the bound grows with the range
            assert err <= tol * max(1.0, mag), (name, err, mag)
            assert rel <= rtol, (name, rel)
        assert np.all(g["dQp"][~live] == 0)
        for name in ("dQ", "dK", "dV"):
            assert np.array_equal(g[name][:, o["perm"]].transpose(0, 2, 1, 3), g[name + "p"])
    return g, o


# ----------------------------------------------------------------------------------- configs
@pytest.mark.parametrize("kind", ["1d", "2d", "3d"])
@pytest.mark.parametrize("tau", [0.25, 0.5])
def test_tiny_config_fp32(kind, tau):
    c = synth.CONFIGS["tiny"]
    Q, K, V, dO = synth.make_qkv("tiny")
    bt, bh, bw, chunk = c["partitions"][kind]
    compare_layer(Q, K, V, dO, c["grid"], (bt, bh, bw), chunk, tau, torch.float32, f"tiny-{kind}")


@pytest.mark.parametrize("grid,block,chunk,D", [
    ((5, 7, 9), (2, 3, 4), 0, 64),          # ragged in all three axes, blocks of 1..24 tokens
    ((3, 5, 7), (0, 0, 0), 25, 128),        # 1D chunks with a short tail, D = 128
    ((6, 10, 12), (6, 5, 4), 0, 64),        # the paper's 2D case: a spatial tile through all frames
    ((4, 4, 5), (4, 4, 1), 0, 64),          # 5 blocks: every 16-byte group of a row of P straddles two rows
    ((2, 4, 33), (2, 4, 1), 0, 64),         # 33 blocks: two mask words per row, groups straddle words and rows
    ((1, 9, 13), (0, 0, 0), 9, 64),         # 13 blocks, S * N_b odd: rows of P not 16-byte aligned
])
def test_ragged_grids_fp32(grid, block, chunk, D):
    S = grid[0] * grid[1] * grid[2]
    Q, K, V, dO = (synth.iid_normal(70 + i, (1, S, 2, D)) for i in range(4))
    compare_layer(Q, K, V, dO, grid, block, chunk, 0.3, torch.float32, "ragged")


# ------------------------------------------------------------ block-choice variants (Sec. 4.3, App. A)
@pytest.mark.parametrize("kind,topk", [("1d", 1), ("2d", 2), ("3d", 4), ("3d", 16), ("3d", 99)])
def test_local_topk_fp32(kind, topk):
    """Per-query top-k, the setting of the training-free runs; k = 16 and 99 keep every block."""
    c = synth.CONFIGS["tiny"]
    Q, K, V, dO = synth.make_qkv("tiny")
    bt, bh, bw, chunk = c["partitions"][kind]
    g, o = compare_layer(Q, K, V, dO, c["grid"], (bt, bh, bw), chunk, 0.25, torch.float32, f"local-topk-{kind}",
                         mode=vb.LOCAL_TOPK, topk=topk)
    assert np.all(g["mask"].sum(-1) == min(topk, g["nb"]))


@pytest.mark.parametrize("tau", [0.25, 0.6, 1.0])
def test_local_threshold_fp32(tau):
    c = synth.CONFIGS["tiny"]
    Q, K, V, dO = synth.make_qkv("tiny")
    g, o = compare_layer(Q, K, V, dO, c["grid"], (2, 4, 4), 0, tau, torch.float32, "local-threshold",
                         mode=vb.LOCAL_THRESHOLD)
    assert np.all(g["mask"].sum(-1) >= 1)           # a query always keeps its best block


@pytest.mark.parametrize("topk", [1, 3, 16])
def test_global_topk_fp32(topk):
    c = synth.CONFIGS["tiny"]
    Q, K, V, dO = synth.make_qkv("tiny")
    g, o = compare_layer(Q, K, V, dO, c["grid"], (2, 4, 4), 0, 0.25, torch.float32, "global-topk",
                         mode=vb.GLOBAL_TOPK, topk=topk)
    assert np.all(g["k"] == min(topk, g["nb"]) * 512)


def test_variants_ragged_bf16():
    """The three variants on a ragged grid (blocks of 1..24 tokens, 70 blocks > one mask word) in bfloat16."""
    grid, block = (5, 7, 9), (1, 2, 3)
    S = grid[0] * grid[1] * grid[2]
    Q, K, V, dO = (synth.to_bf16_grid(synth.iid_normal(90 + i, (1, S, 2, 64))) for i in range(4))
    for mode, topk, tau in ((vb.LOCAL_TOPK, 5, 0.25), (vb.LOCAL_THRESHOLD, 0, 0.3), (vb.GLOBAL_TOPK, 7, 0.25)):
        compare_layer(Q, K, V, dO, grid, block, 0, tau, torch.bfloat16, f"ragged-mode{mode}", mode=mode, topk=topk)


@pytest.mark.parametrize("tau", [0.25, 0.6, 1.0])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_pool_softmax_threshold(tau, dtype):
    """One soft-max over the head's whole pool (the other reading of "normalised")."""
    c = synth.CONFIGS["tiny"]
    Q, K, V, dO = (synth.to_bf16_grid(x) for x in synth.make_qkv("tiny"))
    compare_layer(Q, K, V, dO, c["grid"], (2, 4, 4), 0, tau, dtype, "pool-softmax", mode=vb.POOL_SOFTMAX_THRESHOLD)


@pytest.mark.parametrize("mode,topk", [(0, 0), (1, 2), (3, 2), (4, 0)])
def test_own_block_flag(mode, topk):
    """Every query also keeps the block it lies in (ragged grid, so block boundaries fall inside wavefronts)."""
    grid, block = (5, 7, 9), (2, 3, 4)
    S = grid[0] * grid[1] * grid[2]
    Q, K, V, dO = (synth.iid_normal(140 + i, (1, S, 2, 64)) for i in range(4))
    g, o = compare_layer(Q, K, V, dO, grid, block, 0, 0.15, torch.float32, "own-block", mode=mode | vb.SELECT_OWN_BLOCK, topk=topk)
    assert g["mask"].any(-1).all()
    own = np.repeat(np.arange(g["nb"]), np.diff(g["blk_off"]))
    assert g["mask"][0, :, np.arange(S), own].all()


def test_local_topk_with_equal_scores_takes_lowest_indices():
    """All keys equal -> every block scores the same for every query; ties go to the lower block index."""
    S, D = 512, 64
    Q = synth.iid_normal(5, (1, S, 1, D))
    K = np.ones((1, S, 1, D), dtype=np.float32)
    V = synth.iid_normal(6, (1, S, 1, D))
    g = gu.run_gpu(Q, K, V, None, (8, 8, 8), (2, 4, 4), 0, 0.25, torch.float32, mode=vb.LOCAL_TOPK, topk=3)
    assert g["mask"][0, 0][:, :3].all() and not g["mask"][0, 0][:, 3:].any()
    g = gu.run_gpu(Q, K, V, None, (8, 8, 8), (2, 4, 4), 0, 0.25, torch.float32, mode=vb.GLOBAL_TOPK, topk=3)
    m = g["mask"][0, 0].reshape(-1)
    assert m[:3 * S].all() and not m[3 * S:].any()           # pool order: ascending (query, block)


# ------------------------------------------- outputs written in the caller's token order by the kernels
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_fused_io_matches_oracle_and_unfused(dtype):
    """attn_fwd / attn_bwd with a row map (O, dO, dQ, dK, dV in the caller's order): against the oracle,
    and bit-identical to the path through the separate partition calls (same arithmetic, other addresses)."""
    grid, block = (5, 7, 9), (2, 3, 4)
    S = grid[0] * grid[1] * grid[2]
    Q, K, V, dO = (synth.to_bf16_grid(synth.iid_normal(120 + i, (2, S, 3, 64))) for i in range(4))
    g, o = compare_layer(Q, K, V, dO, grid, block, 0, 0.3, dtype, "fused-io", fused_io=True)
    u = gu.run_gpu(Q, K, V, dO, grid, block, 0, 0.3, dtype)
    for n in ("O", "dQ", "dK", "dV", "LSE"):
        assert np.array_equal(g[n], u[n]), n


def test_tau_one_is_dense_attention():
    c = synth.CONFIGS["tiny"]
    Q, K, V, dO = synth.make_qkv("tiny")
    g, o = compare_layer(Q, K, V, dO, c["grid"], (2, 4, 4), 0, 1.0, torch.float32, "tau=1")
    assert g["mask"].all() and int(g["k"][0, 0]) == 512 * 16
    # and against PyTorch's dense attention on the CPU
    q, k, v = (torch.from_numpy(x).double().permute(0, 2, 1, 3) for x in (Q, K, V))
    dense = torch.nn.functional.scaled_dot_product_attention(q, k, v).permute(0, 2, 1, 3).numpy()
    assert np.abs(g["O"] - dense).max() <= 1e-4


def test_hand_worked_two_block_example():
    """The closed-form example of tests/golden, embedded in D = 64 (other channels zero), scale 1."""
    gold = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "two_block_example.json")))
    D = 64
    Q = np.zeros((1, 4, 1, D), np.float32)
    K = np.zeros((1, 4, 1, D), np.float32)
    V = np.zeros((1, 4, 1, D), np.float32)
    Q[0, :, 0, 0] = [0.5 * math.log(3), 0.5 * math.log(1.5), -math.log(2), -0.5 * math.log(7 / 3)]
    K[0, :, 0, 0] = gold["keys"]
    V[0, :, 0, :2] = gold["values"]
    for tau, k_ref in gold["k_by_tau"].items():
        g = gu.run_gpu(Q, K, V, None, (1, 1, 4), chunk=2, tau=float(tau), score_scale=1.0, softmax_scale=1.0)
        assert int(g["k"][0, 0]) == k_ref
        sel = {(int(a), int(b)) for a, b in zip(*np.nonzero(g["mask"][0, 0]))}
        assert sel == {tuple(p) for p in gold["sorted_pairs_q_b"][:k_ref]}
        np.testing.assert_allclose(g["P"][0, 0], gold["P"], atol=3e-7)
        if tau == "0.5":
            for qi, ref in gold["O_tau_0.5"].items():
                np.testing.assert_allclose(g["O"][0, int(qi), 0, :2], ref, atol=1e-5)
            assert g["LSE"][0, 0, 1] == -np.inf
        if tau == "0.75":
            np.testing.assert_allclose(g["O"][0, 1, 0, :2], gold["O_tau_0.75_q1"], atol=1e-5)


def test_all_ties_take_exactly_k_in_index_order():
    """Q = 0 makes every normalised similarity equal 1/N_b: the cut falls inside a run of equal
    values and must take them in ascending (query, block) order, exactly k of them."""
    S, D, nb = 256, 64, 8
    Q = np.zeros((1, S, 2, D), np.float32)
    K, V = (synth.iid_normal(90 + i, (1, S, 2, D)) for i in range(2))
    for tau in (0.25, 0.3):
        g = gu.run_gpu(Q, K, V, None, (1, 1, S), chunk=S // nb, tau=tau)
        k_ref = math.ceil(float(np.float32(tau)) * S * nb - 1e-9)
        for h in range(2):
            assert int(g["k"][0, h]) == k_ref
            flat = g["mask"][0, h].reshape(-1)
            assert flat[:k_ref].all() and not flat[k_ref:].any()
            gu.check_lists(g, 0, h)


@pytest.mark.parametrize("D", [64, 128])
def test_bf16_small(D):
    """bfloat16 / MFMA path on a grid small enough for the full oracle: ragged blocks whose
    lengths are not multiples of the 64-key chunk, query lists with partial tiles, 3 heads."""
    grid, block = (6, 12, 13), (5, 12, 13) if D == 128 else (4, 5, 13)
    S = grid[0] * grid[1] * grid[2]
    Q, K, V, dO = (synth.to_bf16_grid(synth.blurred_noise(300 + i, grid, 3, D, 1.5)) for i in range(4))
    compare_layer(Q, K, V, dO, grid, block, 0, 0.4, torch.bfloat16, f"bf16-small-D{D}")


@pytest.mark.parametrize("block", [(1, 4, 8), (1, 3, 8)])
def test_bf16_blocks_no_longer_than_one_key_group(block):
    """Key blocks of 32 (and 24, ragged: 16) tokens: the forward and dQ kernels see blocks of a single
    32-key group, and dK/dV of every key comes from the kernel for short block tails alone."""
    grid = (4, 8, 16)
    Q, K, V, dO = (synth.to_bf16_grid(synth.blurred_noise(340 + i, grid, 2, 128, 1.5)) for i in range(4))
    compare_layer(Q, K, V, dO, grid, block, 0, 0.4, torch.bfloat16, f"bf16-one-group-{block}")


@pytest.mark.parametrize("tau", [0.5, 0.9])
def test_bf16_many_blocks_per_row(tau):
    """64 blocks of 16 tokens; at tau = 0.9 the query-major entries of 64 consecutive rows exceed what the list
    kernel collects in LDS (it then writes them directly), at 0.5 they fit."""
    grid, block = (4, 16, 16), (1, 4, 4)
    S = grid[0] * grid[1] * grid[2]
    Q, K, V, dO = (synth.to_bf16_grid(synth.iid_normal(310 + i, (1, S, 2, 128))) for i in range(4))
    g, o = compare_layer(Q, K, V, dO, grid, block, 0, tau, torch.bfloat16, f"many-blocks tau={tau}")
    per_64_rows = g["row_ptr"][0, :, 64::64] - g["row_ptr"][0, :, :-64:64]
    assert (per_64_rows.max() > 2048) == (tau > 0.8), per_64_rows.max()


def test_bf16_mid_lite():
    """The mid configuration's grid and 3D blocks (9x30x52, blocks 3x10x13 of 390 tokens) with 2 of
    its 12 heads, so the float64 oracle finishes in seconds."""
    c = synth.CONFIGS["mid"]
    Q, K, V, dO = synth.make_qkv("mid", heads=2)
    compare_layer(Q, K, V, dO, c["grid"], (3, 10, 13), 0, 0.25, torch.bfloat16, "mid-lite")


def test_selection_is_deterministic():
    c = synth.CONFIGS["tiny"]
    Q, K, V, dO = synth.make_qkv("tiny")
    runs = [gu.run_gpu(Q, K, V, dO, c["grid"], (2, 4, 4), 0, 0.25) for _ in range(3)]
    for r in runs[1:]:
        for name in ("mask", "blk_ptr", "row_ptr", "k", "P", "Op", "dQp", "dKp", "dVp"):
            assert np.array_equal(r[name], runs[0][name]), name
        for h in range(2):
            n = int(r["k"][0, h])            # list entries past the head's nnz are never written
            for name in ("q_idx", "col_idx", "pair_pos"):
                assert np.array_equal(r[name][0, h][:n], runs[0][name][0, h][:n]), name


def test_capacity_overflow_is_reported_not_written():
    from paper_2506_23858_amd import binding as vb
    c = synth.CONFIGS["tiny"]
    Q, K, V, _ = synth.make_qkv("tiny")
    plan = vb.LayerPlan(1, 2, 64, c["grid"], (2, 4, 4), 0, 0.25, torch.float32, need_bwd=False)
    q, k, v = (gu.to_dev(x, torch.float32) for x in (Q, K, V))
    plan.partition(q, k, v)
    plan.cap = 100                      # far below what tau = 0.25 selects
    guard = torch.full_like(plan.q_idx, -7)
    plan.q_idx.copy_(guard)
    plan.select()
    torch.cuda.synchronize()
    assert int(plan.dev_status.item()) == vb.VMOBA_ERR_CAPACITY
    qi = plan.q_idx.cpu().numpy()
    assert np.all(qi[200:] == -7)       # nothing beyond the two heads' 100-entry segments
