"""GPU parity tests: the HIP path, called through the C ABI, against the CPU oracle, element by
element, on the same seeded inputs.  Integer results (permutation, block offsets, mask, lists)
must match bit-exactly (mask pairs within 1e-6 of the threshold are exempt); outputs and
gradients within max-abs 1e-4 (float32) / 2e-2 (bfloat16) -- the exact policy per output, and the
record of every measured error, are in tests/gpu_util.py."""
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

def oracle_selection(Q, K, grid, block, chunk, tau, mode, topk):
    """Oracle partition + selection (Steps 1-2) for every head; no attention."""
    B, S, Hh, D = Q.shape
    perm, inv_perm, blk_off = vo.partition_index(*grid, *block, chunk)
    nb = len(blk_off) - 1
    Qp, Kp = vo.gather_rows(Q, perm), vo.gather_rows(K, perm)
    o = dict(perm=perm, inv_perm=inv_perm, blk_off=blk_off, Bmean=np.zeros((B, Hh, nb, D), np.float32),
             P=np.zeros((B, Hh, S, nb), np.float32), mask=np.zeros((B, Hh, S, nb), bool),
             k=np.zeros((B, Hh), np.int64), theta=np.zeros((B, Hh), np.float32))
    for b in range(B):
        for h in range(Hh):
            sel = vo.select_blocks(Qp[b, h], Kp[b, h], blk_off, tau, 1.0 / math.sqrt(D), mode, topk)
            for n in ("Bmean", "P", "mask", "k", "theta"):
                o[n][b, h] = sel[n]
    return o


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


def compare_layer(Q, K, V, dO, grid, block, chunk, tau, dtype, label="", mode=0, topk=0, fused_io=False, q_in_place=False,
                  kv_in_place=False):
    B, S, Hh, D = Q.shape
    case = f"{label} S={S} Hh={Hh} D={D} grid={grid} block={block} chunk={chunk} tau={tau} mode={mode}"
    print(f"[parity] {case} {dtype}", flush=True)
    g = gu.run_gpu(Q, K, V, dO, grid, block, chunk, tau, dtype, mode=mode, topk=topk, fused_io=fused_io, q_in_place=q_in_place,
                   kv_in_place=kv_in_place)
    o = oracle_selection(Q, K, grid, block, chunk, tau, mode, topk)
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
    # --- attention under the GPU's own mask; bounds and the error record: tests/gpu_util.py
    ref = oracle_with_gpu_mask(g, Q, K, V, dO, 1.0 / math.sqrt(D))
    gu.check_output(case, "O", g["Op"], ref["Op"], dtype)
    assert np.array_equal(g["O"][:, o["perm"]].transpose(0, 2, 1, 3), g["Op"])      # inverse permutation is exact
    live = np.isfinite(ref["LSE"])
    assert np.array_equal(np.isfinite(g["LSE"]), live)
    assert np.all(g["LSE"][~live] == -np.inf) and np.all(g["Op"][~live] == 0)
    gu.check_output(case, "LSE", g["LSE"][live], ref["LSE"][live], dtype, rows="rows with keys")
    if dO is not None:
        for name in ("dQ", "dK", "dV"):
            gu.check_output(case, name, g[name + "p"], ref[name + "p"], dtype)
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


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("mode,topk", [(0, 0), (vb.LOCAL_TOPK | vb.SELECT_OWN_BLOCK, 2)])
def test_queries_in_place(dtype, mode, topk):
    """Only K and V are rearranged (Eq. 1 as written); Q is read where the caller has it and queries are numbered by
    token: against the oracle, and against the path that also permutes Q -- every query's O, LSE and dQ bit for bit
    (a query's arithmetic does not depend on its neighbours in a tile), dK and dV to rounding (their sums over the
    queries run in another order).  The own-block flag finds a query's block through its position."""
    grid, block = (5, 7, 9), (2, 3, 4)
    S = grid[0] * grid[1] * grid[2]
    Q, K, V, dO = (synth.to_bf16_grid(synth.iid_normal(160 + i, (2, S, 3, 64))) for i in range(4))
    g, o = compare_layer(Q, K, V, dO, grid, block, 0, 0.3, dtype, "q-in-place", mode=mode, topk=topk, q_in_place=True)
    assert g["plan"].Qp is None
    u = gu.run_gpu(Q, K, V, dO, grid, block, 0, 0.3, dtype, mode=mode, topk=topk, fused_io=True)
    for n in ("P", "mask", "k", "O", "LSE", "dQ"):
        assert np.array_equal(g[n], u[n]), n
    tol = 1e-5 if dtype == torch.float32 else 2e-2
    for n in ("dK", "dV"):
        np.testing.assert_allclose(g[n], u[n], rtol=tol, atol=tol)


@pytest.mark.parametrize("dtype,D", [(torch.float32, 64), (torch.bfloat16, 64), (torch.bfloat16, 128)])
def test_keys_in_place(dtype, D):
    """Nothing is rearranged in memory: the partition call only builds the index arrays and every kernel finds key
    position k at row perm[k] of the caller's K and V.  Against the oracle, and bit for bit against the path that
    rearranges K and V (same rows, same order of work, other addresses)."""
    grid, block = (6, 12, 13), (4, 5, 13)            # ragged; blocks of 130 .. 260 keys: several 32-key groups per tile
    S = grid[0] * grid[1] * grid[2]
    Q, K, V, dO = (synth.to_bf16_grid(synth.iid_normal(180 + i, (2, S, 3, D))) for i in range(4))
    g, o = compare_layer(Q, K, V, dO, grid, block, 0, 0.4, dtype, "kv-in-place", kv_in_place=True)
    u = gu.run_gpu(Q, K, V, dO, grid, block, 0, 0.4, dtype, q_in_place=True)
    for n in ("Bmean", "P", "mask", "k", "O", "LSE", "dQ", "dK", "dV"):
        assert np.array_equal(g[n], u[n]), n


def test_keys_in_place_block_longer_than_the_row_table():
    """A key block of 4000 keys: more than the forward tile kernel's in-LDS table of row numbers holds, so its rows are
    looked up in global memory; next to it a block of 608 keys that uses the table."""
    grid = (2, 48, 48)
    S = grid[0] * grid[1] * grid[2]
    Q, K, V, dO = (synth.to_bf16_grid(synth.iid_normal(190 + i, (1, S, 1, 128))) for i in range(4))
    compare_layer(Q, K, V, dO, grid, (0, 0, 0), 4000, 0.7, torch.bfloat16, "kv-in-place-long-block", kv_in_place=True)


@pytest.mark.parametrize("mode", ["permute", "q_in_place", "kv_in_place"])
def test_strided_inputs_from_a_packed_qkv_tensor(mode):
    """Q, K, V as views into one packed [B, S, 3, Hh, D] projection output (token stride 3 * Hh * D), dO and the outputs
    as every other head of wider tensors: the kernels address everything through the strides, so the results are bit
    for bit those of the contiguous tensors."""
    grid, block, tau, D, Hh = (5, 7, 9), (2, 3, 4), 0.3, 128, 2
    S = grid[0] * grid[1] * grid[2]
    Q, K, V, dO = (synth.to_bf16_grid(synth.iid_normal(200 + i, (2, S, Hh, D))) for i in range(4))
    kw = dict(fused_io=True, q_in_place=mode != "permute", kv_in_place=mode == "kv_in_place")
    ref = gu.run_gpu(Q, K, V, dO, grid, block, 0, tau, torch.bfloat16, **kw)
    plan = vb.LayerPlan(2, Hh, D, grid, block, 0, tau, torch.bfloat16, **kw)
    packed = torch.stack([gu.to_dev(x, torch.bfloat16) for x in (Q, K, V)], dim=2)          # [B, S, 3, Hh, D]
    q, k, v = (packed[:, :, i] for i in range(3))
    assert q.stride(1) == 3 * Hh * D and not q.is_contiguous()
    wide = torch.zeros(2, S, 2 * Hh, D, dtype=torch.bfloat16, device="cuda")
    wide[:, :, ::2] = gu.to_dev(dO, torch.bfloat16)
    g_in = wide[:, :, ::2]                                                                  # head stride 2 * D
    for name in ("O", "dQ", "dK", "dV"):
        setattr(plan, name, torch.zeros(2, S, 2 * Hh, D, dtype=torch.bfloat16, device="cuda")[:, :, 1::2])
    plan.forward(q, k, v)
    plan.backward(g_in)
    torch.cuda.synchronize()
    assert int(plan.dev_status.item()) == 0
    for name in ("O", "dQ", "dK", "dV"):
        assert np.array_equal(gu.np32(getattr(plan, name)), ref[name]), name


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
    """64 blocks of 16 tokens; at tau = 0.9 the query-major entries of 64 consecutive rows exceed the window the list
    kernel collects in LDS (it then takes them in several windows), at 0.5 they fit in one."""
    grid, block = (4, 16, 16), (1, 4, 4)
    S = grid[0] * grid[1] * grid[2]
    Q, K, V, dO = (synth.to_bf16_grid(synth.iid_normal(310 + i, (1, S, 2, 128))) for i in range(4))
    g, o = compare_layer(Q, K, V, dO, grid, block, 0, tau, torch.bfloat16, f"many-blocks tau={tau}")
    per_64_rows = g["row_ptr"][0, :, 64::64] - g["row_ptr"][0, :, :-64:64]
    assert (per_64_rows.max() > 2048) == (tau > 0.8), per_64_rows.max()


@pytest.mark.parametrize("grid,block,mode,topk", [
    ((5, 6, 20), (1, 1, 2), 0, 0),       # 300 blocks: a full chunk of 256 and one of 44
    ((4, 16, 16), (1, 2, 1), 0, 0),      # 512 blocks, the most the library takes
    ((5, 6, 20), (1, 1, 2), 1, 7),       # per-query top-k over 300 blocks
    ((5, 6, 20), (1, 1, 2), 4, 0),       # pool soft-max over 300 blocks (row statistics from the chunked path)
])
def test_bf16_more_than_256_blocks(grid, block, mode, topk):
    """Beyond 256 blocks the score kernel runs once per chunk of 256 blocks and a second kernel normalises the rows;
    mask rows have up to 16 words."""
    S = grid[0] * grid[1] * grid[2]
    Q, K, V, dO = (synth.to_bf16_grid(synth.iid_normal(330 + i, (1, S, 2, 128))) for i in range(4))
    g, o = compare_layer(Q, K, V, dO, grid, block, 0, 0.3, torch.bfloat16, f"many-blocks-{g_nb(grid, block)}", mode=mode, topk=topk)
    assert g["nb"] == g_nb(grid, block) > 256


@pytest.mark.parametrize("grid,block,D", [
    ((6, 11, 4), (1, 1, 2), 128),      # 132 blocks: five 32-block tiles, rows of P 16-byte aligned
    ((5, 6, 10), (1, 1, 2), 128),      # 150 blocks: five tiles, rows of P not aligned (block on the lane)
    ((4, 11, 8), (1, 1, 2), 128),      # 176 blocks: six tiles, aligned
    ((3, 7, 18), (1, 1, 2), 64),       # 189 blocks, the most with the pre-split means; D = 64
    ((2, 5, 38), (1, 1, 2), 128),      # 190 blocks: means kept as float32
    ((3, 101, 2), (1, 1, 2), 128),     # 303 blocks: chunked launches with rows of P not aligned
    ((1, 7, 10), (1, 1, 2), 128),      # 35 blocks: two tiles, not aligned
    ((3, 7, 10), (1, 1, 2), 64),       # 105 blocks: four tiles, not aligned; D = 64
])
def test_bf16_block_counts_across_the_score_kernel_variants(grid, block, D):
    """The matrix-core score kernel has one instantiation per number of 32-block tiles (1 to 6 with the block means
    pre-split in LDS), two accumulator layouts (query on the lane for rows of P that start 16-byte aligned, block on
    the lane otherwise), a float32-means form (190 to 256 blocks) and a chunked form (beyond 256): one case per
    combination the larger tests do not reach, each against the oracle in full."""
    S = grid[0] * grid[1] * grid[2]
    Q, K, V, dO = (synth.to_bf16_grid(synth.iid_normal(350 + i, (1, S, 2, D))) for i in range(4))
    g, o = compare_layer(Q, K, V, dO, grid, block, 0, 0.3, torch.bfloat16, f"score-variants-{g_nb(grid, block)}")
    assert g["nb"] == g_nb(grid, block)


def g_nb(grid, block):
    return math.prod(-(-a // b) for a, b in zip(grid, block))


def test_bf16_mid_all_heads():
    """The mid configuration as written: grid 9x30x52 (14 040 tokens), 12 heads x 128, 3D blocks 3x10x13 of 390
    tokens, tau = 0.25, forward and backward, every head and every row against the float64 oracle."""
    c = synth.CONFIGS["mid"]
    Q, K, V, dO = synth.make_qkv("mid")
    assert Q.shape == (1, 14040, 12, 128)
    compare_layer(Q, K, V, dO, c["grid"], (3, 10, 13), 0, 0.25, torch.bfloat16, "mid")


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


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_attention_after_capacity_overflow_is_contained(dtype):
    """One head selects more pairs than the lists hold (its queries are zero, so its P is uniform and tau = 0.25
    keeps a quarter of the pool; the other head's capacity is the same but its selection fits): the status
    word is set, the attention calls read none of the incomplete lists -- the overflowing head comes out as if it
    had selected nothing -- and the other head still matches the oracle."""
    grid, block, tau, D = (4, 8, 16), (2, 4, 4), 0.25, 64
    S = 512
    Q, K, V, dO = (synth.to_bf16_grid(synth.iid_normal(400 + i, (1, S, 2, D))) for i in range(4))
    Q[:, :, 0, :] *= 8.0                # head 0: peaked rows of P -> few pairs reach tau * S
    Q[:, :, 1, :] = 0.0                 # head 1: uniform P -> exactly ceil(tau * S * N_b) pairs
    plan = vb.LayerPlan(1, 2, D, grid, block, 0, tau, dtype)
    full_cap = plan.cap
    plan.cap = 1500                     # head 1 needs 2048
    dev = [gu.to_dev(x, dtype) for x in (Q, K, V, dO)]
    plan.forward(*dev[:3])
    plan.backward(dev[3])
    torch.cuda.synchronize()
    assert int(plan.dev_status.item()) == vb.VMOBA_ERR_CAPACITY
    k = plan.k_out.cpu().numpy()
    assert k[0] <= 1500 < k[1] <= full_cap
    blk_ptr = plan.blk_ptr.cpu().numpy()
    assert blk_ptr[0, -1] == k[0] and np.all(blk_ptr[1] == 0)
    O, LSE = gu.np32(plan.O)[0], plan.LSE.cpu().numpy()[0]
    dQ, dK, dV = (gu.np32(t)[0] for t in (plan.dQ, plan.dK, plan.dV))
    assert np.all(O[:, 1] == 0) and np.all(LSE[1] == -np.inf)
    assert np.all(dQ[:, 1] == 0) and np.all(dK[:, 1] == 0) and np.all(dV[:, 1] == 0)
    # head 0 against the oracle under its own mask
    perm, _, off = vo.partition_index(*grid, *block, 0)
    mask = gu.unpack_mask(plan.mask.cpu().numpy(), plan.nb)[0, 0]
    Qp, Kp, Vp, dOp = (vo.gather_rows(x[:, :, :1], perm)[0, 0] for x in (Q, K, V, dO))
    O_ref, _ = vo.masked_attention_fwd(Qp, Kp, Vp, mask, off, 1.0 / math.sqrt(D))
    dQ_ref, dK_ref, dV_ref = vo.masked_attention_bwd(Qp, Kp, Vp, mask, off, 1.0 / math.sqrt(D), dOp)
    case = f"overflow-contained {gu.dtype_name(dtype)}"
    for name, got, ref in (("O", O, O_ref), ("dQ", dQ, dQ_ref), ("dK", dK, dK_ref), ("dV", dV, dV_ref)):
        gu.check_output(case, name, got[perm][:, 0], ref, dtype, rows="head 0")
