"""Parity at full size, in the launch configuration bench.py times (480p: 32 760 tokens, 12 heads x
128, bf16) and at the larger shapes (720p forward only, long-sequence stress with ragged blocks).
The float64 oracle needs ~20 s per 480p head, so: selection is compared in full (it is cheap);
attention in full for one whole head per 480p partition kind, and elsewhere on sampled outputs the
oracle computes one group at a time -- all queries that selected one key block: their O, LSE and dQ
rows, and the dK / dV rows of that block, which those queries alone determine.  Bounds and the
record of the measured errors: tests/gpu_util.py."""
import math

import numpy as np
import pytest
import torch

from oracle import vmoba_oracle as vo
from paper_2506_23858_amd import binding as vb, synth
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

_inputs = {}


def get_inputs(name, heads=None):
    key = (name, heads)
    if key not in _inputs:
        _inputs.clear()                       # one configuration resident at a time
        print(f"[fullsize] generating {name} inputs (heads={heads})", flush=True)
        _inputs[key] = synth.make_qkv(name, heads=heads)
    return _inputs[key]


def check_layer_sampled(name, kind, tau, heads=None, bwd=True, sel_heads=None, groups=2, max_rows=20000,
                        mode=0, topk=0, fused_io=False, whole_heads=(), q_in_place=False, kv_in_place=False):
    """sel_heads: heads whose selection is compared in full (default: all).  groups: number of (head, block)
    groups whose attention outputs are compared.  whole_heads: heads whose attention outputs are compared in
    full -- every row of O, LSE, dQ, dK and dV against the float64 oracle under the GPU's mask.
    q_in_place: the library reads Q where the caller has it and numbers queries by token; its query-indexed
    results are brought to block order here before they meet the oracle's."""
    Q, K, V, dO = get_inputs(name, heads)
    c = synth.CONFIGS[name]
    bt, bh, bw, chunk = c["partitions"][kind]
    D, Hh = c["D"], Q.shape[2]
    scale = 1.0 / math.sqrt(D)
    dtype = torch.bfloat16
    q_in_place = q_in_place or kv_in_place
    fused_io = fused_io or q_in_place
    case = f"{name}-{kind} tau={tau} mode={mode} heads={Hh}" + (" kv-in-place" if kv_in_place else " q-in-place" if q_in_place
                                                                  else " fused-io" if fused_io else "")
    print(f"[fullsize] {case} bwd={bwd}: GPU layer", flush=True)
    plan = vb.LayerPlan(1, Hh, D, c["grid"], (bt, bh, bw), chunk, tau, dtype, need_bwd=bwd,
                        mode=mode, topk=topk, fused_io=fused_io, q_in_place=q_in_place, kv_in_place=kv_in_place)
    dev = [gu.to_dev(x, dtype) for x in ((Q, K, V, dO) if bwd else (Q, K, V))]
    plan.forward(*dev[:3])
    if bwd:
        plan.backward(dev[3])
    torch.cuda.synchronize()
    assert int(plan.dev_status.item()) == 0
    S, nb, cap = plan.S, plan.nb, plan.cap
    perm, inv, off = vo.partition_index(*c["grid"], bt, bh, bw, chunk)
    assert np.array_equal(plan.perm.cpu().numpy(), perm)
    assert np.array_equal(plan.blk_off.cpu().numpy(), off)
    mask_q = gu.unpack_mask(plan.mask.cpu().numpy(), nb)[0]              # rows numbered by query id
    mask_gpu = mask_q[:, perm] if q_in_place else mask_q                 # rows in block order
    k_gpu = plan.k_out.cpu().numpy()
    blk_ptr = plan.blk_ptr.cpu().numpy()
    row_ptr = plan.row_ptr.cpu().numpy()
    q_idx = plan.q_idx.cpu().numpy().reshape(Hh, cap)
    col_idx = plan.col_idx.cpu().numpy().reshape(Hh, cap)
    pair_pos = plan.pair_pos.cpu().numpy().reshape(Hh, cap)
    Qp_all, Kp_all, Vp_all = (vo.gather_rows(x, perm)[0] for x in (Q, K, V))
    if not q_in_place:
        assert np.array_equal(gu.np32(plan.Qp.permute(0, 2, 1, 3))[0], Qp_all)          # permutation bit-exact
    if not kv_in_place:
        assert np.array_equal(gu.np32(plan.Kp.permute(0, 2, 1, 3))[0], Kp_all)
    LSE = plan.LSE.cpu().numpy()[0]
    if q_in_place:
        LSE = LSE[:, perm]

    def block_order(t):          # caller layout [1, S, Hh, D] on the device -> [Hh, S, D] in block order
        return np.ascontiguousarray(gu.np32(t)[0][perm].transpose(1, 0, 2))

    if fused_io:                 # the attention kernels wrote the caller's layout themselves
        Op = block_order(plan.O)
    else:
        Op = gu.np32(plan.Op.permute(0, 2, 1, 3))[0]
        assert np.array_equal(block_order(plan.O), Op)                          # inverse permutation exact
    if bwd:
        dOp_all = vo.gather_rows(dO, perm)[0]
        if fused_io:
            dQp, dKp, dVp = (block_order(t) for t in (plan.dQ, plan.dK, plan.dV))
        else:
            assert np.array_equal(gu.np32(plan.dOp.permute(0, 2, 1, 3))[0], dOp_all)
            dQp, dKp, dVp = (gu.np32(t.permute(0, 2, 1, 3))[0] for t in (plan.dQp, plan.dKp, plan.dVp))
            assert np.array_equal(block_order(plan.dK), dKp)

    # ---- selection, in full, for the chosen heads; list consistency for every head
    g = dict(mask=mask_q[None], k=k_gpu.reshape(1, Hh), blk_ptr=blk_ptr.reshape(1, Hh, nb + 1),
             row_ptr=row_ptr.reshape(1, Hh, S + 1), q_idx=q_idx[None], col_idx=col_idx[None], pair_pos=pair_pos[None])
    P_gpu = plan.P.cpu().numpy()[0]
    if q_in_place:
        P_gpu = P_gpu[:, perm]
    for h in range(Hh):
        gu.check_lists(g, 0, h)
    for h in (range(Hh) if sel_heads is None else sel_heads):
        sel = vo.select_blocks(Qp_all[h], Kp_all[h], off, tau, scale, mode, topk)
        o = dict(P=sel["P"][None, None], theta=np.array([[sel["theta"]]]), mask=sel["mask"][None, None],
                 k=np.array([[sel["k"]]]))
        gh = dict(mask=mask_gpu[None, h:h + 1], k=k_gpu[h:h + 1].reshape(1, 1))
        nband, ndiff = gu.check_selection(gh, o, 0, 0, mode=mode, tau=tau, topk=topk)
        assert np.abs(P_gpu[h] - sel["P"]).max() <= 5e-7
        print(f"   head {h}: k_gpu={k_gpu[h]} k_oracle={sel['k']} band={nband} flipped={ndiff} "
              f"pair fraction={k_gpu[h] / (S * nb):.3f} empty rows={(~mask_gpu[h].any(1)).mean():.3f}", flush=True)
    del P_gpu

    # ---- attention, whole heads: every row of every output
    for h in whole_heads:
        print(f"   whole head {h}: float64 oracle over all {S} rows", flush=True)
        m = mask_gpu[h]
        O_ref, LSE_ref = vo.masked_attention_fwd(Qp_all[h], Kp_all[h], Vp_all[h], m, off, scale)
        rows = f"head {h}, all rows"
        gu.check_output(case, "O", Op[h], O_ref, dtype, rows=rows)
        live = np.isfinite(LSE_ref)
        assert np.array_equal(np.isfinite(LSE[h]), live)
        gu.check_output(case, "LSE", LSE[h][live], LSE_ref[live], dtype, rows=rows)
        del O_ref
        if bwd:
            dQ_ref, dK_ref, dV_ref = vo.masked_attention_bwd(Qp_all[h], Kp_all[h], Vp_all[h], m, off, scale, dOp_all[h])
            gu.check_output(case, "dQ", dQp[h], dQ_ref, dtype, rows=rows)
            gu.check_output(case, "dK", dKp[h], dK_ref, dtype, rows=rows)
            gu.check_output(case, "dV", dVp[h], dV_ref, dtype, rows=rows)
            del dQ_ref, dK_ref, dV_ref

    # ---- attention, sampled: all queries of a few (head, block) groups
    rng = np.random.default_rng(17)
    picks = [(0, int(rng.integers(nb))), (Hh - 1, nb - 1), (Hh // 2, int(rng.integers(nb))), (Hh // 3, 0)][:groups]
    for h, j in picks:
        lst = q_idx[h][blk_ptr[h, j]:blk_ptr[h, j + 1]].astype(np.int64)
        if lst.size == 0:
            continue
        if q_in_place:
            lst = np.sort(inv[lst].astype(np.int64))       # token ids -> block-order positions
        complete = lst.size <= max_rows
        lst = lst[:max_rows]
        rows = f"head {h}: the {lst.size} queries that kept block {j} (L={off[j + 1] - off[j]})"
        print(f"   attention group {rows} (complete={complete})", flush=True)
        m = mask_gpu[h][lst]
        O_ref, LSE_ref = vo.masked_attention_fwd(Qp_all[h][lst], Kp_all[h], Vp_all[h], m, off, scale)
        gu.check_output(case, "O", Op[h][lst], O_ref, dtype, rows=rows)
        gu.check_output(case, "LSE", LSE[h][lst], LSE_ref, dtype, rows=rows)
        if not bwd:
            continue
        dQ_ref, dK_ref, dV_ref = vo.masked_attention_bwd(Qp_all[h][lst], Kp_all[h], Vp_all[h], m, off, scale,
                                                         dOp_all[h][lst])
        gu.check_output(case, "dQ", dQp[h][lst], dQ_ref, dtype, rows=rows)
        if complete:          # those queries alone determine dK and dV of block j
            a, b = off[j], off[j + 1]
            gu.check_output(case, "dK", dKp[h][a:b], dK_ref[a:b], dtype, rows=f"head {h}: keys of block {j}")
            gu.check_output(case, "dV", dVp[h][a:b], dV_ref[a:b], dtype, rows=f"head {h}: keys of block {j}")
    # rows that kept nothing
    empty = ~mask_gpu.any(2)
    assert np.all(Op[empty] == 0) and np.all(LSE[empty] == -np.inf)
    if bwd:
        assert np.all(dQp[empty] == 0)


# a whole head for the 3D and the 2D partition (a different head each; the float64 oracle needs ~20 s per head)
WHOLE_HEAD = {"3d": [5], "2d": [8], "1d": []}


@pytest.mark.parametrize("kind", ["3d", "2d", "1d"])
def test_480p_layer(kind):
    """The 480p workload, outputs written in the caller's order by the attention calls: selection of all 12 heads in
    full; for the 3D and 2D partitions one whole head -- all 32 760 rows of O, LSE, dQ, dK, dV -- against the float64
    oracle; and four more (head, block) groups on other heads."""
    check_layer_sampled("480p", kind, 0.25, fused_io=True, whole_heads=WHOLE_HEAD[kind], groups=4)


def test_480p_separate_partition_calls():
    check_layer_sampled("480p", "3d", 0.25, sel_heads=[4], groups=1)


@pytest.mark.parametrize("kind", ["3d", "1d"])
def test_480p_queries_in_place(kind):
    """The configuration bench.py times: only K and V rearranged, Q read where the caller has it (no gather of Q, no
    copy of dO); for the 1D partition a whole head."""
    check_layer_sampled("480p", kind, 0.25, sel_heads=[1, 10], groups=3, q_in_place=True,
                        whole_heads=[2] if kind == "1d" else [])


@pytest.mark.parametrize("kind", ["3d", "2d"])
def test_480p_keys_in_place(kind):
    """Nothing rearranged in memory: K and V read where the caller has them through the partition's row map."""
    check_layer_sampled("480p", kind, 0.25, sel_heads=[3, 7], groups=3, kv_in_place=True)


@pytest.mark.parametrize("kind", ["3d", "2d", "1d"])
def test_480p_tau_half(kind):
    """The workload's second threshold, all three partitions."""
    check_layer_sampled("480p", kind, 0.5, sel_heads=[0, 5, 11], groups=2, fused_io=(kind != "3d"))


@pytest.mark.parametrize("kind,topk,n_blocks", [("1d_tf", 2, 7), ("2d_tf", 6, 24), ("3d_tf", 18, 72)])
def test_480p_local_topk(kind, topk, n_blocks):
    """The training-free setting (App. A, hyperparameter table): per-query top-k with k = 2 | 6 | 18 of
    7 | 24 | 72 blocks for the 1D | 2D | 3D layers at 480p; forward only, as in inference."""
    c = synth.CONFIGS["480p"]
    assert len(vo.partition_index(*c["grid"], *c["partitions"][kind])[2]) - 1 == n_blocks
    check_layer_sampled("480p", kind, 0.25, bwd=False, sel_heads=[0, 6], mode=vb.LOCAL_TOPK, topk=topk, max_rows=12000)


def test_480p_other_variants():
    """Per-query threshold and global top-k at full size, forward and backward."""
    check_layer_sampled("480p", "3d", 0.25, sel_heads=[3], groups=1, mode=vb.LOCAL_THRESHOLD)
    check_layer_sampled("480p", "3d", 0.25, sel_heads=[9], groups=1, mode=vb.GLOBAL_TOPK, topk=18)


@pytest.mark.parametrize("kind", ["1d", "2d", "2d_half", "3d"])
def test_720p_forward_sampled(kind):
    """720p inference shape (75 600 tokens), forward only, every partition of the cycle: chunks of 2100 tokens; the
    2D partition 1x30x40, which does not divide the 45-row frame, so half of its blocks are truncated (1200 and 600
    tokens); its frame-halves reading 1x45x40 (42 blocks of 1800); 3D blocks 3x15x40."""
    check_layer_sampled("720p", kind, 0.25, bwd=False, sel_heads=[0, 7] if kind in ("2d", "3d") else [7],
                        groups=2 if kind in ("2d", "3d") else 1, max_rows=8000)


@pytest.mark.parametrize("name,kind,n_blocks", [
    ("720p", "2d_tf", 40), ("720p", "3d_tf", 36),
    ("train55k", "1d", 8), ("train55k", "2d", 48), ("train55k", "3d", 72),
    ("train56k", "3d", 36),
])
def test_paper_table_block_shapes(name, kind, n_blocks):
    """The block shapes of the paper's hyperparameter table (App. A) on its 720p grid and on the two grids it
    fine-tunes on (24x36x64 = 55 296 and 36x30x52 = 56 160 latent tokens), with its training setting -- global
    threshold, tau = 0.25, forward and backward -- on 2 heads, queries left in place."""
    c = synth.CONFIGS[name]
    assert len(vo.partition_index(*c["grid"], *c["partitions"][kind])[2]) - 1 == n_blocks
    check_layer_sampled(name, kind, 0.25, heads=2, sel_heads=[1], groups=1, max_rows=8000, q_in_place=True)


@pytest.mark.parametrize("tau", [0.25, 0.75])
def test_stress_shape_reduced_heads(tau):
    """Long-sequence stress shape (31x45x80 = 111 600 tokens, blocks 3x15x16: 165 blocks, the last temporal slab
    truncated to one frame) with 3 of its 40 heads (one per blur width), forward and backward, at the low and the high
    end of its threshold sweep.  165 blocks: the matrix-core score kernel keeps the block means in LDS as float32."""
    check_layer_sampled("stress", "3d", tau, heads=3, sel_heads=[0, 1, 2] if tau < 0.5 else [1], groups=2 if tau < 0.5 else 1,
                        max_rows=8000, q_in_place=tau >= 0.5)


def test_selection_invariants_many_heads_long_workgroup_shares():
    """Selection alone at a shape no CPU run can follow (64 heads x 20 480 tokens x 250 blocks: 328 M scores), checked
    through what defines the result (Eq. 4, Eq. 3) with plain torch reductions in float64 on the library's own P.
    The shape is chosen for the score kernel's bookkeeping: a workgroup's share of the (head, tile) list is 20 tiles
    of 256 queries x 256 block columns, more than the 16 after which it must flush its packed histogram words, and
    crosses head boundaries; the refinement passes run with more workgroups per head than compute units / heads."""
    B, Hh, D, grid, chunk, tau = 1, 64, 128, (20, 32, 32), 82, 0.25
    S = grid[0] * grid[1] * grid[2]
    gen = torch.Generator(device="cuda").manual_seed(20250628)
    Q = torch.randn(B, S, Hh, D, generator=gen, device="cuda").to(torch.bfloat16)
    K = (2.0 * torch.randn(B, S, Hh, D, generator=gen, device="cuda")).to(torch.bfloat16)
    plan = vb.LayerPlan(B, Hh, D, grid, (0, 0, 0), chunk, tau, torch.bfloat16, need_bwd=False, kv_in_place=True)
    nb = plan.nb
    assert nb == 250
    plan.partition(Q, K, K)
    plan.select()
    torch.cuda.synchronize()
    assert int(plan.dev_status.item()) == 0
    shifts = torch.arange(32, device="cuda", dtype=torch.int32)
    target = tau * S
    for h in range(Hh):
        P = plan.P[0, h]
        theta = float(plan.theta[h].item())
        k = int(plan.k_out[h].item())
        assert float((P.double().sum(dim=1) - 1.0).abs().max().item()) < 1e-5, h
        sel = ((plan.mask[0, h].unsqueeze(-1) >> shifts) & 1).bool().reshape(S, -1)
        assert not bool(sel[:, nb:].any().item()), h                 # no bit beyond the last block
        sel = sel[:, :nb]
        assert int(sel.sum().item()) == k, h
        assert int(plan.row_ptr[h, S].item()) == k and int(plan.blk_ptr[h, nb].item()) == k, h
        assert bool(sel[P > theta].all().item()), h                   # everything above theta is kept ...
        assert not bool(sel[P < theta].any().item()), h               # ... nothing below it
        mass = float(P[sel].double().sum().item())
        assert mass >= target - 1e-4, (h, mass, target)               # the kept pairs reach tau * S (Eq. 4) ...
        assert mass - theta < target + 1e-4, (h, mass, theta)         # ... and would not without the smallest of them
