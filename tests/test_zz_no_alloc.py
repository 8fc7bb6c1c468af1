"""vmoba_select_static (the entry point for callers that cannot allocate) against vmoba_select: same inputs,
bit-identical outputs, on two calls in a row -- the second on a smaller input, so that whatever the first call left
in the library's static scratch array would show."""
import ctypes as C
import math

import numpy as np
import pytest
import torch

from paper_2506_23858_amd import binding as vb, synth
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

OUTPUTS = ("Bmean", "P", "mask", "blk_ptr", "row_ptr", "k_out", "theta")
LISTS = ("q_idx", "col_idx", "pair_pos")


def select_both_ways(grid, block, chunk, tau, dtype, Hh, D, seed, mode=0, topk=0):
    S = grid[0] * grid[1] * grid[2]
    Q, K, V = (synth.to_bf16_grid(synth.iid_normal(seed + i, (1, S, Hh, D))) for i in range(3))
    results = []
    for static in (False, True):
        plan = vb.LayerPlan(1, Hh, D, grid, block, chunk, tau, dtype, need_bwd=False, mode=mode, topk=topk)
        for name in LISTS:                       # entries past a head's nnz are never written: give them a known value
            getattr(plan, name).fill_(-1)
        plan.partition(*(gu.to_dev(x, dtype) for x in (Q, K, V)))
        torch.cuda.synchronize()
        if static:
            vb.vmoba_select_static(plan.B, plan.Hh, plan.S, plan.D, plan.nb, plan.blk_off, plan.Qp, plan.Kp, plan.tau,
                                   plan.score_scale, plan.mode, plan.topk, plan.Bmean, plan.P, plan.mask, plan.blk_ptr,
                                   plan.q_idx, plan.row_ptr, plan.col_idx, plan.pair_pos, plan.cap, plan.k_out,
                                   plan.theta, plan.dev_status)
        else:
            plan.select()
        torch.cuda.synchronize()
        assert int(plan.dev_status.item()) == 0
        results.append({n: getattr(plan, n).cpu().numpy() for n in OUTPUTS + LISTS})
    ref, got = results
    assert int(ref["k_out"].sum()) > 0
    for n in OUTPUTS + LISTS:
        assert np.array_equal(ref[n], got[n]), n
    return ref


def test_static_scratch_select_matches_workspace_select():
    print("[no-alloc] call 1: 4x8x16 grid, 3D blocks, float32, 2 heads", flush=True)
    a = select_both_ways((4, 8, 16), (2, 4, 4), 0, 0.25, torch.float32, 2, 64, 600)
    print("[no-alloc] call 2 (smaller in tokens, blocks and heads): 3x5x7 grid in chunks of 25, bfloat16, 1 head", flush=True)
    b = select_both_ways((3, 5, 7), (0, 0, 0), 25, 0.3, torch.bfloat16, 1, 128, 610)
    assert b["P"].size < a["P"].size and b["row_ptr"].size < a["row_ptr"].size and b["blk_ptr"].size < a["blk_ptr"].size
    print("[no-alloc] call 3: per-query top-k on a ragged grid with 27 blocks", flush=True)
    select_both_ways((5, 7, 9), (2, 3, 4), 0, 0.3, torch.float32, 2, 64, 620, mode=vb.LOCAL_TOPK, topk=3)


def test_static_scratch_rejects_geometries_beyond_its_size():
    """40 heads x 111 600 tokens need ~135 MB of scratch: rejected on the host, nothing launched."""
    L = vb.lib()
    dummy = C.c_void_p(256)
    t = vb.vmoba_tensor(256, vb.VMOBA_BF16, 111600 * 40 * 128, 40 * 128, 128)
    need = vb.vmoba_workspace_bytes(vb.OP_SELECT, 1, 40, 111600, 128, 165, 1 << 20, vb.VMOBA_BF16)
    assert need > vb.SELECT_STATIC_MAX_BYTES
    rc = L.vmoba_select_static(1, 40, 111600, 128, 165, dummy, C.byref(t), C.byref(t), 0.25, 0.1, 0, 0,
                               *([dummy] * 8), 1 << 20, dummy, dummy, dummy, None, None, None)
    assert rc == vb.VMOBA_ERR_WORKSPACE
