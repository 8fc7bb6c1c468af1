"""CPU-side checks of the C-ABI library: it loads, exports every function the header declares,
and its host-only helpers and argument validation work without a GPU."""
import ctypes as C
import os
import re

import pytest

from paper_2506_23858_amd import binding as vb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(vb.LIB_PATH):
        from paper_2506_23858_amd import build
        build.build_lib(verbose=False)
    return vb.lib()


def test_every_declared_symbol_is_exported(L):
    hdr = open(os.path.join(ROOT, "include", "vmoba.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(vmoba_[a-z_]+)\s*\(", hdr))
    assert {"vmoba_partition", "vmoba_select", "vmoba_attn_fwd", "vmoba_attn_bwd"} <= declared
    for name in declared:
        assert hasattr(L, name), name
    assert declared == set(vb.EXPORTS)


def test_layer_kind_cycle():
    assert [vb.vmoba_layer_kind(l) for l in range(6)] == [0, 1, 2, 0, 1, 2]


@pytest.mark.parametrize("grid,block,chunk,S,nb", [
    ((21, 30, 52), (3, 30, 52), 0, 32760, 7), ((21, 30, 52), (21, 5, 13), 0, 32760, 24),
    ((21, 30, 52), (7, 5, 13), 0, 32760, 72), ((21, 30, 52), (0, 0, 0), 1560, 32760, 21),
    ((21, 45, 80), (1, 30, 40), 0, 75600, 84), ((31, 45, 80), (3, 15, 16), 0, 111600, 165),
    ((5, 7, 9), (2, 3, 4), 0, 315, 27),
    # the block shapes of the paper's hyperparameter table on its 720p and fine-tuning grids
    ((21, 45, 80), (21, 9, 10), 0, 75600, 40), ((21, 45, 80), (7, 15, 20), 0, 75600, 36),
    ((24, 36, 64), (3, 36, 64), 0, 55296, 8), ((24, 36, 64), (24, 6, 8), 0, 55296, 48),
    ((24, 36, 64), (8, 12, 8), 0, 55296, 72), ((36, 30, 52), (12, 10, 13), 0, 56160, 36),
])
def test_partition_dims(grid, block, chunk, S, nb):
    g = vb.make_grid(*grid, *block, chunk)
    assert vb.vmoba_partition_dims(g) == (S, nb)
    from oracle import vmoba_oracle as vo
    assert vo.partition_dims(*grid, *block, chunk) == (S, nb)


def test_named_partitions_have_the_papers_block_counts():
    """synth.CONFIGS' entries for the paper's own block shapes (App. A, hyperparameter table)."""
    from paper_2506_23858_amd import synth
    want = {("480p", "1d_tf"): 7, ("480p", "2d_tf"): 24, ("480p", "3d_tf"): 72,
            ("720p", "1d_tf"): 7, ("720p", "2d_tf"): 40, ("720p", "3d_tf"): 36,
            ("train55k", "1d"): 8, ("train55k", "2d"): 48, ("train55k", "3d"): 72,
            ("train56k", "1d"): 12, ("train56k", "2d"): 24, ("train56k", "3d"): 36}
    for (name, kind), nb in want.items():
        c = synth.CONFIGS[name]
        bt, bh, bw, chunk = c["partitions"][kind]
        assert vb.vmoba_partition_dims(vb.make_grid(*c["grid"], bt, bh, bw, chunk))[1] == nb, (name, kind)


def test_bad_arguments_are_rejected_before_any_launch(L):
    g = vb.make_grid(0, 4, 4, 1, 1, 1)
    S, nb = C.c_int64(), C.c_int32()
    assert L.vmoba_partition_dims(C.byref(g), C.byref(S), C.byref(nb)) == vb.VMOBA_ERR_INVALID_ARG
    g = vb.make_grid(4, 4, 4, 2, 2, 2)
    # null perm
    assert L.vmoba_partition(C.byref(g), 0, 1, 1, 64, 0, None, None, None, None, None, None) == vb.VMOBA_ERR_INVALID_ARG
    # unsupported head dimension
    dummy = C.c_void_p(256)
    assert L.vmoba_partition(C.byref(g), 1, 1, 1, 48, 0, None, None, dummy, None, None, None) == vb.VMOBA_ERR_UNSUPPORTED
    t = vb.vmoba_tensor(256, vb.VMOBA_F32, 64 * 64, 64, 64)
    args = [1, 1, 64, 64, 8, dummy, C.byref(t), C.byref(t)]
    tail = [dummy] * 8 + [100, dummy, dummy, dummy, None, None, dummy, 1 << 30, None]
    assert L.vmoba_select(*args, 0.0, 0.125, 0, 0, *tail) == vb.VMOBA_ERR_INVALID_ARG      # tau = 0
    assert L.vmoba_select(*args, 1.5, 0.125, 0, 0, *tail) == vb.VMOBA_ERR_INVALID_ARG      # tau > 1
    assert L.vmoba_select(*args, 0.25, 0.125, 7, 0, *tail) == vb.VMOBA_ERR_UNSUPPORTED     # unknown mode
    assert L.vmoba_select(*args, 0.25, 0.125, vb.LOCAL_TOPK, 0, *tail) == vb.VMOBA_ERR_INVALID_ARG   # top-k mode, k = 0
    tail_small = [dummy] * 8 + [100, dummy, dummy, dummy, None, None, dummy, 16, None]
    assert L.vmoba_select(*args, 0.25, 0.125, 0, 0, *tail_small) == vb.VMOBA_ERR_WORKSPACE
    assert vb.status_string(vb.VMOBA_ERR_WORKSPACE) == "workspace too small"


def test_workspace_sizes_grow_with_capacity(L):
    a = vb.vmoba_workspace_bytes(vb.OP_ATTN_FWD, 1, 2, 512, 64, 16, 1000, vb.VMOBA_F32)
    b = vb.vmoba_workspace_bytes(vb.OP_ATTN_FWD, 1, 2, 512, 64, 16, 2000, vb.VMOBA_F32)
    assert 0 < a < b
    assert vb.vmoba_workspace_bytes(vb.OP_SELECT, 1, 2, 512, 64, 16, 1000, vb.VMOBA_F32) > 0
    assert vb.vmoba_workspace_bytes(vb.OP_ATTN_BWD, 1, 2, 512, 64, 16, 1000, vb.VMOBA_F32) > 0
    assert vb.vmoba_workspace_bytes(99, 1, 2, 512, 64, 16, 1000, vb.VMOBA_F32) == 0
    assert 2048 < vb.nnz_capacity_for(512, 16, 0.25) <= 2048 + 32
    assert vb.nnz_capacity_for(512, 16, 1.0) == 512 * 16
