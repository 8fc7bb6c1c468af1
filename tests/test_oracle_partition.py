"""Pins for the oracle's block partition and block means (Sec. 3.2, Eq. 1-2)."""
import numpy as np
import pytest

from oracle import vmoba_oracle as vo


def test_layer_cycle():
    # Eq. 1: l mod 3 = 0 / 1 / 2 -> 1D / 2D / 3D
    assert [vo.layer_kind(l) for l in range(7)] == [0, 1, 2, 0, 1, 2, 0]


@pytest.mark.parametrize("grid,block", [
    ((4, 8, 16), (2, 4, 4)), ((4, 8, 16), (1, 4, 8)), ((5, 7, 9), (2, 3, 4)),
    ((3, 5, 7), (3, 5, 7)), ((3, 5, 7), (1, 1, 1)), ((6, 4, 10), (4, 3, 7)),
])
def test_permutation_is_invertible_and_blocks_are_boxes(grid, block):
    T, H, W = grid
    bt, bh, bw = block
    perm, inv, off = vo.partition_index(T, H, W, bt, bh, bw)
    S = T * H * W
    assert sorted(perm.tolist()) == list(range(S))
    assert np.array_equal(perm[inv], np.arange(S))
    assert np.array_equal(inv[perm], np.arange(S))
    assert off[0] == 0 and off[-1] == S and np.all(np.diff(off) > 0)
    nH, nW = -(-H // bh), -(-W // bw)
    for j in range(len(off) - 1):
        tok = perm[off[j]:off[j + 1]]
        t, h, w = tok // (H * W), (tok // W) % H, tok % W
        # brute force: every token of block j has block coordinates that give id j
        ids = ((t // bt) * nH + (h // bh)) * nW + (w // bw)
        assert np.all(ids == j)
        # row-major inside the box: token ids of a box listed (t,h,w)-lexicographically ascend
        assert np.all(np.diff(tok) > 0)


def test_block_id_order_matches_neighbour_statement():
    # Sec. 3.2: in the 3D pattern the first block's neighbours in width, height and time are
    # the 2nd, 3rd and 5th blocks -> on a 2x2x2 block grid their ids are 1, 2, 4.
    T, H, W, bt, bh, bw = 4, 6, 8, 2, 3, 4
    perm, inv, off = vo.partition_index(T, H, W, bt, bh, bw)

    def block_of(t, h, w):
        p = inv[(t * H + h) * W + w]
        return int(np.searchsorted(off, p, side="right") - 1)

    assert block_of(0, 0, 0) == 0
    assert block_of(0, 0, bw) == 1      # width neighbour
    assert block_of(0, bh, 0) == 2      # height neighbour
    assert block_of(bt, 0, 0) == 4      # time neighbour


@pytest.mark.parametrize("grid,b1,b2,b3,n1,n2,n3", [
    # appendix implementation table: latent grid, temporal / spatial / spatio-temporal block
    # sizes and the block counts printed next to them
    ((21, 30, 52), 3, (5, 13), (7, 5, 13), 7, 24, 72),
    ((21, 45, 80), 3, (9, 10), (7, 15, 20), 7, 40, 36),
    ((24, 36, 64), 3, (6, 8), (8, 12, 8), 8, 48, 72),
])
def test_block_counts_of_paper_table(grid, b1, b2, b3, n1, n2, n3):
    T, H, W = grid
    assert vo.partition_dims(T, H, W, b1, H, W)[1] == n1
    assert vo.partition_dims(T, H, W, T, b2[0], b2[1])[1] == n2
    assert vo.partition_dims(T, H, W, *b3)[1] == n3
    assert vo.partition_dims(T, H, W, *b3)[0] == T * H * W


def test_chunk_mode_is_identity():
    perm, inv, off = vo.partition_index(4, 8, 16, 0, 0, 0, chunk=64)
    assert np.array_equal(perm, np.arange(512))
    assert np.array_equal(off, np.arange(0, 513, 64))
    perm, inv, off = vo.partition_index(3, 5, 7, 0, 0, 0, chunk=25)   # ragged tail
    assert np.array_equal(off, [0, 25, 50, 75, 100, 105])
    assert vo.partition_dims(3, 5, 7, 0, 0, 0, 25) == (105, 5)


def test_1d_box_of_whole_frames_is_identity():
    # Eq. 1, first case: (N^T)(s^T H W) keeps the row-major order
    perm, _, off = vo.partition_index(6, 4, 5, 2, 4, 5)
    assert np.array_equal(perm, np.arange(120))
    assert np.array_equal(off, [0, 40, 80, 120])


@pytest.mark.parametrize("grid,block", [((4, 8, 16), (2, 4, 4)), ((6, 4, 10), (6, 2, 5)),
                                        ((4, 6, 6), (1, 3, 2))])
def test_gather_equals_reshape_transpose(grid, block):
    # on divisible grids Eq. 1 is the einops-style reshape + transpose
    T, H, W = grid
    bt, bh, bw = block
    rng = np.random.default_rng(0)
    X = rng.standard_normal((2, T * H * W, 3, 5)).astype(np.float32)
    perm, inv, off = vo.partition_index(T, H, W, bt, bh, bw)
    Xp = vo.gather_rows(X, perm)
    nT, nH, nW = T // bt, H // bh, W // bw
    ref = X.reshape(2, nT, bt, nH, bh, nW, bw, 3, 5).transpose(0, 7, 1, 3, 5, 2, 4, 6, 8)
    ref = ref.reshape(2, 3, T * H * W, 5)
    assert np.array_equal(Xp, ref)
    assert np.array_equal(vo.scatter_rows(Xp, perm), X)


def test_block_means_library_and_constant():
    rng = np.random.default_rng(1)
    K = rng.standard_normal((96, 7)).astype(np.float32)
    off = np.arange(0, 97, 24)
    Bm = vo.block_means(K, off)
    assert Bm.dtype == np.float32
    np.testing.assert_allclose(Bm, K.reshape(4, 24, 7).astype(np.float64).mean(1), rtol=1e-6, atol=1e-7)
    # ragged: divisor is the real block size
    off2 = np.array([0, 10, 96])
    Bm2 = vo.block_means(K, off2)
    np.testing.assert_allclose(Bm2[0], K[:10].astype(np.float64).mean(0), rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(Bm2[1], K[10:].astype(np.float64).mean(0), rtol=1e-6, atol=1e-7)
    const = np.full((96, 7), 0.37, dtype=np.float32)
    assert np.all(vo.block_means(const, off2) == np.float32(0.37))
