"""The two-level dense BMU search (coarse one-product pass, block selection, sorted tiles, split-fp16 pass
over the listed blocks) against the oracle, on the cases its block selection could get wrong: maps of many
node blocks, equal and nearly equal nodes in different blocks (ties go to the lowest index, so the block of
the lower copy must stay in), code books of equal rows (every block listed), sizes that leave ragged tiles
and blocks, tiles whose lists are shorter than the number of workgroups that share them.
"""
import numpy as np
import pytest

from tests import parity as P

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _bmus(W, X, rows, cols, filter="two_level"):
    from paper_1305_1422_amd import Som
    som = Som(rows, cols, W.shape[1], codebook=torch.from_numpy(W), filter=filter)
    b = som.bmus(P.to_dev(X)).cpu().numpy()
    stats = som.stats()
    som.close()
    return b, stats


def _ordered_map(rng, rows, cols, dim, clusters):
    """A code book that looks like a trained map: smooth over the grid, so that the nodes near an instance's BMU
    sit in a few node blocks, and the other blocks are far away."""
    anchors = rng.random((clusters, dim))
    gy, gx = np.divmod(np.arange(rows * cols), cols)
    u = np.stack([gy / max(rows - 1, 1), gx / max(cols - 1, 1)], 1)
    cpos = rng.random((clusters, 2))
    d2 = ((u[:, None, :] - cpos[None, :, :]) ** 2).sum(-1)
    wgt = np.exp(-d2 / 0.01)
    wgt /= wgt.sum(1, keepdims=True)
    return (wgt @ anchors).astype(np.float32), anchors


@pytest.mark.parametrize("n,rows,cols,dim", [(3000, 40, 45, 96), (129, 1, 129, 40), (1, 30, 50, 7), (2500, 64, 64, 200)])
def test_ordered_map_matches_the_oracle(oracle, n, rows, cols, dim):
    rng = np.random.default_rng(4100 + n)
    W, anchors = _ordered_map(rng, rows, cols, dim, 12)
    X = (anchors[rng.integers(12, size=n)] + 0.03 * rng.standard_normal((n, dim))).astype(np.float32)
    b, _ = _bmus(W, X, rows, cols)
    P.check_bmus_dense(oracle, X, W, b)
    b1, _ = _bmus(W, X, rows, cols, "split_f16")
    assert np.array_equal(b, b1)


def test_random_code_book_lists_many_blocks(oracle):
    """Unordered nodes: the candidates of a tile are spread over all blocks, the fine pass runs nearly everywhere."""
    rng = np.random.default_rng(4200)
    rows, cols, dim, n = 37, 41, 64, 2000
    W = rng.random((rows * cols, dim)).astype(np.float32)
    X = rng.random((n, dim)).astype(np.float32)
    b, _ = _bmus(W, X, rows, cols)
    P.check_bmus_dense(oracle, X, W, b)


def test_copies_of_the_best_node_in_other_blocks(oracle):
    """Every instance's nearest node has an exact copy 5 blocks further up and one a block further down: the
    lowest of the three must win, i.e. the coarse selection keeps all three blocks (equal rows have equal coarse
    scores) and the order of the listed blocks is ascending."""
    rng = np.random.default_rng(4300)
    rows, cols, dim, n = 30, 64, 48, 1500                       # 1,920 nodes = 15 blocks
    k = rows * cols
    W = rng.random((k, dim)).astype(np.float32)
    src = rng.integers(640, 1152, size=n)                        # blocks 5 .. 8
    X = (W[src] + 0.001 * rng.standard_normal((n, dim))).astype(np.float32)
    lower = src - 128 * rng.integers(1, 6, size=n)               # a copy 1 .. 5 blocks below
    upper = src + 128 * rng.integers(1, 6, size=n)
    Wc = W.copy()
    for s, lo, up in zip(src, lower, upper):
        Wc[lo] = W[s]
        Wc[up] = W[s]
    W = Wc
    b, _ = _bmus(W, X, rows, cols)
    want = oracle.bmu_dense(X, W)
    assert np.array_equal(b, want)                               # exact ties: no band, the lowest index


def test_equal_rows_everywhere(oracle):
    """All nodes equal: every block is a candidate for every instance, and node 0 wins."""
    rows, cols, dim, n = 40, 40, 33, 700
    rng = np.random.default_rng(4400)
    W = np.tile(rng.random((1, dim)).astype(np.float32), (rows * cols, 1))
    X = rng.random((n, dim)).astype(np.float32)
    b, _ = _bmus(W, X, rows, cols)
    assert np.all(b == 0)


def test_near_copies_across_blocks_are_decided_exactly(oracle):
    """Nodes that differ by a few ulps and lie in different blocks: neither pass can separate them, the exact
    stage must see all of them."""
    rng = np.random.default_rng(4500)
    rows, cols, dim, n = 25, 52, 128, 600                       # 1,300 nodes, 11 blocks (the last one ragged)
    base = rng.random((5, dim)).astype(np.float32)
    W = base[rng.integers(5, size=rows * cols)].copy()
    W += (rng.integers(-2, 3, size=W.shape) * np.float32(2.0 ** -22)).astype(np.float32)
    X = (base[rng.integers(5, size=n)] + rng.normal(0, 0.05, size=(n, dim))).astype(np.float32)
    b, (refined, collected, rescanned) = _bmus(W, X, rows, cols)
    P.check_bmus_dense(oracle, X, W, b)
    assert collected + rescanned > 0


def test_epochs_with_the_two_level_search(oracle):
    """Whole epochs (search + update) from a random code book down to a small radius, registered data: the
    order of the instances and the block lists change every epoch."""
    from paper_1305_1422_amd import Som, capi
    rng = np.random.default_rng(4600)
    rows, cols, dim, n = 36, 36, 50, 4000
    means = rng.random((9, dim))
    X = (means[rng.integers(9, size=n)] + 0.05 * rng.standard_normal((n, dim))).astype(np.float32)
    W = rng.random((rows * cols, dim)).astype(np.float32)
    som = Som(rows, cols, dim, "toroid", "square", codebook=torch.from_numpy(W), filter="two_level")
    Xd = P.to_dev(X)
    capi.som_set_data_dense(som.ctx, Xd)
    for radius in (18.0, 9.0, 4.0, 2.0, 1.0):
        P.epoch_parity_dense(oracle, som, X, Xd, radius, P.MAP["toroid"], P.GRID["square"])
    som.close()


def test_default_filter_is_two_level_on_large_maps_only(oracle):
    """The default picks the two-level search from 1,024 nodes on; results are the same either way."""
    rng = np.random.default_rng(4700)
    for rows, cols in [(20, 20), (32, 40)]:
        dim, n = 24, 900
        W = rng.random((rows * cols, dim)).astype(np.float32)
        X = rng.random((n, dim)).astype(np.float32)
        b_auto, _ = _bmus(W, X, rows, cols, "auto")
        b_split, _ = _bmus(W, X, rows, cols, "split_f16")
        assert np.array_equal(b_auto, b_split)
        P.check_bmus_dense(oracle, X, W, b_auto)


def test_statistics_of_the_second_pass(oracle):
    """som_two_level_stats: the pairs the second pass worked on, out of all (tile, block) pairs; an ordered map
    lists a small share, a code book of equal rows all of them, a one-level search reports (0, 0)."""
    from paper_1305_1422_amd import Som
    rng = np.random.default_rng(4800)
    rows, cols, dim, n = 48, 48, 40, 3000                        # 2,304 nodes = 18 blocks, 24 tiles
    W, anchors = _ordered_map(rng, rows, cols, dim, 10)
    X = (anchors[rng.integers(10, size=n)] + 0.02 * rng.standard_normal((n, dim))).astype(np.float32)
    som = Som(rows, cols, dim, codebook=torch.from_numpy(W), filter="two_level")
    assert som.two_level_stats() == (0, 0)                       # no search yet
    som.bmus(P.to_dev(X))
    listed, pairs = som.two_level_stats()
    assert pairs == 24 * 18 and 24 <= listed < pairs // 2, (listed, pairs)
    som.set_filter("split_f16")
    som.bmus(P.to_dev(X))
    assert som.two_level_stats() == (0, 0)
    som.close()
    W_eq = np.tile(W[:1], (rows * cols, 1))
    som = Som(rows, cols, dim, codebook=torch.from_numpy(W_eq), filter="two_level")
    som.bmus(P.to_dev(X))
    assert som.two_level_stats() == (pairs, pairs)
    som.close()
