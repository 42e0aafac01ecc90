"""Pins of the oracle's batch update (paper: batch equation, neighbourhood equation,
options -g / -m) against closed forms, limits, symmetries and a geometric
construction of the grid distance that does not use the oracle's integer formula.
"""
import math

import numpy as np
import pytest

P, T, SQ, HX = 0, 1, 0, 1
COMBOS = [(P, SQ), (T, SQ), (P, HX), (T, HX)]


def embed(rows, cols, grid):
    """Planar coordinates of every node: odd hexagonal rows shifted by half a cell."""
    y, x = np.divmod(np.arange(rows * cols), cols)
    if grid == HX:
        return np.stack([x + 0.5 * (y % 2), y * math.sqrt(3.0) / 2.0], axis=1)
    return np.stack([x.astype(float), y.astype(float)], axis=1)


def geometric_d2(rows, cols, map_type, grid):
    """Squared distances between embedded nodes; on a torus the nearest periodic image
    (periods: cols along x, rows * row-pitch along y).  Exact for hexagonal tori with an
    even number of rows, where the lattice is periodic."""
    pos = embed(rows, cols, grid)
    pitch = math.sqrt(3.0) / 2.0 if grid == HX else 1.0
    diff = pos[:, None, :] - pos[None, :, :]
    if map_type == P:
        return np.sum(diff ** 2, axis=-1)
    best = np.full((rows * cols, rows * cols), np.inf)
    for sx in (-1, 0, 1):
        for sy in (-1, 0, 1):
            d = diff + np.array([sx * cols, sy * rows * pitch])
            best = np.minimum(best, np.sum(d ** 2, axis=-1))
    return best


@pytest.mark.parametrize("map_type,grid", COMBOS)
def test_grid_distance_matches_geometric_embedding(oracle, map_type, grid):
    rows, cols = 6, 5
    k = rows * cols
    want = geometric_d2(rows, cols, map_type, grid)
    got = np.array([[oracle.grid_q(rows, cols, map_type, grid, i, b) for b in range(k)]
                    for i in range(k)], dtype=np.float64) / 4.0
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-9)


@pytest.mark.parametrize("map_type,grid", COMBOS)
def test_update_matches_dense_kernel_matrix_from_embedding(oracle, map_type, grid):
    """w_i = sum_b H[i,b] S_b / sum_b H[i,b] C_b with H built from embedded coordinates."""
    rows, cols, dim, n, r = 6, 7, 5, 300, 1.7
    k = rows * cols
    rng = np.random.default_rng(11)
    X = rng.standard_normal((n, dim)).astype(np.float32)
    W = rng.random((k, dim)).astype(np.float32)
    bmu = rng.integers(k, size=n).astype(np.int32)
    S, C = oracle.accumulate_dense(X, bmu, k)
    Wn, D = oracle.update(S, C, W, rows, cols, map_type, grid, r)
    H = np.exp(-geometric_d2(rows, cols, map_type, grid) / (2.0 * r * r))
    onehot = np.zeros((n, k))
    onehot[np.arange(n), bmu] = 1.0
    weights = onehot @ H                      # weight of instance j for node i
    want = (weights.T @ X.astype(np.float64)) / weights.sum(axis=0)[:, None]
    np.testing.assert_allclose(D, weights.sum(axis=0), rtol=1e-12)
    np.testing.assert_allclose(Wn, want.astype(np.float32), rtol=2e-7, atol=1e-9)


def test_three_node_line_closed_form(oracle):
    """1x3 planar square map, r = 1, two instances sitting on the end nodes:
    w0 = (a + e^-2 b)/(1 + e^-2), w1 = (a + b)/2, w2 = (e^-2 a + b)/(1 + e^-2)."""
    a, b = np.array([2.0, -1.0]), np.array([-4.0, 3.0])
    X = np.stack([a, b]).astype(np.float32)
    W = np.zeros((3, 2), dtype=np.float32)
    S, C = oracle.accumulate_dense(X, np.array([0, 2], dtype=np.int32), 3)
    Wn, D = oracle.update(S, C, W, 1, 3, P, SQ, 1.0)
    e2 = math.exp(-2.0)
    want = np.stack([(a + e2 * b) / (1 + e2), (a + b) / 2, (e2 * a + b) / (1 + e2)])
    np.testing.assert_allclose(Wn, want.astype(np.float32), rtol=1e-7)
    np.testing.assert_allclose(D, [1 + e2, 2 * math.exp(-0.5), 1 + e2], rtol=1e-14)


def test_two_row_hexagonal_closed_form(oracle):
    """2x2 planar hexagonal map, one instance on node 0.  Squared distances from node 0:
    node 1 -> 1, node 2 (row 1, shifted half a cell) -> 1/4 + 3/4 = 1, node 3 -> 9/4 + 3/4 = 3."""
    X = np.array([[1.0]], dtype=np.float32)
    S, C = oracle.accumulate_dense(X, np.array([0], dtype=np.int32), 4)
    _, D = oracle.update(S, C, np.zeros((4, 1), np.float32), 2, 2, P, HX, 0.8)
    r2 = 2 * 0.8 * 0.8
    np.testing.assert_allclose(D, [1.0, math.exp(-1 / r2), math.exp(-1 / r2), math.exp(-3 / r2)],
                               rtol=1e-14)


@pytest.mark.parametrize("map_type,grid", COMBOS)
def test_radius_to_zero_gives_kmeans_centroids(oracle, map_type, grid):
    rows, cols, dim, n = 6, 6, 4, 400
    k = rows * cols
    rng = np.random.default_rng(21)
    X = rng.random((n, dim)).astype(np.float32)
    W = rng.random((k, dim)).astype(np.float32)
    bmu = rng.integers(0, k // 2, size=n).astype(np.int32) * 2      # odd nodes never hit
    S, C = oracle.accumulate_dense(X, bmu, k)
    Wn, D = oracle.update(S, C, W, rows, cols, map_type, grid, 1e-3)
    sums = np.zeros((k, dim))
    np.add.at(sums, bmu, X.astype(np.float64))
    cnt = np.bincount(bmu, minlength=k)
    hit = cnt > 0
    np.testing.assert_array_equal(Wn[hit], (sums[hit] / cnt[hit, None]).astype(np.float32))
    np.testing.assert_array_equal(Wn[~hit], W[~hit])            # zero mass: weights kept bit-exactly
    assert np.all(D[~hit] < 1e-20) and np.all(D[hit] >= 1.0)


def test_zero_mass_nodes_keep_weights_and_near_nodes_move(oracle):
    """40x1 planar line, r = 1: mass at distance d is exp(-d^2/2), below 1e-20 from d = 10 on."""
    rows, cols = 1, 40
    W = np.random.default_rng(3).random((cols, 3)).astype(np.float32)
    X = np.array([[5.0, 6.0, 7.0]], dtype=np.float32)
    S, C = oracle.accumulate_dense(X, np.array([0], dtype=np.int32), cols)
    Wn, D = oracle.update(S, C, W, rows, cols, P, SQ, 1.0)
    d = np.arange(cols)
    np.testing.assert_allclose(D, np.exp(-d * d / 2.0), rtol=1e-13)
    moved = D >= 1e-20
    assert moved[:10].all() and not moved[10:].any()        # exp(-50) = 1.9e-22 < 1e-20 <= exp(-40.5)
    np.testing.assert_array_equal(Wn[~moved], W[~moved])
    np.testing.assert_allclose(Wn[moved], np.broadcast_to(X, (10, 3)), rtol=1e-7)


@pytest.mark.parametrize("map_type,grid", COMBOS)
def test_identical_instances_pull_every_reached_node_onto_them(oracle, map_type, grid):
    rows, cols, dim = 4, 5, 3
    k = rows * cols
    x0 = np.array([0.25, -3.0, 8.5], dtype=np.float32)
    X = np.tile(x0, (9, 1))
    W = np.random.default_rng(1).random((k, dim)).astype(np.float32)
    bmu = np.array([0, 3, 3, 7, 19, 19, 19, 11, 0], dtype=np.int32)
    S, C = oracle.accumulate_dense(X, bmu, k)
    Wn, D = oracle.update(S, C, W, rows, cols, map_type, grid, 2.0)
    assert np.all(D >= 1e-20)
    np.testing.assert_allclose(Wn, np.broadcast_to(x0, (k, dim)), rtol=3e-7)


def test_huge_radius_gives_global_mean(oracle):
    rows, cols, dim, n = 5, 4, 6, 200
    k = rows * cols
    rng = np.random.default_rng(8)
    X = rng.standard_normal((n, dim)).astype(np.float32)
    bmu = rng.integers(k, size=n).astype(np.int32)
    S, C = oracle.accumulate_dense(X, bmu, k)
    Wn, _ = oracle.update(S, C, np.zeros((k, dim), np.float32), rows, cols, T, HX, 1e7)
    np.testing.assert_allclose(Wn, np.broadcast_to(X.astype(np.float64).mean(0), (k, dim)),
                               rtol=1e-5, atol=1e-7)


@pytest.mark.parametrize("map_type,grid", COMBOS)
def test_affine_equivariance_and_range(oracle, map_type, grid):
    rows, cols, dim, n = 5, 6, 4, 250
    k = rows * cols
    rng = np.random.default_rng(9)
    X = rng.random((n, dim)).astype(np.float32)
    bmu = rng.integers(k, size=n).astype(np.int32)
    W = np.zeros((k, dim), np.float32)
    S, C = oracle.accumulate_dense(X, bmu, k)
    Wn, _ = oracle.update(S, C, W, rows, cols, map_type, grid, 1.3)
    assert np.all(Wn >= X.min(0) - 1e-6) and np.all(Wn <= X.max(0) + 1e-6)   # weighted mean
    X2 = (X * np.float32(4.0) + np.float32(2.0)).astype(np.float32)           # exact in fp32
    S2, C2 = oracle.accumulate_dense(X2, bmu, k)
    Wn2, _ = oracle.update(S2, C2, W, rows, cols, map_type, grid, 1.3)
    np.testing.assert_allclose(Wn2, Wn * 4.0 + 2.0, rtol=1e-6)


def test_learning_rate_cancels(oracle):
    """A constant factor on the neighbourhood weight drops out of the batch equation."""
    rows, cols, dim, n = 4, 4, 3, 100
    rng = np.random.default_rng(10)
    X = rng.random((n, dim)).astype(np.float32)
    bmu = rng.integers(rows * cols, size=n).astype(np.int32)
    S, C = oracle.accumulate_dense(X, bmu, rows * cols)
    W = np.zeros((rows * cols, dim), np.float32)
    W1, D1 = oracle.update(S, C, W, rows, cols, P, SQ, 1.5, scale=1.0)
    W2, D2 = oracle.update(S, C, W, rows, cols, P, SQ, 1.5, scale=0.013)
    np.testing.assert_allclose(W2, W1, rtol=2e-7)
    np.testing.assert_array_equal(D1, D2)


@pytest.mark.parametrize("grid,rows,cols,dy,dx", [(SQ, 5, 7, 2, 3), (HX, 6, 5, 2, 4), (HX, 6, 5, 4, 1)])
def test_torus_translation_symmetry(oracle, grid, rows, cols, dy, dx):
    """Shifting every BMU by a torus translation shifts the new code book with it, bit for bit
    (hexagonal: even number of rows, even row shift, so row parities are preserved)."""
    k, dim, n = rows * cols, 4, 150
    rng = np.random.default_rng(12)
    X = rng.random((n, dim)).astype(np.float32)
    bmu = rng.integers(k, size=n).astype(np.int32)
    y, x = np.divmod(np.arange(k), cols)
    tau = (((y + dy) % rows) * cols + (x + dx) % cols).astype(np.int32)
    W = np.zeros((k, dim), np.float32)
    S, C = oracle.accumulate_dense(X, bmu, k)
    S2, C2 = oracle.accumulate_dense(X, tau[bmu], k)
    W1, D1 = oracle.update(S, C, W, rows, cols, T, grid, 1.1)
    W2, D2 = oracle.update(S2, C2, W, rows, cols, T, grid, 1.1)
    np.testing.assert_allclose(D2[tau], D1, rtol=1e-13)
    np.testing.assert_allclose(W2[tau], W1, rtol=2e-7)


def test_torus_mass_conservation(oracle):
    rows, cols, n = 6, 8, 77
    k = rows * cols
    bmu = np.random.default_rng(13).integers(k, size=n).astype(np.int32)
    X = np.ones((n, 1), np.float32)
    S, C = oracle.accumulate_dense(X, bmu, k)
    _, D = oracle.update(S, C, np.zeros((k, 1), np.float32), rows, cols, T, HX, 1.4)
    h0 = sum(oracle.neighbourhood(rows, cols, T, HX, i, 0, 1.4) for i in range(k))
    np.testing.assert_allclose(D.sum(), n * h0, rtol=1e-12)


def test_sparse_accumulation_equals_dense(oracle):
    from gen import sparse_zipf_csr
    dim, n, k = 300, 90, 16
    csr = sparse_zipf_csr(n, dim, 4, mean_len=10.0, max_len=30)
    X = np.zeros((n, dim), np.float32)
    for j in range(n):
        X[j, csr[1][csr[0][j]:csr[0][j + 1]]] = csr[2][csr[0][j]:csr[0][j + 1]]
    bmu = np.random.default_rng(5).integers(k, size=n).astype(np.int32)
    S1, C1 = oracle.accumulate_csr(csr, dim, bmu, k)
    S2, C2 = oracle.accumulate_dense(X, bmu, k)
    np.testing.assert_array_equal(S1, S2)
    np.testing.assert_array_equal(C1, C2)
    np.testing.assert_array_equal(C1, np.bincount(bmu, minlength=k).astype(np.float64))


def test_whole_epoch_is_bmu_then_update(oracle):
    rows, cols, dim, n = 5, 5, 6, 120
    rng = np.random.default_rng(14)
    X = rng.random((n, dim)).astype(np.float32)
    W = rng.random((rows * cols, dim)).astype(np.float32)
    bmu, Wn = oracle.epoch_dense(X, W, rows, cols, P, HX, 2.0)
    assert np.array_equal(bmu, oracle.bmu_dense(X, W))        # BMUs refer to the incoming code book
    S, C = oracle.accumulate_dense(X, bmu, rows * cols)
    np.testing.assert_array_equal(Wn, oracle.update(S, C, W, rows, cols, P, HX, 2.0)[0])


def test_subset_update_equals_full_update(oracle):
    rows, cols, dim, n = 6, 5, 4, 90
    k = rows * cols
    rng = np.random.default_rng(15)
    X = rng.random((n, dim)).astype(np.float32)
    W = rng.random((k, dim)).astype(np.float32)
    bmu = rng.integers(0, 6, size=n).astype(np.int32)            # far nodes get no mass at r = 0.3
    S, C = oracle.accumulate_dense(X, bmu, k)
    full, D = oracle.update(S, C, W, rows, cols, P, HX, 0.3)
    nodes = np.array([0, 3, 7, 29, 14], dtype=np.int32)
    sub, Dsub = oracle.update_nodes(S, C, W, rows, cols, P, HX, 0.3, nodes)
    np.testing.assert_array_equal(sub, full[nodes])
    np.testing.assert_array_equal(Dsub, D[nodes])
    assert (D < 1e-20).any() and (D >= 1e-20).any()
