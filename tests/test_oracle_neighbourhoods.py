"""Pins of the oracle's bubble and compact-support neighbourhoods (options -n and -p of the paper's
command line) against things other than the oracle: node counts that geometry fixes, an
independent numpy evaluation from real-valued node positions, the k-means limit, and the
identity with the plain Gaussian when the support covers the whole map."""
import numpy as np
import pytest


def _positions(rows, cols, hexagonal):
    y, x = np.divmod(np.arange(rows * cols), cols)
    if hexagonal:
        return np.stack([x + 0.5 * (y % 2), y * np.sqrt(3.0) / 2.0], axis=1)
    return np.stack([x.astype(float), y.astype(float)], axis=1)


def _dist2(rows, cols, hexagonal, toroid):
    """Squared distances between all nodes from their embedded coordinates; on a torus the
    minimum over the nine periodic images (rows even for the hexagonal torus)."""
    p = _positions(rows, cols, hexagonal)
    px = cols
    py = rows * (np.sqrt(3.0) / 2.0 if hexagonal else 1.0)
    best = None
    for sx in ((-1, 0, 1) if toroid else (0,)):
        for sy in ((-1, 0, 1) if toroid else (0,)):
            d = p[:, None, :] - (p[None, :, :] + np.array([sx * px, sy * py]))
            d2 = (d ** 2).sum(-1)
            best = d2 if best is None else np.minimum(best, d2)
    return best


def test_nodes_inside_the_bubble(oracle):
    # interior node of a planar map: itself and its 4 (square) or 6 (hexagonal) neighbours at radius 1
    for grid, want1, want15 in ((oracle.SQUARE, 5, 9), (oracle.HEXAGONAL, 7, 7)):
        rows, cols = 9, 9
        i = 4 * cols + 4
        for r, want in ((1.0, want1), (1.5, want15), (0.9, 1)):
            inside = sum(oracle.neighbourhood_kind(rows, cols, oracle.PLANAR, grid, i, b, r, oracle.BUBBLE)
                         for b in range(rows * cols))
            assert inside == want, (grid, r, inside)


@pytest.mark.parametrize("map_type,grid_type,rows,cols", [("planar", "square", 5, 7), ("toroid", "square", 6, 5),
                                                          ("planar", "hexagonal", 6, 5), ("toroid", "hexagonal", 6, 7)])
@pytest.mark.parametrize("function,compact", [(1, False), (0, True)])
def test_weights_match_real_coordinates(oracle, map_type, grid_type, rows, cols, function, compact):
    mt, gt = oracle.MAP_TYPES[map_type], oracle.GRID_TYPES[grid_type]
    d2 = _dist2(rows, cols, grid_type == "hexagonal", map_type == "toroid")
    r = 2.3                                     # no pair of nodes is at distance exactly 2.3
    assert np.abs(np.sqrt(d2) - r).min() > 1e-6
    inside = d2 <= r * r
    want = inside.astype(float) if function == 1 else np.where(inside, np.exp(-d2 / (2 * r * r)), 0.0)
    k = rows * cols
    got = np.array([[oracle.neighbourhood_kind(rows, cols, mt, gt, i, b, r, function, compact) for b in range(k)]
                    for i in range(k)])
    assert np.allclose(got, want, rtol=0, atol=1e-12)


def test_bubble_below_one_is_kmeans(oracle):
    rng = np.random.default_rng(3)
    rows, cols, dim, n = 4, 5, 6, 200
    k = rows * cols
    X = rng.random((n, dim)).astype(np.float32)
    W = rng.random((k, dim)).astype(np.float32)
    bmu = rng.integers(0, k - 3, size=n).astype(np.int32)           # the last three nodes get nothing
    S, C = oracle.accumulate_dense(X, bmu, k)
    Wn, D = oracle.update(S, C, W, rows, cols, oracle.TOROID, oracle.HEXAGONAL, 0.9, function=oracle.BUBBLE)
    for i in range(k):
        sel = bmu == i
        if sel.any():
            assert np.allclose(Wn[i], X[sel].astype(np.float64).mean(0), rtol=1e-6)
            assert D[i] == sel.sum()
        else:
            assert np.array_equal(Wn[i], W[i]) and D[i] == 0.0


def test_update_with_bubble_matches_numpy(oracle):
    rng = np.random.default_rng(4)
    rows, cols, dim, n = 6, 5, 4, 300
    k = rows * cols
    X = rng.standard_normal((n, dim)).astype(np.float32)
    W = rng.random((k, dim)).astype(np.float32)
    bmu = rng.integers(0, k, size=n).astype(np.int32)
    S, C = oracle.accumulate_dense(X, bmu, k)
    for function, compact in ((1, False), (0, True)):
        r = 1.7
        d2 = _dist2(rows, cols, True, True)
        H = (d2 <= r * r).astype(float)
        if function == 0:
            H = H * np.exp(-d2 / (2 * r * r))
        Wn, D = oracle.update(S, C, W, rows, cols, oracle.TOROID, oracle.HEXAGONAL, r, function=function,
                              compact=compact)
        num, den = H @ S, H @ C
        assert np.allclose(D, den, rtol=1e-12)
        upd = den >= oracle.EPS_MASS
        assert np.allclose(Wn[upd], (num[upd] / den[upd][:, None]).astype(np.float32), rtol=2e-7, atol=1e-9)
        assert np.array_equal(Wn[~upd], W[~upd])


def test_compact_support_wider_than_the_map_is_the_plain_gaussian(oracle):
    rng = np.random.default_rng(5)
    rows, cols, dim = 5, 6, 3
    k = rows * cols
    S = rng.standard_normal((k, dim))
    C = rng.integers(0, 4, size=k).astype(np.float64)
    W = rng.random((k, dim)).astype(np.float32)
    a, Da = oracle.update(S, C, W, rows, cols, oracle.PLANAR, oracle.SQUARE, 9.0)
    b, Db = oracle.update(S, C, W, rows, cols, oracle.PLANAR, oracle.SQUARE, 9.0, compact=True)
    assert np.array_equal(a, b) and np.array_equal(Da, Db)
    c, Dc = oracle.update(S, C, W, rows, cols, oracle.PLANAR, oracle.SQUARE, 2.0, compact=True)
    assert not np.array_equal(a, c)
