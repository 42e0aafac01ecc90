"""Pins of the oracle's best-matching-unit search (paper: BMU equation and the
inequality below it; sparse file format paragraph of the command-line interface).

None of these retype the oracle's loop: they use planted answers, a k-d tree
from scipy (a different nearest-neighbour algorithm), scipy's cdist, and the
equality of the sparse and dense formulations.
"""
import os

import numpy as np
import pytest
from scipy.spatial import cKDTree
from scipy.spatial.distance import cdist

from gen import sparse_zipf_csr

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def densify(csr, dim):
    indptr, indices, values = csr
    n = len(indptr) - 1
    X = np.zeros((n, dim), dtype=np.float32)
    for j in range(n):
        X[j, indices[indptr[j]:indptr[j + 1]]] = values[indptr[j]:indptr[j + 1]]
    return X


def test_instances_equal_to_nodes_map_to_themselves(oracle):
    rng = np.random.default_rng(1)
    W = rng.random((36, 8)).astype(np.float32)
    order = rng.permutation(36)
    bmu, d2 = oracle.bmu_dense(W[order], W, want_d2=True)
    assert np.array_equal(bmu, order.astype(np.int32))
    assert np.all(d2 == 0.0)


def test_duplicate_nodes_resolve_to_lowest_index(oracle):
    rng = np.random.default_rng(2)
    W = rng.random((20, 5)).astype(np.float32)
    W[13] = W[4]
    W[17] = W[4]
    W[9] = W[2]
    X = np.vstack([W[17], W[9], W[13] + np.float32(1e-4)]).astype(np.float32)
    bmu = oracle.bmu_dense(X, W)
    assert bmu.tolist() == [4, 2, 4]


def test_planted_nearest_node(oracle):
    rng = np.random.default_rng(3)
    k, dim = 30, 6
    W = (10.0 * rng.integers(0, 50, size=(k, dim))).astype(np.float32)   # nodes >= 10 apart or equal
    W = np.unique(W, axis=0)
    k = W.shape[0]
    target = rng.integers(k, size=64)
    X = (W[target] + rng.uniform(-1, 1, size=(64, dim))).astype(np.float32)
    assert np.array_equal(oracle.bmu_dense(X, W), target.astype(np.int32))


@pytest.mark.parametrize("n,k,dim,seed", [(64, 36, 3, 0), (50, 25, 8, 1), (33, 7, 2, 2)])
def test_against_kdtree(oracle, n, k, dim, seed):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, dim)).astype(np.float32)
    W = rng.standard_normal((k, dim)).astype(np.float32)
    bmu, d2 = oracle.bmu_dense(X, W, want_d2=True)
    dist, idx = cKDTree(W.astype(np.float64)).query(X.astype(np.float64), k=1)
    assert np.array_equal(bmu, idx.astype(np.int32))
    np.testing.assert_allclose(np.sqrt(d2), dist, rtol=1e-12, atol=0)


def test_against_cdist_in_high_dimension(oracle):
    rng = np.random.default_rng(5)
    X = rng.random((40, 300)).astype(np.float32)
    W = rng.random((90, 300)).astype(np.float32)
    bmu, d2 = oracle.bmu_dense(X, W, want_d2=True)
    D = cdist(X.astype(np.float64), W.astype(np.float64), metric="sqeuclidean")
    assert np.array_equal(bmu, D.argmin(axis=1).astype(np.int32))
    np.testing.assert_allclose(d2, D.min(axis=1), rtol=1e-12)


def test_pair_distances_match_cdist(oracle):
    rng = np.random.default_rng(6)
    X = rng.random((10, 17)).astype(np.float32)
    W = rng.random((12, 17)).astype(np.float32)
    inst = np.repeat(np.arange(10), 12)
    node = np.tile(np.arange(12), 10)
    got = oracle.sqdist_pairs_dense(X, W, inst, node).reshape(10, 12)
    np.testing.assert_allclose(got, cdist(X.astype(np.float64), W.astype(np.float64), "sqeuclidean"),
                               rtol=1e-12)


def test_sparse_file_example_is_zero_based():
    """The paper's one printed data example: [1.2 0 0 3.4] <-> 0:1.2 3:3.4."""
    lines = [l.strip() for l in open(os.path.join(GOLDEN, "libsvm_example.txt")) if not l.startswith("#")]
    dense = np.array([float(t) for t in lines[0].split(":", 1)[1].split()], dtype=np.float32)
    pairs = [t.split(":") for t in lines[1].split(":", 1)[1].split()]
    indices = np.array([int(p[0]) for p in pairs], dtype=np.int32)
    values = np.array([float(p[1]) for p in pairs], dtype=np.float32)
    csr = (np.array([0, len(pairs)], dtype=np.int64), indices, values)
    assert np.array_equal(densify(csr, dense.size)[0], dense)


def test_sparse_example_row_matches_its_dense_form(oracle):
    csr = (np.array([0, 2], dtype=np.int64), np.array([0, 3], dtype=np.int32),
           np.array([1.2, 3.4], dtype=np.float32))
    W = np.array([[0, 0, 0, 0], [1.2, 0, 0, 3.0], [1.0, 0.1, 0, 3.4], [3.4, 0, 0, 1.2]], dtype=np.float32)
    bmu, d2 = oracle.bmu_csr(csr, 4, W, want_d2=True)
    assert bmu.tolist() == [2]          # a one-based reading would pick another node
    x = np.array([1.2, 0, 0, 3.4], dtype=np.float32).astype(np.float64)
    np.testing.assert_allclose(d2[0], np.sum((x - W[2].astype(np.float64)) ** 2), rtol=1e-12)


@pytest.mark.parametrize("seed", [0, 1])
def test_sparse_equals_densified(oracle, seed):
    dim, n, k = 400, 120, 48
    csr = sparse_zipf_csr(n, dim, seed, mean_len=12.0, max_len=40)
    rng = np.random.default_rng(100 + seed)
    W = rng.random((k, dim)).astype(np.float32) * np.float32(0.2)
    X = densify(csr, dim)
    b_sparse, d_sparse = oracle.bmu_csr(csr, dim, W, want_d2=True)
    b_dense, d_dense = oracle.bmu_dense(X, W, want_d2=True)
    assert np.array_equal(b_sparse, b_dense)
    np.testing.assert_allclose(d_sparse, d_dense, rtol=1e-11)
    inst = np.arange(n).repeat(3)
    node = np.tile(np.array([0, 7, k - 1]), n)
    np.testing.assert_allclose(oracle.sqdist_pairs_csr(csr, dim, W, inst, node),
                               oracle.sqdist_pairs_dense(X, W, inst, node), rtol=1e-10, atol=1e-12)


def test_sparse_distance_has_the_bits_of_the_dense_distance(oracle):
    """The sparse distance is the BMU equation's plain sum over all coordinates: bit for bit what
    the dense routine gives on the densified row, also with a large common offset in the weights
    (where a regrouped |w|^2 - 2 x.w + ... form would lose digits)."""
    dim, n, k = 700, 60, 20
    csr = sparse_zipf_csr(n, dim, 11, mean_len=15.0, max_len=50)
    rng = np.random.default_rng(12)
    W = (rng.random((k, dim)) * 0.3 + 40.0).astype(np.float32)
    X = densify(csr, dim)
    inst = np.arange(n).repeat(k)
    node = np.tile(np.arange(k), n)
    a = oracle.sqdist_pairs_csr(csr, dim, W, inst, node)
    b = oracle.sqdist_pairs_dense(X, W, inst, node)
    assert np.array_equal(a, b)
    b_s, d_s = oracle.bmu_csr(csr, dim, W, want_d2=True)
    b_d, d_d = oracle.bmu_dense(X, W, want_d2=True)
    assert np.array_equal(b_s, b_d) and np.array_equal(d_s, d_d)


def test_sparse_instance_on_a_node_is_at_distance_zero(oracle):
    """An instance that coincides with a weight vector is at distance exactly 0 (not at the rounding
    noise of a cancelling sum), and near-copies of it are told apart at any offset of the map."""
    dim, n = 5000, 40
    csr = sparse_zipf_csr(n, dim, 21, mean_len=80.0, max_len=160)
    X = densify(csr, dim)
    rng = np.random.default_rng(22)
    W = rng.random((3 * n, dim)).astype(np.float32)
    W[n:2 * n] = X                                   # node n + j is instance j itself
    W[:n] = X
    W[:n, 0] = np.nextafter(X[:, 0], np.float32(9.0))          # node j: one ulp off in one coordinate
    bmu, d2 = oracle.bmu_csr(csr, dim, W, want_d2=True)
    assert np.array_equal(bmu, np.arange(n, 2 * n).astype(np.int32))
    assert np.all(d2 == 0.0)
    near = oracle.sqdist_pairs_csr(csr, dim, W, np.arange(n), np.arange(n).astype(np.int32))
    ulp = (W[:n, 0].astype(np.float64) - X[:, 0].astype(np.float64)) ** 2
    assert np.array_equal(near, ulp) and np.all(near > 0.0)
    dist, qe = oracle.bmu_distances_csr(csr, dim, W, bmu)
    assert np.all(dist == 0.0) and qe == 0.0


def test_empty_sparse_row_goes_to_smallest_norm_node(oracle):
    csr = (np.array([0, 0, 1], dtype=np.int64), np.array([2], dtype=np.int32),
           np.array([5.0], dtype=np.float32))
    W = np.array([[1, 1, 1], [0.1, 0.2, 0.1], [0, 0, 4], [0.1, 0.2, 0.1]], dtype=np.float32)
    assert oracle.bmu_csr(csr, 3, W).tolist() == [1, 2]


def test_generated_sparse_rows_are_sorted_unique_unit_length():
    indptr, indices, values = sparse_zipf_csr(200, 3000, 7, mean_len=30.0, max_len=90)
    assert indptr[0] == 0 and np.all(np.diff(indptr) >= 1)
    for j in range(200):
        c = indices[indptr[j]:indptr[j + 1]]
        assert np.all(np.diff(c) > 0) and c[0] >= 0 and c[-1] < 3000
        v = values[indptr[j]:indptr[j + 1]].astype(np.float64)
        assert abs(np.sum(v * v) - 1.0) < 1e-5
