"""Pins of the oracle's post-training outputs: the distance of every instance to its best
matching unit and the mean of those distances (quantisation error; the paper lists the BMUs,
the code book and the U-matrix as results and prints no formula for a quality figure, so the
usual definition is taken).

The pins use planted geometry (right triangles, instances on nodes), scipy's cdist, the minimum
the BMU search reports (a different function of the oracle with its own pins), scaling, and the
equality of the sparse and dense formulations.
"""
import numpy as np
from scipy.spatial.distance import cdist

from gen import sparse_zipf_csr


def densify(csr, dim):
    indptr, indices, values = csr
    n = len(indptr) - 1
    X = np.zeros((n, dim), dtype=np.float32)
    for j in range(n):
        X[j, indices[indptr[j]:indptr[j + 1]]] = values[indptr[j]:indptr[j + 1]]
    return X


def test_right_triangles(oracle):
    W = np.zeros((3, 4), dtype=np.float32)
    W[1] = [1, 1, 1, 1]
    W[2] = [0, 0, 0, 2]
    X = np.array([[3, 4, 0, 0],          # to node 0: 5
                  [1, 1, 4, 5],          # to node 1: sqrt(0+0+9+16) = 5
                  [5, 12, 0, 2],         # to node 2: 13
                  [0, 0, 0, 2]], dtype=np.float32)   # on node 2: 0
    bmu = np.array([0, 1, 2, 2], dtype=np.int32)
    dist, qe = oracle.bmu_distances_dense(X, W, bmu)
    assert np.array_equal(dist, [5.0, 5.0, 13.0, 0.0])
    assert qe == 23.0 / 4.0


def test_distance_is_to_the_named_node_not_to_the_nearest(oracle):
    W = np.array([[0, 0], [10, 0]], dtype=np.float32)
    X = np.array([[1, 0]], dtype=np.float32)
    d0, _ = oracle.bmu_distances_dense(X, W, np.array([0], dtype=np.int32))
    d1, _ = oracle.bmu_distances_dense(X, W, np.array([1], dtype=np.int32))
    assert d0[0] == 1.0 and d1[0] == 9.0


def test_instances_on_their_nodes_have_zero_error(oracle):
    rng = np.random.default_rng(3)
    W = rng.standard_normal((25, 7)).astype(np.float32)
    order = rng.integers(0, 25, 60).astype(np.int32)
    dist, qe = oracle.bmu_distances_dense(W[order], W, order)
    assert np.all(dist == 0.0) and qe == 0.0


def test_agrees_with_the_minimum_of_the_bmu_search_and_with_cdist(oracle):
    rng = np.random.default_rng(4)
    X = rng.random((200, 33)).astype(np.float32)
    W = rng.random((48, 33)).astype(np.float32)
    bmu, d2 = oracle.bmu_dense(X, W, want_d2=True)
    dist, qe = oracle.bmu_distances_dense(X, W, bmu)
    np.testing.assert_allclose(dist, np.sqrt(d2), rtol=1e-15)
    full = cdist(X.astype(np.float64), W.astype(np.float64))
    np.testing.assert_allclose(dist, full.min(axis=1), rtol=1e-12)
    np.testing.assert_allclose(qe, full.min(axis=1).mean(), rtol=1e-12)
    # any other assignment is no better
    other = rng.integers(0, 48, 200).astype(np.int32)
    d_other, qe_other = oracle.bmu_distances_dense(X, W, other)
    np.testing.assert_allclose(d_other, full[np.arange(200), other], rtol=1e-12)
    assert qe_other >= qe


def test_scaling_by_a_power_of_two_scales_the_distances_exactly(oracle):
    rng = np.random.default_rng(5)
    X = rng.standard_normal((50, 12)).astype(np.float32)
    W = rng.standard_normal((9, 12)).astype(np.float32)
    bmu = rng.integers(0, 9, 50).astype(np.int32)
    d1, q1 = oracle.bmu_distances_dense(X, W, bmu)
    d4, q4 = oracle.bmu_distances_dense(X * np.float32(4), W * np.float32(4), bmu)
    assert np.array_equal(d4, 4.0 * d1)
    assert q4 == 4.0 * q1


def test_sparse_equals_dense_on_densified_rows(oracle):
    n, dim = 120, 90
    csr = sparse_zipf_csr(n, dim, 6, mean_len=8.0, max_len=30)
    X = densify(csr, dim)
    rng = np.random.default_rng(7)
    W = rng.random((30, dim)).astype(np.float32)
    bmu = rng.integers(0, 30, n).astype(np.int32)
    dd, qd = oracle.bmu_distances_dense(X, W, bmu)
    ds, qs = oracle.bmu_distances_csr(csr, dim, W, bmu)
    np.testing.assert_allclose(ds, dd, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(qs, qd, rtol=1e-12)


def test_sparse_row_on_its_node_and_empty_row(oracle):
    dim = 6
    W = np.array([[0, 2, 0, 0, 0, 1.5], [0, 0, 0, 0, 3, 4]], dtype=np.float32)
    indptr = np.array([0, 2, 2], dtype=np.int64)            # row 0 = node 0, row 1 empty
    indices = np.array([1, 5], dtype=np.int32)
    values = np.array([2.0, 1.5], dtype=np.float32)
    dist, qe = oracle.bmu_distances_csr((indptr, indices, values), dim, W, np.array([0, 1], dtype=np.int32))
    assert dist[0] == 0.0 and dist[1] == 5.0 and qe == 2.5


def test_no_instances(oracle):
    W = np.ones((4, 3), dtype=np.float32)
    dist, qe = oracle.bmu_distances_dense(np.zeros((0, 3), dtype=np.float32), W, np.zeros(0, dtype=np.int32))
    assert dist.shape == (0,) and qe == 0.0
