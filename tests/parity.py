"""Parity protocol between the HIP path and the CPU oracle (helpers for the ``gpu`` tests).

Tolerances (stated by the benchmark spec):
  * BMU indices bit-exact, except where the oracle's fp64 squared distances of the two
    answers differ by less than 1e-5 relative (near-tie band); with an exact zero best
    distance the other answer must be at distance zero too (dense and sparse rows alike: the
    oracle's sparse distance is the plain sum over all coordinates);
  * code book within 1e-5 absolute + 1e-4 relative after each epoch, computed by the oracle
    from the same input code book and from the (validated) GPU BMU vector.  Nodes whose
    neighbourhood mass is within 1e-3 relative of the keep/update floor are skipped.
"""
from __future__ import annotations

import numpy as np

BAND = 1e-5
ATOL, RTOL = 1e-5, 1e-4
MAP = {"planar": 0, "toroid": 1}
GRID = {"square": 0, "hexagonal": 1}


def check_bmus_dense(oracle, X, W, gpu_bmus, rows=None):
    """All instances, or the listed ``rows`` only.  Returns the number of in-band mismatches."""
    X = np.asarray(X)
    gpu_bmus = np.asarray(gpu_bmus)
    if rows is not None:
        rows = np.asarray(rows, dtype=np.int64)
        X, gpu_bmus = X[rows], gpu_bmus[rows]
    assert gpu_bmus.min() >= 0 and gpu_bmus.max() < W.shape[0], "BMU index out of range"
    want, d2 = oracle.bmu_dense(X, W, want_d2=True)
    bad = np.nonzero(want != gpu_bmus)[0]
    if bad.size:
        dg = oracle.sqdist_pairs_dense(X, W, bad, gpu_bmus[bad])
        _assert_in_band(bad, gpu_bmus, want, dg, d2)
    return int(bad.size)


def check_bmus_csr(oracle, csr, dim, W, gpu_bmus, rows=None):
    """Sparse rows, same rule: the oracle's distances are the BMU equation's plain sum with implicit zeros."""
    gpu_bmus = np.asarray(gpu_bmus)
    if rows is not None:
        csr = csr_take_rows(csr, rows)
        gpu_bmus = gpu_bmus[np.asarray(rows, dtype=np.int64)]
    assert gpu_bmus.min() >= 0 and gpu_bmus.max() < W.shape[0], "BMU index out of range"
    want, d2 = oracle.bmu_csr(csr, dim, W, want_d2=True)
    bad = np.nonzero(want != gpu_bmus)[0]
    if bad.size:
        dg = oracle.sqdist_pairs_csr(csr, dim, W, bad, gpu_bmus[bad])
        _assert_in_band(bad, gpu_bmus, want, dg, d2)
    return int(bad.size)


def _assert_in_band(bad, gpu_bmus, want, d2_gpu_choice, d2_best):
    for t, j in enumerate(bad):
        best, got = d2_best[j], d2_gpu_choice[t]
        ok = (got == 0.0) if best == 0.0 else (got - best < BAND * best)
        assert ok, (f"instance {j}: GPU BMU {gpu_bmus[j]} (d2={got!r}) vs oracle {want[j]} (d2={best!r}) "
                    f"is outside the near-tie band")


def csr_take_rows(csr, rows):
    indptr, indices, values = csr
    rows = np.asarray(rows, dtype=np.int64)
    lens = indptr[rows + 1] - indptr[rows]
    out_ptr = np.zeros(rows.size + 1, dtype=np.int64)
    np.cumsum(lens, out=out_ptr[1:])
    idx = np.concatenate([np.arange(indptr[r], indptr[r + 1]) for r in rows]) if rows.size else np.zeros(0, np.int64)
    return out_ptr, indices[idx.astype(np.int64)], values[idx.astype(np.int64)]


def check_codebook(oracle, S, C, W_in, W_gpu, rows, cols, map_type, grid_type, radius, nodes=None,
                   function=0, compact=False):
    """Oracle update from the given per-node sums against the GPU code book.
    Returns (number of nodes compared, number skipped as knife-edge)."""
    W_gpu = np.asarray(W_gpu)
    if nodes is None:
        want, D = oracle.update(S, C, W_in, rows, cols, map_type, grid_type, radius, function=function,
                                compact=compact)
        got = W_gpu
    else:
        assert function == 0 and not compact
        nodes = np.asarray(nodes, dtype=np.int32)
        want, D = oracle.update_nodes(S, C, W_in, rows, cols, map_type, grid_type, radius, nodes)
        got = W_gpu[nodes]
    knife = np.abs(D / oracle.EPS_MASS - 1.0) < 1e-3
    keep = ~knife
    err = np.abs(got[keep].astype(np.float64) - want[keep].astype(np.float64))
    tol = ATOL + RTOL * np.abs(want[keep].astype(np.float64))
    worst = np.unravel_index(np.argmax(err - tol), err.shape) if err.size else None
    assert np.all(err <= tol), (f"code book mismatch: worst |err|={err[worst]:.3e} tol={tol[worst]:.3e} at "
                                f"kept node #{worst[0]}, column {worst[1]}")
    # nodes below the floor must be untouched, bit for bit
    below = keep & (D < oracle.EPS_MASS)
    if below.any():
        src = W_in if nodes is None else np.asarray(W_in)[nodes]
        assert np.array_equal(got[below], np.asarray(src)[below]), "a zero-mass node changed its weights"
    return int(keep.sum()), int(knife.sum())


def epoch_parity_dense(oracle, som, X_host, X_dev, radius, map_type, grid_type, scale=1.0):
    """Run one GPU epoch from som.codebook and check BMUs and the new code book."""
    import torch
    W_in = som.codebook.cpu().numpy().copy()
    bmus = som.train_epoch(X_dev, radius, scale)
    torch.cuda.synchronize()
    b = bmus.cpu().numpy()
    mism = check_bmus_dense(oracle, X_host, W_in, b)
    S, C = oracle.accumulate_dense(X_host, b, som.k)
    check_codebook(oracle, S, C, W_in, som.codebook.cpu().numpy(), som.rows, som.cols, map_type, grid_type, radius)
    return mism


def epoch_parity_csr(oracle, som, csr_host, csr_dev, dim, radius, map_type, grid_type, scale=1.0):
    import torch
    W_in = som.codebook.cpu().numpy().copy()
    bmus = som.train_epoch(csr_dev, radius, scale)
    torch.cuda.synchronize()
    b = bmus.cpu().numpy()
    mism = check_bmus_csr(oracle, csr_host, dim, W_in, b)
    S, C = oracle.accumulate_csr(csr_host, dim, b, som.k)
    check_codebook(oracle, S, C, W_in, som.codebook.cpu().numpy(), som.rows, som.cols, map_type, grid_type, radius)
    return mism


def to_dev(a, device="cuda:0"):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


def csr_to_dev(csr, device="cuda:0"):
    return tuple(to_dev(a, device) for a in csr)
