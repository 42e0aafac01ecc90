"""ctypes front end of the C oracle (``som_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's CPU-baseline leg.  Argument marshalling only; all arithmetic is in
the C file, which cites the passages of the paper it follows.
"""
from __future__ import annotations

import ctypes as C
from typing import Optional, Tuple

import numpy as np

from . import build as _build

PLANAR, TOROID = 0, 1
SQUARE, HEXAGONAL = 0, 1
LINEAR, EXPONENTIAL = 0, 1
GAUSSIAN, BUBBLE = 0, 1
EPS_MASS = 1e-20          # neighbourhood mass below which a node keeps its weights

MAP_TYPES = {"planar": PLANAR, "toroid": TOROID}
GRID_TYPES = {"square": SQUARE, "hexagonal": HEXAGONAL}
COOLING = {"linear": LINEAR, "exponential": EXPONENTIAL}

_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(_build.build())
        f32p, f64p = C.POINTER(C.c_float), C.POINTER(C.c_double)
        i32p, i64p = C.POINTER(C.c_int32), C.POINTER(C.c_int64)
        L.oracle_num_threads.restype = C.c_int
        L.oracle_grid_q.restype = C.c_int64
        L.oracle_grid_q.argtypes = [C.c_int] * 6
        L.oracle_neighbourhood.restype = C.c_double
        L.oracle_neighbourhood.argtypes = [C.c_int] * 6 + [C.c_double]
        L.oracle_bmu_dense.restype = None
        L.oracle_bmu_dense.argtypes = [f32p, C.c_int64, C.c_int, f32p, C.c_int, i32p, f64p]
        L.oracle_bmu_csr.restype = None
        L.oracle_bmu_csr.argtypes = [i64p, i32p, f32p, C.c_int64, C.c_int, f32p, C.c_int, i32p, f64p]
        L.oracle_sqdist_pairs_dense.restype = None
        L.oracle_sqdist_pairs_dense.argtypes = [f32p, C.c_int, f32p, C.c_int64, i64p, i32p, f64p]
        L.oracle_sqdist_pairs_csr.restype = None
        L.oracle_sqdist_pairs_csr.argtypes = [i64p, i32p, f32p, C.c_int, f32p, C.c_int64, i64p, i32p, f64p]
        L.oracle_accumulate_dense.restype = None
        L.oracle_accumulate_dense.argtypes = [f32p, C.c_int64, C.c_int, i32p, C.c_int, f64p, f64p]
        L.oracle_accumulate_csr.restype = None
        L.oracle_accumulate_csr.argtypes = [i64p, i32p, f32p, C.c_int64, C.c_int, i32p, C.c_int, f64p, f64p]
        L.oracle_neighbourhood_kind.restype = C.c_double
        L.oracle_neighbourhood_kind.argtypes = [C.c_int] * 6 + [C.c_double, C.c_int, C.c_int]
        L.oracle_update.restype = None
        L.oracle_update.argtypes = [f64p, f64p, f32p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                    C.c_double, C.c_double, C.c_double, f64p]
        L.oracle_update_kind.restype = None
        L.oracle_update_kind.argtypes = [f64p, f64p, f32p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                         C.c_double, C.c_double, C.c_double, f64p, C.c_int, C.c_int]
        L.oracle_update_nodes.restype = None
        L.oracle_update_nodes.argtypes = [f64p, f64p, f32p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                          C.c_double, C.c_double, C.c_double, i32p, C.c_int, f32p, f64p]
        L.oracle_epoch_dense.restype = C.c_int
        L.oracle_epoch_dense.argtypes = [f32p, C.c_int64, C.c_int, f32p, C.c_int, C.c_int, C.c_int,
                                         C.c_int, C.c_double, C.c_double, C.c_double, i32p]
        L.oracle_epoch_csr.restype = C.c_int
        L.oracle_epoch_csr.argtypes = [i64p, i32p, f32p, C.c_int64, C.c_int, f32p, C.c_int, C.c_int,
                                       C.c_int, C.c_int, C.c_double, C.c_double, C.c_double, i32p]
        L.oracle_cool.restype = C.c_double
        L.oracle_bmu_distances_dense.argtypes = [f32p, C.c_int64, C.c_int, f32p, i32p, f64p]
        L.oracle_bmu_distances_dense.restype = C.c_double
        L.oracle_bmu_distances_csr.argtypes = [i64p, i32p, f32p, C.c_int64, C.c_int, f32p, i32p, f64p]
        L.oracle_bmu_distances_csr.restype = C.c_double
        L.oracle_cool.argtypes = [C.c_double, C.c_double, C.c_int, C.c_int, C.c_int]
        L.oracle_umatrix.restype = None
        L.oracle_umatrix.argtypes = [f32p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, f64p]
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray], ct):
    return None if a is None else a.ctypes.data_as(C.POINTER(ct))


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _csr(csr) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    indptr, indices, values = csr
    return (np.ascontiguousarray(indptr, dtype=np.int64),
            np.ascontiguousarray(indices, dtype=np.int32),
            np.ascontiguousarray(values, dtype=np.float32))


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def grid_q(rows: int, cols: int, map_type: int, grid_type: int, i: int, b: int) -> int:
    """4 x squared grid distance between nodes i and b (an exact integer)."""
    return int(lib().oracle_grid_q(rows, cols, map_type, grid_type, i, b))


def neighbourhood(rows, cols, map_type, grid_type, i, b, radius) -> float:
    return float(lib().oracle_neighbourhood(rows, cols, map_type, grid_type, i, b, float(radius)))


def bmu_dense(X, W, want_d2: bool = False):
    X, W = _f32(X), _f32(W)
    n, dim = X.shape
    k = W.shape[0]
    assert W.shape[1] == dim
    bmu = np.empty(n, dtype=np.int32)
    d2 = np.empty(n, dtype=np.float64) if want_d2 else None
    lib().oracle_bmu_dense(_p(X, C.c_float), n, dim, _p(W, C.c_float), k, _p(bmu, C.c_int32),
                           _p(d2, C.c_double))
    return (bmu, d2) if want_d2 else bmu


def bmu_csr(csr, dim: int, W, want_d2: bool = False):
    indptr, indices, values = _csr(csr)
    W = _f32(W)
    n, k = indptr.shape[0] - 1, W.shape[0]
    assert W.shape[1] == dim
    bmu = np.empty(n, dtype=np.int32)
    d2 = np.empty(n, dtype=np.float64) if want_d2 else None
    lib().oracle_bmu_csr(_p(indptr, C.c_int64), _p(indices, C.c_int32), _p(values, C.c_float),
                         n, dim, _p(W, C.c_float), k, _p(bmu, C.c_int32), _p(d2, C.c_double))
    return (bmu, d2) if want_d2 else bmu


def sqdist_pairs_dense(X, W, inst, node) -> np.ndarray:
    X, W = _f32(X), _f32(W)
    inst = np.ascontiguousarray(inst, dtype=np.int64)
    node = np.ascontiguousarray(node, dtype=np.int32)
    out = np.empty(inst.shape[0], dtype=np.float64)
    lib().oracle_sqdist_pairs_dense(_p(X, C.c_float), X.shape[1], _p(W, C.c_float), inst.shape[0],
                                    _p(inst, C.c_int64), _p(node, C.c_int32), _p(out, C.c_double))
    return out


def sqdist_pairs_csr(csr, dim: int, W, inst, node) -> np.ndarray:
    indptr, indices, values = _csr(csr)
    W = _f32(W)
    inst = np.ascontiguousarray(inst, dtype=np.int64)
    node = np.ascontiguousarray(node, dtype=np.int32)
    out = np.empty(inst.shape[0], dtype=np.float64)
    lib().oracle_sqdist_pairs_csr(_p(indptr, C.c_int64), _p(indices, C.c_int32), _p(values, C.c_float),
                                  dim, _p(W, C.c_float), inst.shape[0], _p(inst, C.c_int64),
                                  _p(node, C.c_int32), _p(out, C.c_double))
    return out


def accumulate_dense(X, bmu, k: int):
    X = _f32(X)
    n, dim = X.shape
    bmu = np.ascontiguousarray(bmu, dtype=np.int32)
    S = np.empty((k, dim), dtype=np.float64)
    Cn = np.empty(k, dtype=np.float64)
    lib().oracle_accumulate_dense(_p(X, C.c_float), n, dim, _p(bmu, C.c_int32), k,
                                  _p(S, C.c_double), _p(Cn, C.c_double))
    return S, Cn


def accumulate_csr(csr, dim: int, bmu, k: int):
    indptr, indices, values = _csr(csr)
    n = indptr.shape[0] - 1
    bmu = np.ascontiguousarray(bmu, dtype=np.int32)
    S = np.empty((k, dim), dtype=np.float64)
    Cn = np.empty(k, dtype=np.float64)
    lib().oracle_accumulate_csr(_p(indptr, C.c_int64), _p(indices, C.c_int32), _p(values, C.c_float),
                                n, dim, _p(bmu, C.c_int32), k, _p(S, C.c_double), _p(Cn, C.c_double))
    return S, Cn


def neighbourhood_kind(rows, cols, map_type, grid_type, i, b, radius, function=0, compact=False) -> float:
    """Neighbourhood weight for the Gaussian (function 0) or bubble (1) function, optionally with
    compact support (options -n and -p)."""
    return float(lib().oracle_neighbourhood_kind(rows, cols, map_type, grid_type, i, b, float(radius),
                                                 int(function), int(bool(compact))))


def update(S, Cn, W, rows: int, cols: int, map_type: int, grid_type: int, radius: float,
           scale: float = 1.0, eps_mass: float = EPS_MASS, function: int = 0, compact: bool = False):
    """Returns (new code book float32 [k, dim], neighbourhood mass D float64 [k])."""
    S = np.ascontiguousarray(S, dtype=np.float64)
    Cn = np.ascontiguousarray(Cn, dtype=np.float64)
    Wn = _f32(W).copy()
    k, dim = Wn.shape
    assert k == rows * cols and S.shape == (k, dim) and Cn.shape == (k,)
    D = np.empty(k, dtype=np.float64)
    lib().oracle_update_kind(_p(S, C.c_double), _p(Cn, C.c_double), _p(Wn, C.c_float), rows, cols, dim,
                             map_type, grid_type, float(radius), float(scale), float(eps_mass),
                             _p(D, C.c_double), int(function), int(bool(compact)))
    return Wn, D


def update_nodes(S, Cn, W, rows: int, cols: int, map_type: int, grid_type: int, radius: float, nodes,
                 scale: float = 1.0, eps_mass: float = EPS_MASS):
    """New vectors and masses of the listed nodes only: (float32 [len(nodes), dim], float64 [len(nodes)])."""
    S = np.ascontiguousarray(S, dtype=np.float64)
    Cn = np.ascontiguousarray(Cn, dtype=np.float64)
    W = _f32(W)
    nodes = np.ascontiguousarray(nodes, dtype=np.int32)
    k, dim = W.shape
    assert k == rows * cols and S.shape == (k, dim) and Cn.shape == (k,)
    out = np.empty((nodes.shape[0], dim), dtype=np.float32)
    D = np.empty(nodes.shape[0], dtype=np.float64)
    lib().oracle_update_nodes(_p(S, C.c_double), _p(Cn, C.c_double), _p(W, C.c_float), rows, cols, dim,
                              map_type, grid_type, float(radius), float(scale), float(eps_mass),
                              _p(nodes, C.c_int32), nodes.shape[0], _p(out, C.c_float), _p(D, C.c_double))
    return out, D


def epoch_dense(X, W, rows, cols, map_type, grid_type, radius, scale=1.0, eps_mass=EPS_MASS):
    """Returns (bmus against the incoming code book, new code book)."""
    X = _f32(X)
    Wn = _f32(W).copy()
    n, dim = X.shape
    bmu = np.empty(n, dtype=np.int32)
    rc = lib().oracle_epoch_dense(_p(X, C.c_float), n, dim, _p(Wn, C.c_float), rows, cols, map_type,
                                  grid_type, float(radius), float(scale), float(eps_mass),
                                  _p(bmu, C.c_int32))
    if rc:
        raise MemoryError("oracle_epoch_dense")
    return bmu, Wn


def epoch_csr(csr, dim, W, rows, cols, map_type, grid_type, radius, scale=1.0, eps_mass=EPS_MASS):
    indptr, indices, values = _csr(csr)
    Wn = _f32(W).copy()
    n = indptr.shape[0] - 1
    bmu = np.empty(n, dtype=np.int32)
    rc = lib().oracle_epoch_csr(_p(indptr, C.c_int64), _p(indices, C.c_int32), _p(values, C.c_float),
                                n, dim, _p(Wn, C.c_float), rows, cols, map_type, grid_type,
                                float(radius), float(scale), float(eps_mass), _p(bmu, C.c_int32))
    if rc:
        raise MemoryError("oracle_epoch_csr")
    return bmu, Wn


def bmu_distances_dense(X, W, bmu):
    """(distance of every instance to node bmu[j], their mean = quantisation error)."""
    X, W = _f32(X), _f32(W)
    bmu = np.ascontiguousarray(bmu, dtype=np.int32)
    n, dim = X.shape
    assert bmu.shape == (n,) and (n == 0 or (bmu.min() >= 0 and bmu.max() < W.shape[0]))
    dist = np.empty(n, dtype=np.float64)
    qe = lib().oracle_bmu_distances_dense(_p(X, C.c_float), n, dim, _p(W, C.c_float), _p(bmu, C.c_int32),
                                          _p(dist, C.c_double))
    return dist, float(qe)


def bmu_distances_csr(csr, dim: int, W, bmu):
    indptr, indices, values = _csr(csr)
    W = _f32(W)
    bmu = np.ascontiguousarray(bmu, dtype=np.int32)
    n = indptr.shape[0] - 1
    assert bmu.shape == (n,) and (n == 0 or (bmu.min() >= 0 and bmu.max() < W.shape[0]))
    dist = np.empty(n, dtype=np.float64)
    qe = lib().oracle_bmu_distances_csr(_p(indptr, C.c_int64), _p(indices, C.c_int32), _p(values, C.c_float),
                                        n, dim, _p(W, C.c_float), _p(bmu, C.c_int32), _p(dist, C.c_double))
    return dist, float(qe)


def cool(v0: float, vN: float, n_epochs: int, epoch: int, kind: int = LINEAR) -> float:
    return float(lib().oracle_cool(float(v0), float(vN), int(n_epochs), int(epoch), int(kind)))


def umatrix(W, rows: int, cols: int, map_type: int, grid_type: int) -> np.ndarray:
    W = _f32(W)
    k, dim = W.shape
    assert k == rows * cols
    U = np.empty(k, dtype=np.float64)
    lib().oracle_umatrix(_p(W, C.c_float), rows, cols, dim, map_type, grid_type, _p(U, C.c_double))
    return U.reshape(rows, cols)
