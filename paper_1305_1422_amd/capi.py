"""ctypes binding of ``libsom.so``: the same names as ``include/som.h``, torch tensors in.

Argument marshalling only - every step of the epoch runs in the HIP library.  Tensors must
be contiguous CUDA(ROCm) tensors of the stated dtype; they are passed as raw device pointers
and stay owned by the caller.  There is no CPU fallback: importing works without a GPU (so
that the exported symbols can be checked), calling needs one.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SOM_LIB_PATH", os.path.join(HERE, "libsom.so"))

SOM_OK, SOM_ERR_INVALID_ARG, SOM_ERR_ALLOC, SOM_ERR_DEVICE, SOM_ERR_STATE = 0, 1, 2, 3, 4
SOM_MAP_PLANAR, SOM_MAP_TOROID = 0, 1
SOM_GRID_SQUARE, SOM_GRID_HEXAGONAL = 0, 1
SOM_COOL_AS_RADIUS, SOM_COOL_LINEAR, SOM_COOL_EXPONENTIAL = -1, 0, 1
SOM_FILTER_FP32, SOM_FILTER_SPLIT_F16, SOM_FILTER_TWO_LEVEL, SOM_FILTER_AUTO = 0, 1, 2, 3
SOM_NEIGHBORHOOD_GAUSSIAN, SOM_NEIGHBORHOOD_BUBBLE = 0, 1
SOM_SMOOTH_AUTO, SOM_SMOOTH_VECTOR, SOM_SMOOTH_MATRIX, SOM_SMOOTH_MATRIX_SPLIT = 0, 1, 2, 3

EXPORTS = [
    "som_init", "som_destroy", "som_last_error",
    "som_train_epoch_dense", "som_train_epoch_csr",
    "som_bmus_dense", "som_bmus_csr",
    "som_update_dense", "som_update_csr",
    "som_set_data_dense", "som_set_data_csr", "som_train", "som_train_snapshots",
    "som_bmu_distances_dense", "som_bmu_distances_csr", "som_bmu_distances_dense_static",
    "som_cool_schedule", "som_umatrix", "som_get_stats", "som_two_level_stats",
    "som_profile_enable", "som_profile_read",
    "som_set_filter", "som_set_smoothing", "som_set_sparse_hot_block", "som_sparse_hot_block_active", "som_set_sparse_dense_filter", "som_sparse_dense_filter_active", "som_set_neighborhood", "som_set_scale_cooling", "som_validate_csr", "som_debug_scores_dense", "som_debug_scores_csr", "som_debug_mfma_f16", "som_debug_xcc_ids",
]
PROFILE_STAGES = ("bmu_dense_filter", "bmu_csr_filter", "bmu_exact", "node_sums", "smooth_divide", "prepare_dense")


class SomError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"libsom error {code}: {message}")
        self.code = code


_lib = None


def load():
    """Load the built library; raise if it has not been built (no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_1305_1422_amd.build` first")
    L = C.CDLL(LIB_PATH)
    vp, i64, i32, f32, u64 = C.c_void_p, C.c_int64, C.c_int, C.c_float, C.c_uint64
    L.som_init.restype = i32
    L.som_init.argtypes = [C.POINTER(vp), i32, i32, i32, i32, i32, vp, u64, vp]
    L.som_destroy.restype = None
    L.som_destroy.argtypes = [vp]
    L.som_last_error.restype = C.c_char_p
    L.som_last_error.argtypes = [vp]
    L.som_train_epoch_dense.restype = i32
    L.som_train_epoch_dense.argtypes = [vp, vp, i64, vp, f32, f32, vp]
    L.som_train_epoch_csr.restype = i32
    L.som_train_epoch_csr.argtypes = [vp, vp, vp, vp, i64, i64, vp, f32, f32, vp]
    L.som_bmus_dense.restype = i32
    L.som_bmus_dense.argtypes = [vp, vp, i64, vp, vp]
    L.som_bmus_csr.restype = i32
    L.som_bmus_csr.argtypes = [vp, vp, vp, vp, i64, i64, vp, vp]
    L.som_update_dense.restype = i32
    L.som_update_dense.argtypes = [vp, vp, i64, vp, vp, f32, f32]
    L.som_update_csr.restype = i32
    L.som_update_csr.argtypes = [vp, vp, vp, vp, i64, i64, vp, vp, f32, f32]
    L.som_set_data_dense.restype = i32
    L.som_set_data_dense.argtypes = [vp, vp, i64]
    L.som_set_data_csr.restype = i32
    L.som_set_data_csr.argtypes = [vp, vp, vp, vp, i64, i64]
    L.som_train.restype = i32
    L.som_train.argtypes = [vp, i32, f32, f32, f32, f32, i32, vp, vp]
    L.som_cool_schedule.restype = i32
    L.som_cool_schedule.argtypes = [vp, i32, f32, f32, f32, f32, i32, vp, vp]
    L.som_train_snapshots.restype = i32
    L.som_train_snapshots.argtypes = [vp, i32, f32, f32, f32, f32, i32, vp, vp, i32, vp, vp, vp]
    L.som_bmu_distances_dense.restype = i32
    L.som_bmu_distances_dense.argtypes = [vp, vp, i64, vp, vp, vp, vp]
    L.som_bmu_distances_csr.restype = i32
    L.som_bmu_distances_csr.argtypes = [vp, vp, vp, vp, i64, i64, vp, vp, vp, vp]
    L.som_bmu_distances_dense_static.restype = i32
    L.som_bmu_distances_dense_static.argtypes = [vp, i64, i32, vp, i32, vp, vp, vp, vp]
    L.som_umatrix.restype = i32
    L.som_umatrix.argtypes = [vp, vp, vp]
    L.som_get_stats.restype = i32
    L.som_get_stats.argtypes = [vp, C.POINTER(i64)]
    L.som_two_level_stats.restype = i32
    L.som_two_level_stats.argtypes = [vp, C.POINTER(i64)]
    L.som_profile_enable.restype = i32
    L.som_profile_enable.argtypes = [vp, i32]
    L.som_profile_read.restype = i32
    L.som_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i64)]
    L.som_set_scale_cooling.restype = i32
    L.som_set_scale_cooling.argtypes = [vp, i32]
    L.som_validate_csr.restype = i32
    L.som_validate_csr.argtypes = [vp, vp, vp, vp, i64, i64]
    L.som_set_sparse_hot_block.restype = i32
    L.som_set_sparse_hot_block.argtypes = [vp, i32]
    L.som_sparse_hot_block_active.restype = i32
    L.som_sparse_hot_block_active.argtypes = [vp]
    L.som_set_sparse_dense_filter.restype = i32
    L.som_set_sparse_dense_filter.argtypes = [vp, i32]
    L.som_sparse_dense_filter_active.restype = i32
    L.som_sparse_dense_filter_active.argtypes = [vp]
    L.som_set_smoothing.restype = i32
    L.som_set_smoothing.argtypes = [vp, i32]
    L.som_set_filter.restype = i32
    L.som_set_filter.argtypes = [vp, i32]
    L.som_set_neighborhood.restype = i32
    L.som_set_neighborhood.argtypes = [vp, i32, i32]
    L.som_debug_scores_dense.restype = i32
    L.som_debug_scores_dense.argtypes = [vp, vp, i64, vp, vp, vp, vp]
    L.som_debug_scores_csr.restype = i32
    L.som_debug_scores_csr.argtypes = [vp, vp, vp, vp, i64, i64, vp, vp, vp, vp]
    L.som_debug_xcc_ids.restype = i32
    L.som_debug_xcc_ids.argtypes = [vp, i32, vp]
    L.som_debug_mfma_f16.restype = i32
    L.som_debug_mfma_f16.argtypes = [vp, vp, vp, vp, i32, vp]
    _lib = L
    return L


def _ptr(t, dtype, name: str, allow_none: bool = False):
    import torch
    if t is None:
        if allow_none:
            return None
        raise TypeError(f"{name} is None")
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a CUDA/ROCm torch tensor (device memory)")
    if t.dtype != dtype:
        raise TypeError(f"{name} must have dtype {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise TypeError(f"{name} must be contiguous")
    return C.c_void_p(t.data_ptr())


def _check(ctx, rc: int):
    if rc != SOM_OK:
        msg = load().som_last_error(ctx)
        raise SomError(rc, msg.decode() if msg else "")


def som_init(rows: int, cols: int, dim: int, map_type: int, grid_type: int, codebook, seed: int = 0,
             stream: Optional[int] = None):
    """Returns the context handle.  ``stream``: a hipStream_t as int (e.g.
    ``torch.cuda.current_stream().cuda_stream``); None or 0 = the default stream."""
    import torch
    L = load()
    ctx = C.c_void_p()
    cb = C.c_void_p(0) if codebook is None else _ptr(codebook, torch.float32, "codebook")
    rc = L.som_init(C.byref(ctx), rows, cols, dim, map_type, grid_type, cb, seed, C.c_void_p(stream or 0))
    if rc != SOM_OK:
        msg = L.som_last_error(None)
        raise SomError(rc, msg.decode() if msg else "")
    return ctx


def som_destroy(ctx) -> None:
    load().som_destroy(ctx)


def som_last_error(ctx) -> str:
    msg = load().som_last_error(ctx)
    return msg.decode() if msg else ""


def som_train_epoch_dense(ctx, data, codebook, radius: float, scale: float, bmus) -> None:
    import torch
    _check(ctx, load().som_train_epoch_dense(ctx, _ptr(data, torch.float32, "data"), data.shape[0],
                                             _ptr(codebook, torch.float32, "codebook"), radius, scale,
                                             _ptr(bmus, torch.int32, "bmus")))


def som_train_epoch_csr(ctx, indptr, indices, values, codebook, radius: float, scale: float, bmus) -> None:
    import torch
    _check(ctx, load().som_train_epoch_csr(ctx, _ptr(indptr, torch.int64, "indptr"),
                                           _ptr(indices, torch.int32, "indices", True),
                                           _ptr(values, torch.float32, "values", True),
                                           indptr.shape[0] - 1, 0 if indices is None else indices.shape[0],
                                           _ptr(codebook, torch.float32, "codebook"), radius, scale,
                                           _ptr(bmus, torch.int32, "bmus")))


def som_bmus_dense(ctx, data, codebook, bmus) -> None:
    import torch
    _check(ctx, load().som_bmus_dense(ctx, _ptr(data, torch.float32, "data"), data.shape[0],
                                      _ptr(codebook, torch.float32, "codebook"), _ptr(bmus, torch.int32, "bmus")))


def som_bmus_csr(ctx, indptr, indices, values, codebook, bmus) -> None:
    import torch
    _check(ctx, load().som_bmus_csr(ctx, _ptr(indptr, torch.int64, "indptr"),
                                    _ptr(indices, torch.int32, "indices", True),
                                    _ptr(values, torch.float32, "values", True), indptr.shape[0] - 1,
                                    0 if indices is None else indices.shape[0],
                                    _ptr(codebook, torch.float32, "codebook"), _ptr(bmus, torch.int32, "bmus")))


def som_update_dense(ctx, data, bmus, codebook, radius: float, scale: float) -> None:
    import torch
    _check(ctx, load().som_update_dense(ctx, _ptr(data, torch.float32, "data"), data.shape[0],
                                        _ptr(bmus, torch.int32, "bmus"),
                                        _ptr(codebook, torch.float32, "codebook"), radius, scale))


def som_update_csr(ctx, indptr, indices, values, bmus, codebook, radius: float, scale: float) -> None:
    import torch
    _check(ctx, load().som_update_csr(ctx, _ptr(indptr, torch.int64, "indptr"),
                                      _ptr(indices, torch.int32, "indices", True),
                                      _ptr(values, torch.float32, "values", True), indptr.shape[0] - 1,
                                      0 if indices is None else indices.shape[0],
                                      _ptr(bmus, torch.int32, "bmus"), _ptr(codebook, torch.float32, "codebook"),
                                      radius, scale))


def som_set_data_dense(ctx, data) -> None:
    import torch
    _check(ctx, load().som_set_data_dense(ctx, _ptr(data, torch.float32, "data"), data.shape[0]))


def som_set_data_csr(ctx, indptr, indices, values) -> None:
    import torch
    _check(ctx, load().som_set_data_csr(ctx, _ptr(indptr, torch.int64, "indptr"),
                                        _ptr(indices, torch.int32, "indices", True),
                                        _ptr(values, torch.float32, "values", True), indptr.shape[0] - 1,
                                        0 if indices is None else indices.shape[0]))


def som_train(ctx, n_epochs: int, radius0: float, radiusN: float, scale0: float, scaleN: float, cooling: int,
              codebook, bmus) -> None:
    import torch
    _check(ctx, load().som_train(ctx, n_epochs, radius0, radiusN, scale0, scaleN, cooling,
                                 _ptr(codebook, torch.float32, "codebook"), _ptr(bmus, torch.int32, "bmus")))


def som_train_snapshots(ctx, n_epochs: int, radius0: float, radiusN: float, scale0: float, scaleN: float,
                        cooling: int, codebook, bmus, snapshots: int, umatrices, codebooks, bmus_all) -> None:
    import torch
    _check(ctx, load().som_train_snapshots(ctx, n_epochs, radius0, radiusN, scale0, scaleN, cooling,
                                           _ptr(codebook, torch.float32, "codebook"), _ptr(bmus, torch.int32, "bmus"),
                                           snapshots, _ptr(umatrices, torch.float32, "umatrices", True),
                                           _ptr(codebooks, torch.float32, "codebooks", True),
                                           _ptr(bmus_all, torch.int32, "bmus_all", True)))


def som_bmu_distances_dense(ctx, data, codebook, bmus, distances, qerror) -> None:
    import torch
    _check(ctx, load().som_bmu_distances_dense(ctx, _ptr(data, torch.float32, "data"), data.shape[0],
                                               _ptr(codebook, torch.float32, "codebook"),
                                               _ptr(bmus, torch.int32, "bmus"),
                                               _ptr(distances, torch.float32, "distances", True),
                                               _ptr(qerror, torch.float64, "qerror", True)))


def som_bmu_distances_dense_static(data, codebook, bmus, distances, qerror, stream: Optional[int] = None) -> None:
    """The variant without context and without allocations; ``stream``: a hipStream_t as int, None = default."""
    import torch
    _check(None, load().som_bmu_distances_dense_static(_ptr(data, torch.float32, "data"), data.shape[0], data.shape[1],
                                                      _ptr(codebook, torch.float32, "codebook"), codebook.shape[0],
                                                      _ptr(bmus, torch.int32, "bmus"),
                                                      _ptr(distances, torch.float32, "distances", True),
                                                      _ptr(qerror, torch.float64, "qerror", True),
                                                      C.c_void_p(stream or 0)))


def som_bmu_distances_csr(ctx, indptr, indices, values, codebook, bmus, distances, qerror) -> None:
    import torch
    _check(ctx, load().som_bmu_distances_csr(ctx, _ptr(indptr, torch.int64, "indptr"),
                                             _ptr(indices, torch.int32, "indices", True),
                                             _ptr(values, torch.float32, "values", True),
                                             indptr.shape[0] - 1, indices.shape[0],
                                             _ptr(codebook, torch.float32, "codebook"),
                                             _ptr(bmus, torch.int32, "bmus"),
                                             _ptr(distances, torch.float32, "distances", True),
                                             _ptr(qerror, torch.float64, "qerror", True)))


def som_cool_schedule(ctx, n_epochs: int, radius0: float, radiusN: float, scale0: float, scaleN: float,
                      cooling: int, radius_out, scale_out) -> None:
    import torch
    _check(ctx, load().som_cool_schedule(ctx, n_epochs, radius0, radiusN, scale0, scaleN, cooling,
                                         _ptr(radius_out, torch.float64, "radius_out", True),
                                         _ptr(scale_out, torch.float64, "scale_out", True)))


def som_umatrix(ctx, codebook, umatrix) -> None:
    import torch
    _check(ctx, load().som_umatrix(ctx, _ptr(codebook, torch.float32, "codebook"),
                                   _ptr(umatrix, torch.float32, "umatrix")))


def som_get_stats(ctx):
    """(rows_refined, rows_collected, rows_rescanned) of the most recent BMU search; synchronises."""
    out = (C.c_int64 * 3)()
    _check(ctx, load().som_get_stats(ctx, out))
    return int(out[0]), int(out[1]), int(out[2])


def som_two_level_stats(ctx):
    """(listed, all) pairs of (128 instances, 128 nodes) of the most recent dense BMU search's second pass;
    (0, 0) if it ran in one level.  Synchronises."""
    out = (C.c_int64 * 2)()
    _check(ctx, load().som_two_level_stats(ctx, out))
    return int(out[0]), int(out[1])


def som_profile_enable(ctx, on: bool) -> None:
    _check(ctx, load().som_profile_enable(ctx, 1 if on else 0))


def som_profile_read(ctx):
    """{stage name: (total milliseconds, brackets)} since the last read; synchronises the stream."""
    ms = (C.c_double * len(PROFILE_STAGES))()
    cnt = (C.c_int64 * len(PROFILE_STAGES))()
    _check(ctx, load().som_profile_read(ctx, ms, cnt))
    return {name: (float(ms[i]), int(cnt[i])) for i, name in enumerate(PROFILE_STAGES)}


def som_set_neighborhood(ctx, function: int, compact_support: bool) -> None:
    _check(ctx, load().som_set_neighborhood(ctx, function, 1 if compact_support else 0))


def som_set_scale_cooling(ctx, cooling: int) -> None:
    _check(ctx, load().som_set_scale_cooling(ctx, cooling))


def som_validate_csr(ctx, indptr, indices, values) -> None:
    """Raises SomError(SOM_ERR_INVALID_ARG) naming the violation if the CSR structure is not well formed."""
    import torch
    _check(ctx, load().som_validate_csr(ctx, _ptr(indptr, torch.int64, "indptr"),
                                        _ptr(indices, torch.int32, "indices", True),
                                        _ptr(values, torch.float32, "values", True), indptr.shape[0] - 1,
                                        0 if indices is None else indices.shape[0]))


def som_set_sparse_hot_block(ctx, enable: bool) -> None:
    _check(ctx, load().som_set_sparse_hot_block(ctx, 1 if enable else 0))


def som_sparse_hot_block_active(ctx) -> bool:
    return bool(load().som_sparse_hot_block_active(ctx))


def som_set_sparse_dense_filter(ctx, enable: bool) -> None:
    _check(ctx, load().som_set_sparse_dense_filter(ctx, 1 if enable else 0))


def som_sparse_dense_filter_active(ctx) -> bool:
    return bool(load().som_sparse_dense_filter_active(ctx))


def som_set_smoothing(ctx, form: int) -> None:
    _check(ctx, load().som_set_smoothing(ctx, form))


def som_set_filter(ctx, filter: int) -> None:
    _check(ctx, load().som_set_filter(ctx, filter))


def som_debug_scores_dense(ctx, data, codebook, scores, mu_out, margin_out) -> None:
    """Test hook: every score of the dense filter in use, scores [n][k], the centring vector used and the
    margin [n] (float64) the exact stage applies per instance."""
    import torch
    _check(ctx, load().som_debug_scores_dense(ctx, _ptr(data, torch.float32, "data"), data.shape[0],
                                              _ptr(codebook, torch.float32, "codebook"),
                                              _ptr(scores, torch.float32, "scores"),
                                              _ptr(mu_out, torch.float32, "mu_out"),
                                              _ptr(margin_out, torch.float64, "margin_out")))


def som_debug_scores_csr(ctx, indptr, indices, values, codebook, scores, mu_out, margin_out) -> None:
    """Test hook: the same for the sparse sweep."""
    import torch
    _check(ctx, load().som_debug_scores_csr(ctx, _ptr(indptr, torch.int64, "indptr"),
                                            _ptr(indices, torch.int32, "indices", True),
                                            _ptr(values, torch.float32, "values", True), indptr.shape[0] - 1,
                                            0 if indices is None else indices.shape[0],
                                            _ptr(codebook, torch.float32, "codebook"),
                                            _ptr(scores, torch.float32, "scores"),
                                            _ptr(mu_out, torch.float32, "mu_out"),
                                            _ptr(margin_out, torch.float64, "margin_out")))


def som_debug_xcc_ids(out) -> None:
    """Test hook: out[b] = id of the XCD that workgroup b of a launch of out.numel() workgroups ran on."""
    import torch
    rc = load().som_debug_xcc_ids(_ptr(out, torch.int32, "out"), out.numel(), C.c_void_p(0))
    if rc != SOM_OK:
        raise SomError(rc, "som_debug_xcc_ids")


def som_debug_mfma_f16(a, b, c_in, d_out) -> None:
    """Test hook: D = A B^T + C by one 32x32x16 fp16 matrix instruction per problem.
    a, b: [count][32][16] float16; c_in, d_out: [count][32][32] float32 (device tensors)."""
    import torch
    rc = load().som_debug_mfma_f16(_ptr(a, torch.float16, "a"), _ptr(b, torch.float16, "b"),
                                   _ptr(c_in, torch.float32, "c_in"), _ptr(d_out, torch.float32, "d_out"),
                                   a.shape[0], C.c_void_p(torch.cuda.current_stream().cuda_stream))
    if rc != SOM_OK:
        raise SomError(rc, "som_debug_mfma_f16 failed")
