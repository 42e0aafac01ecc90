"""A small object wrapper over the C-ABI binding: holds the context, the code book and the
output buffers as torch tensors on the GPU.  No arithmetic happens here."""
from __future__ import annotations

from typing import Optional, Tuple

import torch

from . import capi

MAP_TYPES = {"planar": capi.SOM_MAP_PLANAR, "toroid": capi.SOM_MAP_TOROID}
GRID_TYPES = {"square": capi.SOM_GRID_SQUARE, "hexagonal": capi.SOM_GRID_HEXAGONAL}
COOLING = {"linear": capi.SOM_COOL_LINEAR, "exponential": capi.SOM_COOL_EXPONENTIAL}
FILTERS = {"fp32": capi.SOM_FILTER_FP32, "split_f16": capi.SOM_FILTER_SPLIT_F16,
           "two_level": capi.SOM_FILTER_TWO_LEVEL, "auto": capi.SOM_FILTER_AUTO}
NEIGHBORHOODS = {"gaussian": capi.SOM_NEIGHBORHOOD_GAUSSIAN, "bubble": capi.SOM_NEIGHBORHOOD_BUBBLE}


def _is_csr(data) -> bool:
    return isinstance(data, (tuple, list)) and len(data) == 3


class Som:
    """rows x cols map over dim-dimensional data on one GPU.

    ``codebook``: optional float32 tensor [rows*cols, dim] (copied to the device) - the
    initial code book; otherwise ``seed`` (non-zero) draws a uniform [0,1) one on the device.
    Dense data: float32 tensor [n, dim].  Sparse data: tuple (indptr int64 [n+1], indices
    int32 [nnz], values float32 [nnz]).
    """

    default_filter: Optional[str] = None     # None = the library's default; tests switch it

    def __init__(self, rows: int, cols: int, dim: int, map_type: str = "planar", grid_type: str = "square",
                 codebook: Optional[torch.Tensor] = None, seed: int = 0, device: str = "cuda:0",
                 filter: Optional[str] = None):
        if not torch.cuda.is_available():
            raise RuntimeError("paper_1305_1422_amd needs a ROCm GPU: there is no CPU fallback")
        self.device = torch.device(device)
        self.rows, self.cols, self.dim, self.k = rows, cols, dim, rows * cols
        if codebook is not None:
            self.codebook = codebook.to(device=self.device, dtype=torch.float32).contiguous().clone()
            seed = 0
        else:
            if seed == 0:
                raise ValueError("give an initial codebook or a non-zero seed")
            self.codebook = torch.empty((self.k, dim), dtype=torch.float32, device=self.device)
        with torch.cuda.device(self.device):
            self.stream = torch.cuda.current_stream(self.device)
            self.ctx = capi.som_init(rows, cols, dim, MAP_TYPES[map_type], GRID_TYPES[grid_type], self.codebook,
                                     seed, self.stream.cuda_stream)
        if filter is None:
            filter = Som.default_filter
        if filter is not None:
            self.set_filter(filter)

    def set_neighborhood(self, function: str = "gaussian", compact_support: bool = False) -> None:
        """Neighbourhood of the batch update: "gaussian" or "bubble"; compact_support cuts the Gaussian
        off beyond the epoch's radius."""
        capi.som_set_neighborhood(self.ctx, NEIGHBORHOODS[function], compact_support)

    def set_scale_cooling(self, cooling: Optional[str]) -> None:
        """Cooling kind of the learning rate where it differs from the radius' ("linear", "exponential");
        None = the same as the radius."""
        capi.som_set_scale_cooling(self.ctx, capi.SOM_COOL_AS_RADIUS if cooling is None else COOLING[cooling])

    def validate_csr(self, csr) -> None:
        """Debug pass: raises capi.SomError if the CSR triple (indptr, indices, values) is malformed."""
        capi.som_validate_csr(self.ctx, csr[0], csr[1], csr[2])

    def set_sparse_hot_block(self, enable: bool) -> None:
        """Allow (default) or forbid the dense block of frequent columns of a registered sparse set."""
        capi.som_set_sparse_hot_block(self.ctx, enable)

    def set_sparse_dense_filter(self, enable: bool) -> None:
        """Allow (default) or forbid the dense filter pass on fp16 planes for a registered sparse set of modest
        dimension."""
        capi.som_set_sparse_dense_filter(self.ctx, enable)

    def set_smoothing(self, form: str) -> None:
        """Units that run the Gaussian smoothing passes: "auto" (default), "vector", "matrix" (fp32 matrix instructions)
        or "matrix_split" (bf16 matrix instructions, operands in three parts); same results to fp32 rounding."""
        capi.som_set_smoothing(self.ctx, {"auto": capi.SOM_SMOOTH_AUTO, "vector": capi.SOM_SMOOTH_VECTOR,
                                          "matrix": capi.SOM_SMOOTH_MATRIX, "matrix_split": capi.SOM_SMOOTH_MATRIX_SPLIT}[form])

    def set_filter(self, filter: str) -> None:
        """Arithmetic of the dense BMU filter pass: "split_f16" (default) or "fp32"; same results."""
        capi.som_set_filter(self.ctx, FILTERS[filter])

    def close(self) -> None:
        if getattr(self, "ctx", None) is not None:
            capi.som_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _n(self, data) -> int:
        return (data[0].shape[0] - 1) if _is_csr(data) else data.shape[0]

    def _new_bmus(self, data) -> torch.Tensor:
        return torch.empty(self._n(data), dtype=torch.int32, device=self.device)

    def train_epoch(self, data, radius: float, scale: float = 1.0, bmus: Optional[torch.Tensor] = None):
        bmus = self._new_bmus(data) if bmus is None else bmus
        if _is_csr(data):
            capi.som_train_epoch_csr(self.ctx, data[0], data[1], data[2], self.codebook, radius, scale, bmus)
        else:
            capi.som_train_epoch_dense(self.ctx, data, self.codebook, radius, scale, bmus)
        return bmus

    def bmus(self, data, bmus: Optional[torch.Tensor] = None):
        bmus = self._new_bmus(data) if bmus is None else bmus
        if _is_csr(data):
            capi.som_bmus_csr(self.ctx, data[0], data[1], data[2], self.codebook, bmus)
        else:
            capi.som_bmus_dense(self.ctx, data, self.codebook, bmus)
        return bmus

    def update(self, data, bmus: torch.Tensor, radius: float, scale: float = 1.0) -> None:
        if _is_csr(data):
            capi.som_update_csr(self.ctx, data[0], data[1], data[2], bmus, self.codebook, radius, scale)
        else:
            capi.som_update_dense(self.ctx, data, bmus, self.codebook, radius, scale)

    def train(self, data, n_epochs: int, radius0: float = 0.0, radiusN: float = 0.0, scale0: float = 0.0,
              scaleN: float = 0.0, cooling: str = "linear", bmus: Optional[torch.Tensor] = None):
        bmus = self._new_bmus(data) if bmus is None else bmus
        if _is_csr(data):
            capi.som_set_data_csr(self.ctx, data[0], data[1], data[2])
        else:
            capi.som_set_data_dense(self.ctx, data)
        self._data = data        # keep the registered tensors alive
        capi.som_train(self.ctx, n_epochs, radius0, radiusN, scale0, scaleN, COOLING[cooling], self.codebook, bmus)
        return bmus

    def train_snapshots(self, data, n_epochs: int, snapshots: int = 1, radius0: float = 0.0, radiusN: float = 0.0,
                        scale0: float = 0.0, scaleN: float = 0.0, cooling: str = "linear"):
        """train() with the interim outputs of option -s: returns (bmus, umatrices[, codebooks, bmus_all])."""
        bmus = self._new_bmus(data)
        if _is_csr(data):
            capi.som_set_data_csr(self.ctx, data[0], data[1], data[2])
        else:
            capi.som_set_data_dense(self.ctx, data)
        self._data = data
        n = bmus.shape[0]
        um = torch.empty((n_epochs, self.rows, self.cols), dtype=torch.float32, device=self.device) \
            if snapshots >= 1 else None
        cbs = torch.empty((n_epochs, self.k, self.dim), dtype=torch.float32, device=self.device) \
            if snapshots == 2 else None
        ball = torch.empty((n_epochs, n), dtype=torch.int32, device=self.device) if snapshots == 2 else None
        capi.som_train_snapshots(self.ctx, n_epochs, radius0, radiusN, scale0, scaleN, COOLING[cooling], self.codebook,
                                 bmus, snapshots, um, cbs, ball)
        return (bmus, um, cbs, ball) if snapshots == 2 else (bmus, um)

    def bmu_distances(self, data, bmus: torch.Tensor) -> Tuple[torch.Tensor, torch.Tensor]:
        """(distance of every instance to node bmus[j] [n] fp32, their mean [1] fp64), both on the device."""
        dist = torch.empty(bmus.shape[0], dtype=torch.float32, device=self.device)
        qe = torch.empty(1, dtype=torch.float64, device=self.device)
        if _is_csr(data):
            capi.som_bmu_distances_csr(self.ctx, data[0], data[1], data[2], self.codebook, bmus, dist, qe)
        else:
            capi.som_bmu_distances_dense(self.ctx, data, self.codebook, bmus, dist, qe)
        return dist, qe

    def cool_schedule(self, n_epochs: int, radius0: float = 0.0, radiusN: float = 0.0, scale0: float = 0.0,
                      scaleN: float = 0.0, cooling: str = "linear") -> Tuple[torch.Tensor, torch.Tensor]:
        r = torch.empty(n_epochs, dtype=torch.float64, device=self.device)
        s = torch.empty(n_epochs, dtype=torch.float64, device=self.device)
        capi.som_cool_schedule(self.ctx, n_epochs, radius0, radiusN, scale0, scaleN, COOLING[cooling], r, s)
        return r, s

    def umatrix(self) -> torch.Tensor:
        u = torch.empty((self.rows, self.cols), dtype=torch.float32, device=self.device)
        capi.som_umatrix(self.ctx, self.codebook, u)
        return u

    def stats(self):
        return capi.som_get_stats(self.ctx)

    def two_level_stats(self):
        """(listed, all) node-block/instance-tile pairs of the last dense search's second pass; (0, 0) if one-level."""
        return capi.som_two_level_stats(self.ctx)
