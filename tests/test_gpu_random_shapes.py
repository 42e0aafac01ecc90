"""Seeded sweep over random valid shapes: dense and sparse data, every filter, every map and grid type,
every neighbourhood, ragged sizes of all kinds, two epochs each, compared with the oracle element by
element (gpu tests, through the C ABI)."""
import numpy as np
import pytest

from gen import sparse_zipf_csr
from tests import parity as P

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

NEIGHBOURHOODS = [("gaussian", False, 0), ("gaussian", True, 0), ("bubble", False, 1)]


@pytest.mark.parametrize("case", range(24))
def test_random_shape(oracle, case):
    from paper_1305_1422_amd import Som
    rng = np.random.default_rng(977_000 + case)
    rows, cols = int(rng.integers(1, 41)), int(rng.integers(1, 41))
    dense = case % 2 == 0
    n = int(rng.integers(1, 3000))
    dim = int(rng.integers(1, 700)) if dense else int(rng.integers(8, 5000))
    map_type = ["planar", "toroid"][int(rng.integers(0, 2))]
    grid = ["square", "hexagonal"][int(rng.integers(0, 2))]
    radius = float(np.float32(rng.uniform(0.3, max(rows, cols))))
    name, compact, function = NEIGHBOURHOODS[case % 3]
    filt = ["split_f16", "fp32", "two_level"][(case // 2) % 3]
    W = (rng.random((rows * cols, dim)) * rng.choice([1.0, 0.05, 20.0])).astype(np.float32)
    if dense:
        X = (rng.random((n, dim)) * rng.choice([1.0, 0.05, 20.0])).astype(np.float32)
        Xd = P.to_dev(X)
    else:
        mean_len = float(min(dim / 2, rng.uniform(2, 60)))
        X = sparse_zipf_csr(n, dim, int(rng.integers(1, 1 << 30)), mean_len=mean_len,
                            max_len=int(min(dim, 4 * mean_len + 1)))
        Xd = P.csr_to_dev(X)
    som = Som(rows, cols, dim, map_type, grid, codebook=torch.from_numpy(W), filter=filt)
    som.set_neighborhood(name, compact)
    for _ in range(2):
        W_in = som.codebook.cpu().numpy().copy()
        b = som.train_epoch(Xd, radius, 0.3).cpu().numpy()
        if dense:
            P.check_bmus_dense(oracle, X, W_in, b)
            S, C = oracle.accumulate_dense(X, b, rows * cols)
        else:
            P.check_bmus_csr(oracle, X, dim, W_in, b)
            S, C = oracle.accumulate_csr(X, dim, b, rows * cols)
        P.check_codebook(oracle, S, C, W_in, som.codebook.cpu().numpy(), rows, cols, P.MAP[map_type], P.GRID[grid],
                         radius, function=function, compact=compact)
        radius = float(np.float32(max(0.3, radius * 0.5)))
    som.close()
