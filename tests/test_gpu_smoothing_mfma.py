"""The matrix-core form of the separable smoothing passes (map lines of 32 nodes and more by default) against the
oracle's plain O(k^2) sum, through som_update_dense: all four map x grid combinations, sides that make one
pass or both run on the matrix cores, output counts that are no multiple of 32, more than seven 32-output
blocks per line (two wavefront tiles), channel counts that are no multiple of 32, few and many chosen nodes.
Sampled nodes (the oracle's update is quadratic in the map size) plus the nodes around the chosen ones."""
import numpy as np
import pytest

from tests import parity as P

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.mark.parametrize("map_type", ["planar", "toroid"])
@pytest.mark.parametrize("grid", ["square", "hexagonal"])
@pytest.mark.parametrize("rows,cols,dim,n,radius", [
    (130, 40, 70, 900, 9.0),        # pass y on the matrix cores, pass x on the vector units
    (40, 129, 33, 900, 2.0),        # the other way round
    (131, 230, 100, 3000, 25.0),    # both; odd row count (hexagonal classes of 66 and 65 rows)
    (226, 128, 32, 400, 60.0),      # eight blocks of outputs along y: two wavefront tiles per line
    (128, 128, 5, 50, 1.0),         # few chosen nodes, narrow neighbourhood: most nodes keep their weights
])
def test_update_matches_oracle(oracle, map_type, grid, rows, cols, dim, n, radius):
    from paper_1305_1422_amd import Som
    rng = np.random.default_rng(rows * 1000 + cols + dim)
    k = rows * cols
    X = rng.standard_normal((n, dim)).astype(np.float32)
    W = rng.random((k, dim)).astype(np.float32)
    bmus = rng.integers(0, k, size=n).astype(np.int32)
    bmus[: n // 4] = bmus[0]                                        # one heavy node
    som = Som(rows, cols, dim, map_type, grid, codebook=torch.from_numpy(W))
    som.update(P.to_dev(X), P.to_dev(bmus), radius)
    torch.cuda.synchronize()
    W_out = som.codebook.cpu().numpy()
    S, C = oracle.accumulate_dense(X, bmus, k)
    hit = np.unique(bmus)
    around = np.concatenate([hit[:8], (hit[:8] + 1) % k, (hit[:8] + cols) % k])
    nodes = np.unique(np.concatenate([rng.choice(k, size=48, replace=False), around,
                                      [0, cols - 1, k - cols, k - 1]]))
    P.check_codebook(oracle, S, C, W, W_out, rows, cols, P.MAP[map_type], P.GRID[grid], radius, nodes=nodes)
    som.close()


@pytest.mark.parametrize("rows,cols", [(140, 150), (30, 50), (12, 20)])
def test_both_forms_agree_on_a_whole_map(oracle, rows, cols):
    """The vector and the matrix-core form of the passes differ only in the order of their fp32 sums; the
    small map takes the matrix cores only when they are asked for."""
    from paper_1305_1422_amd import Som
    dim, n = 64, 5000
    rng = np.random.default_rng(77)
    X = rng.standard_normal((n, dim)).astype(np.float32)
    W = rng.random((rows * cols, dim)).astype(np.float32)
    bmus = rng.integers(0, rows * cols, size=n).astype(np.int32)
    out = []
    for form in ("vector", "matrix", "auto"):
        som = Som(rows, cols, dim, "toroid", "hexagonal", codebook=torch.from_numpy(W))
        som.set_smoothing(form)
        som.update(P.to_dev(X), P.to_dev(bmus), 12.0)
        torch.cuda.synchronize()
        out.append(som.codebook.cpu().numpy())
        som.close()
    np.testing.assert_allclose(out[0], out[1], rtol=2e-5, atol=1e-6)
    if min(rows, cols) >= 32:
        assert np.array_equal(out[2], out[1])
    elif max(rows, cols) < 32:
        assert np.array_equal(out[2], out[0])
    else:                                              # one pass on each kind of unit
        np.testing.assert_allclose(out[2], out[0], rtol=2e-5, atol=1e-6)
