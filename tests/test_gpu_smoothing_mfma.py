"""The matrix-core forms of the separable smoothing passes (map lines of 32 nodes and more by default: fp32 matrix
instructions; from 96 nodes on: bf16 ones with every operand in three parts) against the
oracle's plain O(k^2) sum, through som_update_dense: all four map x grid combinations, sides that make one
pass or both run on the matrix cores, output counts that are no multiple of 32, more than seven 32-output
blocks per line (two wavefront tiles), channel counts that are no multiple of 32, few and many chosen nodes.
Sampled nodes (the oracle's update is quadratic in the map size) plus the nodes around the chosen ones."""
import numpy as np
import pytest

from tests import parity as P

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.mark.parametrize("form", ["auto", "matrix", "matrix_split"])
@pytest.mark.parametrize("map_type", ["planar", "toroid"])
@pytest.mark.parametrize("grid", ["square", "hexagonal"])
@pytest.mark.parametrize("rows,cols,dim,n,radius", [
    (130, 40, 70, 900, 9.0),        # pass y on the matrix cores, pass x on the vector units
    (40, 129, 33, 900, 2.0),        # the other way round
    (131, 230, 100, 3000, 25.0),    # both; odd row count (hexagonal classes of 66 and 65 rows)
    (226, 128, 32, 400, 60.0),      # eight blocks of outputs along y: two wavefront tiles per line
    (128, 128, 5, 50, 1.0),         # few chosen nodes, narrow neighbourhood: most nodes keep their weights
])
def test_update_matches_oracle(oracle, map_type, grid, rows, cols, dim, n, radius, form):
    from paper_1305_1422_amd import Som
    rng = np.random.default_rng(rows * 1000 + cols + dim)
    k = rows * cols
    X = rng.standard_normal((n, dim)).astype(np.float32)
    W = rng.random((k, dim)).astype(np.float32)
    bmus = rng.integers(0, k, size=n).astype(np.int32)
    bmus[: n // 4] = bmus[0]                                        # one heavy node
    som = Som(rows, cols, dim, map_type, grid, codebook=torch.from_numpy(W))
    som.set_smoothing(form)
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
def test_all_forms_agree_on_a_whole_map(oracle, rows, cols):
    """The vector form and the two matrix-core forms of the passes differ only in the order of their fp32 sums
    (and, with three-part bf16 operands, in what is dropped below 2^-23 of a term); the default takes the bf16
    form for lines of 96 nodes and more, the fp32 matrix form from 32 nodes on, else the vector units."""
    from paper_1305_1422_amd import Som
    dim, n = 64, 5000
    rng = np.random.default_rng(77)
    X = rng.standard_normal((n, dim)).astype(np.float32)
    W = rng.random((rows * cols, dim)).astype(np.float32)
    bmus = rng.integers(0, rows * cols, size=n).astype(np.int32)
    out = {}
    for form in ("vector", "matrix", "matrix_split", "auto"):
        som = Som(rows, cols, dim, "toroid", "hexagonal", codebook=torch.from_numpy(W))
        som.set_smoothing(form)
        som.update(P.to_dev(X), P.to_dev(bmus), 12.0)
        torch.cuda.synchronize()
        out[form] = som.codebook.cpu().numpy()
        som.close()
    np.testing.assert_allclose(out["vector"], out["matrix"], rtol=2e-5, atol=1e-6)
    np.testing.assert_allclose(out["vector"], out["matrix_split"], rtol=2e-5, atol=1e-6)
    if min(rows, cols) >= 96:
        assert np.array_equal(out["auto"], out["matrix_split"])
    elif max(rows, cols) < 32:
        assert np.array_equal(out["auto"], out["vector"])
    else:                                              # 30 x 50: pass x on the fp32 matrix cores, pass y on the vector units
        np.testing.assert_allclose(out["auto"], out["vector"], rtol=2e-5, atol=1e-6)


def test_three_part_operands_keep_small_and_large_values(oracle):
    """Channels whose values differ by twelve orders of magnitude, and a narrow neighbourhood on a long line, whose
    far coefficients are around 1e-30: bf16 parts have the exponent range of fp32, so every channel and every node
    above the mass floor keeps its relative accuracy."""
    from paper_1305_1422_amd import Som
    rows, cols, dim, n = 100, 120, 48, 2000
    rng = np.random.default_rng(78)
    scale = np.float32(10.0) ** rng.integers(-6, 7, size=dim).astype(np.float32)
    X = (rng.standard_normal((n, dim)).astype(np.float32) + np.float32(3.0)) * scale
    W = rng.random((rows * cols, dim)).astype(np.float32)
    bmus = rng.integers(0, rows * cols, size=n).astype(np.int32)
    k = rows * cols
    S, C = oracle.accumulate_dense(X, bmus, k)
    for radius in (1.5, 20.0):
        som = Som(rows, cols, dim, "planar", "square", codebook=torch.from_numpy(W))
        som.set_smoothing("matrix_split")
        som.update(P.to_dev(X), P.to_dev(bmus), radius)
        torch.cuda.synchronize()
        got = som.codebook.cpu().numpy()
        som.close()
        nodes = np.unique(np.concatenate([rng.choice(k, size=64, replace=False), bmus[:8], (bmus[:8] + 7) % k]))
        want, D = oracle.update_nodes(S, C, W, rows, cols, oracle.PLANAR, oracle.SQUARE, radius, nodes.astype(np.int32))
        upd = D >= oracle.EPS_MASS * 1.001
        rel = np.abs(got[nodes][upd] - want[upd]) / np.maximum(np.abs(want[upd]), 1e-30)
        assert rel.max() < 1e-4, rel.max()
