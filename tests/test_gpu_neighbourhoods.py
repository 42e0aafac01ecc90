"""Bubble and compact-support neighbourhoods (options -n and -p) on the GPU against the oracle.
The radii are exactly representable in fp32 (the C ABI takes a float), so both sides decide "inside
the radius" from the same number; 1.0 and 2.0 put whole rings of nodes exactly on the boundary."""
import numpy as np
import pytest

from gen import sparse_zipf_csr
from tests import parity as P

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

VARIANTS = [("bubble", False, 1), ("gaussian", True, 0)]


@pytest.mark.parametrize("map_type", ["planar", "toroid"])
@pytest.mark.parametrize("grid_type", ["square", "hexagonal"])
@pytest.mark.parametrize("name,compact,function", VARIANTS)
def test_update_matches_oracle(oracle, map_type, grid_type, name, compact, function):
    from paper_1305_1422_amd import Som
    rng = np.random.default_rng(31)
    rows, cols, dim, n = 12, 19, 70, 900                 # 19 columns: two output tiles, the second ragged
    k = rows * cols
    X = rng.standard_normal((n, dim)).astype(np.float32)
    W = rng.random((k, dim)).astype(np.float32)
    bmu = rng.integers(0, k, size=n).astype(np.int32)
    bmu[bmu % 7 == 3] = 5                                 # empty nodes and one crowded node
    S, C = oracle.accumulate_dense(X, bmu, k)
    Xd, bd = P.to_dev(X), torch.from_numpy(bmu).cuda()
    for radius in (0.75, 1.0, 2.0, 3.5, 40.0):
        som = Som(rows, cols, dim, map_type, grid_type, codebook=torch.from_numpy(W))
        som.set_neighborhood(name, compact)
        som.update(Xd, bd, radius)
        torch.cuda.synchronize()
        kept, knife = P.check_codebook(oracle, S, C, W, som.codebook.cpu().numpy(), rows, cols, P.MAP[map_type],
                                       P.GRID[grid_type], radius, function=function, compact=compact)
        assert kept > 0
        som.close()


@pytest.mark.parametrize("map_type", ["planar", "toroid"])
@pytest.mark.parametrize("grid_type", ["square", "hexagonal"])
@pytest.mark.parametrize("name,compact,function", VARIANTS)
def test_update_on_a_map_wider_than_the_neighbourhood(oracle, map_type, grid_type, name, compact, function):
    """73 columns and radii of 1 to 13: the kernel visits only the stretch of each row's source nodes whose columns
    can be within reach of its 16 destination columns, one that wraps round the seam on a toroid map (first and last
    tiles), is cut at the border on a planar one, and widens to the whole row at the largest radius; sources are
    sparse in some rows (stretches that are empty) and dense in others."""
    from paper_1305_1422_amd import Som
    rng = np.random.default_rng(37)
    rows, cols, dim, n = 22, 73, 40, 2500
    k = rows * cols
    X = rng.standard_normal((n, dim)).astype(np.float32)
    W = rng.random((k, dim)).astype(np.float32)
    bmu = rng.integers(0, k, size=n).astype(np.int32)
    y = bmu // cols
    bmu[(y % 5 == 2) & (bmu % 11 != 0)] = 3                # rows with few sources, and one crowded node
    S, C = oracle.accumulate_dense(X, bmu, k)
    Xd, bd = P.to_dev(X), torch.from_numpy(bmu).cuda()
    for radius in (1.0, 2.5, 6.0, 13.0, 30.0):
        som = Som(rows, cols, dim, map_type, grid_type, codebook=torch.from_numpy(W))
        som.set_neighborhood(name, compact)
        som.update(Xd, bd, radius)
        torch.cuda.synchronize()
        kept, knife = P.check_codebook(oracle, S, C, W, som.codebook.cpu().numpy(), rows, cols, P.MAP[map_type],
                                       P.GRID[grid_type], radius, function=function, compact=compact)
        som.close()


def test_bubble_below_one_is_kmeans_on_the_gpu(oracle):
    from paper_1305_1422_amd import Som
    rng = np.random.default_rng(32)
    rows, cols, dim, n = 8, 8, 33, 500
    k = rows * cols
    X = rng.random((n, dim)).astype(np.float32)
    W = rng.random((k, dim)).astype(np.float32)
    som = Som(rows, cols, dim, "toroid", "hexagonal", codebook=torch.from_numpy(W))
    som.set_neighborhood("bubble")
    b = som.train_epoch(P.to_dev(X), 0.5).cpu().numpy()
    Wn = som.codebook.cpu().numpy()
    for i in range(k):
        sel = b == i
        if sel.any():
            assert np.allclose(Wn[i], X[sel].astype(np.float64).mean(0), rtol=1e-5, atol=1e-6)
        else:
            assert np.array_equal(Wn[i], W[i])
    som.close()


@pytest.mark.parametrize("name,compact,function", VARIANTS)
def test_sparse_epoch_with_compact_neighbourhoods(oracle, name, compact, function):
    from paper_1305_1422_amd import Som
    n, dim, rows, cols = 700, 1500, 9, 11
    csr = sparse_zipf_csr(n, dim, 33, mean_len=40.0, max_len=120)
    W = np.random.default_rng(34).random((rows * cols, dim)).astype(np.float32) * 0.05
    som = Som(rows, cols, dim, "planar", "hexagonal", codebook=torch.from_numpy(W))
    som.set_neighborhood(name, compact)
    b = som.train_epoch(P.csr_to_dev(csr), 2.0).cpu().numpy()
    P.check_bmus_csr(oracle, csr, dim, W, b)
    S, C = oracle.accumulate_csr(csr, dim, b, rows * cols)
    P.check_codebook(oracle, S, C, W, som.codebook.cpu().numpy(), rows, cols, oracle.PLANAR, oracle.HEXAGONAL, 2.0,
                     function=function, compact=compact)
    som.close()


def test_switching_back_to_the_gaussian(oracle):
    from paper_1305_1422_amd import Som
    rng = np.random.default_rng(35)
    rows, cols, dim, n = 7, 9, 20, 300
    X = rng.random((n, dim)).astype(np.float32)
    W = rng.random((rows * cols, dim)).astype(np.float32)
    Xd = P.to_dev(X)
    a = Som(rows, cols, dim, codebook=torch.from_numpy(W))
    b = Som(rows, cols, dim, codebook=torch.from_numpy(W))
    b.set_neighborhood("bubble")
    b.set_neighborhood("gaussian", False)
    a.train_epoch(Xd, 2.0)
    b.train_epoch(Xd, 2.0)
    assert torch.equal(a.codebook, b.codebook)
    a.close()
    b.close()


@pytest.mark.parametrize("kind", ["dense", "csr"])
def test_bubble_plateaus_do_not_reach_the_full_rescan(oracle, kind):
    """Several epochs with a wide bubble: whole regions of the map end up with bit-identical weight vectors.
    The search takes the duplicates out before the filter pass, so no instance needs the exact rescan of all
    nodes, and the BMUs are still the lowest index of the best class."""
    from paper_1305_1422_amd import Som
    rows, cols = 24, 25                                    # 600 nodes, far more than a collected list holds
    if kind == "dense":
        n, dim = 1500, 96
        X = np.random.default_rng(36).random((n, dim)).astype(np.float32)
        Xd = P.to_dev(X)
    else:
        n, dim = 900, 1200
        X = sparse_zipf_csr(n, dim, 37, mean_len=30.0, max_len=90)
        Xd = P.csr_to_dev(X)
    W0 = np.random.default_rng(38).random((rows * cols, dim)).astype(np.float32)
    som = Som(rows, cols, dim, "planar", "square", codebook=torch.from_numpy(W0))
    som.set_neighborhood("bubble")
    duplicates_seen = 0
    for radius in (40.0, 12.0, 6.0, 3.0):                  # 40 covers the map: every updated node = the global mean
        W_in = som.codebook.cpu().numpy().copy()
        b = som.train_epoch(Xd, radius).cpu().numpy()
        duplicates_seen = max(duplicates_seen, rows * cols - len(np.unique(W_in, axis=0)))
        assert som.stats()[2] == 0, f"radius {radius}: {som.stats()[2]} instances fell through to the rescan"
        if kind == "dense":
            P.check_bmus_dense(oracle, X, W_in, b)
        else:
            P.check_bmus_csr(oracle, X, dim, W_in, b)
    assert duplicates_seen > 300, "the schedule produced no large plateau: the test misses its case"
    som.close()


def test_duplicate_rows_with_equal_hash_slots_are_compared_bit_by_bit(oracle):
    """Rows that differ in one bit (here: -0.0 against +0.0, equal as numbers) are not the same row to the
    duplicate search; the result is the exact argmin with the lowest index either way."""
    from paper_1305_1422_amd import Som
    rng = np.random.default_rng(39)
    rows, cols, dim, n = 6, 7, 33, 200
    W = rng.random((rows * cols, dim)).astype(np.float32)
    W[:, 5] = 0.0
    W[10] = W[3]
    W[20] = W[3]
    W[20, 5] = -0.0                                        # bitwise different, numerically identical
    W[30] = W[12]
    X = (W[rng.integers(0, rows * cols, n)] + rng.normal(0, 1e-3, (n, dim))).astype(np.float32)
    som = Som(rows, cols, dim, codebook=torch.from_numpy(W))
    som.set_neighborhood("bubble")
    b = som.bmus(P.to_dev(X)).cpu().numpy()
    want = oracle.bmu_dense(X, W)
    assert np.array_equal(b, want)
    assert not np.isin(b, [10, 20, 30]).any()
    som.close()
