"""Parity of the HIP path against the CPU oracle on dense data (gpu tests, through the C ABI).

Each epoch is checked from the same input code book (the GPU's own previous output), so a
legitimate near-tie flip in one epoch cannot make later epochs diverge.
"""
import numpy as np
import pytest

from gen import make_workload, scaled_workload
from tests import parity as P

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(autouse=True, params=["split_f16", "fp32", "two_level"])
def dense_filter(request):
    """Every test of this module runs with every variant of the dense BMU filter."""
    from paper_1305_1422_amd import Som
    old = Som.default_filter
    Som.default_filter = request.param
    yield request.param
    Som.default_filter = old


def _som(w, codebook):
    from paper_1305_1422_amd import Som
    return Som(w.rows, w.cols, w.dim, w.map_type, w.grid_type, codebook=torch.from_numpy(codebook))


def _run_schedule(oracle, w, epochs=None):
    X = w.data()
    Xd = P.to_dev(X)
    som = _som(w, w.codebook())
    E = w.epochs if epochs is None else epochs
    flips = 0
    for e in range(E):
        r = oracle.cool(w.radius0, w.radiusN, w.epochs, e, oracle.LINEAR)
        flips += P.epoch_parity_dense(oracle, som, X, Xd, r, P.MAP[w.map_type], P.GRID[w.grid_type])
    stats = som.stats()
    som.close()
    return flips, stats


def test_config1_full_schedule(oracle):
    """Configuration 1 as stated: n=1000, dim=10, 20x20 planar square, radius 10 -> 1, 10 epochs."""
    _run_schedule(oracle, make_workload(1))


@pytest.mark.parametrize("cfg,n,dim,rows,cols,epochs", [
    (2, 3000, 200, 12, 10, 4),      # toroid square; dim = 6 chunks + tail of 8; k < one node tile
    (2, 700, 1000, 30, 30, 2),      # full feature width; 900 nodes = 7 tiles + ragged tail
    (3, 2000, 64, 24, 22, 3),       # toroid hexagonal (even rows), 528 nodes
    (3, 1500, 256, 15, 16, 2),      # toroid hexagonal with an odd number of rows (seam)
    (5, 5000, 128, 16, 14, 3),      # planar hexagonal
    (1, 333, 7, 9, 13, 3),          # dim not a multiple of 4: scalar loads
])
def test_scaled_configs(oracle, cfg, n, dim, rows, cols, epochs):
    w = scaled_workload(cfg, n=n, dim=dim, rows=rows, cols=cols, epochs=epochs)
    _run_schedule(oracle, w)


@pytest.mark.parametrize("n,dim,rows,cols", [(1, 1, 1, 1), (1, 5, 3, 2), (129, 4, 1, 130), (257, 33, 17, 1), (2, 3, 2, 2)])
def test_tiny_and_ragged_shapes(oracle, n, dim, rows, cols):
    from paper_1305_1422_amd import Som
    rng = np.random.default_rng(n * 1000 + dim)
    X = rng.random((n, dim)).astype(np.float32)
    W = rng.random((rows * cols, dim)).astype(np.float32)
    for map_type in ("planar", "toroid"):
        for grid in ("square", "hexagonal"):
            som = Som(rows, cols, dim, map_type, grid, codebook=torch.from_numpy(W))
            P.epoch_parity_dense(oracle, som, X, P.to_dev(X), 1.5, P.MAP[map_type], P.GRID[grid])
            som.close()


def test_exact_ties_go_to_lowest_index(oracle):
    """Duplicated nodes and instances that coincide with nodes: the BMU must be the lowest index,
    with no tolerance (the distances tie exactly)."""
    from paper_1305_1422_amd import Som
    rng = np.random.default_rng(7)
    rows, cols, dim = 12, 25, 48                      # 300 nodes: three node tiles
    W = rng.random((rows * cols, dim)).astype(np.float32)
    W[200] = W[17]; W[299] = W[17]; W[150] = W[130]; W[5] = W[3]
    X = np.vstack([W[299], W[200], W[150], W[5], W[17], rng.random((200, dim)).astype(np.float32)])
    som = Som(rows, cols, dim, codebook=torch.from_numpy(W))
    b = som.bmus(P.to_dev(X)).cpu().numpy()
    assert b[:5].tolist() == [17, 17, 130, 3, 17]
    assert np.array_equal(b, oracle.bmu_dense(X, W))
    som.close()


def test_identical_codebook_rows_force_full_rescan(oracle):
    """All nodes equal: every score ties, every instance takes the exact rescan, answer node 0."""
    from paper_1305_1422_amd import Som
    rng = np.random.default_rng(8)
    rows, cols, dim, n = 20, 14, 20, 300
    W = np.tile(rng.random((1, dim)).astype(np.float32), (rows * cols, 1))
    X = rng.random((n, dim)).astype(np.float32)
    som = Som(rows, cols, dim, codebook=torch.from_numpy(W))
    b = som.bmus(P.to_dev(X)).cpu().numpy()
    assert np.all(b == 0)
    refined, collected, rescanned = som.stats()
    assert rescanned == n and collected == n and refined == 0       # 280 equal nodes overflow the lists of 256
    som.close()


def test_many_identical_codebook_rows_fit_the_collected_lists(oracle):
    """140 equal nodes among others: every instance's list holds them all, lowest index wins."""
    from paper_1305_1422_amd import Som
    rng = np.random.default_rng(9)
    rows, cols, dim, n = 10, 20, 24, 300
    W = rng.random((rows * cols, dim)).astype(np.float32) + 3.0      # far from the data
    W[37:177] = rng.random((1, dim)).astype(np.float32)              # 140 copies of one near vector
    X = rng.random((n, dim)).astype(np.float32)
    som = Som(rows, cols, dim, codebook=torch.from_numpy(W))
    b = som.bmus(P.to_dev(X)).cpu().numpy()
    assert np.all(b == 37)
    refined, collected, rescanned = som.stats()
    assert collected == n and rescanned == 0 and refined == 0
    som.close()


def test_near_ties_are_decided_exactly(oracle):
    """Nodes that differ from each other by a few ulps: fp32 scores cannot separate them, the
    exact stage must, and agree with the oracle outside the 1e-5 band (here: everywhere but
    where the fp64 distances themselves tie)."""
    from paper_1305_1422_amd import Som
    rng = np.random.default_rng(9)
    rows, cols, dim, n = 8, 8, 512, 400
    base = rng.random((4, dim)).astype(np.float32)
    W = base[rng.integers(4, size=rows * cols)].copy()
    W += (rng.integers(-2, 3, size=W.shape) * np.float32(2.0 ** -22)).astype(np.float32)   # a few ulps of noise
    X = (base[rng.integers(4, size=n)] + rng.normal(0, 0.05, size=(n, dim))).astype(np.float32)
    som = Som(rows, cols, dim, codebook=torch.from_numpy(W))
    b = som.bmus(P.to_dev(X)).cpu().numpy()
    P.check_bmus_dense(oracle, X, W, b)
    refined, collected, rescanned = som.stats()
    assert collected > 0 and rescanned == 0          # 16 near-copies per base vector: collected lists
    som.close()


def test_update_with_skewed_segments_and_empty_nodes(oracle):
    """All instances on three nodes (one of them takes 90 %): long segments split into many
    chunks; most nodes empty.  Small radius: far nodes have zero mass and must not move."""
    from paper_1305_1422_amd import Som
    rng = np.random.default_rng(10)
    rows, cols, dim, n = 20, 20, 36, 5000
    X = rng.normal(0, 1, size=(n, dim)).astype(np.float32)
    W = rng.random((rows * cols, dim)).astype(np.float32)
    bmus = rng.choice(np.array([7, 211, 399], dtype=np.int32), size=n, p=[0.9, 0.09, 0.01]).astype(np.int32)
    for map_type, grid, radius in [("planar", "square", 0.9), ("toroid", "hexagonal", 0.7), ("planar", "hexagonal", 3.0)]:
        som = Som(rows, cols, dim, map_type, grid, codebook=torch.from_numpy(W))
        som.update(P.to_dev(X), P.to_dev(bmus), radius)
        torch.cuda.synchronize()
        S, C = oracle.accumulate_dense(X, bmus, rows * cols)
        kept, _ = P.check_codebook(oracle, S, C, W, som.codebook.cpu().numpy(), rows, cols, P.MAP[map_type],
                                   P.GRID[grid], radius)
        assert kept > 0
        som.close()


def test_update_radius_to_zero_is_kmeans(oracle):
    """Spec invariant on the GPU: tiny radius -> hit nodes become the centroid of their
    instances, all other nodes keep their weights bit for bit."""
    from paper_1305_1422_amd import Som
    rng = np.random.default_rng(11)
    rows, cols, dim, n = 9, 11, 24, 1200
    X = rng.random((n, dim)).astype(np.float32)
    W = rng.random((rows * cols, dim)).astype(np.float32)
    bmus = (rng.integers(0, rows * cols // 2, size=n) * 2).astype(np.int32)
    som = Som(rows, cols, dim, "toroid", "square", codebook=torch.from_numpy(W))
    som.update(P.to_dev(X), P.to_dev(bmus), 1e-3)
    got = som.codebook.cpu().numpy()
    sums = np.zeros((rows * cols, dim)); np.add.at(sums, bmus, X.astype(np.float64))
    cnt = np.bincount(bmus, minlength=rows * cols)
    hit = cnt > 0
    np.testing.assert_allclose(got[hit], sums[hit] / cnt[hit, None], rtol=1e-4, atol=1e-5)
    assert np.array_equal(got[~hit], W[~hit])
    som.close()


def test_update_is_bit_reproducible(oracle):
    from paper_1305_1422_amd import Som
    w = scaled_workload(2, n=4000, dim=96, rows=10, cols=10)
    X = P.to_dev(w.data())
    outs = []
    for _ in range(2):
        som = _som(w, w.codebook())
        som.train_epoch(X, 3.0)
        outs.append(som.codebook.cpu().numpy().copy())
        som.close()
    assert np.array_equal(outs[0], outs[1])


def test_train_matches_epoch_by_epoch_and_oracle(oracle):
    """som_train (device-side schedule, no host work per epoch) against (a) the same epochs issued
    one by one with radii from the oracle's cooling, bit for bit, and (b) the oracle running free."""
    w = scaled_workload(1, n=600, dim=10, rows=10, cols=10, epochs=6)      # radius 5 -> 1: 5, 4.2, ...
    X = w.data(); Xd = P.to_dev(X)
    a = _som(w, w.codebook())
    last = a.train(Xd, w.epochs, w.radius0, w.radiusN, w.scale0, w.scaleN, "linear")
    b = _som(w, w.codebook())
    Wo = w.codebook()
    for e in range(w.epochs):
        r = oracle.cool(w.radius0, w.radiusN, w.epochs, e, oracle.LINEAR)
        Win = b.codebook.cpu().numpy().copy()
        bm = b.train_epoch(Xd, float(np.float32(r)))
        bo, Wo = oracle.epoch_dense(X, Wo, w.rows, w.cols, P.MAP[w.map_type], P.GRID[w.grid_type], r)
    torch.cuda.synchronize()
    # radii 5, 4.2, 3.4 ... are not all fp32 numbers: allow the last bits to differ between (a) and (b)
    np.testing.assert_allclose(a.codebook.cpu().numpy(), b.codebook.cpu().numpy(), rtol=1e-5, atol=1e-6)
    P.check_bmus_dense(oracle, X, Win, last.cpu().numpy())
    # free-running oracle: same trajectory unless a near-tie flipped, which these sizes do not show
    np.testing.assert_allclose(a.codebook.cpu().numpy(), Wo, rtol=1e-3, atol=1e-4)
    a.close(); b.close()


def test_init_from_seed_is_uniform_and_deterministic(oracle):
    from paper_1305_1422_amd import Som
    a = Som(30, 40, 16, seed=1234)
    b = Som(30, 40, 16, seed=1234)
    c = Som(30, 40, 16, seed=1235)
    A, B, Cc = a.codebook.cpu().numpy(), b.codebook.cpu().numpy(), c.codebook.cpu().numpy()
    assert np.array_equal(A, B) and not np.array_equal(A, Cc)
    assert A.min() >= 0.0 and A.max() < 1.0
    assert abs(A.mean() - 0.5) < 0.01 and abs(A.var() - 1 / 12) < 0.005
    assert np.unique(A).size > 0.99 * A.size * (1 - A.size / 2 ** 25)       # 24-bit values, few repeats
    a.close(); b.close(); c.close()


def test_argument_errors(oracle):
    from paper_1305_1422_amd import Som, capi
    X = P.to_dev(np.zeros((4, 3), np.float32))
    som = Som(2, 2, 3, seed=1)
    with pytest.raises(capi.SomError) as e:
        som.train_epoch(X, 0.0)
    assert e.value.code == capi.SOM_ERR_INVALID_ARG
    with pytest.raises(capi.SomError):
        som.train_epoch(X, 1.0, scale=1.5)
    with pytest.raises(capi.SomError):
        som.train_epoch(X, float("nan"))
    with pytest.raises(capi.SomError) as e:
        capi.som_train(som.ctx, 3, 0.0, 0.0, 0.0, 0.0, 0, som.codebook, torch.empty(4, dtype=torch.int32, device="cuda"))
    assert e.value.code == capi.SOM_ERR_STATE
    with pytest.raises(capi.SomError):
        capi.som_init(0, 5, 3, 0, 0, som.codebook)
    with pytest.raises(capi.SomError):
        capi.som_init(2, 2, 3, 7, 0, som.codebook)
    with pytest.raises(TypeError):
        som.train_epoch(torch.zeros((4, 3)), 1.0)                # host tensor: refused by the binding
    som.close()


def test_registered_data_gives_identical_epochs(oracle):
    """Epoch calls on the registered training set reuse its cached norms: same BMUs and code book
    as on unregistered data, also after other data went through the context in between."""
    from paper_1305_1422_amd import Som, capi
    w = scaled_workload(2, n=2500, dim=120, rows=9, cols=9)
    X = P.to_dev(w.data())
    other = P.to_dev(np.random.default_rng(5).random((700, w.dim)).astype(np.float32) * 7)
    a = _som(w, w.codebook()); b = _som(w, w.codebook())
    capi.som_set_data_dense(b.ctx, X)
    for r in (4.0, 2.0):
        ba = a.train_epoch(X, r).cpu().numpy()
        bb = b.train_epoch(X, r).cpu().numpy()
        assert np.array_equal(ba, bb)
        assert np.array_equal(a.codebook.cpu().numpy(), b.codebook.cpu().numpy())
        b.bmus(other)                                  # overwrites the cached norms; must be noticed
    a.close(); b.close()


def test_non_finite_instances_do_not_leave_the_index_range(oracle):
    """NaN and infinite components: such an instance has no finite distance to any node and a plain scan
    (strict <, starting from +inf) leaves it at node 0; the other instances are unaffected."""
    from paper_1305_1422_amd import Som
    rng = np.random.default_rng(77)
    n, dim, rows, cols = 700, 70, 14, 13
    X = rng.random((n, dim)).astype(np.float32)
    W = rng.random((rows * cols, dim)).astype(np.float32)
    bad = {5: np.nan, 130: np.inf, 131: -np.inf, 699: np.nan}
    for j, v in bad.items():
        X[j, (3 * j) % dim] = v
    X[400, :] = np.inf
    som = Som(rows, cols, dim, codebook=torch.from_numpy(W))
    b = som.bmus(P.to_dev(X)).cpu().numpy()
    want = oracle.bmu_dense(X, W)
    assert b.min() >= 0 and b.max() < rows * cols
    assert np.array_equal(b, want)
    assert all(b[j] == 0 for j in list(bad) + [400])
    # a whole epoch goes through as well: the update must not fault on such rows (node 0 inherits them)
    som.train_epoch(P.to_dev(X), 2.0)
    torch.cuda.synchronize()
    som.close()


@pytest.mark.parametrize("dim", [31, 32, 33, 63, 64, 65, 96, 127, 129, 255, 257, 513])
def test_feature_counts_around_the_chunk_boundaries(oracle, dim):
    """The filter pass walks the features in chunks of 32 and pads the last one; the per-node sums read rows
    as 16-byte vectors when dim % 4 == 0 and element by element otherwise."""
    from paper_1305_1422_amd import Som
    rng = np.random.default_rng(5000 + dim)
    n, rows, cols = 333, 6, 7
    X = rng.normal(0.0, 1.0, (n, dim)).astype(np.float32)
    W = rng.normal(0.0, 1.0, (rows * cols, dim)).astype(np.float32)
    som = Som(rows, cols, dim, "toroid", "hexagonal", codebook=torch.from_numpy(W))
    P.epoch_parity_dense(oracle, som, X, P.to_dev(X), 2.0, P.MAP["toroid"], P.GRID["hexagonal"])
    som.close()


@pytest.mark.parametrize("rows,cols", [(2, 1100), (1030, 3)])
@pytest.mark.parametrize("map_type,grid", [("planar", "square"), ("toroid", "hexagonal")])
def test_map_side_above_the_coefficient_matrix_limit(oracle, rows, cols, map_type, grid):
    """A side of more than 1,024 nodes: the smoothing runs on the filter vectors directly instead of the
    stored coefficient matrices."""
    from paper_1305_1422_amd import Som
    rng = np.random.default_rng(rows * 7 + cols)
    n, dim = 400, 12
    X = rng.random((n, dim)).astype(np.float32)
    W = rng.random((rows * cols, dim)).astype(np.float32)
    som = Som(rows, cols, dim, map_type, grid, codebook=torch.from_numpy(W))
    for radius in (40.0, 3.0):
        P.epoch_parity_dense(oracle, som, X, P.to_dev(X), radius, P.MAP[map_type], P.GRID[grid])
    som.close()


def test_long_instances_take_the_workgroup_per_row_split(oracle):
    """More than 2,048 features: the fp16 planes are written by a workgroup per row instead of a wavefront."""
    from paper_1305_1422_amd import Som
    rng = np.random.default_rng(91)
    n, dim, rows, cols = 150, 2100, 5, 6
    X = rng.normal(0.0, 1.0, (n, dim)).astype(np.float32)
    W = rng.normal(0.0, 1.0, (rows * cols, dim)).astype(np.float32)
    som = Som(rows, cols, dim, codebook=torch.from_numpy(W))
    P.epoch_parity_dense(oracle, som, X, P.to_dev(X), 1.5, P.MAP["planar"], P.GRID["square"])
    som.close()


def test_one_context_serves_growing_and_shrinking_data_and_every_filter(oracle):
    """The per-data scratch grows on demand and is reused for smaller sets; changing the filter variant in
    between must not leave stale planes or candidate arrays behind."""
    from paper_1305_1422_amd import Som
    rng = np.random.default_rng(92)
    dim, rows, cols = 70, 15, 14
    W = rng.random((rows * cols, dim)).astype(np.float32)
    som = Som(rows, cols, dim, codebook=torch.from_numpy(W))
    for n, filt in [(100, "split_f16"), (5000, "two_level"), (300, "fp32"), (7000, "fp32"), (64, "two_level"),
                    (7000, "split_f16"), (9000, "two_level"), (6000, "auto")]:
        som.set_filter(filt)
        X = rng.random((n, dim)).astype(np.float32)
        b = som.bmus(P.to_dev(X)).cpu().numpy()
        P.check_bmus_dense(oracle, X, W, b)
    som.close()
