"""Parity of the sparse (CSR) HIP path against the CPU oracle (gpu tests, through the C ABI)."""
import numpy as np
import pytest

from gen import scaled_workload, sparse_uniform_csr, sparse_zipf_csr
from tests import parity as P

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def densify(csr, dim):
    indptr, indices, values = csr
    X = np.zeros((len(indptr) - 1, dim), dtype=np.float32)
    for j in range(len(indptr) - 1):
        X[j, indices[indptr[j]:indptr[j + 1]]] = values[indptr[j]:indptr[j + 1]]
    return X


@pytest.mark.parametrize("n,dim,rows,cols,epochs,mean_len", [
    (2000, 3000, 12, 10, 4, 100.0),     # configuration 4 scaled: one node sweep per instance
    (600, 900, 24, 22, 2, 30.0),        # 528 nodes: three 256-node slices, the last ragged
    (300, 500, 1, 3, 2, 8.0),           # tiny map
])
def test_scaled_config4(oracle, n, dim, rows, cols, epochs, mean_len):
    from paper_1305_1422_amd import Som
    w = scaled_workload(4, n=n, dim=dim, rows=rows, cols=cols, epochs=epochs)
    csr = sparse_zipf_csr(n, dim, w.data_seed, mean_len=mean_len, max_len=int(4 * mean_len))
    csr_d = P.csr_to_dev(csr)
    som = Som(rows, cols, dim, w.map_type, w.grid_type, codebook=torch.from_numpy(w.codebook()))
    for e in range(epochs):
        r = oracle.cool(w.radius0, w.radiusN, epochs, e, oracle.LINEAR)
        P.epoch_parity_csr(oracle, som, csr, csr_d, dim, r, P.MAP[w.map_type], P.GRID[w.grid_type])
    som.close()


@pytest.mark.parametrize("rows,cols", [(70, 64), (64, 128), (100, 100)])
def test_many_nodes(oracle, rows, cols):
    """4,480 and 8,192 nodes: nine and sixteen scores per lane with one node range per XCD slice;
    10,000 nodes: two ranges per slice."""
    from paper_1305_1422_amd import Som
    dim, n = 300, 150
    csr = sparse_zipf_csr(n, dim, 21, mean_len=12.0, max_len=40)
    W = np.random.default_rng(22).random((rows * cols, dim)).astype(np.float32)
    som = Som(rows, cols, dim, "toroid", "hexagonal", codebook=torch.from_numpy(W))
    b = som.bmus(P.csr_to_dev(csr)).cpu().numpy()
    P.check_bmus_csr(oracle, csr, dim, W, b)
    som.close()


def test_smooth_map_takes_the_second_sweep_over_listed_ranges(oracle):
    """A code book smoothed with a wide neighbourhood has neighbouring nodes closer than the 16-bit
    filter can separate: many instances go to the second sweep, which visits only the node ranges whose
    third-best score is inside the threshold and takes the other ranges' nodes from the first sweep.
    10,000 nodes = two ranges per slice; the result must still be the exact argmin."""
    from paper_1305_1422_amd import Som
    rows, cols, dim, n = 100, 100, 400, 600
    csr = sparse_zipf_csr(n, dim, 41, mean_len=20.0, max_len=60)
    W0 = np.random.default_rng(42).random((rows * cols, dim)).astype(np.float32)
    som = Som(rows, cols, dim, "toroid", "square", codebook=torch.from_numpy(W0))
    csr_d = P.csr_to_dev(csr)
    som.train_epoch(csr_d, 30.0)
    collected = 0
    for radius in (30.0, 12.0):
        W_in = som.codebook.cpu().numpy().copy()
        b = som.train_epoch(csr_d, radius).cpu().numpy()
        collected += som.stats()[1]
        P.check_bmus_csr(oracle, csr, dim, W_in, b)
    assert collected >= 100, f"only {collected} instances took the second sweep: the test misses its case"
    som.close()


def test_sparse_path_equals_dense_path_on_densified_rows(oracle):
    from paper_1305_1422_amd import Som
    n, dim, rows, cols = 500, 640, 9, 8
    csr = sparse_zipf_csr(n, dim, 23, mean_len=25.0, max_len=80)
    X = densify(csr, dim)
    W = (np.random.default_rng(24).random((rows * cols, dim)) * 0.2).astype(np.float32)
    a = Som(rows, cols, dim, "planar", "square", codebook=torch.from_numpy(W))
    b = Som(rows, cols, dim, "planar", "square", codebook=torch.from_numpy(W))
    ba = a.train_epoch(P.csr_to_dev(csr), 2.0).cpu().numpy()
    bb = b.train_epoch(P.to_dev(X), 2.0).cpu().numpy()
    assert np.array_equal(ba, bb)
    np.testing.assert_allclose(a.codebook.cpu().numpy(), b.codebook.cpu().numpy(), rtol=1e-5, atol=1e-6)
    a.close(); b.close()


def test_empty_rows_and_duplicate_nodes(oracle):
    from paper_1305_1422_amd import Som
    dim, rows, cols = 50, 4, 5
    rng = np.random.default_rng(25)
    W = rng.random((rows * cols, dim)).astype(np.float32) + np.float32(0.5)
    W[11] = W[2] = (W[7] * np.float32(0.01))            # nodes 2 and 11: equal, and the smallest norm
    indptr = np.array([0, 0, 3, 3, 5], dtype=np.int64)  # rows 0 and 2 are empty
    indices = np.array([1, 7, 40, 0, 49], dtype=np.int32)
    values = np.array([0.5, -1.0, 2.0, 3.0, 0.25], dtype=np.float32)
    csr = (indptr, indices, values)
    som = Som(rows, cols, dim, codebook=torch.from_numpy(W))
    b = som.bmus(P.csr_to_dev(csr)).cpu().numpy()
    want = oracle.bmu_csr(csr, dim, W)
    assert np.array_equal(b, want) and b[0] == 2 and b[2] == 2
    som.close()


def test_update_csr_given_bmus(oracle):
    from paper_1305_1422_amd import Som
    n, dim, rows, cols = 900, 400, 10, 12
    csr = sparse_zipf_csr(n, dim, 26, mean_len=15.0, max_len=50)
    rng = np.random.default_rng(27)
    W = rng.random((rows * cols, dim)).astype(np.float32)
    bmus = rng.integers(0, rows * cols, size=n).astype(np.int32)
    bmus[: n // 2] = 17                                   # one heavy node
    for map_type, grid, radius in [("toroid", "square", 2.5), ("planar", "hexagonal", 0.8)]:
        som = Som(rows, cols, dim, map_type, grid, codebook=torch.from_numpy(W))
        som.update(P.csr_to_dev(csr), P.to_dev(bmus), radius)
        torch.cuda.synchronize()
        S, C = oracle.accumulate_csr(csr, dim, bmus, rows * cols)
        P.check_codebook(oracle, S, C, W, som.codebook.cpu().numpy(), rows, cols, P.MAP[map_type], P.GRID[grid], radius)
        som.close()


def test_train_csr_schedule_runs_and_matches_last_epoch(oracle):
    from paper_1305_1422_amd import Som
    n, dim, rows, cols, E = 800, 1000, 8, 8, 4
    csr = sparse_zipf_csr(n, dim, 28, mean_len=40.0, max_len=120)
    csr_d = P.csr_to_dev(csr)
    W0 = np.random.default_rng(29).random((rows * cols, dim)).astype(np.float32) * np.float32(0.1)
    a = Som(rows, cols, dim, codebook=torch.from_numpy(W0))
    a.train(csr_d, E, 4.0, 1.0, 1.0, 0.01, "linear")
    b = Som(rows, cols, dim, codebook=torch.from_numpy(W0))
    for e in range(E):
        b.train_epoch(csr_d, oracle.cool(4.0, 1.0, E, e, oracle.LINEAR))      # 4, 3, 2, 1: exact in fp32
    np.testing.assert_allclose(a.codebook.cpu().numpy(), b.codebook.cpu().numpy(), rtol=1e-5, atol=1e-6)
    a.close(); b.close()


def test_non_finite_values_do_not_leave_the_index_range(oracle):
    from paper_1305_1422_amd import Som
    n, dim, rows, cols = 300, 400, 9, 9
    indptr, indices, values = sparse_zipf_csr(n, dim, 78, mean_len=15.0, max_len=40)
    values = values.copy()
    bad_rows = [0, 17, 299]
    for j, v in zip(bad_rows, (np.nan, np.inf, -np.inf)):
        values[indptr[j]] = v
    csr = (indptr, indices, values)
    W = np.random.default_rng(79).random((rows * cols, dim)).astype(np.float32)
    som = Som(rows, cols, dim, codebook=torch.from_numpy(W))
    b = som.bmus(P.csr_to_dev(csr)).cpu().numpy()
    want = oracle.bmu_csr(csr, dim, W)
    assert b.min() >= 0 and b.max() < rows * cols
    assert np.array_equal(b, want)
    assert all(b[j] == 0 for j in bad_rows)
    som.close()


@pytest.mark.parametrize("dim", [16384, 16385])
def test_update_csr_at_the_row_length_where_the_accumulation_changes(oracle, dim):
    """Rows of up to 16,384 columns are summed in LDS per node, longer ones with global atomics; both sides
    of the switch, with one node that holds more instances than one chunk."""
    from paper_1305_1422_amd import Som
    n, rows, cols = 700, 3, 4
    csr = sparse_zipf_csr(n, dim, 43, mean_len=12.0, max_len=40)
    rng = np.random.default_rng(44)
    W = rng.random((rows * cols, dim)).astype(np.float32)
    bmus = rng.integers(0, rows * cols, size=n).astype(np.int32)
    bmus[:400] = 5
    bmus[bmus == 9] = 2                                    # node 9 is chosen by nobody
    som = Som(rows, cols, dim, "planar", "square", codebook=torch.from_numpy(W))
    som.update(P.csr_to_dev(csr), P.to_dev(bmus), 1.0)
    torch.cuda.synchronize()
    S, C = oracle.accumulate_csr(csr, dim, bmus, rows * cols)
    P.check_codebook(oracle, S, C, W, som.codebook.cpu().numpy(), rows, cols, oracle.PLANAR, oracle.SQUARE, 1.0)
    som.close()


def test_sparse_update_on_a_map_side_above_the_coefficient_matrix_limit(oracle):
    """With a side of more than 1,024 nodes the smoothing reads every row of the per-node sums, chosen or
    not: the rows nobody chose have to be zero."""
    from paper_1305_1422_amd import Som
    rows, cols, dim, n = 2, 1040, 60, 500
    csr = sparse_zipf_csr(n, dim, 45, mean_len=8.0, max_len=25)
    W = np.random.default_rng(46).random((rows * cols, dim)).astype(np.float32)
    som = Som(rows, cols, dim, "toroid", "square", codebook=torch.from_numpy(W))
    csr_d = P.csr_to_dev(csr)
    for radius in (25.0, 2.0):
        P.epoch_parity_csr(oracle, som, csr, csr_d, dim, radius, oracle.TOROID, oracle.SQUARE)
    som.close()


@pytest.mark.parametrize("acc", list(range(1, 17)))
def test_every_number_of_scores_per_lane(oracle, acc):
    """512 acc - 7 nodes: acc scores per lane and node range in the sparse sweep (one range per slice), the
    last slice ragged; both sweeps, since the code book rows are nearly alike."""
    from paper_1305_1422_amd import Som
    k = 512 * acc - 7
    rows, cols = 1, k
    dim, n = 120, 70
    csr = sparse_zipf_csr(n, dim, 47 + acc, mean_len=9.0, max_len=30)
    rng = np.random.default_rng(48 + acc)
    W = (rng.random((1, dim)) + 1e-4 * rng.random((k, dim))).astype(np.float32)
    som = Som(rows, cols, dim, "planar", "square", codebook=torch.from_numpy(W))
    b = som.bmus(P.csr_to_dev(csr)).cpu().numpy()
    P.check_bmus_csr(oracle, csr, dim, W, b)
    som.close()


def test_one_context_serves_growing_and_shrinking_sparse_data(oracle):
    from paper_1305_1422_amd import Som
    rng = np.random.default_rng(93)
    dim, rows, cols = 900, 11, 12
    W = (rng.random((rows * cols, dim)) * 0.1).astype(np.float32)
    som = Som(rows, cols, dim, codebook=torch.from_numpy(W))
    for t, n in enumerate([50, 3000, 200, 4000, 10]):
        csr = sparse_zipf_csr(n, dim, 94 + t, mean_len=20.0 + 10 * t, max_len=200)
        b = som.bmus(P.csr_to_dev(csr)).cpu().numpy()
        P.check_bmus_csr(oracle, csr, dim, W, b)
    som.close()


def test_all_rows_empty(oracle):
    """nnz = 0 is legal: every instance is the zero vector and maps to the node of smallest norm
    (lowest index among equals); the update then gives every reachable node the zero vector."""
    from paper_1305_1422_amd import Som
    dim, rows, cols, n = 70, 5, 6, 33
    rng = np.random.default_rng(95)
    W = rng.random((rows * cols, dim)).astype(np.float32) + np.float32(0.25)
    W[19] = W[8] = W[3] * np.float32(0.05)
    csr = (np.zeros(n + 1, dtype=np.int64), np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.float32))
    som = Som(rows, cols, dim, codebook=torch.from_numpy(W))
    csr_d = P.csr_to_dev(csr)
    b = som.bmus(csr_d).cpu().numpy()
    assert np.array_equal(b, oracle.bmu_csr(csr, dim, W)) and np.all(b == 8)
    P.epoch_parity_csr(oracle, som, csr, csr_d, dim, 1.5, oracle.PLANAR, oracle.SQUARE)
    som.close()


def test_instances_that_coincide_with_nodes(oracle):
    """Weight vectors equal to instances, with one-ulp near-copies at lower and higher node indices and a
    long feature space: a distance evaluated as |w|^2 - 2 x.w + ... cancels to its own rounding here and
    cannot tell the copies apart; the search must still return the coincident node, at distance exactly 0."""
    from paper_1305_1422_amd import Som, capi
    dim, n, rows, cols = 12000, 96, 12, 24
    csr = sparse_zipf_csr(n, dim, 96, mean_len=90.0, max_len=300)
    X = densify(csr, dim)
    rng = np.random.default_rng(97)
    W = (rng.random((rows * cols, dim)) * 0.05).astype(np.float32)
    first = csr[1][csr[0][:-1]]                                   # first listed column of every row
    W[n:2 * n] = X                                                # node n + j is instance j
    W[:n] = X
    W[np.arange(n), first] = np.nextafter(X[np.arange(n), first], np.float32(9.0))       # one ulp up
    W[2 * n:3 * n] = X
    W[2 * n + np.arange(n), first] = np.nextafter(X[np.arange(n), first], np.float32(-9.0))   # one ulp down
    som = Som(rows, cols, dim, codebook=torch.from_numpy(W))
    csr_d = P.csr_to_dev(csr)
    b = som.bmus(csr_d).cpu().numpy()
    assert np.array_equal(b, np.arange(n, 2 * n))
    P.check_bmus_csr(oracle, csr, dim, W, b)
    dist, qe = som.bmu_distances(csr_d, P.to_dev(b.astype(np.int32)))
    assert float(qe) == 0.0 and np.all(dist.cpu().numpy() == 0.0)
    som.close()


@pytest.mark.parametrize("nb,compact,radius", [("gaussian", True, 1.0), ("bubble", False, 1.0), ("gaussian", True, 0.5)])
def test_nodes_updated_by_a_single_instance(oracle, nb, compact, radius):
    """More nodes than instances under a neighbourhood of compact support: after an epoch many nodes are the
    weighted mean of ONE instance, i.e. that instance up to an ulp, and so are their neighbours.  The next
    searches meet instances that (nearly) coincide with several nodes; BMUs and code book must keep matching
    the oracle under the plain rule (a best distance of 0 admits only answers at distance 0)."""
    from paper_1305_1422_amd import Som
    dim, n, rows, cols = 6000, 150, 30, 28
    csr = sparse_zipf_csr(n, dim, 98, mean_len=40.0, max_len=160)
    W0 = (np.random.default_rng(99).random((rows * cols, dim)) * 0.02).astype(np.float32)
    som = Som(rows, cols, dim, "toroid", "hexagonal", codebook=torch.from_numpy(W0))
    som.set_neighborhood(nb, compact)
    csr_d = P.csr_to_dev(csr)
    zero_best = 0
    for e in range(4):
        W_in = som.codebook.cpu().numpy().copy()
        b = som.train_epoch(csr_d, radius).cpu().numpy()
        P.check_bmus_csr(oracle, csr, dim, W_in, b)
        zero_best += int(np.count_nonzero(oracle.sqdist_pairs_csr(csr, dim, W_in, np.arange(n), b) < 1e-12))
        S, C = oracle.accumulate_csr(csr, dim, b, rows * cols)
        P.check_codebook(oracle, S, C, W_in, som.codebook.cpu().numpy(), rows, cols, oracle.TOROID, oracle.HEXAGONAL,
                         radius, function=1 if nb == "bubble" else 0, compact=compact)
    assert zero_best >= n // 2, "hardly any instance ever sat on a node: the test misses its case"
    som.close()


def test_validate_csr_names_every_kind_of_violation():
    from paper_1305_1422_amd import Som, capi
    dim, n = 300, 500
    indptr, indices, values = sparse_zipf_csr(n, dim, 61, mean_len=12.0, max_len=40)
    som = Som(3, 3, dim, seed=5)
    som.validate_csr(P.csr_to_dev((indptr, indices, values)))

    def expect(ip, ix, what):
        with pytest.raises(capi.SomError) as err:
            som.validate_csr(P.csr_to_dev((ip, ix, values[: ix.size])))
        assert err.value.code == capi.SOM_ERR_INVALID_ARG and what in str(err.value)

    ip = indptr.copy(); ip[0] = 1
    expect(ip, indices, "indptr[0]")
    ip = indptr.copy(); ip[-1] -= 1
    expect(ip, indices, "indptr[n]")
    ip = indptr.copy(); ip[200] = ip[201] + 3
    expect(ip, indices, "indptr decreases")
    ip = indptr.copy(); ip[77] = -5
    expect(ip, indices, "indptr decreases")
    ix = indices.copy(); ix[indptr[123]] = dim
    expect(indptr, ix, "outside [0, dim)")
    ix = indices.copy(); ix[indptr[400] + 1] = -1
    expect(indptr, ix, "outside [0, dim)")
    j = int(np.argmax(np.diff(indptr) >= 3))
    ix = indices.copy(); ix[indptr[j] + 1], ix[indptr[j] + 2] = ix[indptr[j] + 2], ix[indptr[j] + 1]
    expect(indptr, ix, "strictly increasing")
    ix = indices.copy(); ix[indptr[j] + 1] = ix[indptr[j]]            # a duplicate column
    expect(indptr, ix, "strictly increasing")
    # all rows empty, and a row that ends the array, are well formed
    som.validate_csr(P.csr_to_dev((np.zeros(n + 1, np.int64), indices[:0], values[:0])))
    som.close()


@pytest.mark.parametrize("n,dim,rows,cols,mean_len", [(3000, 4000, 12, 10, 60.0), (700, 1500, 24, 22, 25.0)])
def test_hot_column_block_of_a_registered_set(oracle, n, dim, rows, cols, mean_len):
    """A registered sparse set with skewed column frequencies: its 256 most frequent columns go through the
    matrix cores, the rest through the gather sweep.  BMUs are the exact argmin either way, so they must be
    the same with the split on and off, epoch by epoch, and match the oracle; instances 0 / 1 have no nonzero
    at all / none outside the frequent columns."""
    from paper_1305_1422_amd import Som, capi
    indptr, indices, values = sparse_zipf_csr(n, dim, 71, mean_len=mean_len, max_len=int(4 * mean_len))
    freq = np.bincount(indices, minlength=dim)
    hot = np.sort(np.argsort(-freq, kind="stable")[:256])
    keep = np.ones(indices.size, bool)
    keep[indptr[0]:indptr[1]] = False                                             # row 0: empty
    keep[indptr[1]:indptr[2]] = np.isin(indices[indptr[1]:indptr[2]], hot)        # row 1: frequent columns only
    lens = np.add.reduceat(keep, indptr[:-1]) * (np.diff(indptr) > 0)
    indptr2 = np.zeros(n + 1, np.int64)
    np.cumsum(lens, out=indptr2[1:])
    csr = (indptr2, indices[keep], values[keep])
    assert indptr2[1] == 0 and indptr2[2] > indptr2[1]
    csr_d = P.csr_to_dev(csr)
    W0 = (np.random.default_rng(72).random((rows * cols, dim)) * 0.1).astype(np.float32)
    out = {}
    for on in (True, False):
        som = Som(rows, cols, dim, "toroid", "square", codebook=torch.from_numpy(W0))
        som.set_sparse_hot_block(on)
        capi.som_set_data_csr(som.ctx, *csr_d)
        seq = []
        for radius in (4.0, 2.0, 1.0):
            W_in = som.codebook.cpu().numpy().copy()
            b = som.train_epoch(csr_d, radius).cpu().numpy()
            assert capi.som_sparse_hot_block_active(som.ctx) == on
            P.check_bmus_csr(oracle, csr, dim, W_in, b)
            seq.append(b)
        b = som.bmus(csr_d).cpu().numpy()                      # search only, on the final map
        P.check_bmus_csr(oracle, csr, dim, som.codebook.cpu().numpy(), b)
        seq.append(b)
        out[on] = seq
        som.close()
    assert np.array_equal(out[True][0], out[False][0])         # same input code book: same BMUs, bit for bit


def test_hot_column_block_is_declined_for_evenly_used_columns(oracle):
    from paper_1305_1422_amd import Som, capi
    rng = np.random.default_rng(73)
    n, dim, rows, cols = 400, 2048, 6, 7
    lens = rng.integers(5, 40, n)
    indptr = np.zeros(n + 1, np.int64)
    np.cumsum(lens, out=indptr[1:])
    indices = np.concatenate([np.sort(rng.choice(dim, size=int(l), replace=False)) for l in lens]).astype(np.int32)
    values = rng.random(indices.size).astype(np.float32)
    csr = (indptr, indices, values)
    W = rng.random((rows * cols, dim)).astype(np.float32)
    som = Som(rows, cols, dim, codebook=torch.from_numpy(W))
    csr_d = P.csr_to_dev(csr)
    capi.som_set_data_csr(som.ctx, *csr_d)
    b = som.bmus(csr_d).cpu().numpy()
    assert not capi.som_sparse_hot_block_active(som.ctx)       # 256 of 2,048 evenly used columns hold an eighth
    P.check_bmus_csr(oracle, csr, dim, W, b)
    som.close()


@pytest.mark.parametrize("n,dim,rows,cols,density,filt", [(1500, 600, 30, 40, 0.05, None), (700, 333, 9, 11, 0.2, "split_f16"),
                                                           (2000, 96, 36, 36, 0.5, "two_level")])
def test_dense_planes_of_a_registered_set(oracle, n, dim, rows, cols, density, filt):
    """A registered sparse set of modest dimension and at least 4 % nonzeros is searched through the dense
    filter on fp16 planes of its centred rows; the exact stage and the update stay on the sparse rows.  BMUs
    are the exact argmin either way: the same with the planes on and off, epoch by epoch, equal to the
    oracle's; row 0 is empty, row 1 has a single nonzero."""
    from paper_1305_1422_amd import Som, capi
    indptr, indices, values = sparse_uniform_csr(n, dim, 81, density=density)
    keep = np.ones(indices.size, bool)
    keep[indptr[0]:indptr[1]] = False
    keep[indptr[1] + 1:indptr[2]] = False
    lens = np.add.reduceat(keep, indptr[:-1]) * (np.diff(indptr) > 0)
    indptr2 = np.zeros(n + 1, np.int64)
    np.cumsum(lens, out=indptr2[1:])
    csr = (indptr2, indices[keep], values[keep])
    assert indptr2[1] == 0 and indptr2[2] == 1
    csr_d = P.csr_to_dev(csr)
    W0 = np.random.default_rng(82).random((rows * cols, dim)).astype(np.float32)
    out = {}
    for on in (True, False):
        som = Som(rows, cols, dim, "planar", "hexagonal", codebook=torch.from_numpy(W0), filter=filt)
        som.set_sparse_dense_filter(on)
        capi.som_set_data_csr(som.ctx, *csr_d)
        seq = []
        for radius in (5.0, 2.0, 1.0):
            W_in = som.codebook.cpu().numpy().copy()
            b = som.train_epoch(csr_d, radius).cpu().numpy()
            assert capi.som_sparse_dense_filter_active(som.ctx) == on
            P.check_bmus_csr(oracle, csr, dim, W_in, b)
            seq.append(b)
        b = som.bmus(csr_d).cpu().numpy()                      # search only, on the final map
        P.check_bmus_csr(oracle, csr, dim, som.codebook.cpu().numpy(), b)
        out[on] = seq
        som.close()
    assert np.array_equal(out[True][0], out[False][0])         # same input code book: same BMUs, bit for bit


def test_dense_planes_are_declined_or_dropped(oracle):
    """Not used for long or nearly empty rows, nor with the fp32 filter; and a search over other data on the same
    context (which reuses the plane buffers) makes the next epoch on the registered set build them again."""
    from paper_1305_1422_amd import Som, capi
    rng = np.random.default_rng(83)
    rows, cols = 8, 9
    for n, dim, density, filt in [(300, 5000, 0.05, None), (300, 800, 0.01, None), (300, 800, 0.1, "fp32")]:
        csr = sparse_uniform_csr(n, dim, 84, density=density)
        W = rng.random((rows * cols, dim)).astype(np.float32)
        som = Som(rows, cols, dim, codebook=torch.from_numpy(W), filter=filt)
        csr_d = P.csr_to_dev(csr)
        capi.som_set_data_csr(som.ctx, *csr_d)
        b = som.bmus(csr_d).cpu().numpy()
        assert not capi.som_sparse_dense_filter_active(som.ctx)
        P.check_bmus_csr(oracle, csr, dim, W, b)
        som.close()
    n, dim = 900, 400
    csr = sparse_uniform_csr(n, dim, 85, density=0.08)
    other = rng.random((1300, dim)).astype(np.float32)          # more rows than the registered set: the scratch grows
    W = rng.random((rows * cols, dim)).astype(np.float32)
    som = Som(rows, cols, dim, codebook=torch.from_numpy(W))
    csr_d = P.csr_to_dev(csr)
    capi.som_set_data_csr(som.ctx, *csr_d)
    b1 = som.bmus(csr_d).cpu().numpy()
    assert capi.som_sparse_dense_filter_active(som.ctx)
    bo = som.bmus(P.to_dev(other)).cpu().numpy()
    P.check_bmus_dense(oracle, other, W, bo)
    b2 = som.bmus(csr_d).cpu().numpy()
    assert capi.som_sparse_dense_filter_active(som.ctx)
    assert np.array_equal(b1, b2)
    P.check_bmus_csr(oracle, csr, dim, W, b2)
    som.close()


def test_long_rows_with_hot_column_tables_whole_epochs(oracle):
    """Rows longer than an LDS tile of columns (17,000 > 16,384) on a context that holds the hot-column tables, with
    more than eight instances per node: the per-node sums go through the BMU-sorted chunks with the frequent
    columns in LDS.  Whole epochs against the oracle, registered and - same tables, other rows - unregistered data;
    one node takes half of the instances (many chunks), most nodes none."""
    from paper_1305_1422_amd import Som, capi
    n, dim, rows, cols = 1500, 17000, 5, 6
    csr = sparse_zipf_csr(n, dim, 91, mean_len=50.0, max_len=150)
    csr_d = P.csr_to_dev(csr)
    W0 = (np.random.default_rng(92).random((rows * cols, dim)) * 0.05).astype(np.float32)
    W0[7] += 0.02                                              # a node close to everything at the start
    som = Som(rows, cols, dim, "planar", "square", codebook=torch.from_numpy(W0))
    capi.som_set_data_csr(som.ctx, *csr_d)
    for radius in (2.0, 1.0, 0.6):
        P.epoch_parity_csr(oracle, som, csr, csr_d, dim, radius, P.MAP["planar"], P.GRID["square"])
    assert capi.som_sparse_hot_block_active(som.ctx)
    other = sparse_zipf_csr(900, dim, 93, mean_len=30.0, max_len=90)
    other_d = P.csr_to_dev(other)
    P.epoch_parity_csr(oracle, som, other, other_d, dim, 1.0, P.MAP["planar"], P.GRID["square"])
    som.close()


def _csr_with_row_lengths(lengths, dim, seed):
    rng = np.random.default_rng(seed)
    indptr = np.zeros(len(lengths) + 1, dtype=np.int64)
    np.cumsum(lengths, out=indptr[1:])
    indices = np.concatenate([np.sort(rng.choice(dim, size=m, replace=False)) for m in lengths]).astype(np.int32)
    values = (rng.random(indptr[-1]) + 0.1).astype(np.float32)
    return indptr, indices, values


@pytest.mark.parametrize("copies,rows,cols", [(400, 25, 30), (100, 40, 40), (700, 40, 40)])
def test_full_scan_of_instances_with_hundreds_of_near_copies(oracle, copies, rows, cols):
    """Hundreds of nodes that differ from one another by a few ulps: the candidate lists overflow (or, at 100
    copies on 1,600 nodes, are long enough for the scan of everything to be the cheaper way), and the exact scan of
    all nodes decides.  It reads a transposed copy of the code book; rows of 0, 1, 511, 512, 513 and 1,100
    nonzeros cross its staging buffer of 512, the 750 and 1,600 nodes leave its last round of 512 nodes ragged,
    and instance 6 coincides with three of the nodes (the others are its near-copies), which sends its scan back to
    the row-major code book for the plain sum."""
    from paper_1305_1422_amd import Som
    dim = 3000
    k = rows * cols
    lengths = [0, 1, 40, 511, 512, 513, 1100] * 6 + [60] * 30
    csr = _csr_with_row_lengths(lengths, dim, 7100 + copies)
    X = densify(csr, dim)
    rng = np.random.default_rng(7200 + copies)
    base = X[6]                                                              # a row of 1,100 nonzeros
    W = (rng.random((k, dim)) * 0.3 + 0.5).astype(np.float32)              # the other nodes: far from everything
    near = rng.choice(k, size=copies, replace=False)
    W[near] = base
    W[near] += (rng.integers(-2, 3, size=(copies, dim)) * np.float32(2.0 ** -24)).astype(np.float32)
    exact = np.sort(rng.choice(near, size=3, replace=False))
    W[exact] = base                                                          # instance 6 is these three nodes
    som = Som(rows, cols, dim, codebook=torch.from_numpy(W))
    b = som.bmus(P.csr_to_dev(csr)).cpu().numpy()
    refined, collected, rescanned = som.stats()
    som.close()
    assert rescanned >= 24, (refined, collected, rescanned)                 # the rows of 511 nonzeros and more, at least
    P.check_bmus_csr(oracle, csr, dim, W, b)
    assert b[6] == exact[0]                                                  # exact zero distance: no band, the lowest copy
