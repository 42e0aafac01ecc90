"""Post-training and interim outputs of the HIP path against the CPU oracle (gpu tests, through
the C ABI): distances to the BMUs with their mean, and the per-epoch snapshots of option -s."""
import numpy as np
import pytest

from gen import sparse_zipf_csr
from tests import parity as P

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

DIST_RTOL = 2e-7       # fp64 sums rounded once to fp32 (2^-24) plus the order of the fp64 additions
QE_RTOL = 1e-12        # fp64 throughout; only the order of the additions differs


@pytest.mark.parametrize("n,dim,rows,cols", [(1000, 77, 12, 11), (5000, 300, 7, 9), (3, 5, 2, 2), (4097, 64, 20, 20)])
def test_distances_dense(oracle, n, dim, rows, cols):
    from paper_1305_1422_amd import Som
    rng = np.random.default_rng(n + dim)
    X = rng.standard_normal((n, dim)).astype(np.float32)
    W = rng.standard_normal((rows * cols, dim)).astype(np.float32)
    som = Som(rows, cols, dim, codebook=torch.from_numpy(W))
    Xd = P.to_dev(X)
    b = som.bmus(Xd)
    dist, qe = som.bmu_distances(Xd, b)
    want, want_qe = oracle.bmu_distances_dense(X, W, b.cpu().numpy())
    np.testing.assert_allclose(dist.cpu().numpy(), want, rtol=DIST_RTOL)
    np.testing.assert_allclose(qe.item(), want_qe, rtol=QE_RTOL)
    # any assignment, not only the best one
    other = rng.integers(0, rows * cols, n).astype(np.int32)
    dist, qe = som.bmu_distances(Xd, P.to_dev(other))
    want, want_qe = oracle.bmu_distances_dense(X, W, other)
    np.testing.assert_allclose(dist.cpu().numpy(), want, rtol=DIST_RTOL)
    np.testing.assert_allclose(qe.item(), want_qe, rtol=QE_RTOL)
    som.close()


@pytest.mark.parametrize("n,dim,rows,cols,mean_len", [(700, 900, 9, 8, 30.0), (2500, 3000, 12, 10, 100.0)])
def test_distances_csr(oracle, n, dim, rows, cols, mean_len):
    from paper_1305_1422_amd import Som
    csr = sparse_zipf_csr(n, dim, 51, mean_len=mean_len, max_len=int(4 * mean_len))
    W = (np.random.default_rng(52).random((rows * cols, dim)) * 0.1).astype(np.float32)
    som = Som(rows, cols, dim, codebook=torch.from_numpy(W))
    csr_d = P.csr_to_dev(csr)
    b = som.bmus(csr_d)
    dist, qe = som.bmu_distances(csr_d, b)
    want, want_qe = oracle.bmu_distances_csr(csr, dim, W, b.cpu().numpy())
    # the library regroups the sparse sum only where its rounding is below 1.2e-7 of the result
    np.testing.assert_allclose(dist.cpu().numpy(), want, rtol=DIST_RTOL, atol=1e-9)
    np.testing.assert_allclose(qe.item(), want_qe, rtol=1e-10)
    som.close()


def test_instances_on_nodes_empty_rows_and_bad_indices(oracle):
    from paper_1305_1422_amd import Som
    rng = np.random.default_rng(53)
    W = rng.standard_normal((16, 40)).astype(np.float32)
    som = Som(4, 4, 40, codebook=torch.from_numpy(W))
    order = rng.integers(0, 16, 100).astype(np.int32)
    dist, qe = som.bmu_distances(P.to_dev(W[order]), P.to_dev(order))
    assert float(dist.abs().max()) == 0.0 and qe.item() == 0.0
    # a node index out of range: NaN for that instance and for the mean, the others unaffected
    bad = order.copy()
    bad[7] = 16
    bad[8] = -1
    dist, qe = som.bmu_distances(P.to_dev(W[order]), P.to_dev(bad))
    d = dist.cpu().numpy()
    assert np.isnan(d[7]) and np.isnan(d[8]) and np.isnan(qe.item())
    assert np.all(np.delete(d, [7, 8]) == 0.0)
    # sparse: an empty row lies at |w| from its node
    indptr = np.array([0, 0, 2], dtype=np.int64)
    csr = (indptr, np.array([3, 9], dtype=np.int32), np.array([1.0, -2.0], dtype=np.float32))
    b = np.array([5, 2], dtype=np.int32)
    dist, qe = som.bmu_distances(P.csr_to_dev(csr), P.to_dev(b))
    want, want_qe = oracle.bmu_distances_csr(csr, 40, W, b)
    np.testing.assert_allclose(dist.cpu().numpy(), want, rtol=DIST_RTOL)
    np.testing.assert_allclose(dist.cpu().numpy()[0], np.sqrt((W[5].astype(np.float64) ** 2).sum()), rtol=DIST_RTOL)
    np.testing.assert_allclose(qe.item(), want_qe, rtol=QE_RTOL)
    som.close()


def test_distances_need_an_output():
    from paper_1305_1422_amd import Som, capi
    som = Som(3, 3, 4, seed=1)
    X = torch.zeros((5, 4), dtype=torch.float32, device="cuda:0")
    b = torch.zeros(5, dtype=torch.int32, device="cuda:0")
    with pytest.raises(capi.SomError):
        capi.som_bmu_distances_dense(som.ctx, X, som.codebook, b, None, None)
    som.close()


@pytest.mark.parametrize("kind", ["dense", "csr"])
def test_snapshots_every_epoch(oracle, kind):
    """Option -s 2: after every epoch the U-matrix, the code book and the BMUs that epoch found.  Each epoch
    is checked against the oracle from the snapshot before it; on dense data -s 1 gives the same U-matrices
    and the same final state bit for bit, and -s 0 is som_train."""
    from paper_1305_1422_amd import Som
    rows, cols, E, r0, rN = 9, 7, 4, 4.0, 1.0            # radii 4, 3, 2, 1: exact in fp32
    if kind == "dense":
        n, dim = 900, 48
        X = np.random.default_rng(54).random((n, dim)).astype(np.float32)
        Xd = P.to_dev(X)
    else:
        n, dim = 600, 500
        X = sparse_zipf_csr(n, dim, 55, mean_len=20.0, max_len=60)
        Xd = P.csr_to_dev(X)
    W0 = np.random.default_rng(56).random((rows * cols, dim)).astype(np.float32)
    a = Som(rows, cols, dim, "toroid", "hexagonal", codebook=torch.from_numpy(W0))
    bmus, um, cbs, ball = a.train_snapshots(Xd, E, 2, r0, rN, 1.0, 0.01, "linear")
    torch.cuda.synchronize()
    cbs_h, ball_h, um_h = cbs.cpu().numpy(), ball.cpu().numpy(), um.cpu().numpy()
    mt, gt = P.MAP["toroid"], P.GRID["hexagonal"]
    W_in = W0
    for e in range(E):
        radius = oracle.cool(r0, rN, E, e, oracle.LINEAR)
        if kind == "dense":
            P.check_bmus_dense(oracle, X, W_in, ball_h[e])
            S, C = oracle.accumulate_dense(X, ball_h[e], rows * cols)
        else:
            P.check_bmus_csr(oracle, X, dim, W_in, ball_h[e])
            S, C = oracle.accumulate_csr(X, dim, ball_h[e], rows * cols)
        P.check_codebook(oracle, S, C, W_in, cbs_h[e], rows, cols, mt, gt, radius)
        np.testing.assert_allclose(um_h[e], oracle.umatrix(cbs_h[e], rows, cols, mt, gt), rtol=1e-6, atol=1e-7)
        W_in = cbs_h[e]
    assert np.array_equal(cbs_h[-1], a.codebook.cpu().numpy())
    assert np.array_equal(ball_h[-1], bmus.cpu().numpy())

    if kind == "csr":
        # the sparse per-node sums use floating-point atomics: two runs agree to rounding only, and this
        # small map is nearly collapsed after its first epoch, so the runs drift apart afterwards
        a.close()
        return
    b = Som(rows, cols, dim, "toroid", "hexagonal", codebook=torch.from_numpy(W0))
    bmus1, um1 = b.train_snapshots(Xd, E, 1, r0, rN, 1.0, 0.01, "linear")
    assert torch.equal(um1, um) and torch.equal(bmus1, bmus) and torch.equal(b.codebook, a.codebook)
    c = Som(rows, cols, dim, "toroid", "hexagonal", codebook=torch.from_numpy(W0))
    bmus0 = c.train(Xd, E, r0, rN, 1.0, 0.01, "linear")
    assert torch.equal(bmus0, bmus) and torch.equal(c.codebook, a.codebook)
    a.close(); b.close(); c.close()


def test_snapshot_arguments_are_checked():
    from paper_1305_1422_amd import Som, capi
    som = Som(3, 3, 4, seed=1)
    X = torch.rand((20, 4), dtype=torch.float32, device="cuda:0")
    capi.som_set_data_dense(som.ctx, X)
    b = torch.zeros(20, dtype=torch.int32, device="cuda:0")
    um = torch.zeros((2, 3, 3), dtype=torch.float32, device="cuda:0")
    for snapshots, args in ((3, (um, None, None)), (-1, (um, None, None)), (1, (None, None, None)),
                            (2, (um, None, None))):
        with pytest.raises(capi.SomError):
            capi.som_train_snapshots(som.ctx, 2, 1.5, 1.0, 1.0, 0.01, 0, som.codebook, b, snapshots, *args)
    som.close()
