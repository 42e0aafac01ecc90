"""The entry point that allocates nothing (som_bmu_distances_dense_static) against the entry point it
is a variant of (som_bmu_distances_dense), through the C ABI: same kernels, so the same bits.  Two calls
in a row on the library's static scratch, the second with a smaller input, then a wrong-size call."""
import numpy as np
import pytest

from tests import parity as P

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _both(som, capi, X, W, b):
    n = X.shape[0]
    d_ctx = torch.empty(n, dtype=torch.float32, device="cuda:0")
    q_ctx = torch.empty(1, dtype=torch.float64, device="cuda:0")
    capi.som_bmu_distances_dense(som.ctx, X, W, b, d_ctx, q_ctx)
    d_st = torch.full((n,), -1.0, dtype=torch.float32, device="cuda:0")
    q_st = torch.full((1,), -1.0, dtype=torch.float64, device="cuda:0")
    capi.som_bmu_distances_dense_static(X, W, b, d_st, q_st, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    return d_ctx.cpu().numpy(), q_ctx.item(), d_st.cpu().numpy(), q_st.item()


def test_static_scratch_variant_matches_the_context_variant(oracle):
    from paper_1305_1422_amd import Som, capi
    rng = np.random.default_rng(1234)
    rows, cols, dim = 9, 11, 77
    W = rng.standard_normal((rows * cols, dim)).astype(np.float32)
    som = Som(rows, cols, dim, codebook=torch.from_numpy(W))
    Wd = som.codebook
    for n in (9000, 37):                     # 1,024 partial sums, then 10: stale ones must not be read
        X = rng.standard_normal((n, dim)).astype(np.float32)
        b = rng.integers(0, rows * cols, n).astype(np.int32)
        d_ctx, q_ctx, d_st, q_st = _both(som, capi, P.to_dev(X), Wd, P.to_dev(b))
        assert np.array_equal(d_ctx, d_st) and q_ctx == q_st
        want, want_q = oracle.bmu_distances_dense(X, W, b)
        np.testing.assert_allclose(d_st, want, rtol=2e-7, atol=0)
        np.testing.assert_allclose(q_st, want_q, rtol=1e-12)
    som.close()


def test_static_scratch_variant_rejects_bad_sizes():
    from paper_1305_1422_amd import capi
    L = capi.load()
    x = torch.zeros(4, 3, dtype=torch.float32, device="cuda:0")
    w = torch.zeros(2, 3, dtype=torch.float32, device="cuda:0")
    b = torch.zeros(4, dtype=torch.int32, device="cuda:0")
    q = torch.zeros(1, dtype=torch.float64, device="cuda:0")
    for n, dim, k in ((0, 3, 2), (1 << 31, 3, 2), (4, 0, 2), (4, 3, 0), (4, 3, (1 << 24) + 1)):
        rc = L.som_bmu_distances_dense_static(x.data_ptr(), n, dim, w.data_ptr(), k, b.data_ptr(), None,
                                              q.data_ptr(), None)
        assert rc == capi.SOM_ERR_INVALID_ARG and L.som_last_error(None)
    assert L.som_bmu_distances_dense_static(x.data_ptr(), 4, 3, w.data_ptr(), 2, b.data_ptr(), None, None,
                                            None) == capi.SOM_ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert q.item() == 0.0                   # nothing was enqueued
    # and a valid call with the distances only (no mean): 3-4-5 triangles
    x[:, 0] = 3.0
    w[1, 1] = 4.0
    b[:] = 1
    d = torch.zeros(4, dtype=torch.float32, device="cuda:0")
    capi.som_bmu_distances_dense_static(x, w, b, d, None)
    torch.cuda.synchronize()
    assert d.cpu().tolist() == [5.0] * 4
