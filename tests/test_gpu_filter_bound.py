"""The rounding bounds that the exact BMU stage relies on, checked where they are assumed: every score of
each of the filter passes (split-fp16 MFMA, fp32 MFMA in both of its kernels, the one-product coarse pass of the
two-level search, the 16-bit sparse sweep) is
dumped and compared with its exact value in float64; no error may exceed half the margin the exact stage
applies to that instance (the library reports the margin it uses: same device function, same inputs), and for
the two dense filters the documented closed form of the bound is evaluated here from the inputs alone as well.

Split-fp16 filter (it multiplies centred instances x' = fl(x - mu), so X below is |x'_j| and the term in M
falls away; the closed form evaluated in the test is the centred one, with coef = 2 g + 30):

The split-fp16 filter ranks nodes by scores whose distance from the exact value is bounded by
    B = u [ coef X Wm + sqrt(dim) (sx_j Wm + sw X) + 4 Wm^2 + 6 M Wm ],      u = 2^-24,
(X = |x_j|, Wm = max_i |w'_i|, M = |mu|, sx_j / sw = the powers of two the operands were divided
by, coef = 2 g + 28 with g = 2.5 * 6 f + 9 + ceil(dim / (32 f)) + 2, where f = 4 from 256 features on,
else 2), and that bound in turn prices one 32x32x16 fp16 matrix instruction at 9 u max|product| + 2.5 u (|C| + sum |products|).  Both
statements are tested here against float64 arithmetic: the instruction on random and on
adversarial operands (one dominant term, fifteen just below the truncation point), the scores
of the whole filter on several value distributions.  The expected values are computed in numpy
from the inputs alone.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

U = 2.0 ** -24


def _mfma(a, b, c):
    from paper_1305_1422_amd import capi
    d = torch.empty(c.shape, dtype=torch.float32, device="cuda")
    capi.som_debug_mfma_f16(torch.from_numpy(a).cuda(), torch.from_numpy(b).cuda(), torch.from_numpy(c).cuda(), d)
    torch.cuda.synchronize()
    return d.cpu().numpy()


def _check_mfma(a, b, c):
    got = _mfma(a, b, c).astype(np.float64)
    a64, b64 = a.astype(np.float64), b.astype(np.float64)
    prod = a64[:, :, None, :] * b64[:, None, :, :]                 # [t][row][col][k]
    exact = prod.sum(-1) + c.astype(np.float64)
    model = U * (9.0 * np.abs(prod).max(-1) + 2.5 * (np.abs(c.astype(np.float64)) + np.abs(prod).sum(-1)))
    err = np.abs(got - exact)
    assert np.all(err <= model), f"worst error / model = {(err / np.maximum(model, 1e-300)).max():.3f}"
    return float((err / np.maximum(model, 1e-300)).max())


def test_matrix_instruction_layout_and_rounding_random():
    rng = np.random.default_rng(5)
    count = 64
    for dist in range(3):
        u1, u2 = rng.uniform(-1, 1, (count, 32, 16)), rng.uniform(-1, 1, (count, 32, 16))
        if dist == 1:
            u1, u2 = np.abs(u1), np.abs(u2)
        if dist == 2:
            u1, u2 = 8 * u1 ** 3, 8 * u2 ** 3
        a, b = u1.astype(np.float16), u2.astype(np.float16)
        for cscale in (0.0, 1.0, 300.0):
            c = (cscale * rng.uniform(-1, 1, (count, 32, 32))).astype(np.float32)
            _check_mfma(a, b, c)


def test_matrix_instruction_rounding_adversarial():
    """One dominant term (a product, or the accumulator) and small products of every size from
    2^-20 to 2^-30 of it with several mantissas and sign patterns."""
    mant = np.array([1.0, 1.125, 1.25, 1.5, 1.75, 1.875, 2047 / 1024, 1025 / 1024])
    worst = 0.0
    for dominant_in_c in (False, True):
        for big in (1.0, 2047 / 1024):
            es = list(range(-20, -31, -1))
            a = np.zeros((len(es), 32, 16), np.float16)
            b = np.zeros((len(es), 32, 16), np.float16)
            c = np.zeros((len(es), 32, 32), np.float32)
            for t, e in enumerate(es):
                ea = e // 2
                eb = e - ea
                b[t, :, :] = np.float16(2.0 ** eb)
                for r in range(32):
                    s = -1.0 if (r >> 3) & 1 else 1.0
                    signs = np.where((np.arange(16) & 1) & ((r >> 4) & 1), -s, s)
                    a[t, r, :] = (signs * mant[r & 7] * 2.0 ** ea).astype(np.float16)
                if dominant_in_c:
                    c[t, :, :] = big
                else:
                    a[t, :, 0] = np.float16(big)
                    b[t, :, 0] = np.float16(1.0)
            worst = max(worst, _check_mfma(a, b, c))
    assert worst > 0.2       # the patterns do reach into the model's range: the test is not vacuous


def _pow2_above(m):
    m = np.asarray(m, np.float64)
    e = np.where(m > 0, np.floor(np.log2(np.maximum(m, 1e-300))) + 1, 0)
    return 2.0 ** e


def _score_bound_case(x, w, rows, cols, filter="split_f16"):
    from paper_1305_1422_amd import Som, capi
    n, dim = x.shape
    k = rows * cols
    som = Som(rows, cols, dim, codebook=torch.from_numpy(w), filter=filter)
    xd = torch.from_numpy(x).cuda()
    scores = torch.empty((n, k), dtype=torch.float32, device="cuda")
    mu = torch.empty(dim, dtype=torch.float32, device="cuda")
    margin = torch.empty(n, dtype=torch.float64, device="cuda")
    capi.som_debug_scores_dense(som.ctx, xd, som.codebook, scores, mu, margin)
    torch.cuda.synchronize()
    s_gpu = scores.cpu().numpy().astype(np.float64)
    mu32 = mu.cpu().numpy()
    margin = margin.cpu().numpy()
    som.close()

    wc = (w - mu32[None, :]).astype(np.float32)                   # w' = fl(w - mu), one fp32 rounding
    assert wc.dtype == np.float32
    wc64, mu64, x64 = wc.astype(np.float64), mu32.astype(np.float64), x.astype(np.float64)
    c_i = (wc64 ** 2).sum(1) + 2.0 * wc64 @ mu64
    s_exact = c_i[None, :] - 2.0 * x64 @ wc64.T
    X = np.sqrt((x64 ** 2).sum(1))
    Wm = np.sqrt((wc64 ** 2).sum(1).max())
    M = np.sqrt((mu64 ** 2).sum())
    # the rounding of w - mu is part of the library's bound but not of this comparison (the exact
    # scores above start from the rounded w'), so the bound tested here is slightly larger than needed
    if filter in ("split_f16", "two_level"):
        # this filter multiplies centred instances x' = fl(x - mu): their norms and scales enter the bound,
        # |mu| does not (what the rounding of x - mu adds for all nodes alike cancels in every comparison)
        xc64 = (x - mu32[None, :]).astype(np.float32).astype(np.float64)
        Xc = np.sqrt((xc64 ** 2).sum(1))
        sx = _pow2_above(np.abs(xc64).max(1))
        sw = float(_pow2_above(np.abs(wc64).max()))
        f = 4 if dim >= 256 else 2                                 # chunks of 32 features between two flushes
        g = 2.5 * 6 * f + 9 + np.ceil(dim / (32 * f)) + 2
        # two_level: the scores of its coarse pass, one product of operands rounded to 11 bits
        # (2 (2^14 + 8) u X Wm for the roundings of the two rows, doubled by the factor -2)
        split = 30 if filter == "split_f16" else 2 * (16384 + 8) + 6
        if filter == "two_level":
            g = 2.5 * np.ceil(dim / 16) + 9 + 2                    # one unflushed chain of ceil(dim / 16) instructions
        B = U * ((2 * g + split) * Xc * Wm + np.sqrt(dim) * (sx * Wm + sw * Xc) + 4 * Wm ** 2)
        # the constant 2 delta.x' that the rounding delta of x - mu adds to every score of an instance is no
        # error of the ranking: compare after removing each instance's mean difference
        s_exact = s_exact + np.mean(s_gpu - s_exact, axis=1, keepdims=True)
    else:
        g = 32 + np.ceil(dim / 32) + 2                             # accumulator flushed every 32 features
        B = U * ((2 * g + 4) * X * Wm + 4 * Wm ** 2 + 6 * M * Wm)
    err = np.abs(s_gpu - s_exact)
    ratio = (err / B[:, None]).max()
    assert ratio <= 1.0, f"filter score error exceeds the bound: {ratio:.3f} x"
    # what the exact stage really uses: two scores of an instance are told apart by `margin`, so each may
    # be off by half of it; and the margin is the documented 2.125 B (never less)
    assert np.all(err <= 0.5 * margin[:, None]), f"score error above half the margin: {(err / margin[:, None]).max():.3f}"
    assert np.all(margin >= 2.125 * B * (1 - 1e-6))
    return ratio


def _dense_case(case, rng, rows, cols):
    n, dim = 700, 200
    if case == "uniform":
        x = rng.uniform(0, 1, (n, dim))
        w = rng.uniform(0, 1, (rows * cols, dim))
    elif case == "offset_mixture":
        means = rng.uniform(0, 1, (8, dim)) + 50.0
        x = means[rng.integers(8, size=n)] + 0.05 * rng.standard_normal((n, dim))
        w = means[rng.integers(8, size=rows * cols)] + 0.01 * rng.standard_normal((rows * cols, dim))
    elif case == "heavy_tail":
        x = rng.standard_cauchy((n, dim)).clip(-1e4, 1e4)
        w = rng.standard_cauchy((rows * cols, dim)).clip(-1e3, 1e3)
    elif case == "tiny_and_huge_rows":
        x = rng.standard_normal((n, dim)) * (10.0 ** rng.integers(-12, 6, size=(n, 1)))
        w = rng.standard_normal((rows * cols, dim)) * (10.0 ** rng.integers(-3, 2, size=(rows * cols, 1)))
    elif case == "ragged_dim":
        dim = 1000                                                 # not a multiple of 32 chunks of 64: 16 flushes
        n = 300
        x = rng.uniform(-1, 1, (n, dim))
        w = rng.uniform(-1, 1, (rows * cols, dim))
    else:                                                          # "odd_dim": the register-staged fp32 kernel
        dim = 333
        n = 300
        x = rng.uniform(-1, 1, (n, dim)) + 3.0
        w = rng.uniform(-1, 1, (rows * cols, dim)) + 3.0
    return x.astype(np.float32), w.astype(np.float32)


@pytest.mark.parametrize("filter", ["split_f16", "fp32", "two_level"])
@pytest.mark.parametrize("case", ["uniform", "offset_mixture", "heavy_tail", "tiny_and_huge_rows", "ragged_dim",
                                  "odd_dim"])
def test_filter_scores_stay_within_the_bound(case, filter):
    rng = np.random.default_rng(11)
    rows, cols = 12, 25                                            # 300 nodes: three node blocks, ragged
    x, w = _dense_case(case, rng, rows, cols)
    ratio = _score_bound_case(x, w, rows, cols, filter)
    print(f"{filter} {case}: worst error / bound = {ratio:.4f}")


# ---------------------------------------------------------------- sparse sweep
def _csr_rows(rng, n, dim, lengths, value_kind):
    indptr = np.zeros(n + 1, np.int64)
    np.cumsum(lengths, out=indptr[1:])
    indices = np.concatenate([np.sort(rng.choice(dim, size=int(l), replace=False)) for l in lengths] or
                             [np.zeros(0)]).astype(np.int32)
    nnz = int(indptr[-1])
    if value_kind == "tf":
        values = np.log(2.0 + rng.poisson(2.0, nnz))
    elif value_kind == "signed_wide":
        values = rng.standard_normal(nnz) * 10.0 ** rng.integers(-4, 4, nnz)
    else:
        values = rng.uniform(0.5, 1.5, nnz)
    return indptr, indices, values.astype(np.float32)


@pytest.mark.parametrize("case", ["text_like", "heavy_tailed_columns", "one_huge_column", "constant_columns",
                                  "short_and_long_rows", "signed_wide_values"])
def test_sparse_sweep_scores_stay_within_the_margin(case):
    """Scores of the sparse sweep (code book quantised to 16 bits per column step, values times step, one FMA
    chain per row) against float64: the margin carries 0.51 sum |v_c| step_c for the quantisation plus the fp32
    chain; the error of every score must stay below half of it."""
    from paper_1305_1422_amd import Som, capi
    rng = np.random.default_rng(23)
    rows, cols, dim, n = 20, 35, 3000, 260                         # 700 nodes: eight slices, the last ragged
    k = rows * cols
    w = rng.uniform(0, 1, (k, dim))
    lengths = np.clip(rng.poisson(60, n), 1, 400)
    kind = "tf"
    if case == "heavy_tailed_columns":
        w = w * 10.0 ** rng.uniform(-3, 3, (1, dim))               # column scales over six decades
        w[rng.integers(k, size=40), rng.integers(dim, size=40)] *= 50.0      # and single outliers that set a step
    elif case == "one_huge_column":
        w[:, 7] = rng.standard_normal(k) * 1e6
        lengths[:] = 30
    elif case == "constant_columns":
        w[:, ::3] = 0.25                                           # centred to exactly 0: step falls back to 1
        w[:, 1::3] = rng.uniform(0, 1, (1, len(range(1, dim, 3)))) # constant per column, different values
    elif case == "short_and_long_rows":
        lengths = np.where(np.arange(n) % 3 == 0, 1, np.where(np.arange(n) % 3 == 1, 400, 0))
    elif case == "signed_wide_values":
        kind = "signed_wide"
        w = w - 0.5
    w = w.astype(np.float32)
    csr = _csr_rows(rng, n, dim, lengths, kind)
    if case == "one_huge_column":                                  # every row lists the huge column
        for j in range(n):
            row = csr[1][csr[0][j]:csr[0][j + 1]]
            if 7 not in row:
                row[0] = 7 if row[0] > 7 or row.size == 1 else row[0]
        # keep rows sorted and unique after the edit
        for j in range(n):
            seg = slice(csr[0][j], csr[0][j + 1])
            assert np.all(np.diff(csr[1][seg]) > 0)
    som = Som(rows, cols, dim, codebook=torch.from_numpy(w))
    dev = tuple(torch.from_numpy(a).cuda() for a in csr)
    scores = torch.empty((n, k), dtype=torch.float32, device="cuda")
    mu = torch.empty(dim, dtype=torch.float32, device="cuda")
    margin = torch.empty(n, dtype=torch.float64, device="cuda")
    capi.som_debug_scores_csr(som.ctx, dev[0], dev[1], dev[2], som.codebook, scores, mu, margin)
    torch.cuda.synchronize()
    s_gpu = scores.cpu().numpy().astype(np.float64)
    mu32 = mu.cpu().numpy()
    margin = margin.cpu().numpy()
    som.close()
    wc64 = (w - mu32[None, :]).astype(np.float32).astype(np.float64)
    c_i = (wc64 ** 2).sum(1) + 2.0 * wc64 @ mu32.astype(np.float64)
    worst = 0.0
    for j in range(n):
        seg = slice(csr[0][j], csr[0][j + 1])
        dot = wc64[:, csr[1][seg]] @ csr[2][seg].astype(np.float64)
        err = np.abs(s_gpu[j] - (c_i - 2.0 * dot))
        assert np.all(err <= 0.5 * margin[j]), (f"row {j} (length {seg.stop - seg.start}): score error "
                                                f"{err.max():.3e} above half the margin {margin[j]:.3e}")
        worst = max(worst, float(err.max() / (margin[j] / 2.125)))
    print(f"{case}: worst error / bound = {worst:.4f}")
    assert worst > 1e-4                                            # the comparison is not vacuous


def test_consecutive_workgroups_go_round_the_eight_xcds():
    """What the launch geometry of the dense filter and of the sparse sweep assumes of the dispatcher (it affects
    their L2 hit rates, not their results): workgroup b of a launch runs on the same XCD as workgroup b + 8, and
    eight consecutive workgroups are on eight different XCDs."""
    from paper_1305_1422_amd import capi
    out = torch.full((1024,), -1, dtype=torch.int32, device="cuda")
    capi.som_debug_xcc_ids(out)
    torch.cuda.synchronize()
    ids = out.cpu().numpy()
    assert ids.min() >= 0 and len(set(ids[:8].tolist())) == 8, f"first eight workgroups on XCDs {ids[:8]}"
    assert np.array_equal(ids, np.tile(ids[:8], 128)), "workgroups 8 apart do not share an XCD"
