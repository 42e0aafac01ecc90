"""The rounding bound that the exact BMU stage relies on, checked where it is assumed.

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


def _score_bound_case(x, w, rows, cols):
    from paper_1305_1422_amd import Som, capi
    n, dim = x.shape
    k = rows * cols
    som = Som(rows, cols, dim, codebook=torch.from_numpy(w), filter="split_f16")
    xd = torch.from_numpy(x).cuda()
    scores = torch.empty((n, k), dtype=torch.float32, device="cuda")
    mu = torch.empty(dim, dtype=torch.float32, device="cuda")
    capi.som_debug_scores_dense(som.ctx, xd, som.codebook, scores, mu)
    torch.cuda.synchronize()
    s_gpu = scores.cpu().numpy().astype(np.float64)
    mu32 = mu.cpu().numpy()
    som.close()

    wc = (w - mu32[None, :]).astype(np.float32)                   # w' = fl(w - mu), one fp32 rounding
    assert wc.dtype == np.float32
    wc64, mu64, x64 = wc.astype(np.float64), mu32.astype(np.float64), x.astype(np.float64)
    c_i = (wc64 ** 2).sum(1) + 2.0 * wc64 @ mu64
    s_exact = c_i[None, :] - 2.0 * x64 @ wc64.T
    X = np.sqrt((x64 ** 2).sum(1))
    Wm = np.sqrt((wc64 ** 2).sum(1).max())
    M = np.sqrt((mu64 ** 2).sum())
    sx = _pow2_above(np.abs(x64).max(1))
    sw = float(_pow2_above(np.abs(wc64).max()))
    f = 4 if dim >= 256 else 2                                     # chunks of 32 features between two flushes
    g = 2.5 * 6 * f + 9 + np.ceil(dim / (32 * f)) + 2
    # the rounding of w - mu is part of the library's bound but not of this comparison (the exact
    # scores above start from the rounded w'), so the bound tested here is slightly larger than needed
    B = U * ((2 * g + 28) * X * Wm + np.sqrt(dim) * (sx * Wm + sw * X) + 4 * Wm ** 2 + 6 * M * Wm)
    err = np.abs(s_gpu - s_exact)
    ratio = (err / B[:, None]).max()
    assert ratio <= 1.0, f"filter score error exceeds the bound: {ratio:.3f} x"
    return ratio


@pytest.mark.parametrize("case", ["uniform", "offset_mixture", "heavy_tail", "tiny_and_huge_rows", "ragged_dim"])
def test_filter_scores_stay_within_the_bound(case):
    rng = np.random.default_rng(11)
    rows, cols = 12, 25                                            # 300 nodes: three node blocks, ragged
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
    else:
        dim = 1000                                                 # not a multiple of 32 chunks of 64: 16 flushes
        n = 300
        x = rng.uniform(-1, 1, (n, dim))
        w = rng.uniform(-1, 1, (rows * cols, dim))
    ratio = _score_bound_case(x.astype(np.float32), w.astype(np.float32), rows, cols)
    print(f"{case}: worst error / bound = {ratio:.4f}")
