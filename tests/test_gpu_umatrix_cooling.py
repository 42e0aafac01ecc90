"""U-matrix and cooling schedule of the HIP library against the CPU oracle (gpu tests)."""
import numpy as np
import pytest

from tests import parity as P

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.mark.parametrize("map_type", ["planar", "toroid"])
@pytest.mark.parametrize("grid", ["square", "hexagonal"])
@pytest.mark.parametrize("rows,cols,dim", [(7, 9, 33), (6, 4, 128), (1, 1, 3), (1, 2, 5), (2, 2, 4), (3, 1, 2), (2, 5, 70)])
def test_umatrix(oracle, map_type, grid, rows, cols, dim):
    from paper_1305_1422_amd import Som
    W = np.random.default_rng(rows * 100 + cols).normal(size=(rows * cols, dim)).astype(np.float32)
    som = Som(rows, cols, dim, map_type, grid, codebook=torch.from_numpy(W))
    got = som.umatrix().cpu().numpy()
    want = oracle.umatrix(W, rows, cols, P.MAP[map_type], P.GRID[grid])
    np.testing.assert_allclose(got, want, rtol=1e-6, atol=1e-7)
    som.close()


@pytest.mark.parametrize("cooling", ["linear", "exponential"])
@pytest.mark.parametrize("E,r0,rN,s0,sN", [(10, 10.0, 1.0, 0.1, 0.01), (5, 100.0, 1.0, 1.0, 0.01), (1, 25.0, 1.0, 1.0, 0.01),
                                           (7, 3.5, 0.25, 0.9, 0.3)])
def test_cooling_schedule(oracle, cooling, E, r0, rN, s0, sN):
    from paper_1305_1422_amd import Som
    som = Som(4, 4, 2, seed=3)
    r, s = som.cool_schedule(E, r0, rN, s0, sN, cooling)
    kind = oracle.COOLING[cooling]
    f = lambda v: float(np.float32(v))                    # the ABI carries the end points as fp32
    want_r = [oracle.cool(f(r0), f(rN), E, e, kind) for e in range(E)]
    want_s = [oracle.cool(f(s0), f(sN), E, e, kind) for e in range(E)]
    np.testing.assert_allclose(r.cpu().numpy(), want_r, rtol=1e-13)
    np.testing.assert_allclose(s.cpu().numpy(), want_s, rtol=1e-13)
    som.close()


def test_cooling_defaults_follow_the_papers_command_line(oracle):
    """Defaults in tests/golden/cli_defaults.txt: start radius = half the smaller map side,
    final radius 1, learning rate 1.0 -> 0.01, linear."""
    from paper_1305_1422_amd import Som
    som = Som(30, 50, 2, seed=3)
    r, s = som.cool_schedule(4)
    np.testing.assert_allclose(r.cpu().numpy(), [15.0, 15.0 - 14.0 / 3, 15.0 - 28.0 / 3, 1.0], rtol=1e-13)
    np.testing.assert_allclose(s.cpu().numpy()[[0, -1]], [1.0, float(np.float32(0.01))], rtol=1e-13)
    som.close()


@pytest.mark.parametrize("radius_kind,scale_kind", [("linear", "exponential"), ("exponential", "linear"),
                                                    ("exponential", None)])
def test_radius_and_learning_rate_cool_by_their_own_kinds(oracle, radius_kind, scale_kind):
    """Options -t and -T of the command line are separate: the radius may cool linearly while the
    learning rate cools exponentially, and the other way round."""
    from paper_1305_1422_amd import Som
    E, r0, rN, s0, sN = 9, 20.0, 2.0, 0.5, 0.0625
    som = Som(4, 4, 2, seed=3)
    som.set_scale_cooling(scale_kind)
    r, s = som.cool_schedule(E, r0, rN, s0, sN, radius_kind)
    want_r = [oracle.cool(r0, rN, E, e, oracle.COOLING[radius_kind]) for e in range(E)]
    want_s = [oracle.cool(s0, sN, E, e, oracle.COOLING[scale_kind or radius_kind]) for e in range(E)]
    np.testing.assert_allclose(r.cpu().numpy(), want_r, rtol=1e-13)
    np.testing.assert_allclose(s.cpu().numpy(), want_s, rtol=1e-13)
    som.close()
