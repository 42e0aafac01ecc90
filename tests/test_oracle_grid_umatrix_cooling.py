"""Pins of the oracle's grid geometry (options -g, -m), U-matrix (U-matrix equation)
and cooling schedules (options -t/-T, -r/-R, -l/-L; defaults in tests/golden/cli_defaults.txt).
"""
import math

import numpy as np
import pytest

P, T, SQ, HX = 0, 1, 0, 1
LIN, EXP = 0, 1


def q_from(oracle, rows, cols, m, g, b):
    return np.array([oracle.grid_q(rows, cols, m, g, i, b) for i in range(rows * cols)])


def test_hexagonal_interior_node_has_six_unit_neighbours(oracle):
    rows, cols = 7, 7
    for b in (3 * cols + 3, 2 * cols + 3):            # odd row, even row
        q = q_from(oracle, rows, cols, P, HX, b)
        assert np.sum(q == 4) == 6                     # distance exactly 1
        assert np.sum((q > 0) & (q < 4)) == 0
        assert np.sum(q == 12) == 6                    # next ring: distance sqrt(3)


def test_square_interior_node_has_four_and_four(oracle):
    q = q_from(oracle, 5, 5, P, SQ, 12)
    assert np.sum(q == 4) == 4 and np.sum(q == 8) == 4 and np.sum(q == 0) == 1


def test_hexagonal_neighbour_lists_by_row_parity(oracle):
    rows, cols = 6, 6
    def nb(b):
        return sorted(np.nonzero(q_from(oracle, rows, cols, P, HX, b) == 4)[0].tolist())
    x, y = 2, 2                                        # even row: diagonal neighbours at x-1 and x
    assert nb(y * cols + x) == sorted([y * cols + x - 1, y * cols + x + 1, (y - 1) * cols + x - 1,
                                       (y - 1) * cols + x, (y + 1) * cols + x - 1, (y + 1) * cols + x])
    y = 3                                              # odd row: diagonal neighbours at x and x+1
    assert nb(y * cols + x) == sorted([y * cols + x - 1, y * cols + x + 1, (y - 1) * cols + x,
                                       (y - 1) * cols + x + 1, (y + 1) * cols + x, (y + 1) * cols + x + 1])


@pytest.mark.parametrize("g,rows,cols", [(SQ, 5, 7), (HX, 6, 5)])
def test_torus_distance_is_translation_invariant_and_bounded(oracle, g, rows, cols):
    k = rows * cols
    y, x = np.divmod(np.arange(k), cols)
    base = np.array([[oracle.grid_q(rows, cols, T, g, i, b) for b in range(k)] for i in range(k)])
    assert np.array_equal(base, base.T)
    for dy, dx in [(2, 1), (4, 3)]:
        tau = ((y + dy) % rows) * cols + (x + dx) % cols
        assert np.array_equal(base[np.ix_(tau, tau)], base)
    planar = np.array([[oracle.grid_q(rows, cols, P, g, i, b) for b in range(k)] for i in range(k)])
    assert np.all(base <= planar)
    a_max, m_max = rows // 2, cols                     # half the torus in each direction
    assert base.max() <= m_max * m_max + (3 if g == HX else 4) * a_max * a_max


def test_torus_wraps_to_the_short_way_round(oracle):
    assert oracle.grid_q(1, 10, T, SQ, 0, 9) == 4      # one step across the seam
    assert oracle.grid_q(1, 10, P, SQ, 0, 9) == 4 * 81
    assert oracle.grid_q(10, 1, T, SQ, 0, 7) == 4 * 9
    assert oracle.grid_q(4, 4, T, HX, 0, 3 * 4 + 3) == 4       # (0,0) and (3,3): up-left neighbour through both seams


def test_neighbourhood_value(oracle):
    h = oracle.neighbourhood(3, 9, P, SQ, 0, 2 * 9 + 3, 2.5)   # dx = 3, dy = 2: d^2 = 13
    assert h == pytest.approx(math.exp(-13.0 / (2 * 2.5 * 2.5)), rel=1e-15)


# ------------------------------------------------------------------ U-matrix

@pytest.mark.parametrize("m,g", [(P, SQ), (T, SQ), (P, HX), (T, HX)])
def test_umatrix_of_constant_codebook_is_zero(oracle, m, g):
    W = np.full((4 * 6, 5), 0.37, dtype=np.float32)
    assert np.all(oracle.umatrix(W, 4, 6, m, g) == 0.0)


def test_umatrix_ramp_planar_square(oracle):
    rows, cols, a = 5, 6, 0.75
    x = np.tile(np.arange(cols), rows)
    W = np.zeros((rows * cols, 3), np.float32)
    W[:, 1] = a * x
    U = oracle.umatrix(W, rows, cols, P, SQ)
    np.testing.assert_allclose(U[1:-1, 1:-1], a / 2)          # two of four neighbours differ by a
    np.testing.assert_allclose(U[1:-1, 0], a / 3)
    np.testing.assert_allclose(U[1:-1, -1], a / 3)
    np.testing.assert_allclose(U[0, 1:-1], 2 * a / 3)
    np.testing.assert_allclose(U[-1, 1:-1], 2 * a / 3)
    np.testing.assert_allclose(U[[0, 0, -1, -1], [0, -1, 0, -1]], a / 2)


def test_umatrix_ramp_planar_hexagonal_interior(oracle):
    rows, cols, a = 6, 6, 2.0
    y, x = np.divmod(np.arange(rows * cols), cols)
    W = np.zeros((rows * cols, 2), np.float32)
    W[:, 0] = a * (x + 0.5 * (y % 2))                 # ramp in the embedded x coordinate
    U = oracle.umatrix(W, rows, cols, P, HX)
    np.testing.assert_allclose(U[1:-1, 1:-1], (2 * a + 4 * a / 2) / 6, rtol=1e-12)
    W[:, 0] = a * x                                    # ramp in the column index
    U = oracle.umatrix(W, rows, cols, P, HX)
    np.testing.assert_allclose(U[1:-1, 1:-1], 4 * a / 6, rtol=1e-12)


def test_umatrix_toroid_square_wraps(oracle):
    rows, cols = 4, 5
    W = np.zeros((rows * cols, 1), np.float32)
    W[0, 0] = 1.0                                      # a single spike at node (0, 0)
    U = oracle.umatrix(W, rows, cols, T, SQ)
    assert U[0, 0] == pytest.approx(1.0)
    for yy, xx in [(0, 1), (0, cols - 1), (1, 0), (rows - 1, 0)]:
        assert U[yy, xx] == pytest.approx(0.25)
    assert np.count_nonzero(U) == 5


def test_umatrix_uses_euclidean_distance(oracle):
    W = np.array([[0, 0], [3, 4]], dtype=np.float32)   # 1x2 map: one neighbour each, distance 5
    np.testing.assert_allclose(oracle.umatrix(W, 1, 2, P, SQ), [[5.0, 5.0]])
    assert oracle.umatrix(np.ones((1, 3), np.float32), 1, 1, P, SQ)[0, 0] == 0.0


# ------------------------------------------------------------------ cooling

def test_cooling_end_points_and_monotone(oracle):
    for kind in (LIN, EXP):
        vals = [oracle.cool(25.0, 1.0, 10, e, kind) for e in range(10)]
        assert vals[0] == pytest.approx(25.0) and vals[-1] == pytest.approx(1.0)
        assert all(b < a for a, b in zip(vals, vals[1:]))
        assert oracle.cool(25.0, 1.0, 1, 0, kind) == 25.0


def test_cooling_shapes(oracle):
    assert oracle.cool(10.0, 1.0, 10, 3, LIN) == pytest.approx(7.0)           # 10, 9, 8, 7, ...
    assert oracle.cool(100.0, 1.0, 5, 2, LIN) == pytest.approx(50.5)
    assert oracle.cool(100.0, 1.0, 5, 2, EXP) == pytest.approx(10.0)          # geometric mean at the middle
    ratios = [oracle.cool(8.0, 0.5, 7, e + 1, EXP) / oracle.cool(8.0, 0.5, 7, e, EXP) for e in range(6)]
    np.testing.assert_allclose(ratios, ratios[0], rtol=1e-12)
    assert oracle.cool(1.0, 0.01, 10, 9, LIN) == pytest.approx(0.01)          # default learning-rate range
