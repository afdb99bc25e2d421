"""Pins of the oracle's point quantiser (O6): closed-form cases and an exact-arithmetic
containment check.  No GPU."""
from fractions import Fraction

import numpy as np

from oracle import cpu_oracle as O
from workloads import generators as G


def test_dyadic_points_have_closed_form_cells():
    # voxel size 0.25, origin -3: every value below is exact in single precision, so the cell is
    # known in closed form: cell centres (i + 0.5) * s + o -> i
    i = np.arange(-40, 41)
    centres = ((i + 0.5) * 0.25 - 3.0).astype(np.float32)
    xyz = np.stack([centres, centres[::-1], np.full_like(centres, -3.0 + 0.125)], axis=1)
    ijk, bad = O.points_to_ijk(xyz, [-3.0, -3.0, -3.0], [0.25, 0.25, 0.25])
    assert bad == 0
    assert (ijk[:, 0] == i).all() and (ijk[:, 1] == i[::-1]).all() and (ijk[:, 2] == 0).all()


def test_faces_belong_to_the_upper_cell_and_negatives_floor():
    xyz = np.array([[0.0, 1.0, -1.0], [-0.25, -1e-3, 0.999], [2.0, -2.0, 2.5], [-0.0, 7.75, -7.75]], dtype=np.float32)
    ijk, bad = O.points_to_ijk(xyz, [0, 0, 0], [1, 1, 1])
    assert bad == 0
    assert ijk.tolist() == [[0, 1, -1], [-1, -1, 0], [2, -2, 2], [0, 7, -8]]
    # per-axis voxel sizes and origin
    ijk, _ = O.points_to_ijk(np.array([[1.0, 1.0, 1.0]], np.float32), [0.5, -0.5, 1.0], [0.5, 0.25, 2.0])
    assert ijk.tolist() == [[1, 6, 0]]


def test_invalid_points_are_counted():
    xyz = np.array([[np.nan, 0, 0], [0, np.inf, 0], [0, 0, 3e9], [1, 2, 3], [0, -2.0e9, 0]], dtype=np.float32)
    ijk, bad = O.points_to_ijk(xyz, [0, 0, 0], [1, 1, 1])
    assert bad == 4
    assert ijk[3].tolist() == [1, 2, 3] and (ijk[[0, 1, 2, 4]] == 0).all()
    # the last valid and first invalid magnitudes
    edge = np.array([[1073741823.0, -1073741824.0, 0], [1073741824.0, 0, 0]], dtype=np.float32)   # 2^30-1 rounds to 2^30
    ijk, bad = O.points_to_ijk(edge, [0, 0, 0], [1, 1, 1])
    assert bad == 2
    ok = np.array([[1073741760.0, -1073741824.0, 0]], dtype=np.float32)
    ijk, bad = O.points_to_ijk(ok, [0, 0, 0], [1, 1, 1])
    assert bad == 0 and ijk.tolist() == [[1073741760, -1073741824, 0]]


def test_every_point_lies_in_its_cell_up_to_the_two_roundings():
    # exact rational arithmetic: with d = x - o and t = d / s both rounded to single precision (relative
    # error <= 2^-24 each), the exact quotient q = (x - o) / s satisfies |q - t| <= |q| * 2^-22 roughly, so
    # floor(t) = i implies i - eps <= q < i + 1 + eps with eps = (|q| + 1) * 2^-22
    rng = np.random.default_rng(17)
    xyz = (rng.normal(0.0, 40.0, size=(4000, 3))).astype(np.float32)
    origin = np.array([0.3, -1.7, 12.25], dtype=np.float32)
    size = np.array([0.1, 0.37, 1.5], dtype=np.float32)
    ijk, bad = O.points_to_ijk(xyz, origin, size)
    assert bad == 0
    for p in range(0, 4000, 7):
        for a in range(3):
            q = (Fraction(float(xyz[p, a])) - Fraction(float(origin[a]))) / Fraction(float(size[a]))
            eps = (abs(q) + 1) / 2 ** 22
            assert ijk[p, a] - eps <= q < ijk[p, a] + 1 + eps
    # and away from cell faces the cell is exactly floor(q)
    far = 0
    for p in range(0, 4000, 7):
        for a in range(3):
            q = (Fraction(float(xyz[p, a])) - Fraction(float(origin[a]))) / Fraction(float(size[a]))
            frac = q - (q.numerator // q.denominator)
            if Fraction(1, 1000) < frac < Fraction(999, 1000):
                far += 1
                assert ijk[p, a] == q.numerator // q.denominator
    assert far > 1000


def test_grid_of_a_point_cloud_is_the_grid_of_its_cells():
    pts = G.gaussian_point_cloud(23, 20000, sigma=3.0)
    ijk, bad = O.points_to_ijk(pts, [0, 0, 0], [0.05, 0.05, 0.05])
    assert bad == 0
    g = O.OracleGrid(ijk, np.array([[0, ijk.shape[0]]], dtype=np.int64))
    uniq = np.unique(ijk, axis=0)
    assert g.num_voxels == uniq.shape[0]
    assert (g.lookup(uniq) >= 0).all()
