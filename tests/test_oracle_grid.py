"""Pins for the oracle's index grid (O1): closed forms of Listings 1-2, dense special
cases, invariants, the counting identities of Sec. 3.3 and brute force on tiny grids."""
import itertools

import numpy as np
import pytest

from oracle import cpu_oracle as O
from workloads import generators as G
import paper_forms as P


def _grid(ijk, joffsets=None):
    ijk = np.asarray(ijk, dtype=np.int32).reshape(-1, 3)
    if joffsets is None:
        joffsets = np.array([[0, ijk.shape[0]]], dtype=np.int64)
    return O.OracleGrid(ijk, joffsets)


def _random_cloud(seed, n, lo, hi):
    rng = np.random.default_rng(seed)
    return rng.integers(lo, hi, size=(n, 3)).astype(np.int32)


# ---------------------------------------------------------------- special cases
def test_dense_leaf_at_origin_is_listing1_offset():
    pts = np.array(list(itertools.product(range(8), repeat=3)), dtype=np.int32)
    g = _grid(pts[np.random.default_rng(1).permutation(512)])
    idx = g.lookup(pts)
    expect = (pts[:, 0] << 6) | (pts[:, 1] << 3) | pts[:, 2]
    assert np.array_equal(idx, expect)
    assert g.counts() == (1, 1, 1)


@pytest.mark.parametrize("shift", [(0, 0, 0), (-8, -16, 4096), (-4096, 128, -128)])
def test_dense_16cube_orders_leaves_by_lower_offset(shift):
    base = np.array(list(itertools.product(range(16), repeat=3)), dtype=np.int32)
    pts = base + np.array(shift, dtype=np.int32)
    g = _grid(pts[np.random.default_rng(2).permutation(pts.shape[0])])
    idx = g.lookup(pts)
    # 8 leaves, ordered by lower::off (i slowest), each dense: 512 consecutive indices
    leaf_rank = ((base[:, 0] >> 3) << 2) | ((base[:, 1] >> 3) << 1) | (base[:, 2] >> 3)
    local = ((base[:, 0] & 7) << 6) | ((base[:, 1] & 7) << 3) | (base[:, 2] & 7)
    assert np.array_equal(idx, leaf_rank * 512 + local)
    assert g.counts()[0] == 8


def test_hand_worked_order_across_tiles_and_signs():
    # Hand-derived: tiles order by signed (i>>12, j>>12, k>>12); inside a tile by upper,
    # lower and leaf offsets of Listing 2 / Listing 1.
    pts = [
        (-4097, 5, 5),     # tile (-2, 0, 0)
        (-1, -1, -1),      # tile (-1,-1,-1): upper (31,31,31), lower (15,15,15), leaf (7,7,7)
        (-1, 0, 0),        # tile (-1, 0, 0)
        (0, 0, -1),        # tile (0, 0, -1)
        (0, 0, 0),         # tile (0,0,0) first voxel
        (0, 0, 1),
        (0, 1, 0),
        (1, 0, 0),
        (0, 0, 8),         # next leaf in k (lower k = 1)
        (0, 8, 0),         # lower j = 1
        (8, 0, 0),         # lower i = 1
        (0, 0, 128),       # upper k = 1
        (127, 127, 127),   # upper (0,0,0), lower (15,15,15): ranks before (0,0,128)
        (4095, 4095, 4095),
        (4096, 0, 0),      # tile (1,0,0)
    ]
    expect_order = [
        (-4097, 5, 5), (-1, -1, -1), (-1, 0, 0), (0, 0, -1),
        (0, 0, 0), (0, 0, 1), (0, 1, 0), (1, 0, 0), (0, 0, 8), (0, 8, 0), (8, 0, 0),
        (127, 127, 127), (0, 0, 128), (4095, 4095, 4095), (4096, 0, 0),
    ]
    g = _grid(np.array(pts, dtype=np.int32)[::-1])
    idx = g.lookup(np.array(expect_order, dtype=np.int32))
    assert idx.tolist() == list(range(len(expect_order)))
    assert g.counts()[2] == 6      # six distinct root tiles


# ---------------------------------------------------------------- closed form
@pytest.mark.parametrize("name", ["sphere64", "sheets_small", "lidar_small"])
def test_listing1_on_leaf_records_gives_the_rank(name):
    w = G.workload(name)
    ijk, jo = w.jagged_ijk(dup_fraction=0.02)
    g = O.OracleGrid(ijk, jo)
    coords, jidx = g.ijk()
    leaves = g.leaf_table()
    # map (batch, leaf origin) -> record
    rec = {(int(l["batch"]),) + tuple(int(x) for x in l["origin"]): l for l in leaves}
    step = max(1, coords.shape[0] // 4000)
    for s in range(0, coords.shape[0], step):
        i, j, k = (int(x) for x in coords[s])
        l = rec[(int(jidx[s]), (i >> 3) * 8, (j >> 3) * 8, (k >> 3) * 8)]
        assert P.listing1_get_value(l["offset"], l["prefix"], l["mask"], i, j, k) == s


def test_leaf_table_invariants():
    w = G.workload("sheets_small")
    ijk, jo = w.jagged_ijk()
    g = O.OracleGrid(ijk, jo)
    leaves = g.leaf_table()
    assert leaves.dtype.itemsize == 96 and leaves.dtype.fields["origin"][1] == 80  # 80-byte payload
    pc = np.array([[P.popcount(int(x)) for x in l["mask"]] for l in leaves])
    assert pc.sum() == g.num_voxels
    assert np.array_equal(leaves["offset"], np.concatenate([[0], np.cumsum(pc.sum(1))[:-1]]))
    field6 = (leaves["prefix"] >> np.uint64(54)) & np.uint64(511)
    assert np.array_equal(field6.astype(np.int64) + pc[:, 7], pc.sum(1))
    assert np.all(leaves["prefix"] >> np.uint64(63) == 0)


# ---------------------------------------------------------------- invariants
def test_indices_follow_the_paper_sort_keys_with_negatives_and_batches():
    a = _random_cloud(3, 3000, -300, 300)
    b = _random_cloud(4, 2000, 3900, 4300)          # straddles a tile boundary
    c = np.zeros((0, 3), dtype=np.int32)            # empty grid in the middle
    d = _random_cloud(5, 1000, -5000, -3000)
    ijk, jo = G.make_jagged([a, b, c, d])
    g = O.OracleGrid(ijk, jo)
    expect = []
    for bi, pts in enumerate([a, b, c, d]):
        uniq = {tuple(int(x) for x in p) for p in pts}
        expect += sorted(((bi,) + p for p in uniq), key=lambda t: P.vdb_sort_key(*t))
    coords, jidx = g.ijk()
    got = [(int(jidx[s]),) + tuple(int(x) for x in coords[s]) for s in range(coords.shape[0])]
    assert got == expect
    vj = g.voxel_joffsets()
    sizes = [len({tuple(p) for p in pts.tolist()}) for pts in [a, b, c, d]]
    assert np.array_equal(vj[:, 1] - vj[:, 0], sizes) and vj[0, 0] == 0
    assert np.array_equal(vj[1:, 0], vj[:-1, 1])


def test_permutation_duplicate_and_translation_invariance():
    pts = np.unique(_random_cloud(7, 4000, -200, 200), axis=0)
    g0 = _grid(pts)
    ref = g0.lookup(pts)
    assert sorted(ref.tolist()) == list(range(pts.shape[0]))          # bijection onto [0,N)
    rng = np.random.default_rng(8)
    shuffled = pts[rng.permutation(pts.shape[0])]
    dup = np.concatenate([shuffled, shuffled[:500]], axis=0)
    assert np.array_equal(_grid(dup).lookup(pts), ref)
    for t in [(4096, 0, 0), (-8192, 4096, 12288)]:
        tv = np.array(t, dtype=np.int32)
        assert np.array_equal(_grid(pts + tv).lookup(pts + tv), ref)


def test_node_counts_match_hash_set_counts():
    for seed, lo, hi in [(11, -600, 600), (12, 0, 9000), (13, -70000, 70000)]:
        pts = _random_cloud(seed, 5000, lo, hi)
        g = _grid(pts)
        n_leaf = len({tuple(p) for p in (pts >> 3).tolist()})
        n_lower = len({tuple(p) for p in (pts >> 7).tolist()})
        n_upper = len({tuple(p) for p in (pts >> 12).tolist()})
        assert g.counts() == (n_leaf, n_lower, n_upper)


def test_brute_force_bounding_box_queries():
    pts = _random_cloud(21, 150, -6, 11)
    g = _grid(pts)
    active = {tuple(p) for p in pts.tolist()}
    order = sorted(active, key=lambda p: P.vdb_sort_key(0, *p))
    rank = {p: r for r, p in enumerate(order)}
    box = np.array(list(itertools.product(range(-7, 12), repeat=3)), dtype=np.int32)
    idx = g.lookup(box)
    for p, ix in zip(box.tolist(), idx.tolist()):
        assert ix == rank.get(tuple(p), -1)


def test_empty_batch_and_empty_grid():
    g = O.OracleGrid(np.zeros((0, 3), np.int32), np.zeros((0, 2), np.int64))
    assert g.num_voxels == 0 and g.counts() == (0, 0, 0)
    g = O.OracleGrid(np.zeros((0, 3), np.int32), np.array([[0, 0]], np.int64))
    assert g.num_voxels == 0 and g.voxel_joffsets().tolist() == [[0, 0]]
    assert g.lookup(np.array([[0, 0, 0]], np.int32)).tolist() == [-1]


def test_benchmark_grids_have_the_quoted_sizes():
    w = G.workload("sphere64")
    ijk, jo = w.jagged_ijk()
    g = O.OracleGrid(ijk, jo)
    assert g.num_voxels == 9696 and g.counts() == (216, 1, 1)
