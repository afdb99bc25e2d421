"""GPU parity: index-grid build and queries, bit-exact against the oracle."""
import itertools

import numpy as np
import pytest
import torch

import gpu_common as H
import paper_2407_01781_amd.binding as B
from oracle import cpu_oracle as O
from workloads import generators as G

pytestmark = pytest.mark.gpu


def _cloud(seed, n, lo, hi):
    return np.random.default_rng(seed).integers(lo, hi, size=(n, 3)).astype(np.int32)


@pytest.mark.parametrize("name", ["sphere64", "sheets_small", "lidar_small", "indoor_small"])
def test_workload_grids_match_oracle(name):
    w = G.workload(name)
    ijk, jo = w.jagged_ijk(dup_fraction=0.01)
    g, og = H.both_grids(ijk, jo)
    H.check_grid(g, og)


def test_negative_coordinates_many_tiles_and_empty_grids():
    grids = [_cloud(3, 3000, -300, 300), _cloud(4, 2000, 3900, 4300), np.zeros((0, 3), np.int32),
             _cloud(5, 1000, -5000, -3000), _cloud(6, 500, -70000, 70000)]
    ijk, jo = G.make_jagged(grids)
    g, og = H.both_grids(ijk, jo)
    H.check_grid(g, og)
    assert g.counts()[2] > 20          # many root tiles


def test_sparse_points_overflow_the_first_capacity_guess():
    # one voxel per leaf: more leaves than the first attempt allows, so the build retries
    pts = _cloud(9, 20000, -20000, 20000)
    g, og = H.both_grids(pts, np.array([[0, pts.shape[0]]]))
    H.check_grid(g, og)


def test_large_inputs_take_the_bucket_path_and_agree_with_the_direct_path(fx_opt):
    # above 65536 rows the build scatters the rows into buckets first; the same input through the
    # direct path (one global table) must give the same bits, and both must match the oracle
    grids = [_cloud(31, 60000, -60, 60), np.zeros((0, 3), np.int32), _cloud(32, 50000, 4000, 4200),
             _cloud(33, 30000, -9000, -8800)]
    ijk, jo = G.make_jagged(grids)
    g, og = H.both_grids(ijk, jo)
    H.check_grid(g, og)
    fx_opt("grid_direct", "1")
    g2, _ = H.both_grids(ijk, jo)
    H.check_grid(g2, og)
    assert g.leaf_table().tobytes() == g2.leaf_table().tobytes()


def test_sparse_large_input_overflows_the_bucket_tables():
    # one voxel per leaf and about two thousand rows per bucket: every bucket holds more leaves than
    # its LDS table, so the build repeats through the direct path (and with a larger leaf capacity)
    pts = _cloud(41, 500000, -40000, 40000)
    g, og = H.both_grids(pts, np.array([[0, pts.shape[0]]]))
    H.check_grid(g, og)


def test_empty_batch_and_empty_input():
    g, og = H.both_grids(np.zeros((0, 3), np.int32), np.zeros((0, 2), np.int64))
    assert g.num_voxels == 0 and g.counts() == (0, 0, 0)
    g, og = H.both_grids(np.zeros((0, 3), np.int32), np.array([[0, 0], [0, 0]], np.int64))
    assert g.num_voxels == 0 and g.voxel_joffsets().tolist() == [[0, 0], [0, 0]]
    q = torch.zeros((2, 3), dtype=torch.int32, device="cuda")
    assert g.ijk_to_index(q).cpu().tolist() == [-1, -1]


def test_rows_outside_every_range_are_ignored():
    pts = _cloud(11, 1000, 0, 40)
    jo = np.array([[10, 400], [500, 900]], np.int64)
    g, og = H.both_grids(pts, jo)
    H.check_grid(g, og)


def test_ijk_to_index_matches_oracle_lookup():
    grids = [_cloud(21, 4000, -40, 40), _cloud(22, 3000, 4080, 4120)]
    ijk, jo = G.make_jagged(grids)
    g, og = H.both_grids(ijk, jo)
    rng = np.random.default_rng(23)
    q = np.concatenate([rng.integers(-45, 45, size=(5000, 3)), rng.integers(4070, 4130, size=(5000, 3))]).astype(np.int32)
    jb = rng.integers(-1, 3, size=q.shape[0]).astype(np.int32)      # includes invalid grid ids
    got = g.ijk_to_index(torch.from_numpy(q).cuda(), torch.from_numpy(jb).cuda()).cpu().numpy()
    valid = (jb >= 0) & (jb < 2)
    expect = np.full(q.shape[0], -1, dtype=np.int64)
    expect[valid] = og.lookup(q[valid], jb[valid])
    assert np.array_equal(got, expect)
    # every input row maps to its own voxel; duplicates share an index
    got_in = g.ijk_to_index(torch.from_numpy(ijk).cuda(),
                            torch.from_numpy(np.repeat(np.arange(2, dtype=np.int32), [4000, 3000])).cuda())
    assert np.array_equal(got_in.cpu().numpy(), og.lookup(ijk, np.repeat(np.arange(2, dtype=np.int32), [4000, 3000])))


def test_dense_block_gives_listing1_offsets():
    pts = np.array(list(itertools.product(range(8), repeat=3)), dtype=np.int32)
    g, _ = H.both_grids(pts[np.random.default_rng(1).permutation(512)], np.array([[0, 512]]))
    idx = g.ijk_to_index(torch.from_numpy(pts).cuda()).cpu().numpy()
    assert np.array_equal(idx, (pts[:, 0] << 6) | (pts[:, 1] << 3) | pts[:, 2])


def test_coarsen2_matches_oracle():
    grids = [_cloud(31, 5000, -60, 60), _cloud(32, 3000, 4000, 4200)]
    ijk, jo = G.make_jagged(grids)
    g, og = H.both_grids(ijk, jo)
    H.check_grid(g.coarsen2(), og.coarsen2())


def test_same_input_twice_gives_identical_bits():
    w = G.workload("lidar_small")
    ijk, jo = w.jagged_ijk(dup_fraction=0.01)
    g1, _ = H.both_grids(ijk, jo)
    g2, _ = H.both_grids(ijk, jo)
    assert g1.leaf_table().tobytes() == g2.leaf_table().tobytes()
    assert torch.equal(g1.ijk()[0], g2.ijk()[0])


@pytest.mark.parametrize("name", ["lidar1m", "indoor4"])
def test_full_size_grid_properties_and_sampled_indices(name):
    """Benchmark-size grids: counts, the leaf table's closed-form invariants and sampled
    indices against the oracle (which is fast enough for O1 at this size)."""
    w = G.workload(name)
    ijk, jo = w.jagged_ijk()
    g, og = H.both_grids(ijk, jo)
    H.check_grid(g, og)


def test_released_device_blocks_are_reused_and_can_be_returned():
    # steady-state calls take their device memory from the library's cache of released blocks;
    # returning the cache to the driver must leave later calls working
    pts = _cloud(51, 30000, 0, 200)
    jo = np.array([[0, pts.shape[0]]])
    g1, og = H.both_grids(pts, jo)
    t1 = g1.leaf_table().tobytes()
    del g1
    B.release_cached_memory()
    g2, _ = H.both_grids(pts, jo)
    assert g2.leaf_table().tobytes() == t1 == og.leaf_table().tobytes()
