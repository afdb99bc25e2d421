"""GPU parity: kernel maps, bit-exact against the oracle (decoded from the tiled form the
convolution consumes)."""
import numpy as np
import pytest
import torch

import gpu_common as H
import paper_2407_01781_amd as fx
from oracle import cpu_oracle as O
from workloads import generators as G

pytestmark = pytest.mark.gpu


def _cloud(seed, n, lo, hi):
    return np.random.default_rng(seed).integers(lo, hi, size=(n, 3)).astype(np.int32)


def _check_map(g, og, K, s):
    km = fx.build_kernel_map(g, K, s)
    ogo = O.output_grid(og, K, s)
    H.check_grid(km.g_out, ogo)
    ref = O.kernel_map(og, ogo, K, s)
    got = km.dense().cpu().numpy()
    assert got.dtype == np.int32 and got.shape == ref.shape
    assert np.array_equal(got, ref)
    n_pairs, per = km.info()
    assert n_pairs == int((ref >= 0).sum())
    assert np.array_equal(per, (ref >= 0).sum(axis=0))
    return km, ref


@pytest.mark.parametrize("name,K,s", [("sphere64", 3, 1), ("sheets_small", 3, 1), ("lidar_small", 3, 1),
                                      ("indoor_small", 3, 1), ("lidar_small", 2, 2), ("sheets_small", 1, 1),
                                      ("sphere64", 5, 1), ("sheets_small", 2, 2), ("sheets_small", 3, 2),
                                      ("lidar_small", 3, 2)])
def test_workload_maps_match_oracle(name, K, s):
    w = G.workload(name)
    ijk, jo = w.jagged_ijk(dup_fraction=0.01)
    g, og = H.both_grids(ijk, jo)
    _check_map(g, og, K, s)


def test_map_with_and_without_the_leaf_table_of_the_grid_build(fx_opt):
    # the grid build prepares the table of the leaves around every leaf on its own stream; a 3x3x3 map of the grid
    # onto itself starts from it -- unless it is switched off or the map is built on another stream, in which case the
    # map build makes the table itself.  All three give the oracle's map; so does a grid made from another (padding).
    grids = [_cloud(21, 30000, -40, 40), _cloud(22, 20000, 4000, 4100), _cloud(23, 500, -4100, -4090)]
    ijk, jo = G.make_jagged(grids)
    g, og = H.both_grids(ijk, jo)
    ref = O.kernel_map(og, og, 3, 1)
    assert np.array_equal(fx.build_kernel_map(g, 3, 1).dense().cpu().numpy(), ref)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        km = fx.build_kernel_map(g, 3, 1)
        got = km.dense()
    side.synchronize()
    assert np.array_equal(got.cpu().numpy(), ref)
    gp, ogp = g.pad(1), og.pad(1)
    assert np.array_equal(fx.build_kernel_map(gp, 3, 1).dense().cpu().numpy(), O.kernel_map(ogp, ogp, 3, 1))
    fx_opt("leaf_links", 0)
    g2, _ = H.both_grids(ijk, jo)
    assert np.array_equal(fx.build_kernel_map(g2, 3, 1).dense().cpu().numpy(), ref)


@pytest.mark.parametrize("K,s", [(3, 1), (2, 2), (3, 2)])
def test_negative_coordinates_and_tile_borders(K, s):
    grids = [_cloud(1, 4000, -20, 20), _cloud(2, 4000, 4080, 4112), np.zeros((0, 3), np.int32),
             _cloud(3, 300, -4100, -4090)]
    ijk, jo = G.make_jagged(grids)
    g, og = H.both_grids(ijk, jo)
    _check_map(g, og, K, s)


def test_dense_block_has_many_rows_per_tile():
    # a dense 20^3 block: tiles with the largest number of distinct input rows
    a = np.arange(20, dtype=np.int32)
    pts = np.stack(np.meshgrid(a, a, a, indexing="ij"), axis=-1).reshape(-1, 3)
    g, og = H.both_grids(pts, np.array([[0, pts.shape[0]]]))
    km, ref = _check_map(g, og, 3, 1)
    st = km.tile_stats()
    assert st["mfma_rows_issued"] >= int((ref >= 0).sum())


def test_empty_grid_map():
    g, og = H.both_grids(np.zeros((0, 3), np.int32), np.array([[0, 0]], np.int64))
    km = fx.build_kernel_map(g, 3, 1)
    assert km.n_out == 0 and km.dense().shape == (0, 27) and km.info()[0] == 0


def test_unsupported_kernel_stride_is_reported():
    g, _ = H.both_grids(_cloud(5, 100, 0, 10), np.array([[0, 100]], np.int64))
    for K, s in ((3, 3), (2, 1), (5, 2)):
        with pytest.raises(fx.FxError) as e:
            fx.build_kernel_map(g, K, s)
        assert e.value.status == -2


@pytest.mark.parametrize("name,pairs", [("lidar1m", 7983738), ("indoor4", None), ("lidar1m_down", 986880),
                                        ("sheets4", 1625841), ("volume1m_c64", 26144783), ("dense96", None)])
def test_full_size_maps_match_oracle(name, pairs):
    """Every entry of the map at the benchmark's sizes (the oracle needs a few seconds)."""
    w = G.workload(name)
    ijk, jo = w.jagged_ijk()
    g, og = H.both_grids(ijk, jo)
    km = fx.build_kernel_map(g, w.kernel_size, w.stride)
    ogo = O.output_grid(og, w.kernel_size, w.stride)
    got = km.dense().cpu().numpy()
    ref = O.kernel_map(og, ogo, w.kernel_size, w.stride)
    assert np.array_equal(got, ref)
    n_pairs, per = km.info()
    assert n_pairs == int((ref >= 0).sum()) and np.array_equal(per, (ref >= 0).sum(0))
    if pairs is not None:
        assert n_pairs == pairs
