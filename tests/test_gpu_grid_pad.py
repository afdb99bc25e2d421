"""GPU parity: the padded grid (bit-exact against the oracle) and the stride-1 kernel map and convolution
from a grid onto another one -- the padded grid in particular -- with their gradients.

Tolerances as for the other convolution tests: maps and grids bit-exact; fp32 max-abs <= 1e-4*sqrt(K^3*C);
fp16/bf16 per-row relative L2 <= 2e-2; weight gradient per offset relative to the matrix norm."""
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


@pytest.mark.parametrize("r", [0, 1, 2])
def test_padded_grid_matches_oracle(r):
    grids = [_cloud(801, 4000, -50, 50), np.zeros((0, 3), np.int32), _cloud(802, 2500, 4000, 4100),
             np.array([[-1, -1, -1]], np.int32)]
    ijk, jo = G.make_jagged(grids)
    g, og = H.both_grids(ijk, jo)
    H.check_grid(g.pad(r), og.pad(r))


@pytest.mark.parametrize("name", ["lidar_small", "sheets_small", "volume_small"])
def test_padded_workload_grids(name):
    ijk, jo = G.workload(name).jagged_ijk(dup_fraction=0.01)
    g, og = H.both_grids(ijk, jo)
    H.check_grid(g.pad(1), og.pad(1))


@pytest.mark.parametrize("r", [3, 5, 8])
def test_wide_padding_across_leaves(r):
    """Padding wider than a voxel or two: every leaf reaches all 27 leaves around it at r = 8."""
    grids = [_cloud(861, 250, -20, 20), _cloud(862, 60, 4090, 4102), np.array([[-4097, 7, 8]], np.int32)]
    ijk, jo = G.make_jagged(grids)
    g, og = H.both_grids(ijk, jo)
    H.check_grid(g.pad(r), og.pad(r))


@pytest.mark.parametrize("stride,side", [(64, 18), (128, 14), (4096, 2)])
def test_padding_that_multiplies_the_nodes(stride, side):
    """Voxels on the corners of leaves, of lower nodes and of upper nodes: padding by one voxel puts eight leaves
    (lower nodes, upper nodes) where there was one, which is more than the first attempt of the build leaves room for."""
    ax = (np.arange(side, dtype=np.int64) - side // 2) * stride
    ijk = np.stack(np.meshgrid(ax, ax, ax, indexing="ij"), -1).reshape(-1, 3).astype(np.int32)
    g, og = H.both_grids(ijk, np.array([[0, len(ijk)]]))
    gp, ogp = g.pad(1), og.pad(1)
    H.check_grid(gp, ogp)
    assert gp.num_voxels == 27 * len(ijk) and gp.counts()[0] == 8 * len(ijk)


def test_wide_padding_of_a_large_grid_composes():
    """r = 8 on a grid whose (2r+1)^3 candidates per voxel would not fit 32 bits: no candidate is ever made, and
    padding by 8 is padding by 3 and then by 5 (dilations by cubes compose), leaf record for leaf record."""
    ijk, jo = G.workload("lidar1m").jagged_ijk()
    g = fx.build_index_grid(torch.from_numpy(ijk).cuda(), jo)
    assert 17 ** 3 * g.num_voxels > 2 ** 31 - 1
    p8, p35 = g.pad(8), g.pad(3).pad(5)
    assert p8.num_voxels == p35.num_voxels and p8.counts() == p35.counts()
    assert p8.leaf_table().tobytes() == p35.leaf_table().tobytes()
    assert np.array_equal(p8.voxel_joffsets(), p35.voxel_joffsets())


def test_padding_edge_cases_and_errors():
    e, _ = H.both_grids(np.zeros((0, 3), np.int32), np.array([[0, 0]]))
    assert e.pad(1).num_voxels == 0 and e.pad(0).num_voxels == 0
    one, oone = H.both_grids(np.array([[5, -9, 4095]], np.int32), np.array([[0, 1]]))
    H.check_grid(one.pad(8), oone.pad(8))
    assert one.pad(8).num_voxels == 17 ** 3
    with pytest.raises(fx.FxError):
        one.pad(-1)
    with pytest.raises(fx.FxError):
        one.pad(9)
    edge, _ = H.both_grids(np.array([[0, 0, 2 ** 31 - 1]], np.int32), np.array([[0, 1]]))
    with pytest.raises(fx.FxError, match="coordinate limits"):
        edge.pad(1)
    assert edge.pad(0).num_voxels == 1


def _onto_case(seed, dtype, c_in, c_out, K=3, grids=None, r=1):
    grids = grids if grids is not None else [_cloud(seed, 6000, -40, 40), _cloud(seed + 1, 1500, 300, 330)]
    ijk, jo = G.make_jagged(grids)
    g, og = H.both_grids(ijk, jo)
    gp, ogp = g.pad(r), og.pad(r)
    km = fx.build_kernel_map_onto(g, gp, K)
    feat, wt = G.features_and_weights(seed + 2, og.num_voxels, c_in, c_out, K ** 3, dtype)
    gy = G.round_to_dtype(np.random.default_rng(seed + 3).standard_normal((ogp.num_voxels, c_out)).astype(np.float32), dtype)
    return km, og, ogp, feat, wt, gy


@pytest.mark.parametrize("K", [1, 3, 5])
def test_map_onto_the_padded_grid_is_bit_exact(K):
    km, og, ogp, *_ = _onto_case(811, "f32", 4, 4, K=K, r=K // 2)
    ref = O.kernel_map(og, ogp, K, 1)
    assert km.n_out == ogp.num_voxels
    assert np.array_equal(km.dense().cpu().numpy(), ref)
    assert km.info()[0] == (ref >= 0).sum() == K ** 3 * og.num_voxels      # every (input, offset) pair once


@pytest.mark.parametrize("dtype,c_in,c_out,out_f32", [("bf16", 64, 64, False), ("f16", 32, 128, True), ("f32", 16, 32, False),
                                                     ("f32", 3, 5, False), ("bf16", 24, 40, False)])
def test_convolution_onto_the_padded_grid_and_its_gradients(dtype, c_in, c_out, out_f32):
    km, og, ogp, feat, wt, gy = _onto_case(821, dtype, c_in, c_out)
    odt = torch.float32 if out_f32 else None
    d_x, d_w, d_gy = H.to_device_storage(feat, dtype), H.to_device_storage(wt, dtype), H.to_device_storage(gy, dtype)
    y = fx.sparse_conv_fwd(km, d_x, d_w, out_dtype=odt).float().cpu().numpy()
    H.conv_tolerance_check(y, O.conv(og, ogp, 3, 1, feat, wt), dtype, 27, c_in)
    gx = fx.sparse_conv_bwd_data(km, d_gy, d_w, out_dtype=odt).float().cpu().numpy()
    H.conv_tolerance_check(gx, O.conv_bwd_data(og, ogp, 3, 1, gy, wt), dtype, 27, c_out)
    gw = fx.sparse_conv_bwd_weight(km, d_x, d_gy, out_dtype=odt).float().cpu().numpy().astype(np.float64)
    ref = O.conv_bwd_weight(og, ogp, 3, 1, feat, gy)
    num = np.sqrt(((gw - ref) ** 2).sum(axis=(1, 2)))
    den = np.maximum(np.sqrt((ref ** 2).sum(axis=(1, 2))), 1e-3 * np.sqrt(c_in * c_out))
    assert (num / den).max() <= (1e-4 if dtype == "f32" else (2e-3 if out_f32 else 2e-2))
    # transposed convolution over the same map: features on the padded grid, result on the input grid
    _, wt_t = G.features_and_weights(829, 1, c_out, c_in, 27, dtype)
    up = fx.sparse_conv_transpose_fwd(km, d_gy, H.to_device_storage(wt_t, dtype), out_dtype=odt).float().cpu().numpy()
    H.conv_tolerance_check(up, O.conv_transpose(og, ogp, 3, 1, gy, wt_t), dtype, 27, c_out)
    # the forward map is untouched by the map back that now hangs on it
    assert np.array_equal(km.dense().cpu().numpy(), O.kernel_map(og, ogp, 3, 1))


def test_map_onto_an_unrelated_grid_and_onto_itself():
    a, oa = H.both_grids(_cloud(831, 5000, -30, 30), np.array([[0, 5000]]))
    b, ob = H.both_grids(_cloud(832, 7000, -35, 35), np.array([[0, 7000]]))
    km = fx.build_kernel_map_onto(a, b, 3)
    assert np.array_equal(km.dense().cpu().numpy(), O.kernel_map(oa, ob, 3, 1))
    feat, wt = G.features_and_weights(833, oa.num_voxels, 32, 64, 27, "bf16")
    y = fx.sparse_conv_fwd(km, H.to_device_storage(feat, "bf16"), H.to_device_storage(wt, "bf16")).float().cpu().numpy()
    H.conv_tolerance_check(y, O.conv(oa, ob, 3, 1, feat, wt), "bf16", 27, 32)
    same = fx.build_kernel_map_onto(a, a, 3)
    assert np.array_equal(same.dense().cpu().numpy(), fx.build_kernel_map(a, 3, 1).dense().cpu().numpy())
    two, _ = H.both_grids(*G.make_jagged([_cloud(834, 10, 0, 4), _cloud(835, 10, 0, 4)]))
    with pytest.raises(fx.FxError, match="batch members"):
        fx.build_kernel_map_onto(a, two, 3)
    with pytest.raises(fx.FxError):
        fx.build_kernel_map_onto(a, b, 2)


def test_onto_edge_cases():
    # empty input grid onto an empty grid; single voxel; batch with an empty member
    e, _ = H.both_grids(np.zeros((0, 3), np.int32), np.array([[0, 0]]))
    km = fx.build_kernel_map_onto(e, e.pad(1), 3)
    assert km.n_out == 0
    km, og, ogp, feat, wt, gy = _onto_case(841, "bf16", 32, 64, grids=[np.array([[-1, 0, 7]], np.int32), np.zeros((0, 3), np.int32)])
    assert km.n_out == 27
    y = fx.sparse_conv_fwd(km, H.to_device_storage(feat, "bf16"), H.to_device_storage(wt, "bf16")).float().cpu().numpy()
    H.conv_tolerance_check(y, O.conv(og, ogp, 3, 1, feat, wt), "bf16", 27, 32)
    gx = fx.sparse_conv_bwd_data(km, H.to_device_storage(gy, "bf16"), H.to_device_storage(wt, "bf16")).float().cpu().numpy()
    H.conv_tolerance_check(gx, O.conv_bwd_data(og, ogp, 3, 1, gy, wt), "bf16", 27, 64)


def test_full_size_padded_lidar_grid_sampled():
    """Benchmark-size grid: the padded grid's size and sampled indices, and sampled rows of the map and of the
    convolution onto it."""
    w = G.workload("lidar1m")
    ijk, jo = w.jagged_ijk()
    g, og = H.both_grids(ijk, jo)
    gp, ogp = g.pad(1), og.pad(1)
    assert gp.num_voxels == ogp.num_voxels and gp.counts() == ogp.counts()
    rng = np.random.default_rng(851)
    oc, ob = ogp.ijk()
    rows = np.sort(rng.choice(ogp.num_voxels, 4096, replace=False))
    got = gp.ijk_to_index(torch.from_numpy(oc[rows]).cuda(), torch.from_numpy(ob[rows]).cuda()).cpu().numpy()
    assert np.array_equal(got, rows)
    km = fx.build_kernel_map_onto(g, gp, 3)
    ref = O.kernel_map(og, ogp, 3, 1)
    assert np.array_equal(km.dense().cpu().numpy()[rows], ref[rows])
    assert km.info()[0] == 27 * og.num_voxels
    feat, wt = G.features_and_weights(w.feat_seed, og.num_voxels, 64, 64, 27, "bf16")
    y = fx.sparse_conv_fwd(km, H.to_device_storage(feat, "bf16"), H.to_device_storage(wt, "bf16")).float().cpu().numpy()
    f64, w64 = feat.astype(np.float64), wt.astype(np.float64)
    want = np.zeros((rows.size, 64))
    for n, o in enumerate(rows):
        for kappa in np.nonzero(ref[o] >= 0)[0]:
            want[n] += f64[ref[o, kappa]] @ w64[kappa]
    H.conv_tolerance_check(y[rows], want, "bf16", 27, 64)
