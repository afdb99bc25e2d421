"""GPU parity: the map-free low-depth convolution (Sec. 3.5 scenario 1) against the oracle's
3x3x3 submanifold convolution, at the fp32 bar; and against the kernel-map path."""
import numpy as np
import pytest
import torch

import gpu_common as H
import paper_2407_01781_amd as fx
from oracle import cpu_oracle as O
from workloads import generators as G

pytestmark = pytest.mark.gpu


def _leaf_vs_oracle(grids, c_in, c_out, seed, dup=0.01, dtype="f32", out_f32=False):
    ijk, jo = G.make_jagged([G.shuffle_and_duplicate(g, seed + b, dup) for b, g in enumerate(grids)])
    g, og = H.both_grids(ijk, jo)
    feat, wt = G.features_and_weights(seed, og.num_voxels, c_in, c_out, 27, dtype)
    y = fx.sparse_conv_leaf_fwd(g, H.to_device_storage(feat, dtype), H.to_device_storage(wt, dtype),
                                out_dtype=torch.float32 if out_f32 else None)
    ref = O.conv(og, og, 3, 1, feat, wt)
    assert y.shape == ref.shape
    assert y.dtype == (torch.float32 if out_f32 else H.TORCH_DT[dtype])
    H.conv_tolerance_check(y.float().cpu().numpy(), ref, dtype, 27, c_in)
    return g, feat, wt, y


@pytest.mark.parametrize("c_in,c_out", [(8, 16), (4, 16), (12, 32), (16, 32), (16, 16), (8, 32), (16, 8), (8, 4), (12, 24),
                                        (4, 28)])
def test_volumetric_bodies_all_channel_shapes(c_in, c_out):
    w = G.workload("volume_small")
    _leaf_vs_oracle(w.grids, c_in, c_out, w.feat_seed)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("c_in,c_out,out_f32", [(32, 64, False), (64, 64, True), (64, 128, False), (96, 64, False)])
def test_sixteen_bit_window_kernel_on_volumetric_bodies(dtype, c_in, c_out, out_f32):
    w = G.workload("volume_small")
    _leaf_vs_oracle(w.grids, c_in, c_out, w.feat_seed, dtype=dtype, out_f32=out_f32)


@pytest.mark.parametrize("name", ["lidar_small", "sheets_small", "indoor_small"])
def test_sixteen_bit_window_kernel_on_sparse_grids(name):
    w = G.workload(name)
    _leaf_vs_oracle(w.grids, 64, 64, w.feat_seed, dtype="bf16")


def test_sixteen_bit_window_kernel_on_dense_block_and_isolated_voxels():
    a = np.arange(-10, 10)
    blk = np.stack(np.meshgrid(a, a, a, indexing="ij"), axis=-1).reshape(-1, 3)
    rng = np.random.default_rng(6)
    far = (rng.integers(-2000, 2000, size=(200, 3)) * 16).astype(np.int32)
    _leaf_vs_oracle([np.concatenate([blk, blk + np.array([128, 128, 4096])]).astype(np.int32), far], 32, 64, 74,
                    dtype="f16")


@pytest.mark.parametrize("name", ["volume1m_c64", "dense96"])
def test_sixteen_bit_window_kernel_full_size_sampled_rows(name):
    w = G.workload(name)
    ijk, jo = w.jagged_ijk()
    g, og = H.both_grids(ijk, jo)
    feat, wt = w.feats_weights()
    y = fx.sparse_conv_leaf_fwd(g, H.to_device_storage(feat, w.dtype), H.to_device_storage(wt, w.dtype)).float().cpu().numpy()
    n = og.num_voxels
    starts = list(range(0, n - 300, n // 12)) + [n - 300]
    f64, w64 = feat.astype(np.float64), wt.astype(np.float64)
    for s0 in starts:
        ref = O.conv(og, og, 3, 1, f64, w64, s0, s0 + 300)
        H.conv_tolerance_check(y[s0:s0 + 300], ref[s0:s0 + 300], w.dtype, 27, w.c_in)
    assert np.isfinite(y).all()


@pytest.mark.parametrize("name", ["lidar_small", "sheets_small", "indoor_small", "sphere64"])
def test_sparse_and_surface_grids(name):
    # leaves with a handful of voxels, ragged last tiles, batches of several grids
    w = G.workload(name)
    _leaf_vs_oracle(w.grids, 8, 16, w.feat_seed)


def test_dense_block_across_node_boundaries():
    # a dense 20^3 block that straddles the origin, a lower-node boundary (128) and a root-tile
    # boundary (4096): full leaves (512 voxels, 32 full tiles) and neighbours in other nodes
    a = np.arange(-10, 10)
    blk = np.stack(np.meshgrid(a, a, a, indexing="ij"), axis=-1).reshape(-1, 3)
    grids = [np.concatenate([blk, blk + np.array([128, 128, 4096])]).astype(np.int32)]
    _leaf_vs_oracle(grids, 8, 16, 71)


def test_isolated_voxels_and_single_voxel_grid():
    rng = np.random.default_rng(5)
    far = (rng.integers(-2000, 2000, size=(300, 3)) * 16).astype(np.int32)     # no two share a neighbourhood
    one = np.array([[7, 0, -1]], dtype=np.int32)
    _leaf_vs_oracle([far, one], 8, 16, 72, dup=0.0)


def test_empty_grid_and_empty_batch_member():
    w = G.workload("volume_small")
    g, og = H.both_grids(*G.make_jagged([np.zeros((0, 3), np.int32)]))
    y = fx.sparse_conv_leaf_fwd(g, torch.zeros((0, 8), device="cuda"), torch.zeros((27, 8, 16), device="cuda"))
    assert y.shape == (0, 16)
    _leaf_vs_oracle([w.grids[0], np.zeros((0, 3), np.int32), w.grids[1]], 8, 16, 73)


def test_agrees_with_the_kernel_map_path(fx_opt):
    fx_opt("leaf_dispatch", "0")      # keep fx.sparse_conv_fwd on the kernel-map kernels
    w = G.workload("volume_small")
    g, feat, wt, y = _leaf_vs_oracle(w.grids, 8, 16, w.feat_seed)
    km = fx.build_kernel_map(g, 3, 1)
    y2 = fx.sparse_conv_fwd(km, H.to_device_storage(feat, "f32"), H.to_device_storage(wt, "f32"))
    tol = 1e-4 * np.sqrt(27 * 8)
    assert float((y - y2).abs().max()) <= tol


def test_unsupported_shapes_are_refused():
    w = G.workload("volume_small")
    ijk, jo = w.jagged_ijk()
    g, _ = H.both_grids(ijk, jo)
    n = g.num_voxels
    for c_in, c_out, dt in ((8, 36, torch.float32), (20, 16, torch.float32), (6, 16, torch.float32), (8, 18, torch.float32),
                            (8, 16, torch.bfloat16), (32, 32, torch.bfloat16), (48, 64, torch.float16)):
        with pytest.raises(fx.FxError):
            fx.sparse_conv_leaf_fwd(g, torch.zeros((n, c_in), device="cuda", dtype=dt),
                                    torch.zeros((27, c_in, c_out), device="cuda", dtype=dt))


def test_full_size_volume_sampled_rows():
    # the bench configuration: ~1M voxels at > 50 % leaf occupancy; the oracle computes a sample of output rows
    w = G.workload("volume1m")
    ijk, jo = w.jagged_ijk()
    g, og = H.both_grids(ijk, jo)
    feat, wt = w.feats_weights()
    y = fx.sparse_conv_leaf_fwd(g, H.to_device_storage(feat, "f32"), H.to_device_storage(wt, "f32")).cpu().numpy()
    n = og.num_voxels
    starts = list(range(0, n - 300, n // 12)) + [n - 300]
    f64, w64 = feat.astype(np.float64), wt.astype(np.float64)
    for s0 in starts:
        ref = O.conv(og, og, 3, 1, f64, w64, s0, s0 + 300)
        H.conv_tolerance_check(y[s0:s0 + 300], ref[s0:s0 + 300], "f32", 27, w.c_in)
    assert np.isfinite(y).all()


# ---------------------------------------------------------------- input gradient without a kernel map
def _leaf_bwd_vs_oracle(grids, c_in, c_out, seed, dtype, out_f32=False):
    ijk, jo = G.make_jagged([G.shuffle_and_duplicate(g, seed + b, 0.01) for b, g in enumerate(grids)])
    g, og = H.both_grids(ijk, jo)
    _, wt = G.features_and_weights(seed, og.num_voxels, c_in, c_out, 27, dtype)
    gy = G.round_to_dtype(np.random.default_rng(seed + 99).standard_normal((og.num_voxels, c_out)).astype(np.float32), dtype)
    gin = fx.sparse_conv_leaf_bwd_data(g, H.to_device_storage(gy, dtype), H.to_device_storage(wt, dtype),
                                       out_dtype=torch.float32 if out_f32 else None)
    ref = O.conv_bwd_data(og, og, 3, 1, gy, wt)
    assert gin.shape == ref.shape
    # the forward bars with the contracted channel count (here C_out); the rows of the weights W[kappa] . gout
    # have the scale of gout times sqrt(C_out / (27 C_in)) per tap, which the relative bar absorbs
    H.conv_tolerance_check(gin.float().cpu().numpy(), ref, dtype, 27, c_out)
    return g, gy, wt, gin


@pytest.mark.parametrize("c_in,c_out", [(16, 8), (32, 16), (16, 4), (32, 12), (8, 16), (4, 8), (20, 12)])
def test_input_gradient_fp32(c_in, c_out):
    w = G.workload("volume_small")
    _leaf_bwd_vs_oracle(w.grids, c_in, c_out, w.feat_seed, "f32")


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("c_in,c_out,out_f32", [(64, 32, False), (64, 64, True), (128, 64, False)])
def test_input_gradient_sixteen_bit(dtype, c_in, c_out, out_f32):
    w = G.workload("volume_small")
    _leaf_bwd_vs_oracle(w.grids, c_in, c_out, w.feat_seed, dtype, out_f32)


def test_input_gradient_on_sparse_grid_and_against_the_kernel_map_path(fx_opt):
    fx_opt("leaf_dispatch", "0")
    w = G.workload("lidar_small")
    g, gy, wt, gin = _leaf_bwd_vs_oracle(w.grids, 64, 64, w.feat_seed, "bf16")
    km = fx.build_kernel_map(g, 3, 1)
    gin2 = fx.sparse_conv_bwd_data(km, H.to_device_storage(gy, "bf16"), H.to_device_storage(wt, "bf16"))
    d = (gin.float() - gin2.float()).norm(dim=1) / gin2.float().norm(dim=1).clamp_min(1e-3)
    assert float(d.max()) <= 2e-2


def test_input_gradient_is_the_adjoint_of_the_forward():
    # <leaf_fwd(x; W), g> = <x, leaf_bwd_data(g; W)> in fp32 (both sides computed by the library)
    w = G.workload("volume_small")
    ijk, jo = w.jagged_ijk()
    g, og = H.both_grids(ijk, jo)
    n = og.num_voxels
    gen = torch.Generator(device="cpu").manual_seed(5)
    x = torch.randn((n, 8), generator=gen).cuda()
    gy = torch.randn((n, 16), generator=gen).cuda()
    wt = (torch.randn((27, 8, 16), generator=gen) * 0.1).cuda()
    lhs = (fx.sparse_conv_leaf_fwd(g, x, wt).double() * gy.double()).sum()
    rhs = (x.double() * fx.sparse_conv_leaf_bwd_data(g, gy, wt).double()).sum()
    assert abs(float(lhs - rhs)) <= 1e-4 * abs(float(lhs)) + 1e-3


# ---------------------------------------------------------------- dispatch from the kernel-map entry points
@pytest.mark.parametrize("switch,expect_leaf", [(None, True), ("0", False), ("1", True)])
def test_kernel_map_entry_points_take_the_leaf_kernels_on_dense_grids(switch, expect_leaf, fx_opt):
    # a dense block: by default fx.sparse_conv_fwd / bwd_data on its (3,1) map run the leaf-window kernels; the
    # switch keeps the tile kernels.  Both must meet the oracle; which kernel ran is read from the profile slots.
    if switch is not None:
        fx_opt("leaf_dispatch", switch)
    a = np.arange(-12, 12, dtype=np.int32)
    blk = np.stack(np.meshgrid(a, a, a, indexing="ij"), axis=-1).reshape(-1, 3)
    g, og = H.both_grids(blk, np.array([[0, blk.shape[0]]]))
    km = fx.build_kernel_map(g, 3, 1)
    feat, wt = G.features_and_weights(81, og.num_voxels, 64, 64, 27, "bf16")
    gy = G.round_to_dtype(np.random.default_rng(82).standard_normal((og.num_voxels, 64)).astype(np.float32), "bf16")
    fx.profile_enable(True)
    fx.profile_reset()
    y = fx.sparse_conv_fwd(km, H.to_device_storage(feat, "bf16"), H.to_device_storage(wt, "bf16"))
    gx = fx.sparse_conv_bwd_data(km, H.to_device_storage(gy, "bf16"), H.to_device_storage(wt, "bf16"))
    torch.cuda.synchronize()
    slots = fx.profile_read()
    fx.profile_enable(False)
    assert ("k_conv_leaf" in slots) == expect_leaf
    if switch is not None:          # left alone, the block's partly filled border leaves go to the tile kernel (per-leaf dispatch)
        assert ("k_conv_mfma" in slots) == (not expect_leaf)
    H.conv_tolerance_check(y.float().cpu().numpy(), O.conv(og, og, 3, 1, feat, wt), "bf16", 27, 64)
    H.conv_tolerance_check(gx.float().cpu().numpy(), O.conv_bwd_data(og, og, 3, 1, gy, wt), "bf16", 27, 64)


def test_sparse_grids_stay_on_the_kernel_map_kernels():
    w = G.workload("lidar_small")
    ijk, jo = w.jagged_ijk()
    g, og = H.both_grids(ijk, jo)
    km = fx.build_kernel_map(g, 3, 1)
    feat, wt = w.feats_weights()
    fx.profile_enable(True)
    fx.profile_reset()
    fx.sparse_conv_fwd(km, H.to_device_storage(feat, w.dtype), H.to_device_storage(wt, w.dtype))
    torch.cuda.synchronize()
    slots = fx.profile_read()
    fx.profile_enable(False)
    assert "k_conv_mfma" in slots and "k_conv_leaf" not in slots


# ---------------------------------------------------------------------------------- weight gradient from the leaf window
def _wgrad_rel(gw, ref):
    gw = gw.astype(np.float64)
    num = np.sqrt(((gw - ref) ** 2).sum(axis=(1, 2)))
    den = np.maximum(np.sqrt((ref ** 2).sum(axis=(1, 2))), 1e-3 * np.sqrt(ref.shape[1] * ref.shape[2]))
    return (num / den).max()


def _leaf_wgrad_vs_oracle(grids, c_in, c_out, seed, dup=0.01):
    """Per offset, ||gw[kappa] - ref||_F <= 1e-4 ||ref||_F (fp32 data, fp32 sums)."""
    ijk, jo = G.make_jagged([G.shuffle_and_duplicate(g, seed + b, dup) for b, g in enumerate(grids)])
    g, og = H.both_grids(ijk, jo)
    feat, _ = G.features_and_weights(seed, og.num_voxels, c_in, c_out, 27, "f32")
    gy = np.random.default_rng(seed + 11).standard_normal((og.num_voxels, c_out)).astype(np.float32)
    gw = fx.sparse_conv_leaf_bwd_weight(g, H.to_device_storage(feat, "f32"), H.to_device_storage(gy, "f32"))
    assert gw.shape == (27, c_in, c_out) and gw.dtype == torch.float32
    ref = O.conv_bwd_weight(og, og, 3, 1, feat, gy)
    assert _wgrad_rel(gw.cpu().numpy(), ref) <= 1e-4
    return g, og, feat, gy, gw


@pytest.mark.parametrize("c_in,c_out", [(8, 16), (4, 16), (4, 32), (8, 32), (12, 16), (16, 16), (8, 12), (16, 4), (4, 4),
                                        (12, 8), (8, 28), (16, 32), (12, 24), (16, 20)])
def test_weight_gradient_all_channel_shapes(c_in, c_out):
    w = G.workload("volume_small")
    _leaf_wgrad_vs_oracle(w.grids, c_in, c_out, w.feat_seed)


@pytest.mark.parametrize("name", ["lidar_small", "sheets_small", "sphere64"])
def test_weight_gradient_on_sparse_and_surface_grids(name):
    w = G.workload(name)
    _leaf_wgrad_vs_oracle(w.grids, 8, 16, w.feat_seed)


def test_weight_gradient_edge_cases_and_reproducibility():
    # a batch with an empty member, isolated voxels (every leaf holds one voxel: only the centre tap sums), a dense
    # block across node boundaries
    a = np.arange(-9, 9)
    blk = np.stack(np.meshgrid(a, a, a, indexing="ij"), axis=-1).reshape(-1, 3).astype(np.int32)
    far = (np.random.default_rng(9).integers(-3000, 3000, size=(300, 3)) * 16).astype(np.int32)
    g, og, feat, gy, gw = _leaf_wgrad_vs_oracle([blk + np.array([4090, 120, -8], np.int32), np.zeros((0, 3), np.int32), far], 8, 16, 91)
    again = fx.sparse_conv_leaf_bwd_weight(g, H.to_device_storage(feat, "f32"), H.to_device_storage(gy, "f32"))
    assert torch.equal(gw, again)                       # fixed summation order: identical bits
    _, _, _, _, gw1 = _leaf_wgrad_vs_oracle([np.array([[3, -4, 5]], np.int32)], 16, 16, 92, dup=0.0)
    assert (gw1.cpu().numpy()[np.arange(27) != 13] == 0).all()
    # empty grid: all zeros
    e, _ = H.both_grids(np.zeros((0, 3), np.int32), np.array([[0, 0]]))
    z = fx.sparse_conv_leaf_bwd_weight(e, torch.zeros((0, 8), device="cuda"), torch.zeros((0, 16), device="cuda"))
    assert z.shape == (27, 8, 16) and (z == 0).all()
    # shapes the kernel does not serve
    for c_in, c_out, dt in ((16, 36, torch.float32), (8, 6, torch.float32), (6, 16, torch.float32), (8, 16, torch.bfloat16)):
        with pytest.raises(fx.FxError):
            fx.sparse_conv_leaf_bwd_weight(g, torch.zeros((g.num_voxels, c_in), device="cuda", dtype=dt),
                                           torch.zeros((g.num_voxels, c_out), device="cuda", dtype=dt))


@pytest.mark.parametrize("switch", [None, "0"])
def test_kernel_map_weight_gradient_takes_the_leaf_kernel_at_low_depth(switch, fx_opt):
    if switch is not None:
        fx_opt("leaf_dispatch", switch)
    w = G.workload("volume_small")
    ijk, jo = w.jagged_ijk()
    g, og = H.both_grids(ijk, jo)
    km = fx.build_kernel_map(g, 3, 1)
    feat, _ = G.features_and_weights(5, og.num_voxels, 8, 16, 27, "f32")
    gy = np.random.default_rng(6).standard_normal((og.num_voxels, 16)).astype(np.float32)
    d_x, d_gy = H.to_device_storage(feat, "f32"), H.to_device_storage(gy, "f32")
    fx.profile_enable(True); fx.profile_reset()
    gw = fx.sparse_conv_bwd_weight(km, d_x, d_gy)
    torch.cuda.synchronize()
    fx.profile_enable(False)
    assert _wgrad_rel(gw.cpu().numpy(), O.conv_bwd_weight(og, og, 3, 1, feat, gy)) <= 1e-4
    leaf = fx.sparse_conv_leaf_bwd_weight(g, d_x, d_gy)
    assert torch.equal(gw, leaf) == (switch is None)      # the same kernel, or the scalar one


def test_weight_gradient_full_size_volume():
    """volume1m, 8 -> 16 fp32 (1.03 M voxels, 26 M pairs): the whole gradient against the oracle."""
    w = G.workload("volume1m")
    ijk, jo = w.jagged_ijk()
    g, og = H.both_grids(ijk, jo)
    feat, _ = G.features_and_weights(w.feat_seed, og.num_voxels, 8, 16, 27, "f32")
    gy = np.random.default_rng(w.feat_seed + 3).standard_normal((og.num_voxels, 16)).astype(np.float32)
    gw = fx.sparse_conv_leaf_bwd_weight(g, H.to_device_storage(feat, "f32"), H.to_device_storage(gy, "f32"))
    assert _wgrad_rel(gw.cpu().numpy(), O.conv_bwd_weight(og, og, 3, 1, feat, gy)) <= 1e-4


# ---------------------------------------------------------------------------------- weight gradient, 16-bit types at depth >= 32
def _leaf_wgrad16_vs_oracle(grids, dtype, c_in, c_out, out_f32, seed, dup=0.01):
    """Per offset, ||gw[kappa] - ref||_F relative to ||ref||_F: products are exact and summed in fp32, so the error is
    the one rounding of the result (2e-2 in the storage type) or the fp32 summation order (2e-3 with an fp32 result)."""
    ijk, jo = G.make_jagged([G.shuffle_and_duplicate(g, seed + b, dup) for b, g in enumerate(grids)])
    g, og = H.both_grids(ijk, jo)
    feat, _ = G.features_and_weights(seed, og.num_voxels, c_in, c_out, 27, dtype)
    gy = G.round_to_dtype(np.random.default_rng(seed + 11).standard_normal((og.num_voxels, c_out)).astype(np.float32), dtype)
    d_x, d_gy = H.to_device_storage(feat, dtype), H.to_device_storage(gy, dtype)
    gw = fx.sparse_conv_leaf_bwd_weight(g, d_x, d_gy, out_dtype=torch.float32 if out_f32 else None)
    assert gw.shape == (27, c_in, c_out)
    ref = O.conv_bwd_weight(og, og, 3, 1, feat, gy)
    assert _wgrad_rel(gw.float().cpu().numpy(), ref) <= (2e-3 if out_f32 else 2e-2)
    return g, og, d_x, d_gy, gw


@pytest.mark.parametrize("name", ["volume_small", "lidar_small", "sheets_small"])
@pytest.mark.parametrize("dtype,c_in,c_out,out_f32", [("bf16", 64, 64, False), ("f16", 32, 128, True), ("bf16", 96, 64, True)])
def test_weight_gradient_16_bit_from_the_leaf_window(name, dtype, c_in, c_out, out_f32):
    w = G.workload(name)
    _leaf_wgrad16_vs_oracle(w.grids, dtype, c_in, c_out, out_f32, w.feat_seed)


def test_weight_gradient_16_bit_edge_cases_and_reproducibility():
    a = np.arange(-9, 9)
    blk = np.stack(np.meshgrid(a, a, a, indexing="ij"), axis=-1).reshape(-1, 3).astype(np.int32)
    far = (np.random.default_rng(9).integers(-3000, 3000, size=(300, 3)) * 16).astype(np.int32)
    g, og, d_x, d_gy, gw = _leaf_wgrad16_vs_oracle([blk + np.array([4090, 120, -8], np.int32), np.zeros((0, 3), np.int32), far],
                                                    "bf16", 32, 64, True, 93)
    assert torch.equal(gw, fx.sparse_conv_leaf_bwd_weight(g, d_x, d_gy, out_dtype=torch.float32))     # fixed order: identical bits
    _, _, _, _, gw1 = _leaf_wgrad16_vs_oracle([np.array([[3, -4, 5]], np.int32)], "f16", 32, 64, True, 94, dup=0.0)
    assert (gw1.cpu().numpy()[np.arange(27) != 13] == 0).all()
    # a leaf whose voxel count is not a multiple of 32, next to full leaves: 8x8x8 plus a 3x3x3 corner in the next leaf
    c = np.arange(0, 8)
    full = np.stack(np.meshgrid(c, c, c, indexing="ij"), axis=-1).reshape(-1, 3).astype(np.int32)
    d = np.arange(8, 11)
    corner = np.stack(np.meshgrid(d, d, d, indexing="ij"), axis=-1).reshape(-1, 3).astype(np.int32)
    _leaf_wgrad16_vs_oracle([np.concatenate([full, corner])], "bf16", 64, 64, True, 95, dup=0.0)
    e, _ = H.both_grids(np.zeros((0, 3), np.int32), np.array([[0, 0]]))
    z = fx.sparse_conv_leaf_bwd_weight(e, torch.zeros((0, 32), device="cuda", dtype=torch.bfloat16),
                                       torch.zeros((0, 64), device="cuda", dtype=torch.bfloat16))
    assert z.shape == (27, 32, 64) and (z == 0).all()
    for c_in, c_out in ((48, 64), (32, 32), (8, 16)):
        with pytest.raises(fx.FxError):
            fx.sparse_conv_leaf_bwd_weight(g, torch.zeros((g.num_voxels, c_in), device="cuda", dtype=torch.float16),
                                           torch.zeros((g.num_voxels, c_out), device="cuda", dtype=torch.float16))


@pytest.mark.parametrize("switch", [None, "0", "1"])
def test_kernel_map_weight_gradient_takes_the_leaf_kernel_on_dense_grids(switch, fx_opt):
    """A solid 24^3 block is locally dense (the forward pass takes its leaf-window kernel there): so does the weight
    gradient, unless leaf_dispatch = 0; on the sparse LiDAR grid it does only when leaf_dispatch = 1."""
    if switch is not None:
        fx_opt("leaf_dispatch", switch)
    a = np.arange(0, 24)
    block = np.stack(np.meshgrid(a, a, a, indexing="ij"), axis=-1).reshape(-1, 3).astype(np.int32) + np.array([-8, 4096, 40], np.int32)
    for name, dense in (("block", True), ("lidar_small", False)):
        if name == "block":
            ijk, jo = G.make_jagged([block])
        else:
            ijk, jo = G.workload(name).jagged_ijk()
        g, og = H.both_grids(ijk, jo)
        km = fx.build_kernel_map(g, 3, 1)
        feat, _ = G.features_and_weights(7, og.num_voxels, 64, 64, 27, "bf16")
        gy = G.round_to_dtype(np.random.default_rng(8).standard_normal((og.num_voxels, 64)).astype(np.float32), "bf16")
        d_x, d_gy = H.to_device_storage(feat, "bf16"), H.to_device_storage(gy, "bf16")
        gw = fx.sparse_conv_bwd_weight(km, d_x, d_gy, out_dtype=torch.float32)
        assert _wgrad_rel(gw.cpu().numpy(), O.conv_bwd_weight(og, og, 3, 1, feat, gy)) <= 2e-3
        leaf = fx.sparse_conv_leaf_bwd_weight(g, d_x, d_gy, out_dtype=torch.float32)
        taken = switch == "1" or (switch is None and dense)
        assert torch.equal(gw, leaf) == taken
