"""GPU parity: input and weight gradients of the sparse convolution against the oracle.

Tolerances.  Input gradient: the forward bars with the roles of the channel counts swapped
(fp32: max-abs <= 1e-4*sqrt(K^3*C_out); fp16/bf16: per-row relative L2 <= 2e-2).  Weight
gradient: every gw[kappa] sums one product per active pair of that offset in fp32, so its error
is measured per offset against the size of that matrix: ||gw[kappa] - ref||_F <= tol * ||ref||_F
(+ a floor), tol = 1e-4 for fp32 outputs of fp32 data, 2e-2 when the result is rounded to
fp16/bf16, 2e-3 for fp32 outputs of fp16/bf16 data (exact products, fp32 sums)."""
import numpy as np
import pytest
import torch

import gpu_common as H
import paper_2407_01781_amd as fx
from oracle import cpu_oracle as O
from workloads import generators as G

pytestmark = pytest.mark.gpu


def _setup(w: G.Workload, c_in=None, c_out=None, dtype=None, dup=0.01):
    c_in, c_out, dtype = c_in or w.c_in, c_out or w.c_out, dtype or w.dtype
    ijk, jo = w.jagged_ijk(dup_fraction=dup)
    g, og = H.both_grids(ijk, jo)
    km = fx.build_kernel_map(g, w.kernel_size, w.stride)
    ogo = O.output_grid(og, w.kernel_size, w.stride)
    feat, wt = G.features_and_weights(w.feat_seed, og.num_voxels, c_in, c_out, w.k3, dtype)
    gy = G.round_to_dtype(np.random.default_rng(w.feat_seed + 7).standard_normal((ogo.num_voxels, c_out)).astype(np.float32), dtype)
    return km, og, ogo, feat, wt, gy, dtype, c_in, c_out


def _wgrad_check(gw: np.ndarray, ref: np.ndarray, tol: float):
    gw = gw.astype(np.float64)
    num = np.sqrt(((gw - ref) ** 2).sum(axis=(1, 2)))
    den = np.maximum(np.sqrt((ref ** 2).sum(axis=(1, 2))), 1e-3 * np.sqrt(ref.shape[1] * ref.shape[2]))
    rel = (num / den).max()
    assert rel <= tol, rel
    return rel


def _check_both(w, out_f32=False, **kw):
    km, og, ogo, feat, wt, gy, dtype, c_in, c_out = _setup(w, **kw)
    odt = torch.float32 if out_f32 else None
    d_gy, d_w, d_x = H.to_device_storage(gy, dtype), H.to_device_storage(wt, dtype), H.to_device_storage(feat, dtype)
    gx = fx.sparse_conv_bwd_data(km, d_gy, d_w, out_dtype=odt).float().cpu().numpy()
    ref_gx = O.conv_bwd_data(og, ogo, w.kernel_size, w.stride, gy, wt)
    H.conv_tolerance_check(gx, ref_gx, dtype, w.k3, c_out)
    gw = fx.sparse_conv_bwd_weight(km, d_x, d_gy, out_dtype=odt).float().cpu().numpy()
    ref_gw = O.conv_bwd_weight(og, ogo, w.kernel_size, w.stride, feat, gy)
    _wgrad_check(gw, ref_gw, 1e-4 if dtype == "f32" else (2e-3 if out_f32 else 2e-2))
    return km, d_x, d_gy


def test_config1_sphere_fp32():
    _check_both(G.workload("sphere64"))


@pytest.mark.parametrize("name", ["indoor_small", "lidar_small", "lidar_small_down", "sheets_small"])
@pytest.mark.parametrize("out_f32", [False, True])
def test_mfma_paths_small_workloads(name, out_f32):
    _check_both(G.workload(name), out_f32=out_f32)


@pytest.mark.parametrize("name", ["lidar_small", "lidar_small_down"])
def test_scalar_paths_agree_with_the_oracle_too(name, fx_opt):
    fx_opt("force_scalar", "1")
    _check_both(G.workload(name), c_in=16, c_out=24)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("c_in,c_out", [(64, 192), (128, 64), (32, 64), (64, 32), (48, 40)])
def test_channel_shapes(dtype, c_in, c_out):
    _check_both(G.workload("sheets_small"), c_in=c_in, c_out=c_out, dtype=dtype)


def test_strided_channel_shapes():
    _check_both(G.workload("lidar_small_down"), c_in=128, c_out=64)
    _check_both(G.workload("lidar_small_down"), c_in=64, c_out=96)


def test_strided_input_gradient_with_weights_fetched_per_step(fx_opt):
    # the kernel that keeps the weights in LDS serves up to 128 contracted channels; the switch and a deeper layer
    # both lead to the one that fetches them per step
    _check_both(G.workload("lidar_small_down"), c_in=64, c_out=320)
    fx_opt("gather_lds", 0)
    _check_both(G.workload("lidar_small_down"), c_in=64, c_out=128)
    _check_both(G.workload("lidar_small_down"), c_in=64, c_out=128, out_f32=True)


def test_weight_gradient_is_reproducible_bit_for_bit():
    km, d_x, d_gy = _check_both(G.workload("lidar_small"), out_f32=True)
    a = fx.sparse_conv_bwd_weight(km, d_x, d_gy, out_dtype=torch.float32)
    b = fx.sparse_conv_bwd_weight(km, d_x, d_gy, out_dtype=torch.float32)
    assert torch.equal(a, b)


def test_exact_special_cases_in_bf16():
    """gout = one-hot column pattern and all-ones data give integer sums that every type holds
    exactly: gw[kappa][ci][co] = number of pairs of offset kappa; gin = C_out x (pairs of the row)."""
    w = G.workload("lidar_small")
    ijk, jo = w.jagged_ijk()
    g, og = H.both_grids(ijk, jo)
    km = fx.build_kernel_map(g, 3, 1)
    nb = O.kernel_map(og, og, 3, 1)
    n = og.num_voxels
    ones_x = torch.ones((n, 64), dtype=torch.bfloat16, device="cuda")
    ones_w = torch.ones((27, 64, 64), dtype=torch.bfloat16, device="cuda")
    gw = fx.sparse_conv_bwd_weight(km, ones_x, ones_x, out_dtype=torch.float32).cpu().numpy()
    pairs = (nb >= 0).sum(0).astype(np.float32)
    assert np.array_equal(gw, np.broadcast_to(pairs[:, None, None], gw.shape))
    gx = fx.sparse_conv_bwd_data(km, ones_x, ones_w, out_dtype=torch.float32).cpu().numpy()
    assert np.array_equal(gx, np.repeat(64.0 * (nb >= 0).sum(1)[:, None].astype(np.float32), 64, axis=1))


def test_empty_and_tiny_grids():
    g, og = H.both_grids(np.zeros((0, 3), np.int32), np.array([[0, 0]], np.int64))
    km = fx.build_kernel_map(g, 3, 1)
    z = torch.zeros((0, 64), dtype=torch.bfloat16, device="cuda")
    gw = fx.sparse_conv_bwd_weight(km, z, z)
    assert gw.shape == (27, 64, 64) and not gw.float().abs().max().item()
    assert fx.sparse_conv_bwd_data(km, z, torch.zeros((27, 64, 64), dtype=torch.bfloat16, device="cuda")).shape == (0, 64)
    pts = np.array([[0, 0, 0], [0, 0, 1], [5, 5, 5], [-1, 0, 0]], dtype=np.int32)
    g, og = H.both_grids(pts, np.array([[0, 4]], np.int64))
    km = fx.build_kernel_map(g, 3, 1)
    feat, wt = G.features_and_weights(7, 4, 64, 64, 27, "bf16")
    gy = G.round_to_dtype(np.random.default_rng(8).standard_normal((4, 64)).astype(np.float32), "bf16")
    gw = fx.sparse_conv_bwd_weight(km, H.to_device_storage(feat, "bf16"), H.to_device_storage(gy, "bf16"),
                                   out_dtype=torch.float32).cpu().numpy()
    _wgrad_check(gw, O.conv_bwd_weight(og, og, 3, 1, feat, gy), 2e-3)


@pytest.mark.parametrize("dims,out_f32", [((16, 16, 16), False), ((40, 24, 8), True), ((26, 26, 26), True)])
def test_sparse_grid_with_a_few_dense_spots(dims, out_f32, fx_opt):
    # a sparse cloud (leaf occupancy far below 0.2) with one solid block.  A tile in the block's interior has more
    # rows than the tile kernel stages in LDS (a full leaf with both neighbours on two axes: 10 x 10 x 8 = 800 > 792):
    # none in 16^3 (every leaf is a corner: 9^3 = 729 rows), a few in 40 x 24 x 8 -- spread over one workgroup per
    # column block beside the sixteen-wave launch for the staged tiles --, more than 16 in 26^3, which sends the whole
    # map to the one launch that takes every tile.  Every element against the oracle, and twice with identical bits.
    fx_opt("leaf_dispatch", "0")
    rng = np.random.default_rng(90 + dims[0])
    cloud = rng.integers(-300, 300, size=(40000, 3)).astype(np.int32)
    ax = [np.arange(d, dtype=np.int32) + 1000 for d in dims]
    block = np.stack(np.meshgrid(*ax, indexing="ij"), axis=-1).reshape(-1, 3)
    pts = np.concatenate([cloud, block])[rng.permutation(40000 + block.shape[0])]
    g, og = H.both_grids(pts, np.array([[0, pts.shape[0]]]))
    km = fx.build_kernel_map(g, 3, 1)
    feat, wt = G.features_and_weights(13, og.num_voxels, 64, 64, 27, "bf16")
    gy = G.round_to_dtype(np.random.default_rng(14).standard_normal((og.num_voxels, 64)).astype(np.float32), "bf16")
    d_x, d_gy = H.to_device_storage(feat, "bf16"), H.to_device_storage(gy, "bf16")
    odt = torch.float32 if out_f32 else None
    gw = fx.sparse_conv_bwd_weight(km, d_x, d_gy, out_dtype=odt)
    _wgrad_check(gw.float().cpu().numpy(), O.conv_bwd_weight(og, og, 3, 1, feat, gy), 2e-3 if out_f32 else 2e-2)
    assert torch.equal(gw, fx.sparse_conv_bwd_weight(km, d_x, d_gy, out_dtype=odt))


def test_dense_block_with_rows_beyond_the_lds_budget(fx_opt):
    fx_opt("leaf_dispatch", "0")      # this test is about the tile kernel's general variant
    a = np.arange(24, dtype=np.int32)
    pts = np.stack(np.meshgrid(a, a, a, indexing="ij"), axis=-1).reshape(-1, 3)
    g, og = H.both_grids(pts, np.array([[0, pts.shape[0]]]))
    km = fx.build_kernel_map(g, 3, 1)
    feat, wt = G.features_and_weights(11, og.num_voxels, 64, 64, 27, "bf16")
    gy = G.round_to_dtype(np.random.default_rng(12).standard_normal((og.num_voxels, 64)).astype(np.float32), "bf16")
    gw = fx.sparse_conv_bwd_weight(km, H.to_device_storage(feat, "bf16"), H.to_device_storage(gy, "bf16"),
                                   out_dtype=torch.float32).cpu().numpy()
    _wgrad_check(gw, O.conv_bwd_weight(og, og, 3, 1, feat, gy), 2e-3)
    gx = fx.sparse_conv_bwd_data(km, H.to_device_storage(gy, "bf16"), H.to_device_storage(wt, "bf16")).float().cpu().numpy()
    H.conv_tolerance_check(gx, O.conv_bwd_data(og, og, 3, 1, gy, wt), "bf16", 27, 64)


@pytest.mark.parametrize("name", ["lidar1m", "lidar1m_down", "lidar1m_down3"])
def test_full_size_adjoint_identity(name):
    """A consistency check of the three entry points among themselves at full size, next to the element-by-element
    comparison with the oracle in test_full_size_every_gradient_element: the bilinear forms that the pinned
    oracle satisfies exactly, <conv(x;W), g> = <x, bwd_data(g;W)> = <W, bwd_weight(x,g)>, evaluated in float64 on
    the HIP path's fp32 outputs; the weight-gradient contribution of an output range compared directly, and
    sampled input-gradient rows of the submanifold map (by its symmetry the forward oracle on gout with
    mirrored offsets and transposed weights)."""
    w = G.workload(name)
    ijk, jo = w.jagged_ijk()
    g, og = H.both_grids(ijk, jo)
    km = fx.build_kernel_map(g, w.kernel_size, w.stride)
    ogo = O.output_grid(og, w.kernel_size, w.stride)
    feat, wt = w.feats_weights()
    gy = G.round_to_dtype(np.random.default_rng(99).standard_normal((ogo.num_voxels, w.c_out)).astype(np.float32), w.dtype)
    d_x, d_w, d_gy = (H.to_device_storage(a, w.dtype) for a in (feat, wt, gy))
    y = fx.sparse_conv_fwd(km, d_x, d_w, out_dtype=torch.float32).double()
    gx = fx.sparse_conv_bwd_data(km, d_gy, d_w, out_dtype=torch.float32).double()
    gw = fx.sparse_conv_bwd_weight(km, d_x, d_gy, out_dtype=torch.float32).double()
    lhs = float((y * d_gy.double()).sum())
    scale = float((y.abs() * d_gy.double().abs()).sum())
    assert abs(lhs - float((gx * d_x.double()).sum())) <= 1e-5 * scale
    assert abs(lhs - float((gw * d_w.double()).sum())) <= 1e-5 * scale
    # a weight gradient restricted to the first 2000 outputs, from zeroing gout elsewhere
    gy_head = gy.copy()
    gy_head[2000:] = 0
    gw_head = fx.sparse_conv_bwd_weight(km, d_x, H.to_device_storage(gy_head, w.dtype), out_dtype=torch.float32).cpu().numpy()
    ref = O.conv_bwd_weight(og, ogo, w.kernel_size, w.stride, feat, gy, 0, 2000)
    _wgrad_check(gw_head, ref, 2e-3)
    if w.stride == 1:
        wm = np.ascontiguousarray(wt[::-1].transpose(0, 2, 1))
        gxs = gx.float().cpu().numpy()
        n = og.num_voxels
        for s in (0, n // 3, n - 300):
            ref = O.conv(og, og, w.kernel_size, 1, gy.astype(np.float64), wm.astype(np.float64), s, s + 300)
            H.conv_tolerance_check(gxs[s:s + 300], ref[s:s + 300], w.dtype, w.k3, w.c_out)


def test_3x3x3_stride_2_backward_edge_cases():
    # empty grid, a batch with an empty member, a single voxel with negative coordinates: the inverse map is
    # built on the first backward call of each map
    for grids in ([np.zeros((0, 3), np.int32)],
                  [G.workload("lidar_small").grids[0][:3000], np.zeros((0, 3), np.int32), np.array([[-1, -2, -3]], np.int32)],
                  [np.array([[7, 0, -1]], np.int32)]):
        ijk, jo = G.make_jagged(grids)
        g, og = H.both_grids(ijk, jo)
        km = fx.build_kernel_map(g, 3, 2)
        ogc = og.coarsen2()
        assert km.n_out == ogc.num_voxels
        _, wt = G.features_and_weights(5, 1, 32, 64, 27, "bf16")
        gy = G.round_to_dtype(np.random.default_rng(6).standard_normal((ogc.num_voxels, 64)).astype(np.float32), "bf16")
        gx = fx.sparse_conv_bwd_data(km, H.to_device_storage(gy, "bf16"), H.to_device_storage(wt, "bf16"))
        assert gx.shape == (og.num_voxels, 32)
        if og.num_voxels:
            H.conv_tolerance_check(gx.float().cpu().numpy(), O.conv_bwd_data(og, ogc, 3, 2, gy, wt), "bf16", 27, 64)
        _, wt_t = G.features_and_weights(7, 1, 64, 32, 27, "bf16")
        up = fx.sparse_conv_transpose_fwd(km, H.to_device_storage(gy, "bf16"), H.to_device_storage(wt_t, "bf16"))
        assert up.shape == (og.num_voxels, 32)
        if og.num_voxels:
            H.conv_tolerance_check(up.float().cpu().numpy(), O.conv_transpose(og, ogc, 3, 2, gy, wt_t), "bf16", 27, 64)
        # the forward map is untouched by the inverse that now hangs on it
        assert np.array_equal(km.dense().cpu().numpy(), O.kernel_map(og, ogc, 3, 2))


@pytest.mark.parametrize("name", ["lidar1m", "lidar1m_down", "sheets4"])
def test_full_size_every_gradient_element(name):
    """Configs 3, 4 and 5 at full size: every row of the input gradient and every element of the weight gradient
    against the oracle (the weight gradient of config 3 sums ~3e5 products per element in fp32 in the kernel's
    fixed order).  Outputs are NaN before the calls."""
    w = G.workload(name)
    ijk, jo = w.jagged_ijk()
    g, og = H.both_grids(ijk, jo)
    km = fx.build_kernel_map(g, w.kernel_size, w.stride)
    ogo = O.output_grid(og, w.kernel_size, w.stride)
    feat, wt = w.feats_weights()
    gy = G.round_to_dtype(np.random.default_rng(199).standard_normal((ogo.num_voxels, w.c_out)).astype(np.float32), w.dtype)
    d_x, d_w, d_gy = (H.to_device_storage(a, w.dtype) for a in (feat, wt, gy))
    gx = H.nan_filled((og.num_voxels, w.c_in), H.TORCH_DT[w.dtype])
    fx.sparse_conv_bwd_data(km, d_gy, d_w, out=gx)
    gx = gx.float().cpu().numpy()
    assert np.isfinite(gx).all()
    ref_gx = O.conv_bwd_data(og, ogo, w.kernel_size, w.stride, gy, wt, threads=min(4, H.ORACLE_THREADS))
    print(f"[row-error] {name} input gradient: {H.row_error_report(gx, ref_gx):.3e}", flush=True)
    H.conv_tolerance_check(gx, ref_gx, w.dtype, w.k3, w.c_out)
    del ref_gx
    gw = H.nan_filled((w.k3, w.c_in, w.c_out), torch.float32)
    fx.sparse_conv_bwd_weight(km, d_x, d_gy, out_dtype=torch.float32, out=gw)
    gw = gw.cpu().numpy()
    assert np.isfinite(gw).all()
    ref_gw = O.conv_bwd_weight(og, ogo, w.kernel_size, w.stride, feat, gy, threads=H.ORACLE_THREADS)
    print(f"[wgrad-error] {name}: max relative Frobenius error per offset {_wgrad_check(gw, ref_gw, 2e-3):.3e}", flush=True)


@pytest.mark.parametrize("c_in,c_out", [(512, 64), (64, 512)])
def test_many_work_items_per_workgroup_backward(c_in, c_out):
    """lidar_small (196 tiles) at 512 channels on one side: the input gradient runs 1568 work items on at most 256
    persistent workgroups (c_in = 512 produced channels), and the weight gradient walks a dozen tiles per
    workgroup; both compared element by element, outputs NaN before the calls."""
    w = G.workload("lidar_small")
    km, og, ogo, feat, wt, gy, dtype, _, _ = _setup(w, c_in=c_in, c_out=c_out)
    d_x, d_w, d_gy = (H.to_device_storage(a, dtype) for a in (feat, wt, gy))
    gx = H.nan_filled((og.num_voxels, c_in), torch.bfloat16)
    fx.sparse_conv_bwd_data(km, d_gy, d_w, out=gx)
    gx = gx.float().cpu().numpy()
    assert np.isfinite(gx).all()
    H.conv_tolerance_check(gx, O.conv_bwd_data(og, ogo, 3, 1, gy, wt, threads=min(4, H.ORACLE_THREADS)), dtype, 27, c_out)
    gw = H.nan_filled((27, c_in, c_out), torch.float32)
    fx.sparse_conv_bwd_weight(km, d_x, d_gy, out_dtype=torch.float32, out=gw)
    gw = gw.cpu().numpy()
    assert np.isfinite(gw).all()
    _wgrad_check(gw, O.conv_bwd_weight(og, ogo, 3, 1, feat, gy, threads=H.ORACLE_THREADS), 2e-3)
