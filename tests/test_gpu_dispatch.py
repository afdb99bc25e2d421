"""GPU parity of per-leaf dispatch: one call of the 3x3x3 submanifold convolution (or its input gradient) on a grid
that mixes locally dense leaves with sparse ones runs the leaf-window kernel on the dense leaves and the tile kernel
on everything else; every output row against the oracle, outputs NaN before the call."""
import numpy as np
import pytest
import torch

import gpu_common as H
import paper_2407_01781_amd as fx
from oracle import cpu_oracle as O
from workloads import generators as G

pytestmark = pytest.mark.gpu


def _kernels_of(fn):
    fx.profile_enable(True)
    fx.profile_reset()
    out = fn()
    torch.cuda.synchronize()
    slots = fx.profile_read()
    fx.profile_enable(False)
    return out, slots


def _check_forward_and_input_gradient(pts, jo, dtype, c_in, c_out, expect_both, seed=61):
    g, og = H.both_grids(pts, jo)
    km = fx.build_kernel_map(g, 3, 1)
    feat, wt = G.features_and_weights(seed, og.num_voxels, c_in, c_out, 27, dtype)
    gy = G.round_to_dtype(np.random.default_rng(seed + 1).standard_normal((og.num_voxels, c_out)).astype(np.float32), dtype)
    d_x, d_w, d_gy = (H.to_device_storage(a, dtype) for a in (feat, wt, gy))
    out = H.nan_filled((og.num_voxels, c_out), H.TORCH_DT[dtype])
    _, slots = _kernels_of(lambda: fx.sparse_conv_fwd(km, d_x, d_w, out=out))
    if expect_both:
        assert "k_conv_leaf" in slots and "k_conv_mfma" in slots
    y = out.float().cpu().numpy()
    assert np.isfinite(y).all()
    H.conv_tolerance_check(y, O.conv(og, og, 3, 1, feat, wt, threads=H.ORACLE_THREADS), dtype, 27, c_in)
    gx = H.nan_filled((og.num_voxels, c_in), torch.float32)
    fx.sparse_conv_bwd_data(km, d_gy, d_w, out_dtype=torch.float32, out=gx)
    gx = gx.cpu().numpy()
    assert np.isfinite(gx).all()
    H.conv_tolerance_check(gx, O.conv_bwd_data(og, og, 3, 1, gy, wt, threads=min(4, H.ORACLE_THREADS)), dtype, 27, c_out)
    # the weight gradient is split the same way: dense leaves' pairs from the leaf window, the others from the tiles
    gw, wslots = _kernels_of(lambda: fx.sparse_conv_bwd_weight(km, d_x, d_gy, out_dtype=torch.float32))
    ref = O.conv_bwd_weight(og, og, 3, 1, feat, gy)
    num = np.sqrt(((gw.cpu().numpy().astype(np.float64) - ref) ** 2).sum(axis=(1, 2)))
    den = np.maximum(np.sqrt((ref ** 2).sum(axis=(1, 2))), 1e-3 * np.sqrt(c_in * c_out))
    assert (num / den).max() <= 2e-3
    assert torch.equal(gw, fx.sparse_conv_bwd_weight(km, d_x, d_gy, out_dtype=torch.float32))      # fixed order of the sums
    return g


@pytest.mark.parametrize("switch", [None, 2])
@pytest.mark.parametrize("dtype,c_in,c_out", [("bf16", 64, 64), ("f16", 32, 128)])
def test_mixed_grid_is_split_between_the_two_kernels(switch, dtype, c_in, c_out, fx_opt):
    if switch is not None:
        fx_opt("leaf_dispatch", switch)
    w = G.workload("mixed_small")
    ijk, jo = w.jagged_ijk(dup_fraction=0.01)
    g = _check_forward_and_input_gradient(ijk, jo, dtype, c_in, c_out, expect_both=True)
    cnt = np.diff(np.append(g.leaf_table()["offset"], g.num_voxels))
    assert 0.1 < cnt[cnt >= 205].sum() / g.num_voxels < 0.9          # the automatic rule applies to this grid


def test_forced_split_with_no_dense_leaf_and_with_only_dense_leaves(fx_opt):
    fx_opt("leaf_dispatch", 2)
    w = G.workload("lidar_small")                                   # no leaf reaches 205 voxels: the leaf kernel gets an empty list
    ijk, jo = w.jagged_ijk()
    _check_forward_and_input_gradient(ijk, jo, "bf16", 64, 64, expect_both=False)
    a = np.arange(-16, 16, dtype=np.int32)                            # 64 full leaves: every tile of the split map is empty
    blk = np.stack(np.meshgrid(a, a, a, indexing="ij"), axis=-1).reshape(-1, 3)
    _check_forward_and_input_gradient(blk, np.array([[0, blk.shape[0]]], np.int64), "bf16", 64, 64, expect_both=False)
    # a batch: one member dense, one sparse, one empty
    grids = [blk[:8192], w.grids[0][:20000], np.zeros((0, 3), np.int32)]
    pts, jo = G.make_jagged(grids)
    _check_forward_and_input_gradient(pts, jo, "f16", 32, 64, expect_both=False)


def test_full_size_mixed_grid_every_row():
    """697 301 voxels, 62 % of them in locally dense leaves, mean leaf occupancy 0.16: the automatic rule splits it."""
    w = G.workload("mixed1m")
    ijk, jo = w.jagged_ijk()
    g, og = H.both_grids(ijk, jo)
    km = fx.build_kernel_map(g, 3, 1)
    feat, wt = w.feats_weights()
    out = H.nan_filled((og.num_voxels, w.c_out), torch.bfloat16)
    _, slots = _kernels_of(lambda: fx.sparse_conv_fwd(km, H.to_device_storage(feat, "bf16"), H.to_device_storage(wt, "bf16"), out=out))
    assert "k_conv_leaf" in slots and "k_conv_mfma" in slots
    y = out.float().cpu().numpy()
    assert np.isfinite(y).all()
    H.conv_tolerance_check(y, O.conv(og, og, 3, 1, feat, wt, threads=H.ORACLE_THREADS), "bf16", 27, 64)
