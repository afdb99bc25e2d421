"""GPU test of fx_set_allocator: with PyTorch's caching allocator behind the library, the whole hot path still meets
the oracle, the library's device memory shows up in PyTorch's accounting, and it goes back when the handles die."""
import gc

import numpy as np
import pytest
import torch

import gpu_common as H
import paper_2407_01781_amd as fx
from oracle import cpu_oracle as O
from workloads import generators as G

pytestmark = pytest.mark.gpu


def test_hot_path_on_the_callers_allocator():
    gc.collect()
    fx.use_torch_allocator(True)
    try:
        w = G.workload("lidar_small")
        ijk, jo = w.jagged_ijk(dup_fraction=0.01)
        d_ijk = torch.from_numpy(ijk).cuda()
        feat, wt = w.feats_weights()
        d_x, d_w = H.to_device_storage(feat, w.dtype), H.to_device_storage(wt, w.dtype)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        g = fx.build_index_grid(d_ijk, jo)
        km = fx.build_kernel_map(g, 3, 1)
        held = torch.cuda.memory_allocated() - before
        assert held >= 96 * g.counts()[0]              # at least the leaf table lives in PyTorch's pool now
        og = O.OracleGrid(ijk, jo)
        H.check_grid(g, og)
        assert np.array_equal(km.dense().cpu().numpy(), O.kernel_map(og, og, 3, 1))
        y = fx.sparse_conv_fwd(km, d_x, d_w)
        H.conv_tolerance_check(y.float().cpu().numpy(), O.conv(og, og, 3, 1, feat, wt, threads=H.ORACLE_THREADS), w.dtype, 27, w.c_in)
        gx = fx.sparse_conv_bwd_data(km, d_x, d_w)
        assert gx.shape == d_x.shape
        del km, g, y, gx
        gc.collect()
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() <= before + (1 << 20)      # everything was handed back
    finally:
        gc.collect()
        fx.use_torch_allocator(False)
    # and the library's own cache serves the next call
    g = fx.build_index_grid(d_ijk, jo)
    assert g.num_voxels == og.num_voxels
