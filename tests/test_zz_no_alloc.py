"""GPU test of fx_sparse_conv_fwd_noalloc, the convolution entry point for callers that cannot allocate device
memory: same kernels as fx_sparse_conv_fwd with the packed weights and work-list counters in a static device
array.  Two calls in a row, the second on a smaller input, each compared bit for bit with the allocating entry
point and with the oracle at the convolution's bar; the limits are rejected with a status, not a fault."""
import numpy as np
import pytest
import torch

import gpu_common as H
import paper_2407_01781_amd as fx
from oracle import cpu_oracle as O
from workloads import generators as G

pytestmark = pytest.mark.gpu


def _case(w, c_in, c_out, dtype, out_f32):
    ijk, jo = w.jagged_ijk(dup_fraction=0.01)
    g, og = H.both_grids(ijk, jo)
    km = fx.build_kernel_map(g, w.kernel_size, w.stride)
    ogo = O.output_grid(og, w.kernel_size, w.stride)
    feat, wt = G.features_and_weights(w.feat_seed + 31, og.num_voxels, c_in, c_out, w.k3, dtype)
    d_x, d_w = H.to_device_storage(feat, dtype), H.to_device_storage(wt, dtype)
    odt = torch.float32 if out_f32 else H.TORCH_DT[dtype]
    ref = O.conv(og, ogo, w.kernel_size, w.stride, feat, wt, threads=H.ORACLE_THREADS)
    return km, d_x, d_w, odt, ref, dtype, w.k3, c_in, c_out


def _check(case):
    km, d_x, d_w, odt, ref, dtype, k3, c_in, c_out = case
    out = H.nan_filled((km.n_out, c_out), odt)
    fx.sparse_conv_fwd_noalloc(km, d_x, d_w, out)
    same = fx.sparse_conv_fwd(km, d_x, d_w, out_dtype=odt)
    assert torch.equal(out, same)
    H.conv_tolerance_check(out.float().cpu().numpy(), ref, dtype, k3, c_in)


def test_two_calls_in_a_row_the_second_smaller(fx_opt):
    # small fp32 grids: the allocating entry point would pick its scalar kernel (another summation order); the
    # switch keeps it on the matrix-unit kernel that the no-allocation entry point always takes
    fx_opt("fp32_tiles", "1")
    big = _case(G.workload("lidar_small"), 64, 128, "bf16", False)          # 196 tiles x 2 slices, 27 x 64 x 128 weights
    small = _case(G.workload("sphere64"), 32, 64, "f16", True)              # 19 tiles, fewer and smaller weights
    strided = _case(G.workload("lidar_small_down"), 64, 128, "bf16", False)   # the gather kernel's tiles
    fp32 = _case(G.workload("sphere64"), 32, 32, "f32", True)               # fp32 rows on the matrix units
    for case in (big, small, strided, fp32, big, small):
        _check(case)


def test_limits_are_reported_not_faulted():
    w = G.workload("sphere64")
    ijk, jo = w.jagged_ijk()
    g, _ = H.both_grids(ijk, jo)
    km = fx.build_kernel_map(g, 3, 1)
    n = g.num_voxels
    # 27 x 512 x 512 x 2 bytes = 13.5 MiB of packed weights: beyond the static buffer
    x = torch.zeros((n, 512), dtype=torch.bfloat16, device="cuda")
    wt = torch.zeros((27, 512, 512), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(fx.FxError) as e:
        fx.sparse_conv_fwd_noalloc(km, x, wt, torch.empty((n, 512), dtype=torch.bfloat16, device="cuda"))
    assert e.value.status == -5 and "static buffer" in str(e.value)
    # a shape the matrix-unit kernels do not take (the allocating entry point sends it to the scalar kernel)
    x = torch.zeros((n, 8), dtype=torch.bfloat16, device="cuda")
    wt = torch.zeros((27, 8, 16), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(fx.FxError) as e:
        fx.sparse_conv_fwd_noalloc(km, x, wt, torch.empty((n, 16), dtype=torch.bfloat16, device="cuda"))
    assert e.value.status == -2
    # a 5x5x5 map has no tiled form
    km5 = fx.build_kernel_map(g, 5, 1)
    x = torch.zeros((n, 32), dtype=torch.bfloat16, device="cuda")
    wt = torch.zeros((125, 32, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(fx.FxError) as e:
        fx.sparse_conv_fwd_noalloc(km5, x, wt, torch.empty((n, 64), dtype=torch.bfloat16, device="cuda"))
    assert e.value.status == -2
    # and the entry point still works after the refusals
    _check(_case(w, 32, 64, "bf16", False))


def test_small_fp32_grid_meets_the_fp32_bar():
    # without the switch the two entry points run different kernels here; both meet the oracle at the fp32 bar
    km, d_x, d_w, odt, ref, dtype, k3, c_in, c_out = _case(G.workload("sphere64"), 32, 32, "f32", True)
    out = H.nan_filled((km.n_out, c_out), odt)
    fx.sparse_conv_fwd_noalloc(km, d_x, d_w, out)
    H.conv_tolerance_check(out.cpu().numpy(), ref, dtype, k3, c_in)
    H.conv_tolerance_check(fx.sparse_conv_fwd(km, d_x, d_w).cpu().numpy(), ref, dtype, k3, c_in)
