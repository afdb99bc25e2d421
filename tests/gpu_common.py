"""Helpers shared by the GPU parity tests: build the HIP path's objects and the oracle's on
the same seeded inputs."""
import os

import numpy as np
import torch

import paper_2407_01781_amd as fx
from oracle import cpu_oracle as O
from workloads import generators as G

TORCH_DT = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
ORACLE_THREADS = max(1, min(16, os.cpu_count() or 1))     # host threads the oracle's range-parallel harness may use


def nan_filled(shape, dtype) -> torch.Tensor:
    """An output buffer no element of which can pass a comparison unless the kernel wrote it."""
    return torch.full(tuple(shape), float("nan"), dtype=dtype, device="cuda")


def row_error_report(y: np.ndarray, ref: np.ndarray) -> float:
    """Largest per-row relative L2 error (the quantity the 16-bit bar bounds), for the test log."""
    num = np.linalg.norm(y.astype(np.float64) - ref, axis=1)
    den = np.maximum(np.linalg.norm(ref, axis=1), 1e-3 * np.sqrt(ref.shape[1]))
    return float((num / den).max()) if y.size else 0.0


def to_device_storage(x_f32: np.ndarray, dtype: str) -> torch.Tensor:
    """fp32 array holding values already rounded to `dtype` -> CUDA tensor of that dtype (same bits)."""
    t = torch.from_numpy(np.ascontiguousarray(x_f32))
    return t.to(TORCH_DT[dtype]).cuda().contiguous()


def both_grids(ijk: np.ndarray, joffsets: np.ndarray):
    d_ijk = torch.from_numpy(np.ascontiguousarray(ijk, dtype=np.int32).reshape(-1, 3)).cuda()
    g = fx.build_index_grid(d_ijk, joffsets)
    og = O.OracleGrid(ijk, joffsets)
    return g, og


def check_grid(g, og, ijk=None):
    assert g.num_voxels == og.num_voxels
    assert g.counts() == og.counts()
    assert np.array_equal(g.voxel_joffsets(), og.voxel_joffsets())
    c, j = g.ijk()
    oc, oj = og.ijk()
    assert np.array_equal(c.cpu().numpy(), oc)
    assert np.array_equal(j.cpu().numpy(), oj)
    lt, olt = g.leaf_table(), og.leaf_table()
    assert lt.tobytes() == olt.tobytes()


def conv_tolerance_check(y: np.ndarray, ref: np.ndarray, dtype: str, k3: int, c_in: int):
    """fp32: max-abs <= 1e-4*sqrt(K^3*C_in); fp16/bf16: per-row relative L2 <= 2e-2 (floor on the
    reference norm: 1e-3*sqrt(C_out))."""
    y = y.astype(np.float64)
    if dtype == "f32":
        err = np.abs(y - ref).max() if y.size else 0.0
        assert err <= 1e-4 * np.sqrt(k3 * c_in), err
        return err
    num = np.linalg.norm(y - ref, axis=1)
    den = np.maximum(np.linalg.norm(ref, axis=1), 1e-3 * np.sqrt(ref.shape[1]))
    rel = (num / den).max() if y.size else 0.0
    assert rel <= 2e-2, rel
    return rel
