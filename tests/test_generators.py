"""The synthetic workloads keep the sizes the design notes quote."""
import numpy as np
import pytest

from workloads import generators as G


def test_sphere_shell_size():
    w = G.workload("sphere64")
    assert w.n_voxels == 9696
    assert w.grids[0].min() >= 0 and w.grids[0].max() < 64


def test_sheets_sizes():
    w = G.workload("sheets4")
    assert [g.shape[0] for g in w.grids] == [47881, 48748, 49025, 48843]


def test_indoor_first_grid_size():
    assert G.indoor_scene(2000).shape[0] == 203132


def test_grids_are_unique_and_int32():
    for name in ("sphere64", "indoor_small", "lidar_small", "sheets_small"):
        for g in G.workload(name).grids:
            assert g.dtype == np.int32
            assert np.unique(g, axis=0).shape[0] == g.shape[0]


def test_jagged_shuffle_and_duplicates():
    w = G.workload("sheets_small")
    ijk, jo = w.jagged_ijk(dup_fraction=0.05)
    assert jo.shape == (2, 2) and jo[0, 0] == 0 and jo[1, 1] == ijk.shape[0]
    for b, g in enumerate(w.grids):
        rows = ijk[jo[b, 0]:jo[b, 1]]
        assert rows.shape[0] > g.shape[0]
        assert np.array_equal(np.unique(rows, axis=0), g)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_rounding_is_idempotent_and_close(dtype):
    x = np.random.default_rng(0).standard_normal(1000).astype(np.float32)
    r = G.round_to_dtype(x, dtype)
    assert np.array_equal(G.round_to_dtype(r, dtype), r)
    rel = 2.0 ** -11 if dtype == "f16" else 2.0 ** -8
    assert np.all(np.abs(r - x) <= np.abs(x) * rel + 1e-7)


def test_bf16_bits_roundtrip():
    x = G.round_to_dtype(np.array([1.0, -2.5, 3.140625, 1e-3], dtype=np.float32), "bf16")
    bits = G.to_storage_bits(x, "bf16")
    back = (bits.astype(np.uint32) << 16).view(np.float32)
    assert np.array_equal(back, x)
