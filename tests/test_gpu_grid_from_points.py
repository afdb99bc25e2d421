"""GPU parity: index grid built from xyz points (Sec. 3.6.2 / 4.1.1) against the oracle's
quantiser + grid, bit for bit."""
import numpy as np
import pytest
import torch

import gpu_common as H
import paper_2407_01781_amd as fx
from oracle import cpu_oracle as O
from workloads import generators as G

pytestmark = pytest.mark.gpu


def _check(clouds, origin, voxel_size):
    xyz = np.concatenate(clouds, axis=0) if clouds else np.zeros((0, 3), np.float32)
    ends = np.cumsum([c.shape[0] for c in clouds])
    jo = np.stack([np.concatenate([[0], ends[:-1]]), ends], axis=1).astype(np.int64) if clouds else np.zeros((0, 2), np.int64)
    ijk, bad = O.points_to_ijk(xyz, origin, voxel_size)
    assert bad == 0
    og = O.OracleGrid(ijk, jo)
    g = fx.build_index_grid_from_points(torch.from_numpy(xyz).cuda(), jo, origin, voxel_size)
    H.check_grid(g, og)
    return g, og


@pytest.mark.parametrize("n,sigma,size", [(1000, 1.0, 0.1), (200000, 2.0, 0.05), (200000, 0.2, 0.05), (1 << 20, 5.0, 0.03)])
def test_gaussian_clouds(n, sigma, size):
    # the input family of the grid-construction benchmark: normally distributed points; small sigma /
    # large voxels give many points per voxel, the opposite gives mostly distinct voxels
    _check([G.gaussian_point_cloud(31, n, sigma)], (0.0, 0.0, 0.0), (size, size, size))


def test_batch_anisotropic_voxels_and_shifted_origin():
    clouds = [G.gaussian_point_cloud(40 + b, 30000 + 7000 * b, 1.0 + b) for b in range(3)]
    clouds.insert(1, np.zeros((0, 3), np.float32))
    _check(clouds, (0.3, -1.7, 12.25), (0.1, 0.37, 0.05))


def test_points_on_cell_faces_and_exact_centres():
    i = np.arange(-300, 300, dtype=np.float32)
    faces = np.stack([i * 0.25, i * 0.5, -i * 0.125], axis=1).astype(np.float32)          # exactly on faces
    centres = faces + np.float32(0.0625)
    g, og = _check([faces, centres], (0.0, 0.0, 0.0), (0.25, 0.5, 0.125))
    assert g.num_voxels == og.num_voxels


def test_same_grid_as_building_from_the_oracles_cells():
    xyz = G.gaussian_point_cloud(55, 100000, 3.0)
    ijk, _ = O.points_to_ijk(xyz, (0, 0, 0), (0.1, 0.1, 0.1))
    jo = np.array([[0, xyz.shape[0]]], dtype=np.int64)
    g1 = fx.build_index_grid_from_points(torch.from_numpy(xyz).cuda(), jo, (0, 0, 0), (0.1, 0.1, 0.1))
    g2 = fx.build_index_grid(torch.from_numpy(ijk).cuda(), jo)
    a, b = g1.ijk(), g2.ijk()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


def test_empty_cloud_and_invalid_points():
    g = fx.build_index_grid_from_points(torch.zeros((0, 3), device="cuda"), np.zeros((0, 2), np.int64))
    assert g.num_voxels == 0
    bad = torch.tensor([[0.0, 0.0, 0.0], [float("nan"), 1.0, 1.0], [1.0, 3e12, 0.0]], device="cuda")
    with pytest.raises(fx.FxError, match="not finite or fall outside"):
        fx.build_index_grid_from_points(bad, np.array([[0, 3]], np.int64))
    # the library still works afterwards
    ok = fx.build_index_grid_from_points(bad[:1].contiguous(), np.array([[0, 1]], np.int64))
    assert ok.num_voxels == 1
