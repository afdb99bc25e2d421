"""Seeded synthetic voxel grids, features and weights.

These stand in for the paper's sparse-convolution benchmark inputs (Sec. 4.1.3:
LiDAR scans, rasterised surfaces, volumetric data), whose data is not available
here; only their structure is kept: leaf occupancy class, stencil neighbour count,
extent and channel depth.

This module holds no arithmetic of the method (no tree, no index, no convolution):
it only produces integer coordinates, random features and random weights.  It is
the one module that both the CPU oracle's tests and the HIP path's tests import.

All randomness is numpy's PCG64 (``numpy.random.default_rng(seed)``), drawn in
exactly the order written below.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np


# ----------------------------------------------------------------------------------
# helpers
# ----------------------------------------------------------------------------------

def _unique_rows(ijk: np.ndarray) -> np.ndarray:
    if ijk.shape[0] == 0:
        return ijk.reshape(0, 3).astype(np.int32)
    return np.unique(ijk.astype(np.int32), axis=0)


def _box_surface(o, s, floor: bool = True) -> np.ndarray:
    """All voxels on the faces of the axis-aligned box [o, o+s) (1 voxel thick).

    ``floor=False`` leaves out the k = o[2] face (a building without a floor)."""
    o = np.asarray(o, dtype=np.int64)
    s = np.asarray(s, dtype=np.int64)
    parts = []
    ax = [np.arange(o[a], o[a] + s[a], dtype=np.int64) for a in range(3)]
    for a in range(3):
        others = [b for b in range(3) if b != a]
        g0, g1 = np.meshgrid(ax[others[0]], ax[others[1]], indexing="ij")
        for side, c in enumerate((o[a], o[a] + s[a] - 1)):
            if a == 2 and side == 0 and not floor:
                continue
            p = np.empty((g0.size, 3), dtype=np.int64)
            p[:, a] = c
            p[:, others[0]] = g0.ravel()
            p[:, others[1]] = g1.ravel()
            parts.append(p)
    return np.concatenate(parts, axis=0)


def _plane_patch(axis: int, c: int, o2, s2) -> np.ndarray:
    others = [b for b in range(3) if b != axis]
    a0 = np.arange(o2[0], o2[0] + s2[0], dtype=np.int64)
    a1 = np.arange(o2[1], o2[1] + s2[1], dtype=np.int64)
    g0, g1 = np.meshgrid(a0, a1, indexing="ij")
    p = np.empty((g0.size, 3), dtype=np.int64)
    p[:, axis] = c
    p[:, others[0]] = g0.ravel()
    p[:, others[1]] = g1.ravel()
    return p


# ----------------------------------------------------------------------------------
# the five grid families
# ----------------------------------------------------------------------------------

def sphere_shell(box: int = 64, radius: float = 28.0, thickness: float = 0.5) -> np.ndarray:
    """Voxelised shell of a sphere centred in a ``box``^3 domain (deterministic)."""
    c = box / 2.0
    a = np.arange(box, dtype=np.float64) + 0.5 - c
    d = np.sqrt(a[:, None, None] ** 2 + a[None, :, None] ** 2 + a[None, None, :] ** 2)
    m = np.abs(d - radius) <= thickness
    return np.argwhere(m).astype(np.int32)


def indoor_scene(seed: int, extent: int = 512, size_div: int = 1) -> np.ndarray:
    """Surfaces of 6-12 random axis-aligned boxes and plane patches in extent^3.

    ``size_div`` > 1 shrinks every primitive by that factor (small test variants);
    the random draws are the same for any value."""
    rng = np.random.default_rng(seed)
    n = int(rng.integers(6, 13))
    parts = []
    for _ in range(n):
        u = rng.random()
        if u < 0.7:
            s = np.minimum(np.maximum(rng.integers(40, 113, size=3) // size_div, 3), extent)
            o = [int(rng.integers(0, extent - int(s[a]) + 1)) for a in range(3)]
            parts.append(_box_surface(o, s, floor=True))
        else:
            ax = int(rng.integers(0, 3))
            c = int(rng.integers(0, extent))
            s = np.minimum(np.maximum(rng.integers(96, 257, size=2) // size_div, 3), extent)
            o = [int(rng.integers(0, extent - int(s[a]) + 1)) for a in range(2)]
            parts.append(_plane_patch(ax, c, o, s))
    return _unique_rows(np.concatenate(parts, axis=0))


def lidar_like(seed: int = 3000, extent_xy: int = 2048, n_rings: int = 64,
               n_boxes: int = 50) -> np.ndarray:
    """Concentric scan rings on a ground plane plus random box obstacles."""
    rng = np.random.default_rng(seed)
    c = extent_xy / 2.0
    a = np.arange(extent_xy, dtype=np.float64) + 0.5 - c
    d = np.sqrt(a[:, None] ** 2 + a[None, :] ** 2)
    r = np.arange(n_rings, dtype=np.float64)
    rho = 16.0 + (c - 32.0) * (r / (n_rings - 1)) ** 1.5
    mask = np.zeros(d.shape, dtype=bool)
    for q in rho:
        mask |= np.abs(d - q) <= 1.0
    ij = np.argwhere(mask)
    ground = np.concatenate([ij, np.full((ij.shape[0], 1), 2, dtype=ij.dtype)], axis=1)
    parts = [ground.astype(np.int64)]
    for _ in range(n_boxes):
        s = (int(rng.integers(32, 97)), int(rng.integers(32, 97)), int(rng.integers(16, 57)))
        o = (int(rng.integers(0, extent_xy - s[0] + 1)),
             int(rng.integers(0, extent_xy - s[1] + 1)), 2)
        parts.append(_box_surface(o, s, floor=False))
    return _unique_rows(np.concatenate(parts, axis=0))


def random_walk_sheets(seed: int, extent: int = 128, n_sheets: int = 3) -> np.ndarray:
    """Height-field sheets whose height follows two random walks (one per axis)."""
    rng = np.random.default_rng(seed)
    parts = []
    for _ in range(n_sheets):
        a = np.cumsum(rng.integers(-1, 2, size=extent))
        b = np.cumsum(rng.integers(-1, 2, size=extent))
        h0 = int(rng.integers(24, 104))
        h = np.clip(h0 + a[:, None] + b[None, :], 0, extent - 1).astype(np.int64)
        ii, jj = np.meshgrid(np.arange(extent), np.arange(extent), indexing="ij")
        parts.append(np.stack([ii.ravel(), jj.ravel(), h.ravel()], axis=1))
        # vertical fill between neighbouring columns, so the sheet stays watertight
        for (di, dj) in ((1, 0), (0, 1)):
            h_a = h[: extent - di, : extent - dj]
            h_b = h[di:, dj:]
            lo = np.minimum(h_a, h_b)
            hi = np.maximum(h_a, h_b)
            i0, j0 = np.meshgrid(np.arange(extent - di), np.arange(extent - dj), indexing="ij")
            for t in (1, 2):
                sel = (hi - lo) > t
                if sel.any():
                    parts.append(np.stack([i0[sel], j0[sel], lo[sel] + t], axis=1))
    return _unique_rows(np.concatenate(parts, axis=0))


def volumetric_bodies(seed: int, extent: int = 192, n_bodies: int = 7, origin: int = 0) -> np.ndarray:
    """Solid balls and thick spherical shells (4-8 voxels thick) at random places in extent^3:
    the densest of the three sparsity classes of Sec. 4.1.3 (rasterised volumes, leaf occupancy
    above 40 %).  ``origin`` shifts the whole scene (negative origins put bodies
    across the coordinate planes)."""
    rng = np.random.default_rng(seed)
    a = np.arange(extent, dtype=np.float64) + 0.5
    m = np.zeros((extent, extent, extent), dtype=bool)
    for b in range(n_bodies):
        r = float(rng.uniform(0.12, 0.22) * extent)
        c = rng.uniform(r + 1, extent - r - 1, size=3)
        d2 = ((a - c[0]) ** 2)[:, None, None] + ((a - c[1]) ** 2)[None, :, None] + ((a - c[2]) ** 2)[None, None, :]
        if b % 2 == 0:
            m |= d2 <= r * r
        else:
            t = float(rng.uniform(4.0, 8.0))
            m |= (d2 <= r * r) & (d2 >= (r - t) ** 2)
    return (np.argwhere(m) + origin).astype(np.int32)


def mixed_scene(seed: int, extent_xy: int = 768, n_rings: int = 24, n_boxes: int = 12, n_balls: int = 4,
                n_shells: int = 4) -> np.ndarray:
    """One grid that mixes the three sparsity classes of Sec. 4.1.3: LiDAR-like ground rings and hollow boxes
    (leaf occupancy of a few per cent), thin spherical shells (one voxel thick) and solid balls (full leaves) --
    the input per-leaf dispatch is for.  Everything lies in extent_xy x extent_xy x 96."""
    rng = np.random.default_rng(seed)
    parts = [lidar_like(seed + 1, extent_xy=extent_xy, n_rings=n_rings, n_boxes=n_boxes)]
    zext = 96
    a = np.arange(zext, dtype=np.float64) + 0.5
    for b in range(n_balls + n_shells):
        r = float(rng.uniform(18.0, 40.0))
        cx, cy = rng.uniform(r + 1, extent_xy - r - 1, size=2)
        cz = float(rng.uniform(r * 0.3, zext - 1))
        lo_x, lo_y = int(cx - r - 1), int(cy - r - 1)
        n = int(2 * r + 3)
        ax, ay = np.arange(lo_x, lo_x + n) + 0.5, np.arange(lo_y, lo_y + n) + 0.5
        d2 = ((ax - cx) ** 2)[:, None, None] + ((ay - cy) ** 2)[None, :, None] + ((a - cz) ** 2)[None, None, :]
        m = d2 <= r * r
        if b >= n_balls:
            m &= d2 >= (r - 1.0) ** 2
        v = np.argwhere(m)
        v[:, 0] += lo_x
        v[:, 1] += lo_y
        parts.append(v.astype(np.int32))
    return _unique_rows(np.concatenate(parts, axis=0))


def gaussian_points(seed: int, n: int, sigma: float = 64.0) -> np.ndarray:
    """Integer coordinates of points drawn from an isotropic normal distribution.

    Mirrors the shape of the paper's grid-construction benchmark input (Sec. 4.1.1);
    may contain duplicates and negative coordinates."""
    rng = np.random.default_rng(seed)
    p = rng.normal(0.0, sigma, size=(n, 3))
    return np.floor(p).astype(np.int32)


def gaussian_point_cloud(seed: int, n: int, sigma: float = 1.0) -> np.ndarray:
    """xyz [n,3] float32 drawn from an isotropic normal distribution: the input of the paper's
    grid-construction benchmark (Sec. 4.1.1) before it is turned into voxel coordinates."""
    rng = np.random.default_rng(seed)
    return rng.normal(0.0, sigma, size=(n, 3)).astype(np.float32)


# ----------------------------------------------------------------------------------
# batches, features, weights
# ----------------------------------------------------------------------------------

def shuffle_and_duplicate(ijk: np.ndarray, seed: int, dup_fraction: float = 0.0) -> np.ndarray:
    """Random row order, optionally with a fraction of rows repeated at random places."""
    rng = np.random.default_rng(seed)
    n = ijk.shape[0]
    out = ijk[rng.permutation(n)]
    if dup_fraction > 0.0 and n > 0:
        m = max(1, int(round(n * dup_fraction)))
        extra = out[rng.integers(0, n, size=m)]
        out = np.concatenate([out, extra], axis=0)
        out = out[rng.permutation(out.shape[0])]
    return np.ascontiguousarray(out.astype(np.int32))


def make_jagged(grids: List[np.ndarray]) -> Tuple[np.ndarray, np.ndarray]:
    """Concatenate per-grid coordinate lists into (jdata [sum N_b, 3], joffsets [B, 2])."""
    B = len(grids)
    joff = np.zeros((B, 2), dtype=np.int64)
    pos = 0
    for b, g in enumerate(grids):
        joff[b, 0] = pos
        pos += g.shape[0]
        joff[b, 1] = pos
    if B == 0:
        return np.zeros((0, 3), dtype=np.int32), joff
    data = np.concatenate([g.reshape(-1, 3) for g in grids], axis=0).astype(np.int32)
    return np.ascontiguousarray(data), joff


def round_to_dtype(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp32 values to the storage dtype (round-to-nearest-even); returns fp32
    values that are exactly representable in that dtype."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "f16":
        return x.astype(np.float16).astype(np.float32)
    if dtype == "bf16":
        u = x.view(np.uint32).astype(np.uint64)
        lsb = (u >> 16) & 1
        u = (u + 0x7FFF + lsb) & 0xFFFF0000
        return u.astype(np.uint32).view(np.float32).reshape(x.shape)
    raise ValueError(dtype)


def to_storage_bits(x: np.ndarray, dtype: str) -> np.ndarray:
    """Bit pattern of already-rounded fp32 values in the storage dtype."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "f16":
        return x.astype(np.float16)
    if dtype == "bf16":
        return (x.view(np.uint32) >> 16).astype(np.uint16)
    raise ValueError(dtype)


def features_and_weights(seed: int, n_voxels: int, c_in: int, c_out: int, k3: int,
                         dtype: str) -> Tuple[np.ndarray, np.ndarray]:
    """feat ~ N(0,1) [n, c_in]; W ~ N(0, 1/(k3*c_in)) [k3, c_in, c_out]; both rounded
    to the storage dtype and returned as fp32 arrays holding those rounded values."""
    rng = np.random.default_rng(seed)
    feat = rng.standard_normal(size=(n_voxels, c_in), dtype=np.float32)
    w = rng.standard_normal(size=(k3, c_in, c_out), dtype=np.float32)
    w *= np.float32(1.0 / np.sqrt(k3 * c_in))
    return round_to_dtype(feat, dtype), round_to_dtype(w, dtype)


@dataclass
class Workload:
    name: str
    grids: List[np.ndarray]           # per-grid unique coordinates, unshuffled
    kernel_size: int
    stride: int
    c_in: int
    c_out: int
    dtype: str                        # "f32" | "f16" | "bf16"
    feat_seed: int
    shuffle_seed: int
    note: str = ""
    _jag: Optional[Tuple[np.ndarray, np.ndarray]] = field(default=None, repr=False)

    def jagged_ijk(self, dup_fraction: float = 0.0) -> Tuple[np.ndarray, np.ndarray]:
        """Shuffled (and optionally duplicated) input coordinates + joffsets."""
        shuffled = [shuffle_and_duplicate(g, self.shuffle_seed + b, dup_fraction)
                    for b, g in enumerate(self.grids)]
        return make_jagged(shuffled)

    @property
    def n_voxels(self) -> int:
        return int(sum(g.shape[0] for g in self.grids))

    @property
    def k3(self) -> int:
        return self.kernel_size ** 3

    def feats_weights(self) -> Tuple[np.ndarray, np.ndarray]:
        return features_and_weights(self.feat_seed, self.n_voxels, self.c_in, self.c_out,
                                    self.k3, self.dtype)


def workload(name: str) -> Workload:
    """The five benchmark configurations plus small variants used by tests."""
    if name == "sphere64":          # config 1
        return Workload(name, [sphere_shell(64, 28.0, 0.5)], 3, 1, 32, 32, "f32", 1000, 1001)
    if name == "indoor4":           # config 2
        seeds = (2000, 2001, 2003, 2004)
        return Workload(name, [indoor_scene(s) for s in seeds], 3, 1, 64, 64, "f16", 2100, 2101)
    if name == "lidar1m":           # config 3
        return Workload(name, [lidar_like(3000)], 3, 1, 64, 64, "bf16", 3100, 3101)
    if name == "lidar1m_down":      # config 4
        return Workload(name, [lidar_like(3000)], 2, 2, 64, 128, "bf16", 4100, 3101)
    if name == "lidar1m_down3":     # the config-3 grid through a 3x3x3 stride-2 layer
        return Workload(name, [lidar_like(3000)], 3, 2, 64, 128, "bf16", 4300, 3101)
    if name == "sheets4":           # config 5
        return Workload(name, [random_walk_sheets(5000 + g) for g in range(4)], 3, 1, 256, 256,
                        "bf16", 5100, 5101)
    # ---- small variants (same recipes at a smaller extent), for tests ----
    if name == "indoor_small":
        return Workload(name, [indoor_scene(2000 + g, extent=128, size_div=4) for g in range(3)], 3, 1, 64, 64,
                        "f16", 2200, 2201)
    if name == "lidar_small":
        return Workload(name, [lidar_like(3001, extent_xy=256, n_rings=12, n_boxes=6)], 3, 1, 64, 64,
                        "bf16", 3200, 3201)
    if name == "lidar_small_down":
        return Workload(name, [lidar_like(3001, extent_xy=256, n_rings=12, n_boxes=6)], 2, 2, 64, 128,
                        "bf16", 4200, 3201)
    if name == "sheets_small":
        return Workload(name, [random_walk_sheets(5100 + g, extent=48, n_sheets=2) for g in range(2)],
                        3, 1, 256, 256, "bf16", 5200, 5201)
    # ---- the volumetric class (Sec. 4.1.3 c) at low depth (Sec. 3.5 scenario 1: 8 -> 16, fp32) ----
    if name == "volume1m":
        return Workload(name, [volumetric_bodies(6000, extent=224, n_bodies=8)], 3, 1, 8, 16, "f32", 6100, 6101)
    # the same volumetric grid and a fully dense block at the depth of the benchmark's middle layers
    if name == "volume1m_c64":
        return Workload(name, [volumetric_bodies(6000, extent=224, n_bodies=8)], 3, 1, 64, 64, "bf16", 6300, 6101)
    if name == "dense96":
        a = np.arange(-48, 48, dtype=np.int32)
        blk = np.stack(np.meshgrid(a, a, a, indexing="ij"), axis=-1).reshape(-1, 3)
        return Workload(name, [blk], 3, 1, 64, 64, "bf16", 6400, 6401)
    # ---- one grid mixing solid bodies, thin shells and LiDAR-like rings: the input of per-leaf dispatch ----
    if name == "mixed1m":
        return Workload(name, [mixed_scene(7100)], 3, 1, 64, 64, "bf16", 7200, 7101)
    if name == "mixed_small":
        return Workload(name, [mixed_scene(7101, extent_xy=192, n_rings=8, n_boxes=4, n_balls=2, n_shells=2)], 3, 1, 64, 64,
                        "bf16", 7300, 7102)
    if name == "volume_small":
        return Workload(name, [volumetric_bodies(6001 + g, extent=40, n_bodies=3, origin=-13 * g) for g in range(2)],
                        3, 1, 8, 16, "f32", 6200, 6201)
    raise KeyError(name)


WORKLOADS = ("sphere64", "indoor4", "lidar1m", "lidar1m_down", "sheets4")
