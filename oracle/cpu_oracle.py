"""ctypes + numpy front end of the CPU oracle (test infrastructure only).

Only tests, ``__graft_entry__.smoke()`` and the benchmark's CPU-baseline leg may
import this module.  Every function marshals arrays and calls fvdb_oracle.c; the
passages each routine follows are cited there.
"""
from __future__ import annotations

import ctypes as C
from typing import Optional, Tuple

import numpy as np

from . import build as _build

_lib = None

LEAF_DTYPE = np.dtype([("offset", "<i8"), ("prefix", "<u8"), ("mask", "<u8", (8,)),
                       ("origin", "<i4", (3,)), ("batch", "<i4")])
assert LEAF_DTYPE.itemsize == 96


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        L.fo_grid_create.restype = vp
        L.fo_grid_create.argtypes = [vp, vp, i32]
        L.fo_grid_destroy.argtypes = [vp]
        L.fo_grid_num_voxels.restype = i64
        L.fo_grid_num_voxels.argtypes = [vp]
        L.fo_grid_batch_size.restype = i32
        L.fo_grid_batch_size.argtypes = [vp]
        L.fo_grid_num_leaves.restype = i64
        L.fo_grid_num_leaves.argtypes = [vp]
        L.fo_grid_counts.argtypes = [vp, vp]
        L.fo_grid_voxel_joffsets.argtypes = [vp, vp]
        L.fo_grid_ijk.argtypes = [vp, vp, vp]
        L.fo_grid_leaf_table.argtypes = [vp, vp]
        L.fo_grid_lookup.argtypes = [vp, vp, vp, i64, vp]
        L.fo_grid_coarsen2.restype = vp
        L.fo_grid_coarsen2.argtypes = [vp]
        L.fo_kernel_map.restype = i64
        L.fo_kernel_map.argtypes = [vp, vp, C.c_int, C.c_int, vp]
        L.fo_conv.restype = i64
        L.fo_conv.argtypes = [vp, vp, C.c_int, C.c_int, vp, vp, C.c_int, C.c_int, vp, i64, i64]
        L.fo_conv_bwd_data.restype = i64
        L.fo_conv_bwd_data.argtypes = [vp, vp, C.c_int, C.c_int, vp, vp, C.c_int, C.c_int, vp, i64, i64]
        L.fo_conv_bwd_weight.restype = i64
        L.fo_conv_bwd_weight.argtypes = [vp, vp, C.c_int, C.c_int, vp, vp, C.c_int, C.c_int, vp, i64, i64]
        L.fo_conv_transpose.restype = i64
        L.fo_conv_transpose.argtypes = [vp, vp, C.c_int, C.c_int, vp, vp, C.c_int, C.c_int, vp]
        L.fo_pool2.restype = i64
        L.fo_pool2.argtypes = [vp, vp, C.c_int, vp, C.c_int, vp]
        L.fo_upsample2.restype = i64
        L.fo_upsample2.argtypes = [vp, vp, vp, C.c_int, vp]
        L.fo_pool2_bwd.restype = i64
        L.fo_pool2_bwd.argtypes = [vp, vp, C.c_int, vp, vp, C.c_int, vp]
        L.fo_upsample2_bwd.restype = i64
        L.fo_upsample2_bwd.argtypes = [vp, vp, vp, C.c_int, vp]
        L.fo_points_to_ijk.restype = i64
        L.fo_points_to_ijk.argtypes = [vp, i64, vp, vp, vp]
        L.fo_grid_subdivide2.restype = vp
        L.fo_grid_subdivide2.argtypes = [vp]
        L.fo_grid_pad.restype = vp
        L.fo_grid_pad.argtypes = [vp, C.c_int]
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class OracleGrid:
    """Index grid of a jagged batch of voxel coordinates (O1)."""

    def __init__(self, ijk: Optional[np.ndarray], joffsets: Optional[np.ndarray], _handle=None):
        L = lib()
        if _handle is not None:
            self._h = _handle
        else:
            ijk = np.ascontiguousarray(ijk, dtype=np.int32).reshape(-1, 3)
            joffsets = np.ascontiguousarray(joffsets, dtype=np.int64).reshape(-1, 2)
            self._h = L.fo_grid_create(_p(ijk), _p(joffsets), joffsets.shape[0])
        if not self._h:
            raise MemoryError("oracle grid allocation failed")

    def __del__(self):
        h = getattr(self, "_h", None)
        if h and _lib is not None:
            _lib.fo_grid_destroy(h)
            self._h = None

    @property
    def num_voxels(self) -> int:
        return int(lib().fo_grid_num_voxels(self._h))

    @property
    def batch_size(self) -> int:
        return int(lib().fo_grid_batch_size(self._h))

    def counts(self) -> Tuple[int, int, int]:
        """(leaf, lower, upper) node counts."""
        c = np.zeros(3, dtype=np.int64)
        lib().fo_grid_counts(self._h, _p(c))
        return int(c[0]), int(c[1]), int(c[2])

    def voxel_joffsets(self) -> np.ndarray:
        out = np.zeros((self.batch_size, 2), dtype=np.int64)
        lib().fo_grid_voxel_joffsets(self._h, _p(out))
        return out

    def ijk(self) -> Tuple[np.ndarray, np.ndarray]:
        """Coordinates [N,3] and batch ids [N] in index order."""
        n = self.num_voxels
        out = np.zeros((n, 3), dtype=np.int32)
        jidx = np.zeros(n, dtype=np.int32)
        lib().fo_grid_ijk(self._h, _p(out), _p(jidx))
        return out, jidx

    def leaf_table(self) -> np.ndarray:
        n = int(lib().fo_grid_num_leaves(self._h))
        out = np.zeros(n, dtype=LEAF_DTYPE)
        lib().fo_grid_leaf_table(self._h, _p(out))
        return out

    def lookup(self, ijk: np.ndarray, jidx: Optional[np.ndarray] = None) -> np.ndarray:
        ijk = np.ascontiguousarray(ijk, dtype=np.int32).reshape(-1, 3)
        if jidx is not None:
            jidx = np.ascontiguousarray(jidx, dtype=np.int32)
        out = np.zeros(ijk.shape[0], dtype=np.int64)
        lib().fo_grid_lookup(self._h, _p(ijk), _p(jidx), ijk.shape[0], _p(out))
        return out

    def coarsen2(self) -> "OracleGrid":
        return OracleGrid(None, None, _handle=lib().fo_grid_coarsen2(self._h))

    def subdivide2(self) -> "OracleGrid":
        """All 8 children of every voxel (O5)."""
        return OracleGrid(None, None, _handle=lib().fo_grid_subdivide2(self._h))

    def pad(self, r: int = 1) -> "OracleGrid":
        """Every voxel within Chebyshev distance r of an active one (O7)."""
        h = lib().fo_grid_pad(self._h, int(r))
        if not h:
            raise ValueError("pad needs r >= 0")
        return OracleGrid(None, None, _handle=h)


def output_grid(gin: OracleGrid, kernel_size: int, stride: int) -> OracleGrid:
    if stride == 1:
        return gin
    if stride == 2:
        return gin.coarsen2()
    raise ValueError("stride must be 1 or 2")


def kernel_map(gin: OracleGrid, gout: OracleGrid, kernel_size: int, stride: int) -> np.ndarray:
    """nbmap [N_out, K^3] int64, -1 = no active input voxel (O2)."""
    k3 = kernel_size ** 3
    out = np.zeros((gout.num_voxels, k3), dtype=np.int64)
    r = lib().fo_kernel_map(gin._h, gout._h, kernel_size, stride, _p(out))
    if r < 0:
        raise ValueError("bad kernel-map arguments")
    return out


def _row_ranges(o_begin: int, o_end: int, threads: int):
    """[o_begin, o_end) cut into at most `threads` contiguous ranges of near-equal length."""
    n = max(0, o_end - o_begin)
    parts = max(1, min(threads, n))
    return [(o_begin + n * t // parts, o_begin + n * (t + 1) // parts) for t in range(parts)]


def conv(gin: OracleGrid, gout: OracleGrid, kernel_size: int, stride: int, feat: np.ndarray,
         w: np.ndarray, o_begin: int = 0, o_end: Optional[int] = None, threads: int = 1) -> np.ndarray:
    """out [N_out, C_out] float64 (O3); rows outside [o_begin, o_end) are zero.

    threads > 1: the same C routine is called on disjoint row ranges from that many host threads (every
    output row is still one plain sum computed by one call, so the values do not depend on `threads`)."""
    feat = np.ascontiguousarray(feat, dtype=np.float64)
    w = np.ascontiguousarray(w, dtype=np.float64)
    k3, c_in, c_out = w.shape
    assert k3 == kernel_size ** 3 and feat.shape == (gin.num_voxels, c_in)
    n_out = gout.num_voxels
    if o_end is None:
        o_end = n_out
    out = np.zeros((n_out, c_out), dtype=np.float64)
    L = lib()

    def run(rng):
        return L.fo_conv(gin._h, gout._h, kernel_size, stride, _p(feat), _p(w), c_in, c_out, _p(out), rng[0], rng[1])

    ranges = _row_ranges(max(0, o_begin), min(n_out, o_end), threads)
    if len(ranges) == 1:
        rs = [run(ranges[0])]
    else:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(len(ranges)) as ex:       # ctypes releases the interpreter lock during the call
            rs = list(ex.map(run, ranges))
    if min(rs) < 0:
        raise ValueError("bad conv arguments")
    return out


def conv_bwd_data(gin: OracleGrid, gout: OracleGrid, kernel_size: int, stride: int, grad_out: np.ndarray,
                  w: np.ndarray, threads: int = 1) -> np.ndarray:
    """Gradient with respect to the input features, [N_in, C_in] float64 (O4).

    threads > 1: the C routine runs on disjoint output ranges in that many host threads, each into its own
    array, and the arrays are added in range order (float64: the regrouping moves a sum by ~1e-16 relative)."""
    grad_out = np.ascontiguousarray(grad_out, dtype=np.float64)
    w = np.ascontiguousarray(w, dtype=np.float64)
    k3, c_in, c_out = w.shape
    assert k3 == kernel_size ** 3 and grad_out.shape == (gout.num_voxels, c_out)
    L = lib()

    def run(rng):
        part = np.zeros((gin.num_voxels, c_in), dtype=np.float64)
        r = L.fo_conv_bwd_data(gin._h, gout._h, kernel_size, stride, _p(grad_out), _p(w), c_in, c_out, _p(part),
                               rng[0], rng[1])
        if r < 0:
            raise ValueError("bad conv_bwd_data arguments")
        return part

    ranges = _row_ranges(0, gout.num_voxels, threads)
    if len(ranges) == 1:
        return run(ranges[0])
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(len(ranges)) as ex:
        parts = list(ex.map(run, ranges))
    out = parts[0]
    for part in parts[1:]:
        out += part
    return out


def conv_bwd_weight(gin: OracleGrid, gout: OracleGrid, kernel_size: int, stride: int, feat: np.ndarray,
                    grad_out: np.ndarray, o_begin: int = 0, o_end: Optional[int] = None, threads: int = 1) -> np.ndarray:
    """Gradient with respect to the weights, [K^3, C_in, C_out] float64 (O4); only the outputs
    in [o_begin, o_end) contribute.

    threads > 1: the C routine runs on disjoint output ranges in that many host threads, each into its own
    array, and the arrays are added in range order (float64: the regrouping moves the sum by ~1e-16 relative)."""
    feat = np.ascontiguousarray(feat, dtype=np.float64)
    grad_out = np.ascontiguousarray(grad_out, dtype=np.float64)
    c_in, c_out = feat.shape[1], grad_out.shape[1]
    assert feat.shape[0] == gin.num_voxels and grad_out.shape[0] == gout.num_voxels
    if o_end is None:
        o_end = gout.num_voxels
    L = lib()

    def run(rng):
        part = np.zeros((kernel_size ** 3, c_in, c_out), dtype=np.float64)
        r = L.fo_conv_bwd_weight(gin._h, gout._h, kernel_size, stride, _p(feat), _p(grad_out), c_in, c_out,
                                 _p(part), rng[0], rng[1])
        if r < 0:
            raise ValueError("bad conv_bwd_weight arguments")
        return part

    ranges = _row_ranges(o_begin, o_end, threads)
    if len(ranges) == 1:
        return run(ranges[0])
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(len(ranges)) as ex:
        parts = list(ex.map(run, ranges))
    out = parts[0]
    for part in parts[1:]:
        out += part
    return out


def conv_transpose(gin: OracleGrid, gout: OracleGrid, kernel_size: int, stride: int, z: np.ndarray,
                   w: np.ndarray) -> np.ndarray:
    """Transposed convolution over the map of a convolution gin -> gout (O5): z [N_out, C_in] lives
    on gout, the result [N_in, C_out] on gin; w [K^3, C_in, C_out]."""
    z = np.ascontiguousarray(z, dtype=np.float64)
    w = np.ascontiguousarray(w, dtype=np.float64)
    k3, c_in, c_out = w.shape
    assert k3 == kernel_size ** 3 and z.shape == (gout.num_voxels, c_in)
    out = np.zeros((gin.num_voxels, c_out), dtype=np.float64)
    if lib().fo_conv_transpose(gin._h, gout._h, kernel_size, stride, _p(z), _p(w), c_in, c_out, _p(out)) < 0:
        raise ValueError("bad conv_transpose arguments")
    return out


def pool2(fine: OracleGrid, coarse: OracleGrid, mode: str, z: np.ndarray) -> np.ndarray:
    """Max ("max") or mean ("avg") over the active children of every coarse voxel (O5)."""
    z = np.ascontiguousarray(z, dtype=np.float64)
    assert z.shape[0] == fine.num_voxels
    out = np.zeros((coarse.num_voxels, z.shape[1]), dtype=np.float64)
    if lib().fo_pool2(fine._h, coarse._h, {"max": 0, "avg": 1}[mode], _p(z), z.shape[1], _p(out)) < 0:
        raise ValueError("bad pool2 arguments")
    return out


def upsample2(fine: OracleGrid, coarse: OracleGrid, z: np.ndarray) -> np.ndarray:
    """Nearest-neighbour upsampling: every fine voxel takes the row of its parent floor(ijk/2) (O5)."""
    z = np.ascontiguousarray(z, dtype=np.float64)
    assert z.shape[0] == coarse.num_voxels
    out = np.zeros((fine.num_voxels, z.shape[1]), dtype=np.float64)
    if lib().fo_upsample2(fine._h, coarse._h, _p(z), z.shape[1], _p(out)) < 0:
        raise ValueError("bad upsample2 arguments")
    return out


def points_to_ijk(xyz: np.ndarray, origin, voxel_size) -> Tuple[np.ndarray, int]:
    """Voxel coordinates of points (O6): ijk [n,3] int32 and the number of invalid points."""
    xyz = np.ascontiguousarray(xyz, dtype=np.float32)
    o = np.ascontiguousarray(origin, dtype=np.float32).reshape(3)
    s = np.ascontiguousarray(voxel_size, dtype=np.float32).reshape(3)
    out = np.zeros((xyz.shape[0], 3), dtype=np.int32)
    bad = lib().fo_points_to_ijk(_p(xyz), xyz.shape[0], _p(o), _p(s), _p(out))
    return out, int(bad)


def pool2_bwd(fine: OracleGrid, coarse: OracleGrid, mode: str, grad_out: np.ndarray,
              z: Optional[np.ndarray] = None) -> np.ndarray:
    """Gradient of pool2 with respect to its input: grad_out [N_coarse, C] -> [N_fine, C] (O5);
    max pooling needs the forward input z."""
    g = np.ascontiguousarray(grad_out, dtype=np.float64)
    assert g.shape[0] == coarse.num_voxels
    zz = None if z is None else np.ascontiguousarray(z, dtype=np.float64)
    out = np.zeros((fine.num_voxels, g.shape[1]), dtype=np.float64)
    if lib().fo_pool2_bwd(fine._h, coarse._h, {"max": 0, "avg": 1}[mode], _p(zz), _p(g), g.shape[1], _p(out)) < 0:
        raise ValueError("bad pool2_bwd arguments")
    return out


def upsample2_bwd(fine: OracleGrid, coarse: OracleGrid, grad_out: np.ndarray) -> np.ndarray:
    """Gradient of upsample2: grad_out [N_fine, C] -> [N_coarse, C], the sum over the children (O5)."""
    g = np.ascontiguousarray(grad_out, dtype=np.float64)
    assert g.shape[0] == fine.num_voxels
    out = np.zeros((coarse.num_voxels, g.shape[1]), dtype=np.float64)
    if lib().fo_upsample2_bwd(fine._h, coarse._h, _p(g), g.shape[1], _p(out)) < 0:
        raise ValueError("bad upsample2_bwd arguments")
    return out
