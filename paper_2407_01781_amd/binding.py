"""Thin ctypes binding of the C ABI in include/fvdb_hotpath.h.

Argument marshalling only: every step of the path runs inside the HIP library.  PyTorch is
used for device memory and for the current stream.  There is no CPU fallback: if the built
library is missing, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfvdb_hotpath.so")

FX_OK = 0
DTYPES = {"f32": 0, "f16": 1, "bf16": 2}
_TORCH_DT = {torch.float32: 0, torch.float16: 1, torch.bfloat16: 2}
STATUS_NAMES = {0: "FX_OK", -1: "FX_EINVAL", -2: "FX_EUNSUPPORTED", -3: "FX_ENOMEM", -4: "FX_EDEVICE",
                -5: "FX_ERANGE"}

LEAF_DTYPE = np.dtype([("offset", "<i8"), ("prefix", "<u8"), ("mask", "<u8", (8,)),
                       ("origin", "<i4", (3,)), ("batch", "<i4")])


class FxError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2407_01781_amd.build` "
            "(there is no fallback implementation)")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    L.fx_version.restype = C.c_char_p
    L.fx_last_error.restype = C.c_char_p
    L.fx_init.restype = C.c_int
    L.fx_build_index_grid.restype = C.c_int
    L.fx_build_index_grid.argtypes = [vp, i64, vp, i32, vp, C.POINTER(vp)]
    L.fx_build_index_grid_from_points.restype = C.c_int
    L.fx_build_index_grid_from_points.argtypes = [vp, i64, vp, i32, vp, vp, vp, C.POINTER(vp)]
    L.fx_grid_info.restype = C.c_int
    L.fx_grid_info.argtypes = [vp, C.POINTER(i64), C.POINTER(i32), vp, vp]
    L.fx_grid_ijk.restype = C.c_int
    L.fx_grid_ijk.argtypes = [vp, vp, vp, vp]
    L.fx_grid_ijk_to_index.restype = C.c_int
    L.fx_grid_ijk_to_index.argtypes = [vp, vp, vp, i64, vp, vp]
    L.fx_grid_leaf_table.restype = C.c_int
    L.fx_grid_leaf_table.argtypes = [vp, vp, C.c_size_t, vp]
    L.fx_grid_coarsen2.restype = C.c_int
    L.fx_grid_coarsen2.argtypes = [vp, vp, C.POINTER(vp)]
    L.fx_grid_retain.argtypes = [vp]
    L.fx_grid_destroy.argtypes = [vp]
    L.fx_build_kernel_map_onto.restype = C.c_int
    L.fx_build_kernel_map_onto.argtypes = [vp, vp, i32, vp, C.POINTER(vp)]
    L.fx_build_kernel_map.restype = C.c_int
    L.fx_build_kernel_map.argtypes = [vp, i32, i32, vp, C.POINTER(vp), C.POINTER(vp)]
    L.fx_kmap_info.restype = C.c_int
    L.fx_kmap_info.argtypes = [vp, C.POINTER(i64), C.POINTER(i32), C.POINTER(i64), vp]
    L.fx_kmap_dense.restype = C.c_int
    L.fx_kmap_dense.argtypes = [vp, vp, vp]
    L.fx_kmap_tile_stats.restype = C.c_int
    L.fx_kmap_tile_stats.argtypes = [vp, vp]
    L.fx_kmap_tiled_bytes.restype = C.c_int
    L.fx_kmap_tiled_bytes.argtypes = [vp, C.POINTER(i64)]
    L.fx_kmap_destroy.argtypes = [vp]
    L.fx_sparse_conv_fwd.restype = C.c_int
    L.fx_sparse_conv_fwd.argtypes = [vp, vp, C.c_int, vp, i32, i32, vp, C.c_int, vp]
    L.fx_sparse_conv_fwd_noalloc.restype = C.c_int
    L.fx_sparse_conv_fwd_noalloc.argtypes = [vp, vp, C.c_int, vp, i32, i32, vp, C.c_int, vp]
    L.fx_sparse_conv_bwd_data.restype = C.c_int
    L.fx_sparse_conv_bwd_data.argtypes = [vp, vp, C.c_int, vp, i32, i32, vp, C.c_int, vp]
    L.fx_sparse_conv_bwd_weight.restype = C.c_int
    L.fx_sparse_conv_bwd_weight.argtypes = [vp, vp, vp, C.c_int, i32, i32, vp, C.c_int, vp]
    L.fx_grid_subdivide2.restype = C.c_int
    L.fx_grid_subdivide2.argtypes = [vp, vp, C.POINTER(vp)]
    L.fx_grid_pad.restype = C.c_int
    L.fx_grid_pad.argtypes = [vp, C.c_int32, vp, C.POINTER(vp)]
    L.fx_sparse_conv_leaf_fwd.restype = C.c_int
    L.fx_sparse_conv_leaf_fwd.argtypes = [vp, vp, C.c_int, vp, i32, i32, vp, C.c_int, vp]
    L.fx_sparse_conv_leaf_bwd_weight.restype = C.c_int
    L.fx_sparse_conv_leaf_bwd_weight.argtypes = [vp, vp, vp, C.c_int, i32, i32, vp, C.c_int, vp]
    L.fx_sparse_conv_leaf_bwd_data.restype = C.c_int
    L.fx_sparse_conv_leaf_bwd_data.argtypes = [vp, vp, C.c_int, vp, i32, i32, vp, C.c_int, vp]
    L.fx_sparse_conv_transpose_fwd.restype = C.c_int
    L.fx_sparse_conv_transpose_fwd.argtypes = [vp, vp, C.c_int, vp, i32, i32, vp, C.c_int, vp]
    L.fx_pool2.restype = C.c_int
    L.fx_pool2.argtypes = [vp, i32, vp, C.c_int, i32, vp, vp]
    L.fx_pool2_bwd.restype = C.c_int
    L.fx_pool2_bwd.argtypes = [vp, C.c_int, vp, vp, C.c_int, i32, vp, vp]
    L.fx_upsample2_bwd.restype = C.c_int
    L.fx_upsample2_bwd.argtypes = [vp, vp, C.c_int, i32, vp, vp]
    L.fx_upsample2.restype = C.c_int
    L.fx_upsample2.argtypes = [vp, vp, C.c_int, i32, vp, vp]
    L.fx_set_option.restype = C.c_int
    L.fx_set_option.argtypes = [C.c_char_p, i32]
    L.fx_get_option.restype = C.c_int
    L.fx_get_option.argtypes = [C.c_char_p, C.POINTER(i32)]
    L.fx_set_allocator.restype = C.c_int
    L.fx_set_allocator.argtypes = [vp, vp, vp]
    L.fx_release_cached_memory.restype = None
    L.fx_profile_enable.argtypes = [C.c_int]
    L.fx_profile_slot_count.restype = C.c_int
    L.fx_profile_slot_name.restype = C.c_char_p
    L.fx_profile_slot_name.argtypes = [C.c_int]
    L.fx_profile_read.restype = C.c_int
    L.fx_profile_read.argtypes = [C.c_int, C.POINTER(C.c_double), C.POINTER(i64)]
    return L


lib = _load()


def _check(status: int):
    if status != FX_OK:
        raise FxError(status, lib.fx_last_error().decode())


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def set_option(name: str, value: int) -> None:
    """Process-wide switch of the library (fx_set_option); -1 restores the automatic choice."""
    _check(lib.fx_set_option(name.encode(), int(value)))


def get_option(name: str) -> int:
    v = C.c_int32()
    _check(lib.fx_get_option(name.encode(), C.byref(v)))
    return v.value


_ALLOC_CB = C.CFUNCTYPE(C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p)
_FREE_CB = C.CFUNCTYPE(None, C.c_void_p, C.c_void_p, C.c_void_p)
_torch_alloc_cbs = None          # the callback objects must outlive their use by the library


def use_torch_allocator(enable: bool = True) -> None:
    """Let PyTorch's caching allocator back all device memory the library needs (fx_set_allocator), or go back
    to the library's own block cache.  Switch while no grid or kernel-map handle is alive."""
    global _torch_alloc_cbs
    if not enable:
        _check(lib.fx_set_allocator(None, None, None))
        _torch_alloc_cbs = None
        return

    def _alloc(nbytes, stream, _ctx):
        try:
            return torch.cuda.caching_allocator_alloc(int(nbytes), stream=int(stream or 0))
        except Exception:          # out of memory: the library reports FX_ENOMEM
            return None

    def _free(ptr, _stream, _ctx):
        torch.cuda.caching_allocator_delete(int(ptr))

    cbs = (_ALLOC_CB(_alloc), _FREE_CB(_free))
    _check(lib.fx_set_allocator(C.cast(cbs[0], C.c_void_p), C.cast(cbs[1], C.c_void_p), None))
    _torch_alloc_cbs = cbs


def version() -> str:
    return lib.fx_version().decode()


def profile_enable(on: bool) -> None:
    lib.fx_profile_enable(1 if on else 0)


def profile_reset() -> None:
    lib.fx_profile_reset()


def profile_read() -> dict:
    """{kernel slot name: (total ms, launches)} for slots with at least one launch."""
    out = {}
    for slot in range(lib.fx_profile_slot_count()):
        ms, cnt = C.c_double(), C.c_int64()
        _check(lib.fx_profile_read(slot, C.byref(ms), C.byref(cnt)))
        if cnt.value:
            out[lib.fx_profile_slot_name(slot).decode()] = (float(ms.value), int(cnt.value))
    return out


class IndexGrid:
    """Handle on a GridBatch built by fx_build_index_grid (or a coarsened / output grid)."""

    def __init__(self, handle: int):
        self._h = C.c_void_p(handle)
        n, b = C.c_int64(), C.c_int32()
        _check(lib.fx_grid_info(self._h, C.byref(n), C.byref(b), None, None))
        self.num_voxels, self.batch_size = int(n.value), int(b.value)

    def __del__(self):
        h = getattr(self, "_h", None)
        if h is not None and h.value:
            lib.fx_grid_destroy(h)
            self._h = None

    def counts(self) -> Tuple[int, int, int]:
        c = np.zeros(3, dtype=np.int64)
        _check(lib.fx_grid_info(self._h, None, None, None, c.ctypes.data_as(C.c_void_p)))
        return int(c[0]), int(c[1]), int(c[2])

    def voxel_joffsets(self) -> np.ndarray:
        out = np.zeros((self.batch_size, 2), dtype=np.int64)
        _check(lib.fx_grid_info(self._h, None, None, out.ctypes.data_as(C.c_void_p), None))
        return out

    def ijk(self) -> Tuple[torch.Tensor, torch.Tensor]:
        out = torch.empty((self.num_voxels, 3), dtype=torch.int32, device="cuda")
        jidx = torch.empty((self.num_voxels,), dtype=torch.int32, device="cuda")
        _check(lib.fx_grid_ijk(self._h, _ptr(out), _ptr(jidx), _stream()))
        return out, jidx

    def ijk_to_index(self, ijk: torch.Tensor, jidx: Optional[torch.Tensor] = None) -> torch.Tensor:
        assert ijk.is_cuda and ijk.dtype == torch.int32 and ijk.is_contiguous()
        n = ijk.shape[0]
        if jidx is not None:
            assert jidx.is_cuda and jidx.dtype == torch.int32 and jidx.is_contiguous() and jidx.shape[0] == n
        out = torch.empty((n,), dtype=torch.int32, device="cuda")
        _check(lib.fx_grid_ijk_to_index(self._h, _ptr(ijk), _ptr(jidx), n, _ptr(out), _stream()))
        return out

    def leaf_table(self) -> np.ndarray:
        n_leaf = self.counts()[0]
        out = np.zeros(n_leaf, dtype=LEAF_DTYPE)
        _check(lib.fx_grid_leaf_table(self._h, out.ctypes.data_as(C.c_void_p), out.nbytes, _stream()))
        return out

    def coarsen2(self) -> "IndexGrid":
        h = C.c_void_p()
        _check(lib.fx_grid_coarsen2(self._h, _stream(), C.byref(h)))
        return IndexGrid(h.value)

    def subdivide2(self) -> "IndexGrid":
        """The grid of all eight children of every voxel."""
        h = C.c_void_p()
        _check(lib.fx_grid_subdivide2(self._h, _stream(), C.byref(h)))
        return IndexGrid(h.value)

    def pad(self, r: int = 1) -> "IndexGrid":
        """The grid of all voxels within Chebyshev distance r of an active one."""
        h = C.c_void_p()
        _check(lib.fx_grid_pad(self._h, int(r), _stream(), C.byref(h)))
        return IndexGrid(h.value)


def build_index_grid(ijk: torch.Tensor, joffsets) -> IndexGrid:
    """ijk: CUDA int32 [n_rows,3]; joffsets: host int64 [B,2]."""
    assert ijk.is_cuda and ijk.dtype == torch.int32 and ijk.is_contiguous()
    jo = np.ascontiguousarray(np.asarray(joffsets, dtype=np.int64).reshape(-1, 2))
    h = C.c_void_p()
    _check(lib.fx_build_index_grid(_ptr(ijk), ijk.shape[0], jo.ctypes.data_as(C.c_void_p), jo.shape[0],
                                   _stream(), C.byref(h)))
    return IndexGrid(h.value)


def build_index_grid_from_points(xyz: torch.Tensor, joffsets, origin=(0.0, 0.0, 0.0),
                                 voxel_size=(1.0, 1.0, 1.0)) -> IndexGrid:
    """xyz: CUDA float32 [n_rows,3]; voxel (i,j,k) is the cell [origin + i*s, origin + (i+1)*s)."""
    assert xyz.is_cuda and xyz.dtype == torch.float32 and xyz.is_contiguous()
    jo = np.ascontiguousarray(np.asarray(joffsets, dtype=np.int64).reshape(-1, 2))
    o = np.ascontiguousarray(np.broadcast_to(np.asarray(origin, dtype=np.float32), (3,)))
    s = np.ascontiguousarray(np.broadcast_to(np.asarray(voxel_size, dtype=np.float32), (3,)))
    h = C.c_void_p()
    _check(lib.fx_build_index_grid_from_points(_ptr(xyz), xyz.shape[0], jo.ctypes.data_as(C.c_void_p), jo.shape[0],
                                               o.ctypes.data_as(C.c_void_p), s.ctypes.data_as(C.c_void_p),
                                               _stream(), C.byref(h)))
    return IndexGrid(h.value)


class KernelMap:
    def __init__(self, handle: int, g_in: IndexGrid, g_out: IndexGrid, kernel_size: int, stride: int):
        self._h = C.c_void_p(handle)
        self.g_in, self.g_out = g_in, g_out
        self.kernel_size, self.stride = kernel_size, stride
        self.k3 = kernel_size ** 3
        self.n_out = g_out.num_voxels

    def __del__(self):
        h = getattr(self, "_h", None)
        if h is not None and h.value:
            lib.fx_kmap_destroy(h)
            self._h = None

    def info(self) -> Tuple[int, np.ndarray]:
        """(number of active pairs, pairs per offset [K^3])."""
        n_out, k3, n_pairs = C.c_int64(), C.c_int32(), C.c_int64()
        per = np.zeros(self.k3, dtype=np.int64)
        _check(lib.fx_kmap_info(self._h, C.byref(n_out), C.byref(k3), C.byref(n_pairs),
                                per.ctypes.data_as(C.c_void_p)))
        return int(n_pairs.value), per

    def tile_stats(self) -> dict:
        s = np.zeros(4, dtype=np.int64)
        _check(lib.fx_kmap_tile_stats(self._h, s.ctypes.data_as(C.c_void_p)))
        return {"mfma_rows_issued": int(s[0]), "n_tiles": int(s[1]), "staged_rows": int(s[2]), "tile": int(s[3])}

    def tiled_bytes(self) -> int:
        b = C.c_int64()
        _check(lib.fx_kmap_tiled_bytes(self._h, C.byref(b)))
        return int(b.value)

    def dense(self) -> torch.Tensor:
        out = torch.empty((self.n_out, self.k3), dtype=torch.int32, device="cuda")
        _check(lib.fx_kmap_dense(self._h, _ptr(out), _stream()))
        return out


def release_cached_memory() -> None:
    """Return the device blocks the library keeps for reuse to the driver (waits for the device)."""
    lib.fx_release_cached_memory()


def build_kernel_map(g_in: IndexGrid, kernel_size: int, stride: int) -> KernelMap:
    hg, hk = C.c_void_p(), C.c_void_p()
    _check(lib.fx_build_kernel_map(g_in._h, kernel_size, stride, _stream(), C.byref(hg), C.byref(hk)))
    g_out = IndexGrid(hg.value)
    return KernelMap(hk.value, g_in, g_out, kernel_size, stride)


def build_kernel_map_onto(g_in: IndexGrid, g_out: IndexGrid, kernel_size: int) -> KernelMap:
    """Stride-1 map from the voxels of g_out (any grid of the same batch size) into g_in."""
    hk = C.c_void_p()
    _check(lib.fx_build_kernel_map_onto(g_in._h, g_out._h, kernel_size, _stream(), C.byref(hk)))
    return KernelMap(hk.value, g_in, g_out, kernel_size, 1)


def sparse_conv_fwd(kmap: KernelMap, feat: torch.Tensor, weights: torch.Tensor,
                    out_dtype: Optional[torch.dtype] = None, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """feat [N_in, C_in], weights [K^3, C_in, C_out] (same dtype, CUDA, contiguous)."""
    assert feat.is_cuda and weights.is_cuda and feat.is_contiguous() and weights.is_contiguous()
    assert feat.dtype == weights.dtype and feat.dtype in _TORCH_DT
    k3, c_in, c_out = weights.shape
    assert k3 == kmap.k3 and feat.shape == (kmap.g_in.num_voxels, c_in)
    out_dtype = out_dtype or feat.dtype
    if out is None:
        out = torch.empty((kmap.n_out, c_out), dtype=out_dtype, device="cuda")
    assert out.is_cuda and out.is_contiguous() and out.shape == (kmap.n_out, c_out) and out.dtype == out_dtype
    _check(lib.fx_sparse_conv_fwd(kmap._h, _ptr(feat), _TORCH_DT[feat.dtype], _ptr(weights), c_in, c_out,
                                  _ptr(out), _TORCH_DT[out_dtype], _stream()))
    return out


def sparse_conv_fwd_noalloc(kmap: KernelMap, feat: torch.Tensor, weights: torch.Tensor, out: torch.Tensor) -> torch.Tensor:
    """sparse_conv_fwd through the entry point that allocates nothing; the caller supplies `out` [N_out, C_out]."""
    assert feat.is_cuda and weights.is_cuda and feat.is_contiguous() and weights.is_contiguous()
    assert feat.dtype == weights.dtype and feat.dtype in _TORCH_DT
    k3, c_in, c_out = weights.shape
    assert k3 == kmap.k3 and feat.shape == (kmap.g_in.num_voxels, c_in)
    assert out.is_cuda and out.is_contiguous() and out.shape == (kmap.n_out, c_out) and out.dtype in _TORCH_DT
    _check(lib.fx_sparse_conv_fwd_noalloc(kmap._h, _ptr(feat), _TORCH_DT[feat.dtype], _ptr(weights), c_in, c_out,
                                          _ptr(out), _TORCH_DT[out.dtype], _stream()))
    return out


def sparse_conv_bwd_data(kmap: KernelMap, grad_out: torch.Tensor, weights: torch.Tensor,
                         out_dtype: Optional[torch.dtype] = None, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """grad_out [N_out, C_out], weights [K^3, C_in, C_out] -> gradient of the input features [N_in, C_in]."""
    assert grad_out.is_cuda and weights.is_cuda and grad_out.is_contiguous() and weights.is_contiguous()
    assert grad_out.dtype == weights.dtype and grad_out.dtype in _TORCH_DT
    k3, c_in, c_out = weights.shape
    assert k3 == kmap.k3 and grad_out.shape == (kmap.n_out, c_out)
    out_dtype = out_dtype or grad_out.dtype
    gin = out if out is not None else torch.empty((kmap.g_in.num_voxels, c_in), dtype=out_dtype, device="cuda")
    assert gin.is_cuda and gin.is_contiguous() and gin.shape == (kmap.g_in.num_voxels, c_in) and gin.dtype == out_dtype
    _check(lib.fx_sparse_conv_bwd_data(kmap._h, _ptr(grad_out), _TORCH_DT[grad_out.dtype], _ptr(weights), c_in, c_out,
                                       _ptr(gin), _TORCH_DT[out_dtype], _stream()))
    return gin


def sparse_conv_bwd_weight(kmap: KernelMap, feat: torch.Tensor, grad_out: torch.Tensor,
                           out_dtype: Optional[torch.dtype] = None, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """feat [N_in, C_in], grad_out [N_out, C_out] -> gradient of the weights [K^3, C_in, C_out]."""
    assert feat.is_cuda and grad_out.is_cuda and feat.is_contiguous() and grad_out.is_contiguous()
    assert feat.dtype == grad_out.dtype and feat.dtype in _TORCH_DT
    c_in, c_out = feat.shape[1], grad_out.shape[1]
    assert feat.shape[0] == kmap.g_in.num_voxels and grad_out.shape[0] == kmap.n_out
    out_dtype = out_dtype or feat.dtype
    gw = out if out is not None else torch.empty((kmap.k3, c_in, c_out), dtype=out_dtype, device="cuda")
    assert gw.is_cuda and gw.is_contiguous() and gw.shape == (kmap.k3, c_in, c_out) and gw.dtype == out_dtype
    _check(lib.fx_sparse_conv_bwd_weight(kmap._h, _ptr(feat), _ptr(grad_out), _TORCH_DT[feat.dtype], c_in, c_out,
                                         _ptr(gw), _TORCH_DT[out_dtype], _stream()))
    return gw


def sparse_conv_transpose_fwd(kmap: KernelMap, feat: torch.Tensor, weights: torch.Tensor,
                              out_dtype: Optional[torch.dtype] = None) -> torch.Tensor:
    """feat [N_out, C_in] on the map's output grid, weights [K^3, C_in, C_out] -> [N_in, C_out] on its input grid."""
    assert feat.is_cuda and weights.is_cuda and feat.is_contiguous() and weights.is_contiguous()
    assert feat.dtype == weights.dtype and feat.dtype in _TORCH_DT
    k3, c_in, c_out = weights.shape
    assert k3 == kmap.k3 and feat.shape == (kmap.n_out, c_in)
    out_dtype = out_dtype or feat.dtype
    out = torch.empty((kmap.g_in.num_voxels, c_out), dtype=out_dtype, device="cuda")
    _check(lib.fx_sparse_conv_transpose_fwd(kmap._h, _ptr(feat), _TORCH_DT[feat.dtype], _ptr(weights), c_in, c_out,
                                            _ptr(out), _TORCH_DT[out_dtype], _stream()))
    return out


def sparse_conv_leaf_fwd(grid: IndexGrid, feat: torch.Tensor, weights: torch.Tensor,
                         out_dtype: Optional[torch.dtype] = None) -> torch.Tensor:
    """3x3x3 submanifold convolution straight from the grid (no kernel map): feat [N, C_in],
    weights [27, C_in, C_out] -> [N, C_out]; fp32 at low depth, f16 / bf16 at C_in % 32 == 0, C_out % 64 == 0."""
    assert feat.is_cuda and weights.is_cuda and feat.is_contiguous() and weights.is_contiguous()
    assert feat.dtype == weights.dtype and feat.dtype in _TORCH_DT
    k3, c_in, c_out = weights.shape
    assert k3 == 27 and feat.shape == (grid.num_voxels, c_in)
    out_dtype = out_dtype or feat.dtype
    out = torch.empty((grid.num_voxels, c_out), dtype=out_dtype, device="cuda")
    _check(lib.fx_sparse_conv_leaf_fwd(grid._h, _ptr(feat), _TORCH_DT[feat.dtype], _ptr(weights), c_in, c_out,
                                       _ptr(out), _TORCH_DT[out_dtype], _stream()))
    return out


def sparse_conv_leaf_bwd_data(grid: IndexGrid, grad_out: torch.Tensor, weights: torch.Tensor,
                              out_dtype: Optional[torch.dtype] = None) -> torch.Tensor:
    """Input gradient of sparse_conv_leaf_fwd: grad_out [N, C_out], weights [27, C_in, C_out] -> [N, C_in]."""
    assert grad_out.is_cuda and weights.is_cuda and grad_out.is_contiguous() and weights.is_contiguous()
    assert grad_out.dtype == weights.dtype and grad_out.dtype in _TORCH_DT
    k3, c_in, c_out = weights.shape
    assert k3 == 27 and grad_out.shape == (grid.num_voxels, c_out)
    out_dtype = out_dtype or grad_out.dtype
    gin = torch.empty((grid.num_voxels, c_in), dtype=out_dtype, device="cuda")
    _check(lib.fx_sparse_conv_leaf_bwd_data(grid._h, _ptr(grad_out), _TORCH_DT[grad_out.dtype], _ptr(weights), c_in, c_out,
                                            _ptr(gin), _TORCH_DT[out_dtype], _stream()))
    return gin


def sparse_conv_leaf_bwd_weight(grid: IndexGrid, feat: torch.Tensor, grad_out: torch.Tensor,
                                out_dtype: Optional[torch.dtype] = None) -> torch.Tensor:
    """Weight gradient of sparse_conv_leaf_fwd: feat [N, C_in], grad_out [N, C_out] -> [27, C_in, C_out]."""
    assert feat.is_cuda and grad_out.is_cuda and feat.is_contiguous() and grad_out.is_contiguous()
    assert feat.dtype == grad_out.dtype and feat.dtype in _TORCH_DT
    assert feat.shape[0] == grid.num_voxels and grad_out.shape[0] == grid.num_voxels
    c_in, c_out = feat.shape[1], grad_out.shape[1]
    out_dtype = out_dtype or feat.dtype
    gw = torch.empty((27, c_in, c_out), dtype=out_dtype, device="cuda")
    _check(lib.fx_sparse_conv_leaf_bwd_weight(grid._h, _ptr(feat), _ptr(grad_out), _TORCH_DT[feat.dtype], c_in, c_out,
                                              _ptr(gw), _TORCH_DT[out_dtype], _stream()))
    return gw


def pool2(kmap: KernelMap, feat: torch.Tensor, mode: str = "max") -> torch.Tensor:
    """Max / mean over the active children; kmap is a (2,2) map, feat [N_in, C] -> [N_out, C]."""
    assert feat.is_cuda and feat.is_contiguous() and feat.dtype in _TORCH_DT
    assert feat.shape[0] == kmap.g_in.num_voxels
    out = torch.empty((kmap.n_out, feat.shape[1]), dtype=feat.dtype, device="cuda")
    _check(lib.fx_pool2(kmap._h, {"max": 0, "avg": 1}[mode], _ptr(feat), _TORCH_DT[feat.dtype], feat.shape[1],
                        _ptr(out), _stream()))
    return out


def upsample2(kmap: KernelMap, feat: torch.Tensor) -> torch.Tensor:
    """Nearest-neighbour upsampling; kmap is a (2,2) map, feat [N_out, C] -> [N_in, C]."""
    assert feat.is_cuda and feat.is_contiguous() and feat.dtype in _TORCH_DT
    assert feat.shape[0] == kmap.n_out
    out = torch.empty((kmap.g_in.num_voxels, feat.shape[1]), dtype=feat.dtype, device="cuda")
    _check(lib.fx_upsample2(kmap._h, _ptr(feat), _TORCH_DT[feat.dtype], feat.shape[1], _ptr(out), _stream()))
    return out


def pool2_bwd(kmap: KernelMap, grad_out: torch.Tensor, mode: str = "max", feat: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Gradient of pool2: grad_out [N_out, C] -> [N_in, C]; max pooling needs the forward input feat [N_in, C]."""
    assert grad_out.is_cuda and grad_out.is_contiguous() and grad_out.dtype in _TORCH_DT and grad_out.shape[0] == kmap.n_out
    if mode == "max":
        assert feat is not None and feat.is_cuda and feat.is_contiguous() and feat.dtype == grad_out.dtype
        assert feat.shape == (kmap.g_in.num_voxels, grad_out.shape[1])
    gin = torch.empty((kmap.g_in.num_voxels, grad_out.shape[1]), dtype=grad_out.dtype, device="cuda")
    _check(lib.fx_pool2_bwd(kmap._h, {"max": 0, "avg": 1}[mode], _ptr(feat) if mode == "max" else None, _ptr(grad_out),
                            _TORCH_DT[grad_out.dtype], grad_out.shape[1], _ptr(gin), _stream()))
    return gin


def upsample2_bwd(kmap: KernelMap, grad_out: torch.Tensor) -> torch.Tensor:
    """Gradient of upsample2: grad_out [N_in, C] on the fine grid -> [N_out, C], the sum over the children."""
    assert grad_out.is_cuda and grad_out.is_contiguous() and grad_out.dtype in _TORCH_DT
    assert grad_out.shape[0] == kmap.g_in.num_voxels
    gin = torch.empty((kmap.n_out, grad_out.shape[1]), dtype=grad_out.dtype, device="cuda")
    _check(lib.fx_upsample2_bwd(kmap._h, _ptr(grad_out), _TORCH_DT[grad_out.dtype], grad_out.shape[1], _ptr(gin), _stream()))
    return gin
