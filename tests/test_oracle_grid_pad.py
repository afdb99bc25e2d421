"""Pins for the oracle's padded grid (O7) and for the convolution onto it: a library dilation of
the dense occupancy volume, closed forms, composition, and the dense cross-correlation read at
every site the stencil reaches."""
import numpy as np
import pytest
import scipy.ndimage as ndi
import torch

from oracle import cpu_oracle as O
from workloads import generators as G


def _cloud(seed, n, lo, hi):
    return np.unique(np.random.default_rng(seed).integers(lo, hi, size=(n, 3)).astype(np.int32), axis=0)


def _one(pts):
    return O.OracleGrid(pts, np.array([[0, pts.shape[0]]]))


def _same_grid(a, b):
    (ca, ja), (cb, jb) = a.ijk(), b.ijk()
    return np.array_equal(ca, cb) and np.array_equal(ja, jb) and np.array_equal(a.voxel_joffsets(), b.voxel_joffsets())


@pytest.mark.parametrize("r", [1, 2, 3])
def test_matches_binary_dilation_of_the_dense_volume(r):
    pts = _cloud(701, 250, -9, 12)                     # crosses zero and leaf boundaries
    lo = pts.min(0) - r - 1
    shape = pts.max(0) - lo + r + 2
    occ = np.zeros(shape, dtype=bool)
    q = pts - lo
    occ[q[:, 0], q[:, 1], q[:, 2]] = True
    ref = ndi.binary_dilation(occ, structure=np.ones((2 * r + 1,) * 3, dtype=bool))
    g = _one(pts).pad(r)
    # brute force over the whole box: active exactly where the library routine says so
    box = np.stack(np.meshgrid(*[np.arange(s) for s in shape], indexing="ij"), -1).reshape(-1, 3).astype(np.int32)
    idx = g.lookup(box + lo)
    assert np.array_equal(idx >= 0, ref.reshape(-1))
    assert g.num_voxels == int(ref.sum())
    assert np.array_equal(np.sort(idx[idx >= 0]), np.arange(g.num_voxels))     # indices are a bijection


def test_closed_forms():
    one = _one(np.array([[-3, 8, 4095]], np.int32))
    for r in (0, 1, 2, 4):
        g = one.pad(r)
        assert g.num_voxels == (2 * r + 1) ** 3
        c = g.ijk()[0]
        assert (c.min(0) == np.array([-3 - r, 8 - r, 4095 - r])).all() and (c.max(0) == np.array([-3 + r, 8 + r, 4095 + r])).all()
    # a dense a x b x c box grows by r on every side
    a, b, c = 5, 9, 3
    box = np.stack(np.meshgrid(np.arange(a), np.arange(b), np.arange(c), indexing="ij"), -1).reshape(-1, 3).astype(np.int32) + np.array([6, -4, 13], np.int32)
    assert _one(box).pad(2).num_voxels == (a + 4) * (b + 4) * (c + 4)
    # two voxels three apart along one axis: the cubes of r = 1 touch without overlap, those of r = 2 share
    # two 5 x 5 layers
    two = _one(np.array([[0, 0, 0], [3, 0, 0]], np.int32))
    assert two.pad(1).num_voxels == 54
    assert two.pad(2).num_voxels == 2 * 125 - 2 * 25


def test_identity_composition_and_containment():
    pts = _cloud(702, 400, -20, 21)
    g = _one(pts)
    assert _same_grid(g.pad(0), g)
    assert _same_grid(g.pad(1).pad(1), g.pad(2))
    assert _same_grid(g.pad(1).pad(2), g.pad(3))
    c, b = g.ijk()
    assert (g.pad(1).lookup(c, b) >= 0).all()
    # the result does not depend on input order or duplicates
    perm = np.random.default_rng(703).permutation(pts.shape[0])
    dup = np.concatenate([pts[perm], pts[:50]])
    assert _same_grid(_one(dup).pad(1), g.pad(1))
    with pytest.raises(ValueError):
        g.pad(-1)


def test_batch_members_are_padded_apart():
    a, b, e = _cloud(704, 120, 0, 10), _cloud(705, 80, -5, 3), np.zeros((0, 3), np.int32)
    ijk, jo = G.make_jagged([a, e, b])
    g = O.OracleGrid(ijk, jo).pad(1)
    assert g.batch_size == 3
    vj = g.voxel_joffsets()
    c, j = g.ijk()
    for bi, pts in enumerate([a, e, b]):
        gi = _one(pts).pad(1) if pts.shape[0] else None
        n = 0 if gi is None else gi.num_voxels
        assert vj[bi, 1] - vj[bi, 0] == n
        if n:
            assert np.array_equal(c[vj[bi, 0]:vj[bi, 1]], gi.ijk()[0]) and (j[vj[bi, 0]:vj[bi, 1]] == bi).all()


def test_convolution_onto_the_padded_grid_is_the_full_dense_correlation():
    """Stride 1, input grid S, output grid pad(S, 1): every site the 3x3x3 stencil reaches S from gets the
    dense cross-correlation's value there, and the outputs hold everything the input produces (the dense
    result is zero at every other site)."""
    pts = _cloud(706, 300, -6, 7)
    gin = _one(pts)
    gout = gin.pad(1)
    rng = np.random.default_rng(707)
    c_in, c_out = 4, 3
    feat = rng.standard_normal((gin.num_voxels, c_in))
    w = rng.standard_normal((27, c_in, c_out))
    got = O.conv(gin, gout, 3, 1, feat, w)
    ci, co = gin.ijk()[0], gout.ijk()[0]
    lo = co.min(0) - 1
    shape = co.max(0) - lo + 2
    dense = np.zeros((1, c_in) + tuple(shape))
    p = ci - lo
    dense[0, :, p[:, 0], p[:, 1], p[:, 2]] = feat
    wt = torch.from_numpy(w.reshape(3, 3, 3, c_in, c_out)).permute(4, 3, 0, 1, 2).contiguous()
    y = torch.nn.functional.conv3d(torch.from_numpy(dense), wt, padding=1).numpy()[0]
    q = co - lo
    assert np.allclose(got, y[:, q[:, 0], q[:, 1], q[:, 2]].T, rtol=1e-12, atol=1e-12)
    on = np.zeros(shape, dtype=bool)
    on[q[:, 0], q[:, 1], q[:, 2]] = True
    assert np.abs(y[:, ~on]).max() == 0.0
    # the map onto the padded grid has every (input, offset) pair exactly once: 27 pairs per input voxel
    nb = O.kernel_map(gin, gout, 3, 1)
    assert (nb >= 0).sum() == 27 * gin.num_voxels
    for kappa in range(27):
        col = nb[:, kappa]
        assert np.array_equal(np.sort(col[col >= 0]), np.arange(gin.num_voxels))
    # gradients on such a map: adjoint identities against the forward operator
    gy = rng.standard_normal(got.shape)
    gx = O.conv_bwd_data(gin, gout, 3, 1, gy, w)
    gw = O.conv_bwd_weight(gin, gout, 3, 1, feat, gy)
    assert np.isclose((gy * got).sum(), (gx * feat).sum(), rtol=1e-11)
    assert np.isclose((gy * got).sum(), (gw * w).sum(), rtol=1e-11)
    # and the input gradient is itself a dense correlation: of gy with the mirrored, transposed weights
    dy = np.zeros((1, c_out) + tuple(shape))
    dy[0, :, q[:, 0], q[:, 1], q[:, 2]] = gy
    wm = torch.from_numpy(w[::-1].copy().reshape(3, 3, 3, c_in, c_out)).permute(3, 4, 0, 1, 2).contiguous()
    dx = torch.nn.functional.conv3d(torch.from_numpy(dy), wm, padding=1).numpy()[0]
    assert np.allclose(gx, dx[:, p[:, 0], p[:, 1], p[:, 2]].T, rtol=1e-12, atol=1e-12)
