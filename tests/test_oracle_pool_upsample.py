"""Pins for the oracle's transposed convolution, pooling and upsampling (O5): the dense library
routines on a densified box (conv_transpose3d, max_pool3d, sums of 2x2x2 blocks, repeat), the
adjoint identity against the pinned forward oracle, and exact special cases."""
import numpy as np
import pytest
import torch

from oracle import cpu_oracle as O
from workloads import generators as G


def _cloud(seed, n, lo, hi):
    return np.unique(np.random.default_rng(seed).integers(lo, hi, size=(n, 3)).astype(np.int32), axis=0)


def _densify(coords, feat, lo, shape):
    """[C, X, Y, Z] float64 box holding feat at coords - lo and `fill` elsewhere."""
    p = coords - lo
    d = np.zeros((feat.shape[1],) + tuple(shape), dtype=np.float64)
    d[:, p[:, 0], p[:, 1], p[:, 2]] = feat.T
    return d


@pytest.mark.parametrize("K", [2, 3])
@pytest.mark.parametrize("c_in,c_out", [(3, 5), (4, 2)])
def test_transposed_convolution_matches_dense_conv_transpose3d(c_in, c_out, K):
    pts = _cloud(201, 500, -8, 9)
    fine = O.OracleGrid(pts, np.array([[0, pts.shape[0]]]))
    coarse = fine.coarsen2()
    rng = np.random.default_rng(202)
    z = rng.standard_normal((coarse.num_voxels, c_in))
    w = rng.standard_normal((K ** 3, c_in, c_out))
    cc, fc = coarse.ijk()[0], fine.ijk()[0]
    lo = cc.min(0)
    shape = cc.max(0) - lo + 1
    dense = torch.from_numpy(_densify(cc, z, lo, shape))[None]
    # torch's weight layout for conv_transpose3d is [C_in, C_out, kD, kH, kW]
    kern = torch.from_numpy(w.reshape(K, K, K, c_in, c_out)).permute(3, 4, 0, 1, 2).contiguous()
    # fine box starting at 2*lo; for K = 3 the offsets are -1, 0, 1: padding 1 shifts the taps, output_padding 1
    # keeps the last fine row of the box
    y = torch.nn.functional.conv_transpose3d(dense, kern, stride=2, padding=K // 2 if K == 3 else 0,
                                             output_padding=1 if K == 3 else 0)[0].numpy()
    q = fc - 2 * lo
    ref = y[:, q[:, 0], q[:, 1], q[:, 2]].T
    assert np.allclose(O.conv_transpose(fine, coarse, K, 2, z, w), ref, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("K,s", [(2, 2), (3, 1), (3, 2)])
def test_transposed_convolution_is_the_adjoint_of_the_forward_oracle(K, s):
    """<conv(x; W), z> = <x, conv_transpose(z; W^T)> with W^T[kappa] = W[kappa] transposed."""
    w_ = G.workload("sheets_small")
    ijk, jo = w_.jagged_ijk()
    gin = O.OracleGrid(ijk, jo)
    gout = O.output_grid(gin, K, s)
    rng = np.random.default_rng(211)
    x = rng.standard_normal((gin.num_voxels, 3))
    w = rng.standard_normal((K ** 3, 3, 4))
    z = rng.standard_normal((gout.num_voxels, 4))
    lhs = float((O.conv(gin, gout, K, s, x, w) * z).sum())
    rhs = float((x * O.conv_transpose(gin, gout, K, s, z, np.ascontiguousarray(w.transpose(0, 2, 1)))).sum())
    assert np.isclose(lhs, rhs, rtol=1e-11)
    # and it is the oracle's input gradient with the weights of the forward direction
    assert np.allclose(O.conv_transpose(gin, gout, K, s, z, np.ascontiguousarray(w.transpose(0, 2, 1))),
                       O.conv_bwd_data(gin, gout, K, s, z, w), rtol=1e-12, atol=1e-12)


def test_pooling_matches_dense_pooling_of_the_densified_box():
    pts = _cloud(221, 900, -9, 10)
    fine = O.OracleGrid(pts, np.array([[0, pts.shape[0]]]))
    coarse = fine.coarsen2()
    rng = np.random.default_rng(222)
    z = rng.standard_normal((fine.num_voxels, 4))
    fc, cc = fine.ijk()[0], coarse.ijk()[0]
    lo = 2 * cc.min(0)
    shape = 2 * (cc.max(0) - cc.min(0) + 1)
    q = cc - cc.min(0)
    # max: inactive sites hold -inf so that they never win
    p = fc - lo
    d = np.full((4,) + tuple(shape), -np.inf)
    d[:, p[:, 0], p[:, 1], p[:, 2]] = z.T
    mx = torch.nn.functional.max_pool3d(torch.from_numpy(d)[None], 2)[0].numpy()
    assert np.array_equal(O.pool2(fine, coarse, "max", z), mx[:, q[:, 0], q[:, 1], q[:, 2]].T)
    # mean over the active children = (sum over the 2x2x2 block with zeros) / (number of active children)
    dz = _densify(fc, z, lo, shape)
    occ = _densify(fc, np.ones((fine.num_voxels, 1)), lo, shape)
    blk = lambda a: a.reshape(a.shape[0], shape[0] // 2, 2, shape[1] // 2, 2, shape[2] // 2, 2).sum(axis=(2, 4, 6))
    ref = (blk(dz) / np.maximum(blk(occ), 1))[:, q[:, 0], q[:, 1], q[:, 2]].T
    assert np.allclose(O.pool2(fine, coarse, "avg", z), ref, rtol=1e-13, atol=1e-13)


def test_pooling_special_cases():
    # a full 2x2x2 block of distinct values: max is the largest, mean the plain average; a lone voxel is its own pool
    a = np.arange(2, dtype=np.int32)
    pts = np.concatenate([np.stack(np.meshgrid(a, a, a, indexing="ij"), -1).reshape(-1, 3), [[10, -3, 7]]]).astype(np.int32)
    fine = O.OracleGrid(pts, np.array([[0, 9]]))
    coarse = fine.coarsen2()
    assert coarse.num_voxels == 2
    z = np.zeros((9, 1))
    idx = fine.lookup(pts)
    z[idx[:8], 0] = np.arange(1, 9)
    z[idx[8], 0] = -5.0
    o_blk = coarse.lookup(np.array([[0, 0, 0]], np.int32))[0]
    o_one = coarse.lookup(np.array([[5, -2, 3]], np.int32))[0]          # floor(-3/2) = -2
    mx, av = O.pool2(fine, coarse, "max", z), O.pool2(fine, coarse, "avg", z)
    assert mx[o_blk, 0] == 8.0 and av[o_blk, 0] == 4.5
    assert mx[o_one, 0] == -5.0 and av[o_one, 0] == -5.0


def test_upsampling_matches_dense_repeat_and_subdivision_has_all_children():
    pts = _cloud(231, 300, -6, 7)
    coarse = O.OracleGrid(pts, np.array([[0, 120], [120, pts.shape[0]]]))     # a batch of two grids
    fine = coarse.subdivide2()
    assert fine.num_voxels == 8 * coarse.num_voxels and fine.batch_size == 2
    assert np.array_equal(fine.voxel_joffsets(), 8 * coarse.voxel_joffsets())
    # every fine voxel's parent is active and every child of every coarse voxel is active
    fc, fb = fine.ijk()
    assert (coarse.lookup(fc >> 1, fb) >= 0).all()
    z = np.random.default_rng(232).standard_normal((coarse.num_voxels, 3))
    up = O.upsample2(fine, coarse, z)
    assert np.array_equal(up, z[coarse.lookup(fc >> 1, fb)])
    # dense check on the first grid: np.repeat along the three axes
    cc, cb = coarse.ijk()
    sel = cb == 0
    lo = cc[sel].min(0)
    shape = cc[sel].max(0) - lo + 1
    d = _densify(cc[sel], z[sel], lo, shape)
    big = d.repeat(2, axis=1).repeat(2, axis=2).repeat(2, axis=3)
    fsel = fb == 0
    q = fc[fsel] - 2 * lo
    assert np.array_equal(up[fsel], big[:, q[:, 0], q[:, 1], q[:, 2]].T)
    # pooling undoes upsampling exactly (max and mean of eight equal values)
    assert np.array_equal(O.pool2(fine, coarse, "max", up), z)
    assert np.allclose(O.pool2(fine, coarse, "avg", up), z, rtol=1e-15, atol=0)
    # upsampling onto a grid with orphans: rows without an active parent are zero
    extra = np.concatenate([fc[fsel][:5], [[1000, 1000, 1000]]]).astype(np.int32)
    g2 = O.OracleGrid(extra, np.array([[0, 6], [6, 6]]))
    up2 = O.upsample2(g2, coarse, z)
    orphan = g2.lookup(np.array([[1000, 1000, 1000]], np.int32), np.zeros(1, np.int32))[0]
    assert not up2[orphan].any() and np.abs(up2).sum() > 0


# ---------------------------------------------------------------- gradients of pooling and upsampling
def _fine_coarse(seed, n=900, lo=-9, hi=10):
    pts = _cloud(seed, n, lo, hi)
    fine = O.OracleGrid(pts, np.array([[0, pts.shape[0]]]))
    return fine, fine.coarsen2()


def test_pooling_gradients_match_autograd_of_the_dense_pooling():
    fine, coarse = _fine_coarse(241)
    rng = np.random.default_rng(242)
    z = rng.standard_normal((fine.num_voxels, 3))
    g = rng.standard_normal((coarse.num_voxels, 3))
    fc, cc = fine.ijk()[0], coarse.ijk()[0]
    lo = 2 * cc.min(0)
    shape = 2 * (cc.max(0) - cc.min(0) + 1)
    p, q = fc - lo, cc - cc.min(0)
    # max: a library's autograd through max_pool3d of the densified box (inactive sites at -inf never win;
    # random values have no ties)
    d = torch.full((3,) + tuple(int(s) for s in shape), -np.inf, dtype=torch.float64)
    d[:, p[:, 0], p[:, 1], p[:, 2]] = torch.from_numpy(z.T)
    d.requires_grad_(True)
    y = torch.nn.functional.max_pool3d(d[None], 2)[0]
    (y[:, q[:, 0], q[:, 1], q[:, 2]] * torch.from_numpy(g.T)).sum().backward()
    ref = d.grad[:, p[:, 0], p[:, 1], p[:, 2]].numpy().T
    assert np.array_equal(O.pool2_bwd(fine, coarse, "max", g, z), ref)
    # mean: autograd through block sums divided by the (constant) number of active children
    dz = torch.zeros((3,) + tuple(int(s) for s in shape), dtype=torch.float64)
    dz[:, p[:, 0], p[:, 1], p[:, 2]] = torch.from_numpy(z.T)
    dz.requires_grad_(True)
    occ = torch.from_numpy(_densify(fc, np.ones((fine.num_voxels, 1)), lo, shape))
    blk = lambda a: a.reshape(a.shape[0], shape[0] // 2, 2, shape[1] // 2, 2, shape[2] // 2, 2).sum(dim=(2, 4, 6))
    ym = blk(dz) / torch.clamp(blk(occ), min=1)
    (ym[:, q[:, 0], q[:, 1], q[:, 2]] * torch.from_numpy(g.T)).sum().backward()
    refm = dz.grad[:, p[:, 0], p[:, 1], p[:, 2]].numpy().T
    assert np.allclose(O.pool2_bwd(fine, coarse, "avg", g), refm, rtol=1e-13, atol=1e-13)


def test_gradients_are_the_adjoints_of_the_pinned_forward_operators():
    fine, coarse = _fine_coarse(251)
    rng = np.random.default_rng(252)
    z = rng.standard_normal((fine.num_voxels, 4))
    g = rng.standard_normal((coarse.num_voxels, 4))
    gf = rng.standard_normal((fine.num_voxels, 4))
    # mean pooling and upsampling are linear: <op(z), g> = <z, op_bwd(g)>
    assert np.isclose((O.pool2(fine, coarse, "avg", z) * g).sum(), (z * O.pool2_bwd(fine, coarse, "avg", g)).sum(), rtol=1e-11)
    assert np.isclose((O.upsample2(fine, coarse, g) * gf).sum(), (g * O.upsample2_bwd(fine, coarse, gf)).sum(), rtol=1e-11)
    # max pooling is piecewise linear: pool(z) = <selection, z>, and the gradient is that selection applied to g
    gm = O.pool2_bwd(fine, coarse, "max", g, z)
    assert np.isclose((O.pool2(fine, coarse, "max", z) * g).sum(), (z * gm).sum(), rtol=1e-11)
    # every coarse voxel hands each channel's gradient to exactly one child
    assert np.allclose(O.upsample2_bwd(fine, coarse, gm), g, rtol=0, atol=0)
    # upsampling then its gradient counts the children: upsample2_bwd(upsample2(g)) = n(o) * g
    n_children = O.upsample2_bwd(fine, coarse, np.ones((fine.num_voxels, 1)))
    assert np.allclose(O.upsample2_bwd(fine, coarse, O.upsample2(fine, coarse, g)), n_children * g, rtol=1e-13)


def test_max_pooling_gradient_with_ties_goes_to_the_first_child_in_offset_order():
    a = np.arange(2, dtype=np.int32)
    pts = np.stack(np.meshgrid(a, a, a, indexing="ij"), -1).reshape(-1, 3).astype(np.int32)
    fine = O.OracleGrid(pts, np.array([[0, 8]]))
    coarse = fine.coarsen2()
    idx = fine.lookup(pts)                   # offset order kappa = 4a + 2b + c is the order of pts
    z = np.zeros((8, 2))
    z[idx[[2, 5, 7]], 0] = 3.0               # three equal maxima in channel 0: the first (kappa = 2) wins
    z[idx, 1] = np.array([1, 9, 2, 9, 0, 0, 0, 0])      # channel 1: kappa = 1 and 3 tie
    g = np.array([[10.0, -4.0]])
    gin = O.pool2_bwd(fine, coarse, "max", g, z)
    exp = np.zeros((8, 2))
    exp[idx[2], 0] = 10.0
    exp[idx[1], 1] = -4.0
    assert np.array_equal(gin, exp)
    assert np.array_equal(O.pool2_bwd(fine, coarse, "avg", g), np.tile(g / 8.0, (8, 1)))
