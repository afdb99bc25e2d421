"""Pins for the oracle's backward pass (O4): the gradients that a library's autograd gives for
the dense masked 3-D cross-correlation, the adjoint identities against the pinned forward
oracle, central differences of the forward oracle, and exact special cases."""
import numpy as np
import pytest
import torch

from oracle import cpu_oracle as O
from workloads import generators as G


def _cloud(seed, n, lo, hi):
    return np.random.default_rng(seed).integers(lo, hi, size=(n, 3)).astype(np.int32)


def _dense_autograd(coords_in, feat, coords_out, w, gout, K, s):
    """Scatter the features to a dense box, run torch's conv3d in float64, read the outputs at
    the active output sites, and let autograd differentiate <out, gout> with respect to the
    scattered features and the weights."""
    d0 = -(K - 1) // 2 if K % 2 else 0
    lo = np.minimum(coords_in.min(0), coords_out.min(0) * s) + d0 - s
    lo = (lo // s) * s
    hi = np.maximum(coords_in.max(0), coords_out.max(0) * s) + K + s
    shape = tuple(hi - lo + 1)
    c_in, c_out = w.shape[1], w.shape[2]
    x = torch.tensor(feat, dtype=torch.float64, requires_grad=True)
    wt = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    p = torch.from_numpy(coords_in - lo).long()
    flat = (p[:, 0] * shape[1] + p[:, 1]) * shape[2] + p[:, 2]
    dense = torch.zeros((c_in, shape[0] * shape[1] * shape[2]), dtype=torch.float64)
    dense = dense.index_copy(1, flat, x.T).reshape((c_in,) + shape)
    kern = wt.reshape(K, K, K, c_in, c_out).permute(4, 3, 0, 1, 2)
    y = torch.nn.functional.conv3d(dense[None], kern, stride=s, padding=-d0)[0]
    q = torch.from_numpy(coords_out - lo // s).long()
    out = y[:, q[:, 0], q[:, 1], q[:, 2]].T
    (out * torch.from_numpy(gout)).sum().backward()
    return x.grad.numpy(), wt.grad.numpy()


@pytest.mark.parametrize("K,s,c_in,c_out", [(3, 1, 5, 7), (2, 2, 6, 3), (1, 1, 4, 4), (5, 1, 2, 3), (3, 2, 4, 5)])
def test_matches_autograd_of_dense_masked_correlation(K, s, c_in, c_out):
    pts = np.unique(_cloud(131, 600, -7, 8), axis=0)
    gin = O.OracleGrid(pts, np.array([[0, pts.shape[0]]]))
    gout = O.output_grid(gin, K, s)
    rng = np.random.default_rng(132)
    feat = rng.standard_normal((gin.num_voxels, c_in))
    w = rng.standard_normal((K ** 3, c_in, c_out))
    gy = rng.standard_normal((gout.num_voxels, c_out))
    ref_gx, ref_gw = _dense_autograd(gin.ijk()[0], feat, gout.ijk()[0], w, gy, K, s)
    assert np.allclose(O.conv_bwd_data(gin, gout, K, s, gy, w), ref_gx, rtol=1e-12, atol=1e-12)
    assert np.allclose(O.conv_bwd_weight(gin, gout, K, s, feat, gy), ref_gw, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("K,s", [(3, 1), (2, 2)])
def test_adjoint_identities_on_a_jagged_batch(K, s):
    """<conv(x; W), g> = <x, bwd_data(g; W)> = <W, bwd_weight(x, g)> for any x, W, g."""
    w_ = G.workload("sheets_small")
    ijk, jo = w_.jagged_ijk()
    gin = O.OracleGrid(ijk, jo)
    gout = O.output_grid(gin, K, s)
    rng = np.random.default_rng(141)
    x = rng.standard_normal((gin.num_voxels, 3))
    w = rng.standard_normal((K ** 3, 3, 4))
    g = rng.standard_normal((gout.num_voxels, 4))
    lhs = float((O.conv(gin, gout, K, s, x, w) * g).sum())
    assert np.isclose(lhs, float((x * O.conv_bwd_data(gin, gout, K, s, g, w)).sum()), rtol=1e-11)
    assert np.isclose(lhs, float((w * O.conv_bwd_weight(gin, gout, K, s, x, g)).sum()), rtol=1e-11)


def test_central_differences_of_the_forward_oracle():
    pts = np.unique(_cloud(151, 60, 0, 5), axis=0)
    g = O.OracleGrid(pts, np.array([[0, pts.shape[0]]]))
    rng = np.random.default_rng(152)
    x = rng.standard_normal((g.num_voxels, 2))
    w = rng.standard_normal((27, 2, 3))
    gy = rng.standard_normal((g.num_voxels, 3))
    loss = lambda x_, w_: float((O.conv(g, g, 3, 1, x_, w_) * gy).sum())
    gx, gw = O.conv_bwd_data(g, g, 3, 1, gy, w), O.conv_bwd_weight(g, g, 3, 1, x, gy)
    h = 1e-5
    for (i, c) in [(0, 0), (7, 1), (g.num_voxels - 1, 0)]:
        d = np.zeros_like(x)
        d[i, c] = h
        assert np.isclose((loss(x + d, w) - loss(x - d, w)) / (2 * h), gx[i, c], rtol=1e-7, atol=1e-9)
    for (k, ci, co) in [(13, 0, 0), (0, 1, 2), (26, 0, 1), (4, 1, 1)]:
        d = np.zeros_like(w)
        d[k, ci, co] = h
        assert np.isclose((loss(x, w + d) - loss(x, w - d)) / (2 * h), gw[k, ci, co], rtol=1e-7, atol=1e-9)


def test_k1_reduces_to_two_gemms():
    w_ = G.workload("sheets_small")
    ijk, jo = w_.jagged_ijk()
    g = O.OracleGrid(ijk, jo)
    rng = np.random.default_rng(161)
    x = rng.standard_normal((g.num_voxels, 6))
    w = rng.standard_normal((1, 6, 9))
    gy = rng.standard_normal((g.num_voxels, 9))
    assert np.allclose(O.conv_bwd_data(g, g, 1, 1, gy, w), gy @ w[0].T, rtol=1e-13, atol=1e-13)
    assert np.allclose(O.conv_bwd_weight(g, g, 1, 1, x, gy)[0], x.T @ gy, rtol=1e-12, atol=1e-12)


def test_all_ones_count_pairs_per_offset_and_per_input():
    w_ = G.workload("sphere64")
    ijk, jo = w_.jagged_ijk()
    g = O.OracleGrid(ijk, jo)
    nb = O.kernel_map(g, g, 3, 1)
    n = g.num_voxels
    gw = O.conv_bwd_weight(g, g, 3, 1, np.ones((n, 2)), np.ones((n, 3)))
    assert np.array_equal(gw, np.broadcast_to((nb >= 0).sum(0).astype(np.float64)[:, None, None], (27, 2, 3)))
    gx = O.conv_bwd_data(g, g, 3, 1, np.ones((n, 3)), np.ones((27, 2, 3)))
    uses = np.bincount(nb[nb >= 0], minlength=n).astype(np.float64)       # pairs each input takes part in
    assert np.array_equal(gx, np.repeat(3.0 * uses[:, None], 2, axis=1))


def test_strided_map_uses_every_input_once():
    pts = np.unique(_cloud(171, 400, -9, 9), axis=0)
    gin = O.OracleGrid(pts, np.array([[0, pts.shape[0]]]))
    gout = gin.coarsen2()
    nb = O.kernel_map(gin, gout, 2, 2)
    rng = np.random.default_rng(172)
    w = rng.standard_normal((8, 3, 2))
    gy = rng.standard_normal((gout.num_voxels, 2))
    gx = O.conv_bwd_data(gin, gout, 2, 2, gy, w)
    o, kappa = np.nonzero(nb >= 0)
    expect = np.zeros_like(gx)
    expect[nb[o, kappa]] = np.einsum("pic,pc->pi", w[kappa], gy[o])
    assert np.allclose(gx, expect, rtol=1e-13, atol=1e-13)
    assert np.array_equal(np.sort(nb[o, kappa]), np.arange(gin.num_voxels))


def test_weight_gradient_row_ranges_add_up():
    pts = np.unique(_cloud(181, 500, -6, 6), axis=0)
    g = O.OracleGrid(pts, np.array([[0, pts.shape[0]]]))
    rng = np.random.default_rng(182)
    x = rng.standard_normal((g.num_voxels, 4))
    gy = rng.standard_normal((g.num_voxels, 5))
    full = O.conv_bwd_weight(g, g, 3, 1, x, gy)
    a = O.conv_bwd_weight(g, g, 3, 1, x, gy, 0, 100)
    b = O.conv_bwd_weight(g, g, 3, 1, x, gy, 100, g.num_voxels)
    assert np.allclose(a + b, full, rtol=1e-12, atol=1e-12)
