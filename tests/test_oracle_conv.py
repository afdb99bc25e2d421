"""Pins for the oracle's convolution (O3): a dense 3-D cross-correlation (library routine)
masked to the active sites, the K=1 per-voxel GEMM, exact special cases and linearity."""
import numpy as np
import pytest
import torch

from oracle import cpu_oracle as O
from workloads import generators as G


def _cloud(seed, n, lo, hi):
    return np.random.default_rng(seed).integers(lo, hi, size=(n, 3)).astype(np.int32)


def _dense_reference(coords_in, feat, coords_out, w, K, s):
    """Scatter to a dense box, run torch's conv3d (= cross-correlation) in float64, read
    the outputs back at the active output sites."""
    d0 = -(K - 1) // 2 if K % 2 else 0
    lo = np.minimum(coords_in.min(0), coords_out.min(0) * s) + d0 - s
    lo = (lo // s) * s                                       # keep the stride phase
    hi = np.maximum(coords_in.max(0), coords_out.max(0) * s) + K + s
    shape = (hi - lo + 1)
    c_in, c_out = w.shape[1], w.shape[2]
    dense = np.zeros((1, c_in) + tuple(shape), dtype=np.float64)
    p = coords_in - lo
    dense[0, :, p[:, 0], p[:, 1], p[:, 2]] = feat
    wt = torch.from_numpy(w.reshape(K, K, K, c_in, c_out)).permute(4, 3, 0, 1, 2).contiguous()
    # output site p_o reads inputs s*p_o + d0 + (0..K-1): start the window d0 before lo
    x = torch.from_numpy(dense)
    pad = -d0
    y = torch.nn.functional.conv3d(x, wt, stride=s, padding=pad).numpy()[0]
    q = coords_out - lo // s
    return y[:, q[:, 0], q[:, 1], q[:, 2]].T


@pytest.mark.parametrize("K,s,c_in,c_out", [(3, 1, 5, 7), (2, 2, 6, 3), (1, 1, 4, 4), (5, 1, 2, 3), (3, 2, 4, 5)])
def test_matches_dense_masked_correlation(K, s, c_in, c_out):
    pts = np.unique(_cloud(31, 600, -7, 8), axis=0)
    gin = O.OracleGrid(pts, np.array([[0, pts.shape[0]]]))
    gout = O.output_grid(gin, K, s)
    rng = np.random.default_rng(32)
    feat = rng.standard_normal((gin.num_voxels, c_in))
    w = rng.standard_normal((K ** 3, c_in, c_out))
    got = O.conv(gin, gout, K, s, feat, w)
    ref = _dense_reference(gin.ijk()[0], feat, gout.ijk()[0], w, K, s)
    assert np.allclose(got, ref, rtol=1e-12, atol=1e-12)


def test_batches_do_not_mix():
    a = np.unique(_cloud(41, 300, 0, 8), axis=0)
    b = np.unique(_cloud(42, 300, 0, 8), axis=0)
    ijk, jo = G.make_jagged([a, b])
    g = O.OracleGrid(ijk, jo)
    rng = np.random.default_rng(43)
    feat = rng.standard_normal((g.num_voxels, 3))
    w = rng.standard_normal((27, 3, 2))
    both = O.conv(g, g, 3, 1, feat, w)
    vj = g.voxel_joffsets()
    for bi, pts in enumerate([a, b]):
        gi = O.OracleGrid(pts, np.array([[0, pts.shape[0]]]))
        alone = O.conv(gi, gi, 3, 1, feat[vj[bi, 0]:vj[bi, 1]], w)
        assert np.array_equal(alone, both[vj[bi, 0]:vj[bi, 1]])


def test_k1_is_a_per_voxel_gemm():
    w_ = G.workload("sheets_small")
    ijk, jo = w_.jagged_ijk()
    g = O.OracleGrid(ijk, jo)
    rng = np.random.default_rng(51)
    feat = rng.standard_normal((g.num_voxels, 6))
    w = rng.standard_normal((1, 6, 9))
    assert np.allclose(O.conv(g, g, 1, 1, feat, w), feat @ w[0], rtol=1e-13, atol=1e-13)


def test_identity_tap_copies_the_neighbour_row_exactly():
    w_ = G.workload("sphere64")
    ijk, jo = w_.jagged_ijk()
    g = O.OracleGrid(ijk, jo)
    nb = O.kernel_map(g, g, 3, 1)
    feat = G.round_to_dtype(np.random.default_rng(61).standard_normal((g.num_voxels, 8)), "bf16")
    for kappa in (0, 5, 13, 22):
        w = np.zeros((27, 8, 8))
        w[kappa] = np.eye(8)
        out = O.conv(g, g, 3, 1, feat, w)
        expect = np.where(nb[:, kappa:kappa + 1] >= 0, feat[np.maximum(nb[:, kappa], 0)], 0.0)
        assert np.array_equal(out, expect)


def test_all_ones_counts_neighbours():
    w_ = G.workload("sphere64")
    ijk, jo = w_.jagged_ijk()
    g = O.OracleGrid(ijk, jo)
    nb = O.kernel_map(g, g, 3, 1)
    out = O.conv(g, g, 3, 1, np.ones((g.num_voxels, 4)), np.ones((27, 4, 3)))
    assert np.array_equal(out, np.repeat(4.0 * (nb >= 0).sum(1)[:, None], 3, axis=1))


def test_linearity_and_row_range():
    pts = np.unique(_cloud(71, 500, -6, 6), axis=0)
    g = O.OracleGrid(pts, np.array([[0, pts.shape[0]]]))
    rng = np.random.default_rng(72)
    f1, f2 = rng.standard_normal((2, g.num_voxels, 4))
    w1, w2 = rng.standard_normal((2, 27, 4, 5))
    y = O.conv(g, g, 3, 1, 2.0 * f1 - 3.0 * f2, w1)
    assert np.allclose(y, 2.0 * O.conv(g, g, 3, 1, f1, w1) - 3.0 * O.conv(g, g, 3, 1, f2, w1), atol=1e-12)
    y = O.conv(g, g, 3, 1, f1, w1 + 0.5 * w2)
    assert np.allclose(y, O.conv(g, g, 3, 1, f1, w1) + 0.5 * O.conv(g, g, 3, 1, f1, w2), atol=1e-12)
    part = O.conv(g, g, 3, 1, f1, w1, 10, 50)
    full = O.conv(g, g, 3, 1, f1, w1)
    assert np.array_equal(part[10:50], full[10:50]) and not part[:10].any() and not part[50:].any()


def test_host_threads_do_not_change_the_values():
    """The range-parallel harness calls the same routine on disjoint output ranges: forward rows are bit-identical,
    the gradients (sums over ranges regrouped in float64) agree to 1e-12."""
    rng = np.random.default_rng(77)
    pts = rng.integers(-6, 14, size=(3000, 3)).astype(np.int32)
    og = O.OracleGrid(pts, np.array([[0, 1200], [1200, 3000]], np.int64))
    n = og.num_voxels
    feat, wt = rng.standard_normal((n, 5)), rng.standard_normal((27, 5, 7))
    gy = rng.standard_normal((n, 7))
    assert np.array_equal(O.conv(og, og, 3, 1, feat, wt), O.conv(og, og, 3, 1, feat, wt, threads=5))
    a, b = O.conv(og, og, 3, 1, feat, wt, 100, 900), O.conv(og, og, 3, 1, feat, wt, 100, 900, threads=3)
    assert np.array_equal(a, b) and not a[:100].any() and not a[900:].any()
    np.testing.assert_allclose(O.conv_bwd_data(og, og, 3, 1, gy, wt, threads=4), O.conv_bwd_data(og, og, 3, 1, gy, wt),
                               rtol=0, atol=1e-12)
    np.testing.assert_allclose(O.conv_bwd_weight(og, og, 3, 1, feat, gy, threads=4), O.conv_bwd_weight(og, og, 3, 1, feat, gy),
                               rtol=0, atol=1e-10)
