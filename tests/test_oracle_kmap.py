"""Pins for the oracle's kernel map (O2): brute-force neighbour search, identities of the
submanifold map, and the stride-2 output-set definition."""
import numpy as np
import pytest

from oracle import cpu_oracle as O
from workloads import generators as G


def _cloud(seed, n, lo, hi):
    return np.random.default_rng(seed).integers(lo, hi, size=(n, 3)).astype(np.int32)


def _offsets(K):
    d0 = -(K - 1) // 2 if K % 2 else 0
    return [(a + d0, b + d0, c + d0) for a in range(K) for b in range(K) for c in range(K)]


def _brute_nbmap(coords_in, jidx_in, coords_out, jidx_out, K, s):
    """O(N_out * K^3 * N_in) search with plain comparisons."""
    offs = _offsets(K)
    out = np.full((coords_out.shape[0], len(offs)), -1, dtype=np.int64)
    for o in range(coords_out.shape[0]):
        for kappa, d in enumerate(offs):
            q = coords_out[o].astype(np.int64) * s + np.array(d)
            hit = np.nonzero((coords_in == q).all(axis=1) & (jidx_in == jidx_out[o]))[0]
            assert hit.size <= 1
            if hit.size:
                out[o, kappa] = hit[0]
    return out


@pytest.mark.parametrize("K,s", [(3, 1), (1, 1), (2, 2), (5, 1), (3, 2)])
def test_against_brute_force(K, s):
    grids = [_cloud(1, 120, -5, 6), _cloud(2, 90, 4090, 4102), np.zeros((0, 3), np.int32)]
    ijk, jo = G.make_jagged(grids)
    gin = O.OracleGrid(ijk, jo)
    gout = O.output_grid(gin, K, s)
    nb = O.kernel_map(gin, gout, K, s)
    ci, ji = gin.ijk()
    co, jo_ = gout.ijk()
    assert np.array_equal(nb, _brute_nbmap(ci, ji, co, jo_, K, s))


@pytest.mark.parametrize("name", ["sphere64", "sheets_small"])
def test_submanifold_identities(name):
    w = G.workload(name)
    ijk, jo = w.jagged_ijk()
    g = O.OracleGrid(ijk, jo)
    nb = O.kernel_map(g, g, 3, 1)
    n = g.num_voxels
    assert np.array_equal(nb[:, 13], np.arange(n))                     # centre tap = identity
    pairs = (nb >= 0).sum(axis=0)
    assert np.array_equal(pairs, pairs[::-1])                          # pairs[k] = pairs[26-k]
    for kappa in range(27):                                            # nb[o][k]=i <=> nb[i][26-k]=o
        o = np.nonzero(nb[:, kappa] >= 0)[0]
        i = nb[o, kappa]
        assert np.array_equal(nb[i, 26 - kappa], o)
        assert np.unique(i).size == i.size                             # injective per offset


def test_sphere_pair_count():
    w = G.workload("sphere64")
    ijk, jo = w.jagged_ijk()
    g = O.OracleGrid(ijk, jo)
    assert int((O.kernel_map(g, g, 3, 1) >= 0).sum()) == 100944


def test_stride2_output_set_and_single_use_of_inputs():
    grids = [_cloud(5, 3000, -40, 40), _cloud(6, 2000, 4000, 4200)]
    ijk, jo = G.make_jagged(grids)
    gin = O.OracleGrid(ijk, jo)
    gout = O.output_grid(gin, 2, 2)
    co, jb = gout.ijk()
    for b, pts in enumerate(grids):
        expect = {tuple(p) for p in (pts >> 1).tolist()}              # floor, also for negatives
        got = {tuple(p) for p in co[jb == b].tolist()}
        assert got == expect
    nb = O.kernel_map(gin, gout, 2, 2)
    used = nb[nb >= 0]
    assert np.array_equal(np.sort(used), np.arange(gin.num_voxels))    # every input exactly once
    assert np.all((nb >= 0).sum(axis=1) >= 1)
