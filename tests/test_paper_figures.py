"""Pins against figures the paper prints (tests/golden/*.txt, each file cites its passage)."""
import os

import numpy as np

from oracle import cpu_oracle as O

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _read(name):
    out = {}
    for line in open(os.path.join(GOLDEN, name)):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split()
        out[k] = int(v)
    return out


def test_dense_layer_accounting_of_sec_3_5():
    """On a dense N^3 grid every interior voxel has all 27 taps, so the oracle's pair count times
    2*C_in*C_out (the effective-FLOP definition of Sec. 4.1.3) and the per-voxel feature bytes
    must reproduce the paper's 6912 N^3 operations and 96 N^3 bytes."""
    g = _read("sec3_5_dense_layer_accounting.txt")
    n = 12
    ax = np.arange(n, dtype=np.int32)
    ijk = np.stack(np.meshgrid(ax, ax, ax, indexing="ij"), -1).reshape(-1, 3)
    og = O.OracleGrid(ijk, np.array([[0, len(ijk)]], dtype=np.int64))
    nb = O.kernel_map(og, og, g["kernel_size"], 1)
    coords, _ = og.ijk()
    interior = np.all((coords >= 1) & (coords <= n - 2), axis=1)
    taps = (nb >= 0).sum(1)
    assert np.all(taps[interior] == g["kernel_size"] ** 3)
    assert 2 * int(taps[interior][0]) * g["c_in"] * g["c_out"] == g["ops_per_voxel"]
    assert 4 * (g["c_in"] + g["c_out"]) == g["bytes_per_voxel"]
    # boundary voxels have fewer taps: faces 18, edges 12, corners 8
    assert sorted(set(taps.tolist())) == [8, 12, 18, 27]
    # and the convolution itself does that many multiply-adds: all-ones data count them
    feat = np.ones((len(ijk), g["c_in"]))
    w = np.ones((27, g["c_in"], g["c_out"]))
    y = O.conv(og, og, 3, 1, feat, w)
    assert np.array_equal(y[:, 0] * 2 * g["c_out"], taps * 2.0 * g["c_in"] * g["c_out"])


def test_leaf_record_of_sec_3_2():
    g = _read("sec3_2_leaf_record.txt")
    dt = O.LEAF_DTYPE
    payload = dt.fields["offset"][0].itemsize + dt.fields["prefix"][0].itemsize + dt.fields["mask"][0].itemsize
    assert payload == g["leaf_payload_bytes"] and dt.fields["origin"][1] == g["leaf_payload_bytes"]
    assert dt.fields["mask"][0].shape == (g["mask_words"],)
    # a full leaf: the 7 prefix fields hold 64, 128, ..., 448, each within 9 bits
    ax = np.arange(8, dtype=np.int32)
    ijk = np.stack(np.meshgrid(ax, ax, ax, indexing="ij"), -1).reshape(-1, 3)
    og = O.OracleGrid(ijk, np.array([[0, 512]], dtype=np.int64))
    lf = og.leaf_table()[0]
    fields = [(int(lf["prefix"]) >> (g["prefix_field_bits"] * w)) & ((1 << g["prefix_field_bits"]) - 1)
              for w in range(g["prefix_fields"])]
    assert fields == [64 * (w + 1) for w in range(g["prefix_fields"])]
    assert int(lf["prefix"]) >> (g["prefix_field_bits"] * g["prefix_fields"]) == 0
