"""The paper's closed forms, typed out in plain Python for use as pins.

Nothing here is used by the oracle or by the HIP path: these are independent
statements of Listing 1 (sparse index from a leaf record), Listing 2 (node offsets)
and the two sort keys of Sec. 3.3, with the readings the design notes list
(64-bit shift in Listing 1; `(w & mask) == 0`; prefix field n-1 for word n;
21-bit fields of key a biased so that they order as signed numbers).
"""


def leaf_off(i, j, k):                      # Listing 1, `off`
    return (i & 7) << 6 | (j & 7) << 3 | (k & 7)


def lower_off(i, j, k):                     # Listing 2
    a = lambda n: (n & 127) >> 3
    return a(i) << 8 | a(j) << 4 | a(k)


def upper_off(i, j, k):                     # Listing 2
    a = lambda n: (n & 4095) >> 7
    return a(i) << 10 | a(j) << 5 | a(k)


def key_a(i, j, k):                         # Sec. 3.3 step 2, fields ordered as signed
    bias = 1 << 20
    return ((i >> 12) + bias) << 42 | ((j >> 12) + bias) << 21 | ((k >> 12) + bias)


def key_b_low(i, j, k):                     # Sec. 3.3 step 5 without the tile id M
    return upper_off(i, j, k) << 21 | lower_off(i, j, k) << 9 | leaf_off(i, j, k)


def vdb_sort_key(b, i, j, k):
    """(grid, key a, key b): sorting by it is 'sort by a, then by b within a run'."""
    return (b, key_a(i, j, k), key_b_low(i, j, k))


def popcount(x):
    return bin(x).count("1")


def listing1_get_value(m_offset, m_prefix_sum, m_bitmask, i, j, k):
    """Listing 1's getValue on one leaf record, 0-based (returns None if inactive)."""
    m = leaf_off(i, j, k)
    n = m >> 6
    w = int(m_bitmask[n])
    mask = 1 << (m & 63)
    if (w & mask) == 0:
        return None
    s = (int(m_prefix_sum) >> (9 * (n - 1))) & 511 if n else 0
    return s + int(m_offset) + popcount(w & (mask - 1))
