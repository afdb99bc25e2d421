"""What Listings 1 and 2 and the sort keys of Sec. 3.3 mean, stated as arithmetic of their own for use as pins.

Nothing here is used by the oracle or by the HIP path, and nothing follows the listings statement by statement:
node offsets are written as positional numbers over the digits of a coordinate (a voxel coordinate splits, from the
bottom, into a base-8 digit inside its leaf, a base-16 digit inside its lower node, a base-32 digit inside its upper
node and the signed tile number above), and the value a leaf record returns for a voxel is written as the definition
the listing implements: the leaf's first index plus the voxel's rank among the leaf's active voxels in bit order.
The packed prefix field is then checked against that rank (the reading "field n-1 belongs to word n", nine bits per
field, is what makes the two agree).
"""

LEAF, LOWER, UPPER = 8, 16, 32          # fan-out per axis of the three node levels (Sec. 3.1)


def _digits(c):
    """(digit in the leaf, digit in the lower node, digit in the upper node, tile number) of one coordinate;
    floor division keeps the digits non-negative for negative coordinates, as the two's-complement masks do."""
    tile, rest = divmod(c, LEAF * LOWER * UPPER)
    upper, rest = divmod(rest, LEAF * LOWER)
    lower, leaf = divmod(rest, LEAF)
    return leaf, lower, upper, tile


def _positional(di, dj, dk, base):
    return (di * base + dj) * base + dk


def leaf_off(i, j, k):                      # what Listing 1 calls the offset of a voxel in its leaf
    return _positional(_digits(i)[0], _digits(j)[0], _digits(k)[0], LEAF)


def lower_off(i, j, k):                     # Listing 2, leaf inside its lower node
    return _positional(_digits(i)[1], _digits(j)[1], _digits(k)[1], LOWER)


def upper_off(i, j, k):                     # Listing 2, lower node inside its upper node
    return _positional(_digits(i)[2], _digits(j)[2], _digits(k)[2], UPPER)


def key_a(i, j, k):                         # Sec. 3.3 step 2: the tile numbers as three base-2^21 digits that order as signed
    bias = 1 << 20
    return _positional(_digits(i)[3] + bias, _digits(j)[3] + bias, _digits(k)[3] + bias, 1 << 21)


def key_b_low(i, j, k):                     # Sec. 3.3 step 5 without the tile id M: upper, lower, leaf offsets as one number
    return (upper_off(i, j, k) * LOWER ** 3 + lower_off(i, j, k)) * LEAF ** 3 + leaf_off(i, j, k)


def vdb_sort_key(b, i, j, k):
    """(grid, key a, key b): sorting by it is 'sort by a, then by b within a run'."""
    return (b, key_a(i, j, k), key_b_low(i, j, k))


def popcount(x):
    return bin(x).count("1")


def _leaf_bits(m_bitmask):
    """The leaf's 512 activity bits as one integer, bit = offset of the voxel in the leaf."""
    return sum(int(w) << (64 * n) for n, w in enumerate(m_bitmask))


def prefix_fields(m_prefix_sum):
    """The seven 9-bit fields of the packed prefix sum, lowest first."""
    return [(int(m_prefix_sum) >> (9 * f)) & 511 for f in range(7)]


def listing1_get_value(m_offset, m_prefix_sum, m_bitmask, i, j, k):
    """Index of voxel (i, j, k) from one leaf record (None if inactive): the leaf's first index plus the number of
    active voxels of the leaf below this one in bit order.  The count of whole words below the voxel's word must be
    what the record's prefix field for that word says."""
    bits = _leaf_bits(m_bitmask)
    pos = leaf_off(i, j, k)
    if not (bits >> pos) & 1:
        return None
    word = pos // 64
    below_words = popcount(bits & ((1 << (64 * word)) - 1))
    if word:
        assert prefix_fields(m_prefix_sum)[word - 1] == below_words
    return int(m_offset) + popcount(bits & ((1 << pos) - 1))
