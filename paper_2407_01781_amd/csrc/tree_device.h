// Device-side index lookup through the tree (Listing 1's getValue, applied at every level;
// Listing 2's node offsets; Sec. 3.3's root-tile key).
#pragma once
#include "common.h"

namespace fx {

// Root-tile key of Sec. 3.3 step 2: three 21-bit fields holding the signed tile coordinates
// (coord >> 12), each biased by 2^20 so that unsigned order of the key = signed order of
// (i, j, k) tiles.
__device__ __forceinline__ uint64_t tile_key(int i, int j, int k) {
    const uint64_t bias = 1ull << 20;
    return ((uint64_t)((int64_t)(i >> 12) + bias) << 42) | ((uint64_t)((int64_t)(j >> 12) + bias) << 21) |
           (uint64_t)((int64_t)(k >> 12) + bias);
}
__device__ __forceinline__ int upper_off(int i, int j, int k) {  // Listing 2
    return (((i & 4095) >> 7) << 10) | (((j & 4095) >> 7) << 5) | ((k & 4095) >> 7);
}
__device__ __forceinline__ int lower_off(int i, int j, int k) {  // Listing 2
    return (((i & 127) >> 3) << 8) | (((j & 127) >> 3) << 4) | ((k & 127) >> 3);
}
__device__ __forceinline__ int leaf_off(int i, int j, int k) {  // Listing 1
    return ((i & 7) << 6) | ((j & 7) << 3) | (k & 7);
}

// upper node (= rank of the root tile in (batch, key) order) or -1
__device__ __forceinline__ int find_upper(const uint64_t* __restrict__ root_key,
                                          const int32_t* __restrict__ root_batch, int n_upper, int b,
                                          uint64_t key) {
    int lo = 0, hi = n_upper;
    while (lo < hi) {
        int mid = (lo + hi) >> 1;
        int mb = root_batch[mid];
        uint64_t mk = root_key[mid];
        bool less = (mb < b) || (mb == b && mk < key);
        if (less) lo = mid + 1; else hi = mid;
    }
    if (lo < n_upper && root_batch[lo] == b && root_key[lo] == key) return lo;
    return -1;
}

// The same with a shortcut for a single root tile (the usual case): one round of independent loads instead of the
// search's dependent ones.  For the latency-bound launches of the grid build and the neighbour-leaf table; the
// leaf-window kernels keep the plain search (with the shortcut inlined their prologue ran 8 % slower).
__device__ __forceinline__ int find_upper_short(const uint64_t* __restrict__ root_key,
                                                const int32_t* __restrict__ root_batch, int n_upper, int b,
                                                uint64_t key) {
    if (n_upper == 1) return (root_batch[0] == b && root_key[0] == key) ? 0 : -1;
    return find_upper(root_key, root_batch, n_upper, b, key);
}

// child id below one node: masks/prefix are the node's word arrays
__device__ __forceinline__ int child_of(const uint64_t* __restrict__ mask, const uint32_t* __restrict__ prefix,
                                        int off) {
    const uint64_t w = mask[off >> 6];
    const uint64_t bit = 1ull << (off & 63);
    if (!(w & bit)) return -1;
    return (int)(prefix[off >> 6] + (uint32_t)__popcll(w & (bit - 1)));
}

template <bool SHORT = false>
__device__ __forceinline__ int find_leaf(const TreeView& t, int b, int i, int j, int k) {
    int u = SHORT ? find_upper_short(t.root_key, t.root_batch, t.n_upper, b, tile_key(i, j, k))
                  : find_upper(t.root_key, t.root_batch, t.n_upper, b, tile_key(i, j, k));
    if (u < 0) return -1;
    int l = child_of(t.upper_mask + (size_t)u * kUpperWords, t.upper_prefix + (size_t)u * kUpperWords,
                     upper_off(i, j, k));
    if (l < 0) return -1;
    return child_of(t.lower_mask + (size_t)l * kLowerWords, t.lower_prefix + (size_t)l * kLowerWords,
                    lower_off(i, j, k));
}

// Listing 1: index of voxel (i,j,k) inside a leaf record, or -1 if inactive.
__device__ __forceinline__ int leaf_value(const fx_leaf* __restrict__ lf, int i, int j, int k) {
    const int m = leaf_off(i, j, k), n = m >> 6;
    const uint64_t w = lf->mask[n];
    const uint64_t bit = 1ull << (m & 63);
    if (!(w & bit)) return -1;
    const uint64_t sum = n ? (lf->prefix >> (9 * (n - 1))) & 511 : 0;
    return (int)(lf->offset + (int64_t)sum + __popcll(w & (bit - 1)));
}

__device__ __forceinline__ int get_value(const TreeView& t, int b, int i, int j, int k) {
    int f = find_leaf(t, b, i, j, k);
    if (f < 0) return -1;
    return leaf_value(t.leaf + f, i, j, k);
}

}  // namespace fx
