// Kernel-map build (Sec. 3.5): neighbour lookup through the tree for every output voxel and
// stencil offset, and the tiled form the MFMA convolution consumes.
#include "kmap.h"
#include "dev_timing.h"
#include "tree_device.h"

#include <string.h>

#include <algorithm>
#include <new>

namespace fx {

__host__ __device__ constexpr int delta_min(int K) { return (K & 1) ? -(K - 1) / 2 : 0; }

// ---------------------------------------------------------------------------------- leaf-centric lookup
// The unit of lookup work is one OUTPUT leaf handled by one wave (Sec. 3.5 scenario 1: gather
// offsets come straight from the tree's light metadata, amortised over the leaf).  The wave
// resolves the <= 27 input leaves that the leaf's stencil footprint can touch once, keeps
// their 80-byte records in LDS, lists the leaf's active voxels with mask popcounts, and then
// every lane evaluates Listing 1 for one (voxel, offset) entry at a time.
struct NbLeafLds {
    uint64_t mask[27][8];
    uint64_t prefix[27];
    int32_t offset[27];   // -1: no such leaf
    uint16_t active[512];
};

// Stage the neighbour records of output leaf `lf` (wave-wide; lanes 0..26 do one tree descent
// each) and list its active voxels.  Returns the number of active voxels.
template <int K>
__device__ __forceinline__ int stage_leaf(const TreeView& tin, const fx_leaf* __restrict__ lf, int stride, int lane,
                                          NbLeafLds& lds) {
    constexpr int D0 = delta_min(K);
    const int b = lf->batch;
    const int oi = lf->origin[0], oj = lf->origin[1], ok = lf->origin[2];
    const int bi = (stride * oi + D0) >> 3, bj = (stride * oj + D0) >> 3, bk = (stride * ok + D0) >> 3;
    if (lane < 27) {
        const int a = lane / 9, c = (lane / 3) % 3, d = lane % 3;
        const int hi_i = (stride * (oi + 7) + D0 + K - 1) >> 3, hi_j = (stride * (oj + 7) + D0 + K - 1) >> 3,
                  hi_k = (stride * (ok + 7) + D0 + K - 1) >> 3;
        int id = -1;
        if (bi + a <= hi_i && bj + c <= hi_j && bk + d <= hi_k)
            id = find_leaf(tin, b, (bi + a) * 8, (bj + c) * 8, (bk + d) * 8);
        if (id >= 0) {
            const fx_leaf* nl = tin.leaf + id;
#pragma unroll
            for (int w = 0; w < 8; ++w) lds.mask[lane][w] = nl->mask[w];
            lds.prefix[lane] = nl->prefix;
            lds.offset[lane] = (int32_t)nl->offset;
        } else {
#pragma unroll
            for (int w = 0; w < 8; ++w) lds.mask[lane][w] = 0;
            lds.prefix[lane] = 0;
            lds.offset[lane] = -1;
        }
    }
    int n_act = 0;
    const uint64_t lt = (1ull << lane) - 1;
#pragma unroll
    for (int w = 0; w < 8; ++w) {
        const uint64_t m = lf->mask[w];
        if ((m >> lane) & 1) lds.active[n_act + __popcll(m & lt)] = (uint16_t)(w * 64 + lane);
        n_act += __popcll(m);
    }
    return n_act;
}

// map entry (active voxel v of the staged leaf, offset kappa)
template <int K>
__device__ __forceinline__ int lookup_entry(const NbLeafLds& lds, int oi, int oj, int ok, int stride, int v, int kappa) {
    constexpr int D0 = delta_min(K);
    const int bi = (stride * oi + D0) >> 3, bj = (stride * oj + D0) >> 3, bk = (stride * ok + D0) >> 3;
    const int loc = lds.active[v];
    const int da = kappa / (K * K), db = (kappa / K) % K, dc = kappa % K;
    const int qi = stride * (oi + (loc >> 6)) + D0 + da;
    const int qj = stride * (oj + ((loc >> 3) & 7)) + D0 + db;
    const int qk = stride * (ok + (loc & 7)) + D0 + dc;
    const int slot = (((qi >> 3) - bi) * 3 + ((qj >> 3) - bj)) * 3 + ((qk >> 3) - bk);
    const int n = qi & 7;
    const uint64_t w = lds.mask[slot][n];
    const uint64_t bit = 1ull << (((qj & 7) << 3) | (qk & 7));
    if (!(w & bit)) return -1;
    const uint64_t sum = n ? (lds.prefix[slot] >> (9 * (n - 1))) & 511 : 0;
    return lds.offset[slot] + (int)sum + __popcll(w & (bit - 1));
}

// Neighbour-leaf table: for every output leaf, the ids of the <= 27 input leaves its stencil
// footprint can touch (-1: none).  One thread per (leaf, slot): a million independent tree
// descents run at full occupancy here instead of inside the latency-bound tile builder.
// The thread of slot 0 also notes, for every tile of kTileT consecutive outputs that starts inside
// its leaf, that the tile's first voxel lies in this leaf.
// INV: the table of the INVERSE of a 3x3x3 stride-2 map.  The "outputs" are then the fine voxels p and their
// "neighbours" the coarse voxels (p - delta) / 2 for the offsets delta in {-1,0,1}^3 with p - delta even on
// every axis (exactly the pairs (coarse o, offset delta) of the forward map with 2 o + delta = p); tin is
// the coarse grid.  A fine leaf at origin 8t touches coarse coordinates 4t-1 .. 4t+4: two leaves per axis.
template <int K, bool INV>
__device__ __forceinline__ void leaf_neighbors_item(const TreeView& tin, const TreeView& tout, int stride, int64_t n_out,
                                                    int64_t e, int32_t* __restrict__ nbr, int32_t* __restrict__ tile_first_leaf,
                                                    int dense_min, int32_t* __restrict__ dense_leaves, int32_t* __restrict__ n_dense) {
    constexpr int D0 = delta_min(K);
    const int f = (int)(e / 27), slot = (int)(e - (int64_t)f * 27);
    const fx_leaf* lf = tout.leaf + f;
    if (slot == 0) {
        const int64_t begin = lf->offset, end = f + 1 < tout.n_leaf ? tout.leaf[f + 1].offset : n_out;
        for (int64_t t = (begin + kTileT - 1) / kTileT; t * kTileT < end; ++t) tile_first_leaf[t] = f;
        // per-leaf dispatch: the locally dense leaves are listed for the leaf-window kernel
        if (dense_min > 0 && (int)(end - begin) >= dense_min) dense_leaves[atomicAdd(n_dense, 1)] = f;
    }
    const int oi = lf->origin[0], oj = lf->origin[1], ok = lf->origin[2];
    const int bi = INV ? ((oi - 1) >> 1) >> 3 : (stride * oi + D0) >> 3, bj = INV ? ((oj - 1) >> 1) >> 3 : (stride * oj + D0) >> 3,
              bk = INV ? ((ok - 1) >> 1) >> 3 : (stride * ok + D0) >> 3;
    const int hi_i = INV ? ((oi + 8) >> 1) >> 3 : (stride * (oi + 7) + D0 + K - 1) >> 3,
              hi_j = INV ? ((oj + 8) >> 1) >> 3 : (stride * (oj + 7) + D0 + K - 1) >> 3,
              hi_k = INV ? ((ok + 8) >> 1) >> 3 : (stride * (ok + 7) + D0 + K - 1) >> 3;
    const int a = slot / 9, c = (slot / 3) % 3, d = slot % 3;
    int id = -1;
    if (bi + a <= hi_i && bj + c <= hi_j && bk + d <= hi_k)
        id = find_leaf<true>(tin, lf->batch, (bi + a) * 8, (bj + c) * 8, (bk + d) * 8);
    nbr[e] = id;
}

template <int K, bool INV = false>
__global__ void k_leaf_neighbors(TreeView tin, TreeView tout, int stride, int64_t n_out, int32_t* __restrict__ nbr,
                                 int32_t* __restrict__ tile_first_leaf, int dense_min, int32_t* __restrict__ dense_leaves,
                                 int32_t* __restrict__ n_dense) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= (int64_t)tout.n_leaf * 27) return;
    leaf_neighbors_item<K, INV>(tin, tout, stride, n_out, e, nbr, tile_first_leaf, dense_min, dense_leaves, n_dense);
}

// The table of the map that is expected next, launched by the grid build before the host knows the counts of the
// grid it has just built (tout): they come from the device header (the view's own are not set) and the launch covers
// the leaf capacity.  self: the map of the grid onto itself (tin is ignored).
template <int K>
__global__ void k_leaf_links(TreeView tin, TreeView tout, int self, int stride, const GridHeader* __restrict__ hdr,
                             int32_t* __restrict__ nbr, int32_t* __restrict__ tile_first_leaf) {
    if (hdr->overflow) return;                 // a level did not fit: the tree is incomplete and the build is repeated
    tout.n_upper = hdr->n_upper; tout.n_lower = hdr->n_lower; tout.n_leaf = hdr->n_leaf;
    if (self) tin = tout;
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= (int64_t)tout.n_leaf * 27) return;
    leaf_neighbors_item<K, false>(tin, tout, stride, hdr->n_voxels, e, nbr, tile_first_leaf, 0, nullptr, nullptr);
}

// stage_leaf with the neighbour leaves read from the table
__device__ __forceinline__ int stage_leaf_from_table(const TreeView& tin, const fx_leaf* __restrict__ lf,
                                                     const int32_t* __restrict__ nbr_row, int lane, NbLeafLds& lds) {
    if (lane < 27) {
        const int id = nbr_row[lane];
        if (id >= 0) {
            const fx_leaf* nl = tin.leaf + id;
#pragma unroll
            for (int w = 0; w < 8; ++w) lds.mask[lane][w] = nl->mask[w];
            lds.prefix[lane] = nl->prefix;
            lds.offset[lane] = (int32_t)nl->offset;
        } else {
#pragma unroll
            for (int w = 0; w < 8; ++w) lds.mask[lane][w] = 0;
            lds.prefix[lane] = 0;
            lds.offset[lane] = -1;
        }
    }
    int n_act = 0;
    const uint64_t lt = (1ull << lane) - 1;
#pragma unroll
    for (int w = 0; w < 8; ++w) {
        const uint64_t m = lf->mask[w];
        if ((m >> lane) & 1) lds.active[n_act + __popcll(m & lt)] = (uint16_t)(w * 64 + lane);
        n_act += __popcll(m);
    }
    return n_act;
}

// LDS traffic of one wave is processed in order, so a wave that writes its own staging area and
// then reads it only needs the compiler to keep that order.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// ---------------------------------------------------------------------------------- dense map
// [n_out, K^3] int32, written offset-minor so that consecutive lanes write consecutive entries.
constexpr int kNbWavesPerBlock = 4;

template <int K>
__global__ void __launch_bounds__(64 * kNbWavesPerBlock)
k_nbmap(TreeView tin, TreeView tout, int stride, int32_t* __restrict__ nbmap) {
    constexpr int K3 = K * K * K;
    __shared__ NbLeafLds lds_all[kNbWavesPerBlock];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int f_raw = blockIdx.x * kNbWavesPerBlock + wave;
    const bool valid = f_raw < tout.n_leaf;
    const int f = valid ? f_raw : tout.n_leaf - 1;  // surplus waves repeat the last leaf's set-up, write nothing
    NbLeafLds& lds = lds_all[wave];
    const fx_leaf* lf = tout.leaf + f;
    const int n_act = stage_leaf<K>(tin, lf, stride, lane, lds);
    __syncthreads();
    const int oi = lf->origin[0], oj = lf->origin[1], ok = lf->origin[2];
    const int64_t out0 = lf->offset * (int64_t)K3;
    const int total = valid ? n_act * K3 : 0;
    for (int e = lane; e < total; e += 64) {
        const int v = e / K3, kappa = e - v * K3;
        nbmap[out0 + e] = lookup_entry<K>(lds, oi, oj, ok, stride, v, kappa);
    }
}

// ---------------------------------------------------------------------------------- tiled form
constexpr int kPackThreads = kTileT;          // one thread per output slot
constexpr int kPackWaves = kPackThreads / 64;
constexpr int kHaloHashSlots = 2048;
constexpr int kLdsLeafRows = 56;             // leaves of a tile whose neighbour rows are kept in LDS
constexpr int kRecHashSlots = 512;           // de-duplication of the neighbour leaves of those rows
constexpr int kMaxRecs = 80;                 // distinct neighbour-leaf records kept in LDS
// Provisional 16-bit entry codes of the index pass: a window row (< kTileT), kCodeNear | offset of a row in the
// index neighbourhood of the window, kCodeHalo | hash slot of a row farther away, or none.
constexpr uint32_t kCodeNone = 0xFFFFu, kCodeHalo = 0x8000u, kCodeNear = 0x4000u;
// Rows just outside a submanifold tile's own index range (in VDB order nearly all of a tile's outside rows lie within a
// few thousand indices of it) are marked in a bitmap over [o0 - kNearSpan, o0 + kTileT + kNearSpan): one LDS atomic
// without a return value per reference, and the bitmap's prefix popcounts are the ascending order.  Only rows
// beyond that go through the hash.
constexpr int kNearSpan = 4096;
constexpr int kNearBits = 2 * kNearSpan + kTileT, kNearWords = kNearBits / 32;
static_assert(kHaloHashSlots <= 0x4000 && kTileT <= 0x4000 && kNearBits <= 0x4000, "entry codes are 16 bits");
static_assert(kNearWords <= kTileT, "one thread per bitmap word");

typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;
typedef __attribute__((ext_vector_type(4))) int32_t i32x4_t;
typedef __attribute__((ext_vector_type(16))) uint32_t u32x16_t;

// LDS of one tile builder.  Regions, who writes and who reads them, phase by phase (every phase boundary below
// is a __syncthreads()):
//   staging    writes stage.leaf_off, stage.rec_hash / slot_rec / rec_id, then rec_mask / rec_base / nbr_rows
//   mask pass  reads  stage.leaf_off, nbr_rows, rec_mask;            writes vox, slot_mask
//   sort       reads  slot_mask;                                      writes key (scratch, then slot per position)
//   index pass reads  key, vox, slot_mask, nbr_rows, rec_mask, rec_base;  writes halo.* (or reads slot_base)
//   halo rank  reads  halo.halo, halo.halo_slot, halo.near_bits;      writes slot_rank (over rec_mask, dead by then), near_prefix
//   emission   reads  slot_rank, near_bits, near_prefix
// The three arms of `u` are never live together: stage ends with the mask pass, halo / slot_base begin after
// the sort.
struct PackLds {
    uint64_t rec_mask[(kMaxRecs + 1) * 8];    // mBitMask of Listing 1 per staged record; record kMaxRecs stays all zero
    int32_t rec_base[(kMaxRecs + 1) * 8];     // per mask word: mOffset + the prefix-sum field that precedes it
    int16_t nbr_rows[kLdsLeafRows * 27];      // neighbours of the tile's first leaves: >= 0 record, -1 none, -2 not staged
    uint32_t vox[kTileT];                     // per slot: leaf of the tile | word << 9 | bit << 12 | origin parities << 18
    uint32_t slot_mask[kTileT];               // per slot: taps with an active input
    uint32_t key[kTileT];                     // sort scratch, then the slot at every position of the final order
    union alignas(16) {
        struct {
            int32_t leaf_off[kTileT];         // first index of every leaf of the tile
            int32_t rec_hash[kRecHashSlots];  // leaf id or -1
            uint16_t slot_rec[kRecHashSlots]; // hash slot -> record, 0xFFFF: not staged
            int32_t rec_id[kMaxRecs];
        } stage;
        struct {
            int32_t hash[kHaloHashSlots];     // open addressing over the rows outside the window
            int32_t halo[kMaxHalo];           // the distinct ones in insertion order
            uint16_t halo_slot[kMaxHalo];     // and their hash slots
            uint32_t near_bits[kNearWords];   // rows near the window: bit (row - (o0 - kNearSpan))
            uint32_t near_prefix[kNearWords]; // rows marked in the words before each word
        } halo;
        uint32_t slot_base[kTileT];           // direct tiles: first list entry of each column
    } u;
    uint32_t group_mask[kGroupsPerTile];
    uint32_t group_dst[kGroupsPerTile];      // final position (tile_group_of(wave, slot)) of each block of the mask-sorted order
    uint32_t wave_mask[kTileWaves];
    uint32_t wave_block0[kTileWaves];
    uint32_t wave_sums[kPackWaves];
    int32_t n_halo, n_blocks, n_pair_blocks, overflow, n_rec, any_left_out;
};
static_assert(sizeof(PackLds) <= 40 * 1024, "four tile builders per compute unit");
static_assert(sizeof(uint16_t) * kHaloHashSlots <= sizeof(uint64_t) * kMaxRecs * 8, "slot_rank lives in rec_mask");

__device__ __forceinline__ uint64_t shfl_xor_u64(uint64_t v, int j) {
    const uint32_t lo = (uint32_t)__shfl_xor((int)(uint32_t)v, j);
    const uint32_t hi = (uint32_t)__shfl_xor((int)(uint32_t)(v >> 32), j);
    return ((uint64_t)hi << 32) | lo;
}

// bitonic sort of one key per thread over the whole block (ascending by thread id)
__device__ __forceinline__ uint32_t block_sort_keys32(uint32_t v, uint32_t* lds) {
    const int tid = threadIdx.x;
    for (int k = 2; k <= kPackThreads; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            uint32_t o;
            if (j >= 64) {
                lds[tid] = v;
                __syncthreads();
                o = lds[tid ^ j];
                __syncthreads();
            } else {
                o = (uint32_t)__shfl_xor((int)v, j);
            }
            const bool up = ((tid & k) == 0), lower = ((tid & j) == 0);
            const bool take_min = (lower == up);
            v = take_min ? (v < o ? v : o) : (v > o ? v : o);
        }
    }
    return v;
}

// exclusive scan of one value per thread over the block
__device__ __forceinline__ uint32_t block_scan_excl(uint32_t v, uint32_t* wave_sums, uint32_t* total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t incl = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_up(incl, d);
        if (lane >= d) incl += o;
    }
    if (lane == 63) wave_sums[wave] = incl;
    __syncthreads();
    uint32_t base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kPackWaves; ++w) {
        const uint32_t s = wave_sums[w];
        if (w < wave) base += s;
        tot += s;
    }
    __syncthreads();
    *total = tot;
    return base + incl - v;
}

// position of the r-th (0-based) set bit of m (r < popcount(m))
__device__ __forceinline__ int select64(uint64_t m, int r) {
    uint32_t x = (uint32_t)m;
    int pos = 0;
    int c = __popc(x);
    if (r >= c) { r -= c; x = (uint32_t)(m >> 32); pos = 32; }
#pragma unroll
    for (int sh = 16; sh >= 1; sh >>= 1) {
        c = __popc(x & ((1u << sh) - 1u));
        if (r >= c) { r -= c; x >>= sh; pos += sh; }
    }
    return pos;
}

// Where tap (a, b, c) of the voxel at word wn, row j, column k of its leaf looks: the slot 0..26 of the
// neighbour-leaf table, the mask word n2 and the bit inside it (Listing 1's offset, split), all relative to
// the voxel's own leaf, whose origin is a multiple of 8 and drops out.  The three axes are independent, so a
// thread packs, once, one byte per tap coordinate and axis: bits 0-1 the leaf step s (0..2) along the axis, bits
// 2-4 the coordinate inside that leaf, bit 5 "this tap coordinate exists" (TapAxes); a tap is then three byte
// extractions with wave-uniform positions.
//   forward maps   query = stride * p + D0 + (a, b, c); the table's first slot is the leaf of stride * origin + D0
//   INV            (the inverse of the 3x3x3 stride-2 map) tap (a, b, c) of fine voxel p names the coarse voxel
//                  (p + 1 - (a, b, c)) / 2 and only when that is even on every axis; the table's first slot is the
//                  leaf of (origin - 1) / 2, so the parity of origin / 8 (one bit per axis) comes in
struct TapAxes { uint32_t i, j, k; };

template <int K, bool INV>
__device__ __forceinline__ uint32_t tap_axis(int stride, int x, int par) {      // x: the voxel's coordinate inside its leaf
    uint32_t packed = 0;
#pragma unroll
    for (int a = 0; a < K; ++a) {
        int step, in, ok = 1;
        if (INV) {
            const int t = x + 1 - a, u = 4 * par + (t >> 1);
            ok = !(t & 1);
            step = (u >> 3) + 1 - par;
            in = u & 7;
        } else {
            constexpr int D0 = delta_min(K), S0 = D0 < 0 ? -1 : 0;      // floor(D0 / 8)
            const int t = stride * x + D0 + a;
            step = (t >> 3) - S0;
            in = t & 7;
        }
        packed |= (uint32_t)(step | (in << 2) | (ok << 5)) << (8 * a);
    }
    return packed;
}

template <int K, bool INV>
__device__ __forceinline__ TapAxes tap_axes(int stride, int wn, int j, int k, int par) {
    return TapAxes{tap_axis<K, INV>(stride, wn, par & 1), tap_axis<K, INV>(stride, j, (par >> 1) & 1),
                   tap_axis<K, INV>(stride, k, (par >> 2) & 1)};
}

// tap (a, b, c), wave-uniform: slot of the neighbour-leaf table, mask word, bit, and whether the tap exists
__device__ __forceinline__ void tap_query(const TapAxes& t, int a, int b, int c, int& slot, int& n2, int& bit6, bool& ok) {
    const uint32_t qi = (t.i >> (8 * a)) & 0xFFu, qj = (t.j >> (8 * b)) & 0xFFu, qk = (t.k >> (8 * c)) & 0xFFu;
    slot = (int)((qi & 3u) * 9u + (qj & 3u) * 3u + (qk & 3u));
    n2 = (int)((qi >> 2) & 7u);
    bit6 = (int)((((qj >> 2) & 7u) << 3) | ((qk >> 2) & 7u));
    ok = ((qi & qj & qk) >> 5) & 1u;
}

// Mask word n2 of the neighbour leaf in slot `slot` of tile-leaf `lo` and the index of that word's first voxel
// (Listing 1: mOffset + prefix field).  A missing leaf reads the all-zero record; a leaf whose record is not
// staged (rows beyond kLdsLeafRows, records beyond kMaxRecs) is fetched from the grid.
__device__ __forceinline__ void neighbour_word(const PackLds& L, const TreeView& tin, const int32_t* __restrict__ nbr_row_global,
                                               int lo, int slot, int n2, uint64_t& w, int32_t& base) {
    const int v = lo < kLdsLeafRows ? (int)L.nbr_rows[lo * 27 + slot] : -2;
    const int rec = v >= 0 ? v : kMaxRecs;
    w = L.rec_mask[rec * 8 + n2];
    base = L.rec_base[rec * 8 + n2];
    if (__builtin_expect(v == -2, 0)) {
        const int id = nbr_row_global[slot];
        if (id >= 0) {
            const fx_leaf* nl = tin.leaf + id;
            w = nl->mask[n2];
            const uint64_t npre = nl->prefix;
            base = (int32_t)nl->offset + (n2 ? (int32_t)((npre >> (9 * (n2 - 1))) & 511) : 0);
        }
    }
}

// a fresh read of an LDS word that other waves update with atomics
__device__ __forceinline__ int32_t lds_peek(const int32_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

__device__ __forceinline__ uint32_t popc_below(uint64_t w, int bit6) {   // set bits of w below position bit6
    const uint32_t wlo = (uint32_t)w, whi = (uint32_t)(w >> 32);
    const uint32_t mlo = bit6 >= 32 ? 0xFFFFFFFFu : ((1u << bit6) - 1u);
    const uint32_t mhi = bit6 >= 32 ? ((1u << (bit6 - 32)) - 1u) : 0u;
    return (uint32_t)(__popc(wlo & mlo) + __popc(whi & mhi));
}

// One workgroup per tile of kTileT consecutive outputs.  SUBM: input grid == output grid, so the tile's own
// index range is the window; otherwise there is no window.  DEDUP: rows outside the window are de-duplicated in
// the halo table (a stride-1 map between two grids: no window, all rows in the table); without it the tile is
// "direct".  Phases:
//   staging     the distinct neighbour leaves of the tile's leaves, their records into LDS
//   mask pass   thread = output voxel: which of its K^3 taps have an active input (bit tests only; for the 3x3x3
//               stride-1 stencil three taps per mask-word read)
//   sort, deal  voxels ordered by tap mask, cut into column blocks, blocks dealt to the convolution's waves
//   index pass  thread = column of the final order, laid out as the id blocks are (voxel column, wave slot):
//               Listing 1's prefix + popcount for the taps of the wave's union mask, one uniform step per offset;
//               rows outside the window enter the halo table; the 16-bit entries stay in registers
//   halo rank, emission   the halo rows ranked; every thread writes its own entries, a wave 128 consecutive bytes
template <int K, bool SUBM, bool INV = false, bool DEDUP = SUBM>
__global__ void __launch_bounds__(kPackThreads, 8)
k_build_tiles(TreeView tin, TreeView tout, int stride, const int32_t* __restrict__ leaf_nbr,
              const int32_t* __restrict__ tile_first_leaf, int64_t n_out, TileHeader* __restrict__ tile_hdr,
              uint16_t* __restrict__ tile_perm, int32_t* __restrict__ tile_rows, int row_stride,
              uint16_t* __restrict__ tile_blocks, int block_stride, int dense_min) {
    constexpr int K3 = K * K * K;
    static_assert(K3 <= kMaxK3Tiled, "tiled path supports up to 27 offsets");
    extern __shared__ __align__(16) unsigned char lds_raw[];
    PackLds& L = *reinterpret_cast<PackLds*>(lds_raw);
    const int tid = threadIdx.x;
    const int64_t tile = blockIdx.x;
    const int64_t o0 = tile * kTileT;
    const int n_valid = (int)min((int64_t)kTileT, n_out - o0);

    FX_STAMP(0);
    FX_STAMP_HWID(8);
    // ---- which output leaves overlap [o0, o0 + n_valid): from the one holding the tile's first voxel to the one
    // holding the next tile's first voxel.  That last leaf may start exactly at the tile's end and hold none of
    // the tile's voxels; kTileT voxels lie in at most kTileT leaves, so the count is cut there.
    const int f_lo = tile_first_leaf[tile];
    const int f_hi = (tile + 1) * kTileT < n_out ? tile_first_leaf[tile + 1] : tout.n_leaf - 1;
    const int n_leaves = min(f_hi + 1 - f_lo, kTileT);
    static_assert(sizeof(L.u.stage.leaf_off) / sizeof(int32_t) >= kTileT, "one entry per possible leaf of a tile");
    if (tid == 0) { L.n_halo = 0; L.n_blocks = 0; L.n_pair_blocks = 0; L.overflow = 0; L.n_rec = 0; L.any_left_out = 0; }
    if (tid < kTileWaves) L.wave_mask[tid] = 0;
    for (int e = tid; e < kRecHashSlots; e += kPackThreads) { L.u.stage.rec_hash[e] = -1; L.u.stage.slot_rec[e] = 0xFFFF; }
    if (tid < 8) { L.rec_mask[kMaxRecs * 8 + tid] = 0; L.rec_base[kMaxRecs * 8 + tid] = 0; }
    for (int li = tid; li < n_leaves; li += kPackThreads) L.u.stage.leaf_off[li] = (int32_t)tout.leaf[f_lo + li].offset;
    __syncthreads();

    // ---- staging.  The 80-byte records (Listing 1) of the distinct neighbour leaves go to LDS, so that no
    // lookup chases a pointer through global memory: (1) de-duplicate the neighbour ids of the tile's leaves in
    // a hash, (2) number the distinct ones, (3) fetch their records with independent loads and rewrite the
    // neighbour rows as record numbers.
    {
        constexpr int kCandPerThread = (kLdsLeafRows * 27 + kPackThreads - 1) / kPackThreads;
        const int n_cand = min(n_leaves, kLdsLeafRows) * 27;
        const int32_t* src = leaf_nbr + (int64_t)f_lo * 27;
        int32_t cand_id[kCandPerThread];
        int cand_slot[kCandPerThread];
#pragma unroll
        for (int q = 0; q < kCandPerThread; ++q) {
            const int e = tid + q * kPackThreads;
            cand_id[q] = e < n_cand ? src[e] : -1;
        }
#pragma unroll
        for (int q = 0; q < kCandPerThread; ++q) {
            cand_slot[q] = -1;
            if (cand_id[q] < 0) continue;
            uint32_t h = ((uint32_t)cand_id[q] * 0x9E3779B1u) >> 23;   // 9 bits
            for (int probe = 0; probe < kRecHashSlots; ++probe) {
                const int32_t cur = lds_peek(&L.u.stage.rec_hash[h]);
                if (cur == cand_id[q]) { cand_slot[q] = (int)h; break; }
                if (cur < 0) {
                    const int32_t old = atomicCAS(&L.u.stage.rec_hash[h], -1, cand_id[q]);
                    if (old < 0 || old == cand_id[q]) { cand_slot[q] = (int)h; break; }
                }
                h = (h + 1) & (kRecHashSlots - 1);
            }
        }
        __syncthreads();
        if (tid < kRecHashSlots && L.u.stage.rec_hash[tid] >= 0) {
            const int r = atomicAdd(&L.n_rec, 1);
            if (r < kMaxRecs) { L.u.stage.slot_rec[tid] = (uint16_t)r; L.u.stage.rec_id[r] = L.u.stage.rec_hash[tid]; }
        }
        __syncthreads();
        const int n_rec = min(L.n_rec, kMaxRecs);
        for (int e = tid; e < n_rec * 8; e += kPackThreads) {
            const int r = e >> 3, w = e & 7;
            const fx_leaf* nl = tin.leaf + L.u.stage.rec_id[r];
            L.rec_mask[e] = nl->mask[w];
            L.rec_base[e] = (int32_t)nl->offset + (w ? (int32_t)((nl->prefix >> (9 * (w - 1))) & 511) : 0);
        }
#pragma unroll
        for (int q = 0; q < kCandPerThread; ++q) {
            const int e = tid + q * kPackThreads;
            if (e >= n_cand) continue;
            int v = -1;
            if (cand_id[q] >= 0) {
                const uint16_t r = cand_slot[q] >= 0 ? L.u.stage.slot_rec[cand_slot[q]] : (uint16_t)0xFFFF;
                v = r != 0xFFFF ? (int)r : -2;
            }
            L.nbr_rows[e] = (int16_t)v;
        }
    }
    __syncthreads();
    FX_STAMP(1);

    // ---- mask pass: thread = output voxel (slot tid).  The thread finds its leaf (binary search over the tile's
    // leaf offsets) and its position inside the leaf (select on the leaf mask), then tests its taps.
    uint32_t mask = 0;
    {
        uint32_t vox = 0;
        if (tid < n_valid) {
            const int32_t o = (int32_t)(o0 + tid);
            int lo = 0, hi = n_leaves;   // last leaf of the tile with offset <= o
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (L.u.stage.leaf_off[mid] <= o) lo = mid; else hi = mid;
            }
            const fx_leaf* lf = tout.leaf + (f_lo + lo);
            const int r = o - L.u.stage.leaf_off[lo];           // rank of the voxel inside its leaf
            const uint64_t pre = lf->prefix;
            int wn = 0, before = 0;                 // mask word holding the voxel, active voxels before that word
#pragma unroll
            for (int w = 0; w < 7; ++w) {
                const int fld = (int)((pre >> (9 * w)) & 511);
                if (fld <= r) { wn = w + 1; before = fld; }
            }
            const int bit = select64(lf->mask[wn], r - before);
            const int j = bit >> 3, k = bit & 7;
            int par = 0;
            if (INV) par = ((lf->origin[0] >> 3) & 1) | (((lf->origin[1] >> 3) & 1) << 1) | (((lf->origin[2] >> 3) & 1) << 2);
            vox = (uint32_t)lo | ((uint32_t)wn << 9) | ((uint32_t)bit << 12) | ((uint32_t)par << 18);
            const int32_t* nbr_row = leaf_nbr + (int64_t)(f_lo + lo) * 27;
            if (K == 3 && !INV && stride == 1) {
                // The 3x3x3 stencil: the taps (a, b, 0..2) are three adjacent bits of one mask-word row, padded
                // at the leaf's k faces with the facing bit of the leaf beyond (read only by the voxels at k = 0
                // and k = 7; the others re-read the row's own word).
                const int side = k == 0 ? -1 : 1, side_bit = k == 0 ? 7 : 0;
#pragma unroll
                for (int a = 0; a < 3; ++a) {
                    const int ti = wn - 1 + a, si = (ti >> 3) + 1, n2 = ti & 7;
#pragma unroll
                    for (int b = 0; b < 3; ++b) {
                        const int tj = j - 1 + b, sj = (tj >> 3) + 1, jr = (tj & 7) << 3;
                        const int sc = (si * 3 + sj) * 3 + 1;
                        uint64_t wc, ws;
                        int32_t unused;
                        neighbour_word(L, tin, nbr_row, lo, sc, n2, wc, unused);
                        neighbour_word(L, tin, nbr_row, lo, sc + side, n2, ws, unused);
                        const uint32_t row8 = (uint32_t)(wc >> jr) & 0xFFu;
                        const uint32_t sbit = (uint32_t)(ws >> (jr + side_bit)) & 1u;
                        const uint32_t row10 = (row8 << 1) | (k == 0 ? sbit : sbit << 9);
                        mask |= ((row10 >> k) & 7u) << (a * 9 + b * 3);
                    }
                }
            } else {
                const TapAxes axes = tap_axes<K, INV>(stride, wn, j, k, par);
#pragma unroll 1
                for (int kappa = 0; kappa < K3; ++kappa) {
                    int slot, n2, bit6;
                    bool ok;
                    tap_query(axes, kappa / (K * K), (kappa / K) % K, kappa % K, slot, n2, bit6, ok);
                    uint64_t w;
                    int32_t unused;
                    neighbour_word(L, tin, nbr_row, lo, slot, n2, w, unused);
                    mask |= (uint32_t)(ok && ((w >> bit6) & 1ull)) << kappa;
                }
            }
        }
        // per-leaf dispatch (dense_min > 0): the outputs of a locally dense leaf are another kernel's; here they
        // have no taps and are never stored
        if (dense_min > 0 && tid < n_valid) {
            const int lo = (int)(vox & 511u);
            const int64_t end = f_lo + lo + 1 < tout.n_leaf ? tout.leaf[f_lo + lo + 1].offset : n_out;
            if ((int)(end - tout.leaf[f_lo + lo].offset) >= dense_min) { mask = 0; vox |= 1u << 21; L.any_left_out = 1; }
        }
        L.vox[tid] = vox;
        L.slot_mask[tid] = mask;
    }
    FX_STAMP(2);

    // ---- order the outputs by mask.  The sort key keeps 23 of the 27 mask bits (the four corner taps of the
    // lowest i-plane weigh least in the order and are dropped) so that key and slot fit 32 bits.  From here on
    // thread tid stands for position tid of the mask-sorted order: column tid % kGroup of sorted block tid / kGroup.
    uint32_t my_slot;
    {
        const uint32_t low9 = mask & 511u;
        const uint32_t key23 = ((mask >> 9) << 5) | ((low9 >> 1) & 1u) | (((low9 >> 3) & 7u) << 1) | (((low9 >> 7) & 1u) << 4);
        my_slot = block_sort_keys32((key23 << 9) | (uint32_t)tid, L.key) & 511u;    // its barriers also publish vox / slot_mask
        mask = L.slot_mask[my_slot];
        // union of the masks of every column block: OR over the 32 lanes that hold it
        uint32_t gm = mask;
#pragma unroll
        for (int d = 1; d < kGroup; d <<= 1) gm |= (uint32_t)__shfl_xor((int)gm, d);
        if ((tid & (kGroup - 1)) == 0) L.group_mask[tid / kGroup] = gm;
    }
    const uint32_t my_vox = L.vox[my_slot];
    __syncthreads();
    FX_STAMP(3);
    // Deal the column blocks to the consumer waves of the convolution by cost (offsets present = multiplies
    // issued): rank the blocks by cost, heaviest first, and deal the ranks to the waves in serpentine order
    // (0 1 2 3 3 2 1 0 ...), which evens out the sums.  Sorted block s becomes block group_dst[s] of the final
    // order (= tile_group_of(wave, wave slot)).  Tiles that list one row per pair go to the one-wave-per-block
    // gather kernels, which gain nothing from the deal and run the mask-sorted order slightly faster: they keep it.
    if (tid < kGroupsPerTile) {
        const int c = __popc(L.group_mask[tid]);
        int rank = 0;
#pragma unroll
        for (int g = 0; g < kGroupsPerTile; ++g) {
            const int cg = __popc(L.group_mask[g]);
            rank += (cg > c) || (cg == c && g < tid);
        }
        const int gi = rank / kTileWaves, r = rank % kTileWaves;
        L.group_dst[tid] = DEDUP ? (uint32_t)tile_group_of((gi & 1) ? kTileWaves - 1 - r : r, gi) : (uint32_t)tid;
    }
    __syncthreads();
    const int my_g = (int)L.group_dst[tid / kGroup];                      // final block of this thread's column
    const int cw = tile_wave_of(my_g), cgi = tile_slot_of(my_g), cn = tid % kGroup;
    if (cn == 0) tile_hdr[tile].group_mask[my_g] = L.group_mask[tid / kGroup];
    tile_perm[tile * kTileT + my_g * kGroup + cn] = ((my_vox >> 21) & 1u) ? (uint16_t)0xFFFF : (uint16_t)my_slot;
    if (tid < kGroupsPerTile) {               // the union over the blocks of every convolution wave (cleared at the top)
        atomicOr(&L.wave_mask[tile_wave_of((int)L.group_dst[tid])], L.group_mask[tid]);
        uint32_t pairs = (uint32_t)__popc(L.group_mask[tid]);
#pragma unroll
        for (int d = 1; d < kGroupsPerTile; d <<= 1) pairs += (uint32_t)__shfl_xor((int)pairs, d);
        if (tid == 0) L.n_pair_blocks = (int32_t)pairs;
    }
    __syncthreads();                         // stage is dead from here on
    const uint32_t my_cwm = L.wave_mask[cw];  // blocks exist for these offsets in this column's convolution wave
    uint32_t blk0 = 0;
#pragma unroll
    for (int w = 0; w < kTileWaves; ++w) blk0 += w < cw ? (uint32_t)__popc(L.wave_mask[w]) : 0u;
    // offsets this hardware wave (two sorted blocks with similar masks) looks up
    const uint32_t um = (uint32_t)__builtin_amdgcn_readfirstlane((int)(L.group_mask[(tid >> 6) * 2] | L.group_mask[(tid >> 6) * 2 + 1]));
    const int n_look = __popc(um);
    FX_STAMP(4);

    // ---- index pass
    const int32_t win_lo = SUBM ? (int32_t)o0 : 0;
    const int32_t win_n = SUBM ? n_valid : 0;
    int32_t* my_rows = tile_rows + tile * (int64_t)row_stride;
    const int lo = (int)(my_vox & 511u);
    const TapAxes axes = tap_axes<K, INV>(stride, (int)((my_vox >> 9) & 7u), (int)((my_vox >> 15) & 7u), (int)((my_vox >> 12) & 7u),
                                          (int)((my_vox >> 18) & 7u));
    const int32_t* nbr_row = leaf_nbr + (int64_t)(f_lo + lo) * 27;
    u32x16_t codes;                           // the thread's entries, two per word, in the order of the wave's offsets
    bool direct = !DEDUP;
    uint32_t n_list = 0;
    for (;;) {
        uint32_t list_base = 0;
        if (direct) {
            list_base = block_scan_excl((uint32_t)__popc(mask), L.wave_sums, &n_list);
        } else {
            for (int e = tid; e < kHaloHashSlots; e += kPackThreads) L.u.halo.hash[e] = -1;
            if (SUBM && tid < kNearWords) L.u.halo.near_bits[tid] = 0;
            __syncthreads();
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) codes[e] = 0;
        uint32_t rest = um;
        for (int kk = 0; kk < n_look; ++kk) {
            const int kappa = __builtin_ctz(rest);
            rest &= rest - 1;
            int slot, n2, bit6;
            bool ok;
            tap_query(axes, kappa / (K * K), (kappa / K) % K, kappa % K, slot, n2, bit6, ok);
            uint64_t w;
            int32_t base;
            neighbour_word(L, tin, nbr_row, lo, slot, n2, w, base);
            uint32_t code = kCodeNone;
            if ((mask >> kappa) & 1u) {
                const int32_t idx = base + (int32_t)popc_below(w, bit6);
                if (direct) {
                    code = list_base + (uint32_t)__popc(mask & ((1u << kappa) - 1u));
                    my_rows[code] = idx;
                } else if ((uint32_t)(idx - win_lo) < (uint32_t)win_n) {
                    code = (uint32_t)(idx - win_lo);
                } else if (SUBM && (uint32_t)(idx - (win_lo - kNearSpan)) < (uint32_t)kNearBits) {
                    const uint32_t off = (uint32_t)(idx - (win_lo - kNearSpan));
                    (void)__hip_atomic_fetch_or(&L.u.halo.near_bits[off >> 5], 1u << (off & 31u), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    code = kCodeNear | off;
                } else {
                    // a row far from the window: into the halo table (or found there)
                    uint32_t h = ((uint32_t)idx * 0x9E3779B1u) >> 21;  // 11 bits
                    for (;;) {
                        const int32_t cur = lds_peek(&L.u.halo.hash[h]);
                        if (cur == idx) { code = kCodeHalo | h; break; }
                        if (cur < 0) {
                            if (lds_peek(&L.overflow)) break;
                            const int32_t old = atomicCAS(&L.u.halo.hash[h], -1, idx);
                            if (old < 0) {
                                const int at = atomicAdd(&L.n_halo, 1);
                                if (at < kMaxHalo) { L.u.halo.halo[at] = idx; L.u.halo.halo_slot[at] = (uint16_t)h; code = kCodeHalo | h; }
                                else L.overflow = 1;
                                break;
                            }
                            if (old == idx) { code = kCodeHalo | h; break; }
                        }
                        h = (h + 1) & (kHaloHashSlots - 1);
                    }
                }
            }
            codes[kk >> 1] |= code << (16 * (kk & 1));
        }
        __syncthreads();
        if (direct || !L.overflow) break;
        direct = true;                        // more rows than the table holds: the tile lists one row per pair
        __syncthreads();                      // everyone has read the flag before the scan reuses LDS
    }
    FX_STAMP(5);

    // ---- the halo list, ascending: first the rows near the window in bitmap order, then the far rows, ranked
    // among themselves by counting (all distinct).  A row's place in the list, offset by win_n, is its local id.
    uint16_t* slot_rank = reinterpret_cast<uint16_t*>(L.rec_mask);      // hash slot -> place; the records are dead
    int n_halo = 0;
    if (!direct) {
        uint32_t n_near = 0;
        if (SUBM) {
            const uint32_t bits = tid < kNearWords ? L.u.halo.near_bits[tid] : 0u;
            uint32_t at = block_scan_excl((uint32_t)__popc(bits), L.wave_sums, &n_near);
            if (tid < kNearWords) L.u.halo.near_prefix[tid] = at;
            for (uint32_t m = bits; m; m &= m - 1) my_rows[at++] = win_lo - kNearSpan + 32 * tid + (__ffs(m) - 1);
        }
        const int n_far = L.n_halo;
        for (int i = tid; i < n_far; i += kPackThreads) {
            const int32_t v = L.u.halo.halo[i];
            int rank = (int)n_near;
            int jx = 0;
            for (; jx + 4 <= n_far; jx += 4) {
                const i32x4_t q = *reinterpret_cast<const i32x4_t*>(&L.u.halo.halo[jx]);
                rank += (q[0] < v) + (q[1] < v) + (q[2] < v) + (q[3] < v);
            }
            for (; jx < n_far; ++jx) rank += (L.u.halo.halo[jx] < v);
            my_rows[rank] = v;
            slot_rank[L.u.halo.halo_slot[i]] = (uint16_t)rank;
        }
        n_halo = (int)n_near + n_far;
        n_list = (uint32_t)n_halo;
    }
    __syncthreads();
    FX_STAMP(6);
    const bool lds_codes = !direct && (win_n + n_halo <= kRowCap);

    // ---- header
    if (tid == 0) {
        TileHeader* H = tile_hdr + tile;
        int run = 0;
#pragma unroll
        for (int w = 0; w < kTileWaves; ++w) { H->wave_mask[w] = L.wave_mask[w]; H->wave_block0[w] = (uint32_t)run; run += __popc(L.wave_mask[w]); }
        const bool empty = L.n_pair_blocks == 0;      // nothing to multiply (all outputs left to another kernel): no rows staged
        H->win_lo = direct ? 0 : win_lo; H->win_n = (direct || empty) ? 0 : win_n; H->n_list = (int32_t)n_list;
        H->n_blocks = run; H->n_out = n_valid;
        H->flags = (direct ? kTileDirect : (lds_codes ? kTileLdsOffsets : 0)) | (L.any_left_out ? kTilePartial : 0);
        H->n_pair_blocks = L.n_pair_blocks; H->pad = 0;
    }

    // ---- id blocks.  Entry [voxel column][wave slot] of block (convolution wave, offset) belongs to this thread
    // for every offset of its convolution wave's mask -- also those its own sorted block does not have (no input).
    // The two sorted blocks of a hardware wave may sit in different convolution waves, so the loop runs over the
    // union of both waves' offsets and every lane places its entry by its own wave's block numbering.
    {
        const uint32_t em = (uint32_t)__builtin_amdgcn_readlane((int)my_cwm, 0) | (uint32_t)__builtin_amdgcn_readlane((int)my_cwm, 32);
        uint16_t* dst = tile_blocks + ((size_t)tile * block_stride + blk0) * kIdBlockElems + cn * kGroupsPerWave + cgi;
        for (uint32_t rest = em; rest; rest &= rest - 1) {
            const int kappa = __builtin_ctz(rest);
            const uint32_t below = (1u << kappa) - 1u;
            uint32_t code = kCodeNone;
            if ((um >> kappa) & 1u) {                      // uniform: the wave looked this offset up
                const int kk = __popc(um & below);
                code = (codes[kk >> 1] >> (16 * (kk & 1))) & 0xFFFFu;
            }
            uint32_t id = kNoRow;
            if (code != kCodeNone) {
                if (code & kCodeHalo) id = (uint32_t)win_n + slot_rank[code & (kCodeHalo - 1u)];
                else if (SUBM && (code & kCodeNear)) {
                    const uint32_t off = code & (kCodeNear - 1u);
                    id = (uint32_t)win_n + L.u.halo.near_prefix[off >> 5] + (uint32_t)__popc(L.u.halo.near_bits[off >> 5] & ((1u << (off & 31u)) - 1u));
                } else id = code;
            }
            if (lds_codes) id = lds_row_code(id == kNoRow ? (uint32_t)kRowCap : id);
            if ((my_cwm >> kappa) & 1u) dst[(size_t)__popc(my_cwm & below) * kIdBlockElems] = (uint16_t)id;
        }
    }
    FX_STAMP(7);
}

// global input row of a tile-local id
__device__ __forceinline__ int32_t tile_global_row(const TileHeader* H, const int32_t* rows, uint32_t id) {
    return id < (uint32_t)H->win_n ? H->win_lo + (int32_t)id : rows[id - (uint32_t)H->win_n];
}

// decode the tiled form back into the dense table and / or count pairs per offset
__global__ void __launch_bounds__(kTileT)
k_tiles_to_dense(const TileHeader* __restrict__ tile_hdr, const uint16_t* __restrict__ tile_perm,
                 const int32_t* __restrict__ tile_rows, int row_stride, const uint16_t* __restrict__ tile_blocks,
                 int block_stride, int K3, int32_t* __restrict__ nbmap, unsigned long long* __restrict__ pairs) {
    __shared__ unsigned int cnt[32];
    if (threadIdx.x < 32) cnt[threadIdx.x] = 0;
    __syncthreads();
    const int64_t tile = blockIdx.x;
    const TileHeader* H = tile_hdr + tile;
    const int n_valid = H->n_out;
    const int g = threadIdx.x / kGroup, sub = threadIdx.x % kGroup;   // blockDim.x == kTileT: one thread per slot
    const int w = tile_wave_of(g), gi = tile_slot_of(g);
    const int local = tile_perm[tile * kTileT + g * kGroup + sub];
    uint32_t wm = H->wave_mask[w];
    size_t blk = (size_t)tile * block_stride + H->wave_block0[w];
    const int32_t* rows = tile_rows + tile * (int64_t)row_stride;
    while (wm) {
        const int kappa = __ffs(wm) - 1;
        wm &= wm - 1;
        uint16_t id = tile_blocks[blk * kIdBlockElems + sub * kGroupsPerWave + gi];
        if (H->flags & kTileLdsOffsets) id = (id / kRowBytes == kRowCap) ? kNoRow : (uint16_t)(id / kRowBytes);
        ++blk;
        if (id != kNoRow && local < n_valid) {
            if (nbmap) nbmap[(tile * kTileT + local) * K3 + kappa] = tile_global_row(H, rows, id);
            if (pairs) atomicAdd(&cnt[kappa], 1u);
        }
    }
    __syncthreads();
    if (pairs && threadIdx.x < K3 && cnt[threadIdx.x])
        atomicAdd(&pairs[threadIdx.x], (unsigned long long)cnt[threadIdx.x]);
}

// The map's tiling statistics, summed over the tile headers on request: stats[0] MFMA columns issued, [1] rows
// staged or listed, [2] direct tiles, [3] bytes of the tiled form (headers, permutations, row lists, id blocks).
__global__ void k_tile_stats(const TileHeader* __restrict__ tile_hdr, int64_t n_tiles, unsigned long long* __restrict__ stats) {
    unsigned long long v[4] = {0, 0, 0, 0};
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < n_tiles; t += (int64_t)gridDim.x * blockDim.x) {
        const TileHeader* H = tile_hdr + t;
        const bool direct = (H->flags & kTileDirect) != 0;
        v[0] += (unsigned long long)H->n_pair_blocks * kGroup;
        v[1] += (unsigned long long)(direct ? H->n_list : H->win_n + H->n_list);
        v[2] += direct ? 1ull : 0ull;
        v[3] += sizeof(TileHeader) + sizeof(uint16_t) * kTileT + sizeof(int32_t) * (size_t)H->n_list +
                sizeof(uint16_t) * kIdBlockElems * (size_t)H->n_blocks;
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        unsigned long long x = v[q];
        for (int d = 32; d >= 1; d >>= 1) x += shfl_xor_u64(x, d);
        if ((threadIdx.x & 63) == 0 && x) atomicAdd(&stats[q], x);
    }
}

__global__ void k_fill_i32(int32_t* __restrict__ p, int64_t n, int32_t v) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += stride) p[e] = v;
}

// pairs per offset from the dense table (maps that are not tiled)
__global__ void k_pair_counts(const int32_t* __restrict__ nbmap, int64_t n_out, int K3,
                              unsigned long long* __restrict__ pairs) {
    __shared__ unsigned int cnt[128];
    for (int e = threadIdx.x; e < 128; e += blockDim.x) cnt[e] = 0;
    __syncthreads();
    const int64_t total = n_out * K3;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += stride)
        if (nbmap[e] >= 0) atomicAdd(&cnt[e % K3], 1u);
    __syncthreads();
    for (int e = threadIdx.x; e < K3; e += blockDim.x)
        if (cnt[e]) atomicAdd(&pairs[e], (unsigned long long)cnt[e]);
}

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// dense [n_out, K3] table computed by the leaf-centric lookup kernel
static hipError_t launch_nbmap(const fx_kmap* km, int32_t* d_nbmap, hipStream_t st) {
    if (km->gout->hdr.n_leaf == 0) return hipSuccess;
    if (km->is_inverse) {        // the lookup rule of an inverse map lives in the tile builder only: decode its tiles
        const int64_t total = km->n_out * km->K3;
        const unsigned nbf = (unsigned)std::min<int64_t>((total + 256 * 8 - 1) / (256 * 8), 8192);
        k_fill_i32<<<nbf, 256, 0, st>>>(d_nbmap, total, -1);
        k_tiles_to_dense<<<(unsigned)km->n_tiles, kTileT, 0, st>>>(km->d_tile_hdr, km->d_tile_perm, km->d_tile_rows,
                                                                  km->row_stride, km->d_tile_blocks, km->block_stride,
                                                                  km->K3, d_nbmap, nullptr);
        return hipGetLastError();
    }
    const unsigned nb = (unsigned)((km->gout->hdr.n_leaf + kNbWavesPerBlock - 1) / kNbWavesPerBlock);
    const TreeView tin = km->gin->view(), tout = km->gout->view();
    ProfScope ps(kProfNbmap, st);
    switch (km->K) {
        case 1: k_nbmap<1><<<nb, 64 * kNbWavesPerBlock, 0, st>>>(tin, tout, km->stride, d_nbmap); break;
        case 2: k_nbmap<2><<<nb, 64 * kNbWavesPerBlock, 0, st>>>(tin, tout, km->stride, d_nbmap); break;
        case 3: k_nbmap<3><<<nb, 64 * kNbWavesPerBlock, 0, st>>>(tin, tout, km->stride, d_nbmap); break;
        default: k_nbmap<5><<<nb, 64 * kNbWavesPerBlock, 0, st>>>(tin, tout, km->stride, d_nbmap); break;
    }
    return hipGetLastError();
}

// The scalar convolution reads the dense table; it is built on first use.
fx_status kmap_ensure_dense(fx_kmap* km, hipStream_t st) {
    if (km->d_nbmap || km->n_out == 0) return FX_OK;
    void* p = nullptr;
    FX_TRY(dev_alloc(&p, sizeof(int32_t) * (size_t)(km->n_out * km->K3), st));
    hipError_t e = launch_nbmap(km, (int32_t*)p, st);
    if (e != hipSuccess) {
        dev_free(p, st);
        set_error("dense kernel-map build failed: %s", hipGetErrorString(e));
        return FX_EDEVICE;
    }
    km->d_nbmap = (int32_t*)p;
    return FX_OK;
}

}  // namespace fx

using namespace fx;

FX_DEV_TIMING_EXPORT(fx_debug_kmap_timing)
#ifdef FX_DEV_TIMING
extern "C" int fx_debug_kmap_occupancy(void) {     // resident tile builders per compute unit
    int n = -1;
    (void)hipFuncSetAttribute((const void*)k_build_tiles<3, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(PackLds));
    (void)hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k_build_tiles<3, true>, kPackThreads, sizeof(PackLds));
    return n;
}
#endif

extern "C" void fx_kmap_destroy(fx_kmap* km) {
    if (!km) return;
    if (km->refs.fetch_sub(1) != 1) return;
    if (km->d_alloc) dev_free(km->d_alloc, km->stream);
    if (km->d_nbmap) dev_free(km->d_nbmap, km->stream);
    if (km->d_unstaged_list) dev_free(km->d_unstaged_list, km->stream);
    if (km->inverse) fx_kmap_destroy(km->inverse);
    if (km->mixed) fx_kmap_destroy(km->mixed);
    if (km->gin) fx_grid_destroy(km->gin);
    if (km->gout) fx_grid_destroy(km->gout);
    free(km->h_pairs);
    delete km;
}

extern "C" fx_status fx_build_kernel_map(fx_grid* g_in, int32_t K, int32_t stride, void* stream, fx_grid** g_out,
                                         fx_kmap** out) {
    if (!g_in || !g_out || !out) { set_error("fx_build_kernel_map: null pointer"); return FX_EINVAL; }
    const bool ok = (stride == 1 && (K == 1 || K == 3 || K == 5)) || (stride == 2 && (K == 2 || K == 3));
    if (!ok) {
        set_error("fx_build_kernel_map: (kernel_size, stride) = (%d, %d) is not supported", K, stride);
        return (K >= 1 && stride >= 1) ? FX_EUNSUPPORTED : FX_EINVAL;
    }
    hipStream_t st = (hipStream_t)stream;
    fx_grid* gout = nullptr;
    if (stride == 1) { gout = g_in; fx_grid_retain(gout); }
    else FX_TRY(grid_coarsen2_for_map(g_in, K, st, &gout));
    fx_kmap* km = nullptr;
    FX_TRY(build_map(g_in, gout, K, stride, false, st, &km, 0, stride != 1));     // takes over the reference to gout
    *g_out = gout;
    fx_grid_retain(gout);
    *out = km;
    return FX_OK;
}

extern "C" fx_status fx_build_kernel_map_onto(fx_grid* g_in, fx_grid* g_out, int32_t K, void* stream, fx_kmap** out) {
    if (!g_in || !g_out || !out) { set_error("fx_build_kernel_map_onto: null pointer"); return FX_EINVAL; }
    if (K != 1 && K != 3 && K != 5) {
        set_error("fx_build_kernel_map_onto: kernel size %d is not supported (stride 1: 1, 3, 5)", K);
        return K >= 1 ? FX_EUNSUPPORTED : FX_EINVAL;
    }
    if (g_in->B != g_out->B) {
        set_error("fx_build_kernel_map_onto: the grids hold %d and %d batch members", g_in->B, g_out->B);
        return FX_EINVAL;
    }
    fx_grid_retain(g_out);
    return build_map(g_in, g_out, K, 1, false, (hipStream_t)stream, out);    // takes over that reference
}

void fx::enqueue_leaf_links(fx_grid* g, hipStream_t st, const fx_grid* g_in, int K, int stride) {
    if (option(kOptLeafLinks) == 0 || g->d_leaf_links || (K != 2 && K != 3)) return;
    void* p = nullptr;
    const size_t n_links = 27 * (size_t)g->cap_leaf, n_first = (size_t)g->cap_leaf + 2;     // runs of 512 voxels <= leaves + 1
    if (dev_alloc(&p, sizeof(int32_t) * (n_links + n_first), st) != FX_OK) return;
    g->d_leaf_links = (int32_t*)p;
    g->d_tile_first_leaf = g->d_leaf_links + n_links;
    g->links_K = K; g->links_stride = stride;
    const unsigned nb = (unsigned)((n_links + 255) / 256);
    const TreeView tout = g->view(), tin = g_in ? g_in->view() : tout;
    if (K == 2) k_leaf_links<2><<<nb, 256, 0, st>>>(tin, tout, g_in ? 0 : 1, stride, g->d_hdr, g->d_leaf_links, g->d_tile_first_leaf);
    else k_leaf_links<3><<<nb, 256, 0, st>>>(tin, tout, g_in ? 0 : 1, stride, g->d_hdr, g->d_leaf_links, g->d_tile_first_leaf);
    if (hipGetLastError() != hipSuccess) { dev_free(p, st); g->d_leaf_links = nullptr; g->d_tile_first_leaf = nullptr; }
}

// The map from the voxels of `gout` (the rows that are produced) to the voxels of `g_in` (the rows that are
// looked up).  Takes over the caller's reference to gout and retains g_in.  inverse: see k_leaf_neighbors.
fx_status fx::build_map(fx_grid* g_in, fx_grid* gout, int K, int stride, bool inverse, hipStream_t st, fx_kmap** out, int dense_min,
                        bool gout_made_for_map) {
    fx_kmap* km = new (std::nothrow) fx_kmap();
    if (!km) { fx_grid_destroy(gout); set_error("host allocation failed"); return FX_ENOMEM; }
    km->stream = st; km->gin = g_in; fx_grid_retain(g_in); km->gout = gout;
    km->K = K; km->stride = stride; km->K3 = K * K * K; km->is_inverse = inverse;
    km->n_in = g_in->hdr.n_voxels; km->n_out = gout->hdr.n_voxels;
    km->h_pairs = (int64_t*)calloc((size_t)km->K3, sizeof(int64_t));
    const bool tiled = km->K3 <= kMaxK3Tiled;
    km->n_tiles = tiled ? (km->n_out + kTileT - 1) / kTileT : 0;
    km->row_stride = kTileT * km->K3;
    km->block_stride = kTileWaves * km->K3;

    // one allocation: stats | tile headers | perm | rows | blocks
    const size_t nt = (size_t)std::max<int64_t>(km->n_tiles, 1);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    const size_t o_st = take(sizeof(int64_t) * (size_t)(4 + km->K3));
    const size_t o_th = take(sizeof(TileHeader) * nt);
    const size_t o_tp = take(sizeof(uint16_t) * kTileT * nt);
    const size_t o_tr = take(tiled ? sizeof(int32_t) * (size_t)km->row_stride * nt : 0);
    const size_t o_tb = take(tiled ? sizeof(uint16_t) * kIdBlockElems * (size_t)km->block_stride * nt : 0);
    // the table the grid build prepared: that of the 3x3x3 map of the grid onto itself, or of the strided map whose
    // build made gout (work on the grid's own stream only: the kernel that fills it may still be running there)
    const bool links = tiled && !inverse && dense_min <= 0 && gout->d_leaf_links && st == gout->stream &&
                       option(kOptLeafLinks) != 0 && gout->links_K == K && gout->links_stride == stride &&
                       (stride == 1 ? (K == 3 && g_in == gout) : gout_made_for_map);
    const size_t o_ln = take(tiled && !links ? sizeof(int32_t) * 27 * (size_t)std::max(gout->hdr.n_leaf, 1) : 0);
    const size_t o_tf = take(tiled && !links ? sizeof(int32_t) * (nt + 1) : 0);
    const size_t o_dl = take(dense_min > 0 ? sizeof(int32_t) * ((size_t)std::max(gout->hdr.n_leaf, 1) + 1) : 0);
    fx_status rc = dev_alloc(&km->d_alloc, off, st);
    if (rc != FX_OK) { fx_kmap_destroy(km); return rc; }
    char* p = (char*)km->d_alloc;
    km->d_stats = (int64_t*)(p + o_st);
    km->d_tile_hdr = (TileHeader*)(p + o_th);
    km->d_tile_perm = (uint16_t*)(p + o_tp);
    km->d_tile_rows = (int32_t*)(p + o_tr);
    km->d_tile_blocks = (uint16_t*)(p + o_tb);
    int32_t* d_leaf_nbr = links ? gout->d_leaf_links : (int32_t*)(p + o_ln);
    int32_t* d_tile_first = links ? gout->d_tile_first_leaf : (int32_t*)(p + o_tf);
    int32_t* d_n_dense = dense_min > 0 ? (int32_t*)(p + o_dl) : nullptr;        // the count, then the list
    int32_t* d_dense = dense_min > 0 ? d_n_dense + 1 : nullptr;
    km->d_n_dense = d_n_dense; km->d_dense_leaves = d_dense;

    hipError_t e = hipSuccess;
    if (d_n_dense) { k_fill_i32<<<1, 64, 0, st>>>(d_n_dense, 1, 0); e = hipGetLastError(); }
    if (e == hipSuccess && km->n_tiles > 0) {
        const size_t lds = sizeof(PackLds);
        const unsigned ntl = (unsigned)km->n_tiles;
        const TreeView tin = g_in->view(), tout = gout->view();
        if (!links) {
            ProfScope ps(kProfLeafNeighbors, st);
            const int64_t ne = (int64_t)gout->hdr.n_leaf * 27;
            const unsigned nbk = (unsigned)((ne + 255) / 256);
            if (K == 1) k_leaf_neighbors<1><<<nbk, 256, 0, st>>>(tin, tout, stride, km->n_out, d_leaf_nbr, d_tile_first, dense_min, d_dense, d_n_dense);
            else if (K == 2) k_leaf_neighbors<2><<<nbk, 256, 0, st>>>(tin, tout, stride, km->n_out, d_leaf_nbr, d_tile_first, dense_min, d_dense, d_n_dense);
            else if (inverse) k_leaf_neighbors<3, true><<<nbk, 256, 0, st>>>(tin, tout, stride, km->n_out, d_leaf_nbr, d_tile_first, dense_min, d_dense, d_n_dense);
            else k_leaf_neighbors<3><<<nbk, 256, 0, st>>>(tin, tout, stride, km->n_out, d_leaf_nbr, d_tile_first, dense_min, d_dense, d_n_dense);
        }
        ProfScope ps(kProfBuildTiles, st);
#define FX_TILES(KV, SUBMV...)                                                                                 \
    do {                                                                                                       \
        e = hipFuncSetAttribute((const void*)k_build_tiles<KV, SUBMV>,                                         \
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                         \
        if (e == hipSuccess)                                                                                   \
            k_build_tiles<KV, SUBMV><<<ntl, kPackThreads, lds, st>>>(tin, tout, stride, d_leaf_nbr, d_tile_first, \
                                                                     km->n_out,                                \
                                                                     km->d_tile_hdr, km->d_tile_perm,          \
                                                                     km->d_tile_rows, km->row_stride,          \
                                                                     km->d_tile_blocks, km->block_stride,      \
                                                                     dense_min);                               \
    } while (0)
        const bool same_grid = g_in == gout;      // a stride-1 map onto another grid has no window of its own rows
        if (K == 1 && same_grid) FX_TILES(1, true);
        else if (K == 1) FX_TILES(1, false);
        else if (K == 2) FX_TILES(2, false);
        else if (stride == 1 && same_grid) FX_TILES(3, true);
        // between two grids: when the outputs outnumber the inputs 2:1 (a padded output grid), a tile's outputs share
        // few input rows and all of them go through the halo table; otherwise (the map back) a tile reaches more
        // rows than the table holds and keeps one row per pair
        else if (stride == 1 && map_shares_rows(km)) FX_TILES(3, false, false, true);
        else if (stride == 1) FX_TILES(3, false);
        else if (inverse) FX_TILES(3, false, true, true);      // 512 fine voxels reach a few hundred coarse rows: staged tiles
        else FX_TILES(3, false);      // 3x3x3 stride 2: windows overlap, still no input row inside the tile's own range
#undef FX_TILES
        if (e == hipSuccess) e = hipGetLastError();
    }
    if (e != hipSuccess) {
        set_error("kernel-map build failed: %s", hipGetErrorString(e));
        fx_kmap_destroy(km);
        return FX_EDEVICE;
    }
    if (!tiled) {
        rc = kmap_ensure_dense(km, st);
        if (rc != FX_OK) { fx_kmap_destroy(km); return rc; }
    }
    *out = km;
    return FX_OK;
}

// The inverse of a 3x3x3 stride-2 map as a tiled map of its own: produced rows = the fine voxels, looked-up
// rows = the coarse voxels, offset kappa of a fine voxel = the coarse voxel whose offset kappa lands on it.
// The inverse of a stride-1 map between two different grids is the ordinary stride-1 map the other way round
// with the offsets mirrored (input p is linked to output p - delta), so its users mirror the weights.
fx_status fx::kmap_ensure_inverse(fx_kmap* km, hipStream_t st) {
    if (km->inverse) return FX_OK;
    const bool strided3 = km->K == 3 && km->stride == 2, onto = km->stride == 1 && km->gin != km->gout;
    if (!(strided3 || onto) || km->is_inverse) { set_error("no inverse map for this (kernel, stride)"); return FX_EUNSUPPORTED; }
    fx_grid_retain(km->gin);                  // build_map takes over one reference to the grid of the produced rows
    return build_map(km->gout, km->gin, km->K, km->stride, strided3, st, &km->inverse);
}

fx_status fx::kmap_ensure_mixed(fx_kmap* km, hipStream_t st) {
    if (km->mixed) return FX_OK;
    if (!(km->K == 3 && km->stride == 1 && km->gin == km->gout) || km->is_inverse) {
        set_error("per-leaf dispatch serves the 3x3x3 submanifold map only");
        return FX_EUNSUPPORTED;
    }
    fx_grid_retain(km->gout);                  // build_map takes over one reference to the grid of the produced rows
    return build_map(km->gin, km->gout, 3, 1, false, st, &km->mixed, kDenseLeafVoxels);
}

// One workgroup: the tiles without kTileLdsOffsets, counted and (the first `cap`) listed in ascending order; the count
// goes to pinned host memory, then the ticket.
__global__ void __launch_bounds__(1024) k_list_unstaged_tiles(const TileHeader* __restrict__ tile_hdr, int64_t n_tiles,
                                                              int32_t* __restrict__ list, int cap, int32_t* __restrict__ host_count,
                                                              int32_t* __restrict__ host_ticket, int32_t ticket) {
    __shared__ uint32_t wave_count[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t base = 0;
    for (int64_t t0 = 0; t0 < n_tiles; t0 += 1024) {
        const int64_t t = t0 + tid;
        const bool hit = t < n_tiles && !(tile_hdr[t].flags & kTileLdsOffsets);
        const uint64_t votes = __ballot(hit);
        if (lane == 0) wave_count[wave] = (uint32_t)__popcll(votes);
        __syncthreads();
        uint32_t before = 0, total = 0;
        for (int w = 0; w < 16; ++w) { const uint32_t c = wave_count[w]; total += c; if (w < wave) before += c; }
        const uint32_t pos = base + before + (uint32_t)__popcll(votes & ((1ull << lane) - 1ull));
        if (hit && pos < (uint32_t)cap) list[pos] = (int32_t)t;
        base += total;
        __syncthreads();
    }
    if (tid == 0) {
        *host_count = (int32_t)base;
        __threadfence_system();
        __hip_atomic_store(host_ticket, ticket, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

fx_status fx::kmap_unstaged_tiles(fx_kmap* km, hipStream_t st) {
    if (km->h_n_unstaged >= 0) return FX_OK;
    if (km->n_tiles == 0) { km->h_n_unstaged = 0; return FX_OK; }
    if (!km->d_unstaged_list) FX_TRY(dev_alloc((void**)&km->d_unstaged_list, sizeof(int32_t) * kMaxListedTiles, st));
    void* stage = nullptr;
    FX_TRY(host_staging(&stage, 128));      // the area of read-backs that the host waits for
    volatile int32_t* h_count = reinterpret_cast<volatile int32_t*>(stage);
    volatile int32_t* h_ticket = reinterpret_cast<volatile int32_t*>((char*)stage + 64);
    static thread_local int32_t next_ticket = 0;
    const int32_t ticket = ++next_ticket == 0 ? ++next_ticket : next_ticket;   // never 0
    *h_ticket = 0;
    k_list_unstaged_tiles<<<1, 1024, 0, st>>>(km->d_tile_hdr, km->n_tiles, km->d_unstaged_list, kMaxListedTiles,
                                               (int32_t*)h_count, (int32_t*)h_ticket, ticket);
    FX_HIP_TRY(hipGetLastError());
    bool seen = false;
    for (int spin = 0; spin < 200000 && !seen; ++spin) {
        seen = (*h_ticket == ticket);
        if (!seen) __builtin_ia32_pause();
    }
    if (!seen) FX_HIP_TRY(hipStreamSynchronize(st));
    std::atomic_thread_fence(std::memory_order_acquire);
    km->h_n_unstaged = *h_count;
    return FX_OK;
}

fx_status fx::kmap_fetch_stats(fx_kmap* km) {
    if (km->stats_valid) return FX_OK;
    hipStream_t st = km->stream;
    unsigned long long* pairs = (unsigned long long*)(km->d_stats + 4);
    FX_HIP_TRY(hipMemsetAsync(km->d_stats, 0, sizeof(int64_t) * (size_t)(4 + km->K3), st));
    if (km->n_tiles > 0) {
        k_tile_stats<<<(unsigned)std::min<int64_t>((km->n_tiles + 255) / 256, 256), 256, 0, st>>>(
            km->d_tile_hdr, km->n_tiles, (unsigned long long*)km->d_stats);
        k_tiles_to_dense<<<(unsigned)km->n_tiles, kTileT, 0, st>>>(km->d_tile_hdr, km->d_tile_perm, km->d_tile_rows,
                                                                  km->row_stride, km->d_tile_blocks, km->block_stride,
                                                                  km->K3, nullptr, pairs);
        FX_HIP_TRY(hipGetLastError());
    } else if (km->n_out > 0) {
        const int64_t total = km->n_out * km->K3;
        const unsigned nb = (unsigned)std::min<int64_t>((total + 256 * 16 - 1) / (256 * 16), 4096);
        k_pair_counts<<<nb, 256, 0, st>>>(km->d_nbmap, km->n_out, km->K3, pairs);
        FX_HIP_TRY(hipGetLastError());
    }
    void* stage = nullptr;
    const size_t bytes = sizeof(int64_t) * (size_t)(4 + km->K3);
    FX_TRY(host_staging(&stage, bytes));
    FX_HIP_TRY(hipMemcpyAsync(stage, km->d_stats, bytes, hipMemcpyDeviceToHost, st));
    FX_HIP_TRY(hipStreamSynchronize(st));
    const int64_t* h = (const int64_t*)stage;
    km->h_stats[0] = h[0]; km->h_stats[1] = km->n_tiles; km->h_stats[2] = h[1]; km->h_stats[3] = kTileT;
    km->h_tiled_bytes = h[3];
    km->h_n_pairs = 0;
    for (int k = 0; k < km->K3; ++k) { km->h_pairs[k] = h[4 + k]; km->h_n_pairs += h[4 + k]; }
    km->stats_valid = true;
    return FX_OK;
}

extern "C" fx_status fx_kmap_info(const fx_kmap* km_, int64_t* n_out, int32_t* k3, int64_t* n_pairs,
                                  int64_t* h_pairs_per_offset) {
    fx_kmap* km = const_cast<fx_kmap*>(km_);
    if (!km) { set_error("fx_kmap_info: null map"); return FX_EINVAL; }
    if (n_out) *n_out = km->n_out;
    if (k3) *k3 = km->K3;
    if (n_pairs || h_pairs_per_offset) {
        FX_TRY(kmap_fetch_stats(km));
        if (n_pairs) *n_pairs = km->h_n_pairs;
        if (h_pairs_per_offset) memcpy(h_pairs_per_offset, km->h_pairs, sizeof(int64_t) * (size_t)km->K3);
    }
    return FX_OK;
}

extern "C" fx_status fx_kmap_tile_stats(const fx_kmap* km_, int64_t* h_stats4) {
    fx_kmap* km = const_cast<fx_kmap*>(km_);
    if (!km || !h_stats4) { set_error("fx_kmap_tile_stats: null pointer"); return FX_EINVAL; }
    FX_TRY(kmap_fetch_stats(km));
    memcpy(h_stats4, km->h_stats, sizeof(km->h_stats));
    return FX_OK;
}

extern "C" fx_status fx_kmap_tiled_bytes(const fx_kmap* km_, int64_t* h_bytes) {
    fx_kmap* km = const_cast<fx_kmap*>(km_);
    if (!km || !h_bytes) { set_error("fx_kmap_tiled_bytes: null pointer"); return FX_EINVAL; }
    FX_TRY(kmap_fetch_stats(km));
    *h_bytes = km->h_tiled_bytes;
    return FX_OK;
}

extern "C" fx_status fx_kmap_dense(const fx_kmap* km, int32_t* d_nbmap, void* stream) {
    if (!km || (!d_nbmap && km->n_out > 0)) { set_error("fx_kmap_dense: null pointer"); return FX_EINVAL; }
    if (km->n_out == 0) return FX_OK;
    hipStream_t st = (hipStream_t)stream;
    const int64_t total = km->n_out * km->K3;
    if (km->n_tiles > 0) {
        const unsigned nb = (unsigned)std::min<int64_t>((total + 256 * 8 - 1) / (256 * 8), 8192);
        k_fill_i32<<<nb, 256, 0, st>>>(d_nbmap, total, -1);
        k_tiles_to_dense<<<(unsigned)km->n_tiles, kTileT, 0, st>>>(km->d_tile_hdr, km->d_tile_perm, km->d_tile_rows,
                                                                  km->row_stride, km->d_tile_blocks, km->block_stride,
                                                                  km->K3, d_nbmap, nullptr);
        FX_HIP_TRY(hipGetLastError());
    } else {
        FX_HIP_TRY(hipMemcpyAsync(d_nbmap, km->d_nbmap, sizeof(int32_t) * (size_t)total, hipMemcpyDeviceToDevice, st));
    }
    return FX_OK;
}
