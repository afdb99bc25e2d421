// Kernel-map build (Sec. 3.5): neighbour lookup through the tree for every output voxel and
// stencil offset, and the tiled form the MFMA convolution consumes.
#include "kmap.h"
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
template <int K, bool INV = false>
__global__ void k_leaf_neighbors(TreeView tin, TreeView tout, int stride, int64_t n_out, int32_t* __restrict__ nbr,
                                 int32_t* __restrict__ tile_first_leaf, unsigned long long* __restrict__ stats) {
    constexpr int D0 = delta_min(K);
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= (int64_t)tout.n_leaf * 27) return;
    const int f = (int)(e / 27), slot = (int)(e - (int64_t)f * 27);
    const fx_leaf* lf = tout.leaf + f;
    if (e == 0)                          // the build's statistics (this is its first launch)
        for (int q = 0; q < 4 + K * K * K; ++q) stats[q] = 0ull;
    if (slot == 0) {
        const int64_t begin = lf->offset, end = f + 1 < tout.n_leaf ? tout.leaf[f + 1].offset : n_out;
        for (int64_t t = (begin + kTileT - 1) / kTileT; t * kTileT < end; ++t) tile_first_leaf[t] = f;
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
        id = find_leaf(tin, lf->batch, (bi + a) * 8, (bj + c) * 8, (bk + d) * 8);
    nbr[e] = id;
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

#ifdef FX_KMAP_TIMING
// development aid: per-workgroup phase timestamps (thread 0), read back with fx_debug_kmap_timing
__device__ unsigned long long g_kmap_timing[4096 * 8];
#define FX_KSTAMP(slot) do { if (threadIdx.x == 0 && blockIdx.x < 4096) g_kmap_timing[blockIdx.x * 8 + (slot)] = __builtin_readcyclecounter(); } while (0)
#else
#define FX_KSTAMP(slot) do { } while (0)
#endif

// ---------------------------------------------------------------------------------- tiled form
constexpr int kPackThreads = kTileT;          // one thread per output slot
constexpr int kPackWaves = kPackThreads / 64;
constexpr int kHaloHashSlots = 2048;
constexpr int kLdsLeafRows = 56;             // leaves of a tile whose neighbour rows are kept in LDS
constexpr int kRecHashSlots = 512;           // de-duplication of the neighbour leaves of those rows
constexpr int kMaxRecs = 128;                // distinct neighbour-leaf records kept in LDS

struct PackScratch {                          // live after the lookup phase
    uint32_t key[kTileT];                     // slot of every position of the mask-sorted order
    int32_t hash[kHaloHashSlots];             // open addressing over halo rows
    int32_t halo[kMaxHalo];                   // distinct halo rows in insertion order
    uint32_t slot_mask[kTileT];
    union {
        uint32_t slot_base[kTileT];           // direct tiles: first list entry of each slot
        uint16_t halo_slot[kMaxHalo];         // other tiles: hash slot of each halo row
    };
    uint16_t slot_rank[kHaloHashSlots];       // hash slot -> rank of its row among the halo rows
};

typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;

struct PackLds {
    int32_t nb[kTileT * kMaxK3Tiled];         // the tile's map entries [slot][kappa]
    union {
        struct {                              // lookup phase
            int32_t leaf_off[kTileT];         // first index of every leaf of the tile
            // neighbours of the tile's first leaves: >= 0 record in `rec`, -1 none, <= -2 leaf id -2-v (not staged)
            int32_t nbr_rows[kLdsLeafRows * 27];
            int32_t rec_hash[kRecHashSlots];  // leaf id or -1
            uint16_t slot_rec[kRecHashSlots]; // hash slot -> record, 0xFFFF: not staged
            int32_t rec_id[kMaxRecs];
            uint64_t rec_mask[(kMaxRecs + 1) * 8];  // mBitMask of Listing 1; record kMaxRecs stays all zero
            int32_t rec_base[(kMaxRecs + 1) * 8];   // per mask word: mOffset + the prefix-sum field that precedes it
        } look;
        PackScratch s;
    } u;
    uint32_t group_mask[kGroupsPerTile];
    uint32_t group_src[kGroupsPerTile];      // column block of the mask-sorted order that takes each final position
    uint32_t wave_mask[kTileWaves];
    uint32_t wave_block0[kTileWaves];
    uint32_t wave_sums[kPackWaves];
    int32_t n_halo, n_blocks, n_pair_blocks, overflow, f_lo, n_leaves, n_rec;
};
static_assert(sizeof(PackLds) <= 80 * 1024, "two tile builders per compute unit");

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

// in-LDS bitonic sort of P (power of two) int32 values
__device__ __forceinline__ void lds_bitonic_sort(int32_t* a, int P) {
    for (int k = 2; k <= P; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int t = threadIdx.x; t < P; t += blockDim.x) {
                const int p = t ^ j;
                if (p > t) {
                    const int32_t x = a[t], y = a[p];
                    const bool up = ((t & k) == 0);
                    if ((x > y) == up) { a[t] = y; a[p] = x; }
                }
            }
            __syncthreads();
        }
    }
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

// One workgroup per tile of kTileT consecutive outputs: lookups (one thread per voxel, straight
// into LDS), mask sort, row de-duplication, block emission.  SUBM: input grid == output grid, so the
// tile's own index range is the window; otherwise there is no window.  DEDUP: rows outside the window are
// de-duplicated in the halo table (a stride-1 map between two grids: no window, all rows in the table);
// without it the tile is "direct".
template <int K, bool SUBM, bool INV = false, bool DEDUP = SUBM>
__global__ void __launch_bounds__(kPackThreads)
k_build_tiles(TreeView tin, TreeView tout, int stride, const int32_t* __restrict__ leaf_nbr,
              const int32_t* __restrict__ tile_first_leaf, int64_t n_out, TileHeader* __restrict__ tile_hdr,
              uint16_t* __restrict__ tile_perm, int32_t* __restrict__ tile_rows, int row_stride,
              uint16_t* __restrict__ tile_blocks, int block_stride, unsigned long long* __restrict__ stats) {
    constexpr int K3 = K * K * K;
    static_assert(K3 <= kMaxK3Tiled, "tiled path supports up to 27 offsets");
    extern __shared__ __align__(16) unsigned char lds_raw[];
    PackLds& L = *reinterpret_cast<PackLds*>(lds_raw);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t tile = blockIdx.x;
    const int64_t o0 = tile * kTileT;
    const int n_valid = (int)min((int64_t)kTileT, n_out - o0);

    FX_KSTAMP(0);
    // ---- which output leaves overlap [o0, o0 + n_valid)
    if (tid == 0) {
        // leaves from the one holding the tile's first voxel to the one holding the next tile's first
        // voxel.  That last leaf may start exactly at the tile's end and hold none of the tile's voxels;
        // kTileT voxels lie in at most kTileT leaves, so the count is cut there (a tile of kTileT one-voxel
        // leaves would otherwise list kTileT + 1 and write past leaf_off)
        const int lo = tile_first_leaf[tile];
        const int a = (tile + 1) * kTileT < n_out ? tile_first_leaf[tile + 1] : tout.n_leaf - 1;
        L.f_lo = lo;
        L.n_leaves = min(a + 1 - lo, kTileT);
        L.n_halo = 0; L.n_blocks = 0; L.n_pair_blocks = 0; L.overflow = 0; L.n_rec = 0;
    }
    for (int e = tid; e < kRecHashSlots; e += kPackThreads) { L.u.look.rec_hash[e] = -1; L.u.look.slot_rec[e] = 0xFFFF; }
    if (tid < 8) { L.u.look.rec_mask[kMaxRecs * 8 + tid] = 0; L.u.look.rec_base[kMaxRecs * 8 + tid] = 0; }
    __syncthreads();

    // ---- lookups: one thread per output voxel.  The thread finds its leaf (binary search over the
    // tile's leaf offsets), its position inside the leaf (select on the leaf mask), and evaluates
    // Listing 1 for its K^3 neighbours through the neighbour-leaf table; the few leaf records a
    // tile touches stay in the L1 cache.
    uint32_t mask = 0, hmask = 0;     // taps of this thread's voxel; those whose row lies outside the window
    {
        const int f_lo = L.f_lo, n_leaves = L.n_leaves;
        for (int li = tid; li < n_leaves; li += kPackThreads) L.u.look.leaf_off[li] = (int32_t)tout.leaf[f_lo + li].offset;
        // The 80-byte records (Listing 1) of the distinct neighbour leaves are staged in LDS, so the
        // 27 lookups of a voxel chase no pointer through global memory: (1) de-duplicate the
        // neighbour ids of the tile's leaves in a hash, (2) number the distinct ones, (3) fetch
        // their records with independent loads and rewrite the neighbour rows as record numbers.
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
                cand_slot[q] = -1;
                if (cand_id[q] < 0) continue;
                uint32_t h = ((uint32_t)cand_id[q] * 0x9E3779B1u) >> 23;   // 9 bits
                for (int probe = 0; probe < kRecHashSlots; ++probe) {
                    const int32_t cur = ((volatile int32_t*)L.u.look.rec_hash)[h];
                    if (cur == cand_id[q]) { cand_slot[q] = (int)h; break; }
                    if (cur < 0) {
                        const int32_t old = atomicCAS(&L.u.look.rec_hash[h], -1, cand_id[q]);
                        if (old < 0 || old == cand_id[q]) { cand_slot[q] = (int)h; break; }
                    }
                    h = (h + 1) & (kRecHashSlots - 1);
                }
            }
            __syncthreads();
            if (tid < kRecHashSlots && L.u.look.rec_hash[tid] >= 0) {
                const int r = atomicAdd(&L.n_rec, 1);
                if (r < kMaxRecs) { L.u.look.slot_rec[tid] = (uint16_t)r; L.u.look.rec_id[r] = L.u.look.rec_hash[tid]; }
            }
            __syncthreads();
            const int n_rec = min(L.n_rec, kMaxRecs);
            for (int e = tid; e < n_rec * 8; e += kPackThreads) {
                const int r = e >> 3, w = e & 7;
                const fx_leaf* nl = tin.leaf + L.u.look.rec_id[r];
                L.u.look.rec_mask[e] = nl->mask[w];
                L.u.look.rec_base[e] = (int32_t)nl->offset + (w ? (int32_t)((nl->prefix >> (9 * (w - 1))) & 511) : 0);
            }
#pragma unroll
            for (int q = 0; q < kCandPerThread; ++q) {
                const int e = tid + q * kPackThreads;
                if (e >= n_cand) continue;
                int32_t v = -1;
                if (cand_id[q] >= 0) {
                    const uint16_t r = cand_slot[q] >= 0 ? L.u.look.slot_rec[cand_slot[q]] : (uint16_t)0xFFFF;
                    v = r != 0xFFFF ? (int32_t)r : -2 - cand_id[q];
                }
                L.u.look.nbr_rows[e] = v;
            }
        }
        __syncthreads();
        int32_t* my_nb = L.nb + tid * K3;
        if (tid < n_valid) {
            const int32_t w_lo = SUBM ? (int32_t)o0 : 0, w_n = SUBM ? n_valid : 0;
            constexpr int D0 = delta_min(K);
            const int32_t o = (int32_t)(o0 + tid);
            int lo = 0, hi = n_leaves;   // last leaf of the tile with offset <= o
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (L.u.look.leaf_off[mid] <= o) lo = mid; else hi = mid;
            }
            const int f = f_lo + lo;
            const fx_leaf* lf = tout.leaf + f;
            int r = o - L.u.look.leaf_off[lo];           // rank of the voxel inside its leaf
            const uint64_t pre = lf->prefix;
            int wn = 0, before = 0;                 // mask word holding the voxel, active voxels before that word
#pragma unroll
            for (int w = 0; w < 7; ++w) {
                const int fld = (int)((pre >> (9 * w)) & 511);
                if (fld <= r) { wn = w + 1; before = fld; }
            }
            const int bit = select64(lf->mask[wn], r - before);
            const int pi = lf->origin[0] + wn, pj = lf->origin[1] + (bit >> 3), pk = lf->origin[2] + (bit & 7);
            // INV (inverse of the 3x3x3 stride-2 map): offset (a,b,c) of fine voxel p names the coarse voxel
            // (p - delta) / 2, delta = (a,b,c) - 1, and only when p - delta is even on every axis
            const int bi = INV ? ((lf->origin[0] - 1) >> 1) >> 3 : (stride * lf->origin[0] + D0) >> 3,
                      bj = INV ? ((lf->origin[1] - 1) >> 1) >> 3 : (stride * lf->origin[1] + D0) >> 3,
                      bk = INV ? ((lf->origin[2] - 1) >> 1) >> 3 : (stride * lf->origin[2] + D0) >> 3;
            const int32_t* nbr_row = leaf_nbr + (int64_t)f * 27;
            const bool row_in_lds = lo < kLdsLeafRows;
            // kept as rolled loops: the fully unrolled form of this divergent body gave wrong entries
            // for the offsets (-1,0,0), (0,-1,0), (0,0,-1) on gfx950 (cause not established; the
            // parity tests against the oracle catch it)
            const int32_t* lds_row = L.u.look.nbr_rows + lo * 27;
            int kappa = 0;
#pragma unroll 1
            for (int a = 0; a < K; ++a) {
                const int qi_full = INV ? pi + 1 - a : stride * pi + D0 + a;
                const bool even_i = INV ? !(qi_full & 1) : true;
                const int qi = INV ? qi_full >> 1 : qi_full;
                const int si = ((qi >> 3) - bi) * 9, n2 = qi & 7;
#pragma unroll 1
                for (int b2 = 0; b2 < K; ++b2) {
                    const int qj_full = INV ? pj + 1 - b2 : stride * pj + D0 + b2;
                    const bool even_ij = INV ? even_i && !(qj_full & 1) : true;
                    const int qj = INV ? qj_full >> 1 : qj_full;
                    const int sij = si + ((qj >> 3) - bj) * 3, bj8 = (qj & 7) << 3;
#pragma unroll 1
                    for (int c = 0; c < K; ++c, ++kappa) {
                        const int qk_full = INV ? pk + 1 - c : stride * pk + D0 + c;
                        const bool even_ijk = INV ? even_ij && !(qk_full & 1) : true;
                        const int qk = INV ? qk_full >> 1 : qk_full;
                        const int slot = sij + ((qk >> 3) - bk);
                        // The common case runs without a branch: a missing neighbour leaf reads the all-zero
                        // record kMaxRecs, whose mask has no bit to find.
                        const int v = row_in_lds ? lds_row[slot] : -2 - nbr_row[slot];   // -2 - (-1) = -1
                        const int rec = v >= 0 ? v : kMaxRecs;
                        uint64_t w = L.u.look.rec_mask[rec * 8 + n2];
                        int32_t base = L.u.look.rec_base[rec * 8 + n2];
                        if (__builtin_expect(v <= -2, 0)) {   // record not staged: three independent global loads
                            const fx_leaf* nl = tin.leaf + (-2 - v);
                            w = nl->mask[n2];
                            const uint64_t npre = nl->prefix;
                            base = (int32_t)nl->offset + (n2 ? (int32_t)((npre >> (9 * (n2 - 1))) & 511) : 0);
                        }
                        const int bit6 = bj8 | (qk & 7);
                        const uint32_t wlo = (uint32_t)w, whi = (uint32_t)(w >> 32);
                        // bits below bit6, per half: all of the low half once bit6 >= 32
                        const uint32_t mlo = bit6 >= 32 ? 0xFFFFFFFFu : ((1u << bit6) - 1u);
                        const uint32_t mhi = bit6 >= 32 ? ((1u << (bit6 - 32)) - 1u) : 0u;
                        const bool present = even_ijk && (((bit6 >= 32 ? whi : wlo) >> (bit6 & 31)) & 1u) != 0;
                        const int idx = base + __popc(wlo & mlo) + __popc(whi & mhi);
                        // entry encoding from here on: -1 none; -2 - id: row win_lo + id of the window;
                        // >= 0: a row outside the window, not yet entered in the halo table
                        const bool in_win = (uint32_t)(idx - w_lo) < (uint32_t)w_n;
                        const int res = present ? (in_win ? -2 - (idx - w_lo) : idx) : -1;
                        mask |= (uint32_t)present << kappa;
                        hmask |= (uint32_t)(present && !in_win) << kappa;
                        my_nb[kappa] = res;
                    }
                }
            }
        } else {
#pragma unroll
            for (int kappa = 0; kappa < K3; ++kappa) my_nb[kappa] = -1;
        }
    }
    __syncthreads();

    FX_KSTAMP(1);
    // ---- per-slot mask; halo rows into the hash
    PackScratch& S = L.u.s;
    for (int e = tid; e < kHaloHashSlots; e += kPackThreads) S.hash[e] = -1;
    __syncthreads();
    const int32_t win_lo = SUBM ? (int32_t)o0 : 0;
    const int32_t win_n = SUBM ? n_valid : 0;
    // rows outside the window go into the halo table; an entry that is in becomes -1024 - (table slot)
    for (uint32_t hm = DEDUP ? hmask : 0u; hm; hm &= hm - 1) {
        const int kappa = __ffs(hm) - 1;
        const int32_t r = L.nb[tid * K3 + kappa];
        uint32_t h = ((uint32_t)r * 0x9E3779B1u) >> 21;  // 11 bits
        bool in = false;
        for (;;) {
            const int32_t cur = ((volatile int32_t*)S.hash)[h];
            if (cur == r) { in = true; break; }
            if (cur < 0) {
                if (((volatile int32_t*)&L.overflow)[0]) break;
                const int32_t old = atomicCAS(&S.hash[h], -1, r);
                if (old < 0) {
                    const int pos = atomicAdd(&L.n_halo, 1);
                    if (pos < kMaxHalo) { S.halo[pos] = r; S.halo_slot[pos] = (uint16_t)h; in = true; } else L.overflow = 1;
                    break;
                }
                if (old == r) { in = true; break; }
            }
            h = (h + 1) & (kHaloHashSlots - 1);
        }
        if (in) L.nb[tid * K3 + kappa] = -1024 - (int32_t)h;
    }
    S.slot_mask[tid] = mask;
    __syncthreads();
    const bool direct = !DEDUP || L.overflow != 0;
    const int n_halo = direct ? 0 : L.n_halo;

    FX_KSTAMP(2);
    // ---- order outputs by mask; order halo rows by index; per-slot list base (direct tiles)
    // The sort key keeps 23 of the 27 mask bits (the four corner taps of the lowest i-plane weigh
    // least in the order and are dropped) so that key and slot fit 32 bits; S.key then holds the
    // slot of every sorted position.
    const uint32_t low9 = mask & 511u;
    const uint32_t key23 = ((mask >> 9) << 5) | ((low9 >> 1) & 1u) | (((low9 >> 3) & 7u) << 1) | (((low9 >> 7) & 1u) << 4);
    const uint32_t sorted = block_sort_keys32((key23 << 9) | (uint32_t)tid, S.key);
    __syncthreads();
    S.key[tid] = sorted & 511u;
    __syncthreads();
    FX_KSTAMP(3);
    int32_t* my_rows = tile_rows + tile * (int64_t)row_stride;
    if (!direct) {
        // rank of every halo row among the halo rows (all distinct): its position in the
        // ascending row list and, offset by win_n, its local id
        for (int i = tid; i < n_halo; i += kPackThreads) {
            const int32_t v = S.halo[i];
            int rank = 0;
            for (int j = 0; j < n_halo; ++j) rank += (S.halo[j] < v);
            my_rows[rank] = v;
            S.slot_rank[S.halo_slot[i]] = (uint16_t)rank;
        }
    }
    FX_KSTAMP(4);
    uint32_t n_list;
    {
        uint32_t total;
        const uint32_t base = block_scan_excl(direct ? (uint32_t)__popc(mask) : 0u, L.wave_sums, &total);
        if (direct) S.slot_base[tid] = base;
        n_list = direct ? total : (uint32_t)n_halo;
    }
    uint32_t my_gm = 0;
    if (tid < kGroupsPerTile) {
        for (int n = 0; n < kGroup; ++n) my_gm |= S.slot_mask[S.key[tid * kGroup + n]];
        L.group_mask[tid] = my_gm;
    }
    __syncthreads();
    // Deal the column blocks to the consumer waves of the convolution by cost (offsets present =
    // multiplies issued): rank the blocks by cost, heaviest first, and deal the ranks to the waves
    // in serpentine order (0 1 2 3 3 2 1 0 ...), which evens out the sums.  Position
    // tile_group_of(w, gi) of the final order takes block group_src[...] of the sorted order.
    if (tid < kGroupsPerTile) {
        const int c = __popc(my_gm);
        int rank = 0;
        for (int g = 0; g < kGroupsPerTile; ++g) {
            const int cg = __popc(L.group_mask[g]);
            rank += (cg > c) || (cg == c && g < tid);
        }
        const int gi = rank / kTileWaves, r = rank % kTileWaves;
        // (tiles without staged rows go to the one-wave-per-block gather kernels, which gain nothing
        // from the deal and run the mask-sorted order slightly faster: they keep it)
        if (direct) L.group_src[tid] = (uint32_t)tid;
        else L.group_src[tile_group_of((gi & 1) ? kTileWaves - 1 - r : r, gi)] = (uint32_t)tid;
    }
    __syncthreads();
    const uint32_t dealt = S.key[L.group_src[tid / kGroup] * kGroup + tid % kGroup];   // slot at final position tid
    if (tid < kGroupsPerTile) my_gm = L.group_mask[L.group_src[tid]];
    __syncthreads();
    S.key[tid] = dealt;
    if (tid < kGroupsPerTile) L.group_mask[tid] = my_gm;
    __syncthreads();
    if (tid == 0) {
        int run = 0, pairs = 0;
        for (int w = 0; w < kTileWaves; ++w) {
            uint32_t wm = 0;
            for (int gi = 0; gi < kGroupsPerWave; ++gi) {
                const uint32_t gm = L.group_mask[tile_group_of(w, gi)];
                wm |= gm;
                pairs += __popc(gm);
            }
            L.wave_mask[w] = wm;
            L.wave_block0[w] = run;
            run += __popc(wm);
        }
        L.n_blocks = run;
        L.n_pair_blocks = pairs;
    }
    __syncthreads();

    FX_KSTAMP(5);
    const bool lds_codes = !direct && (win_n + n_halo <= kRowCap);

    // ---- header, permutation, row list
    TileHeader* H = tile_hdr + tile;
    if (tid == 0) {
        H->win_lo = direct ? 0 : win_lo; H->win_n = direct ? 0 : win_n; H->n_list = (int32_t)n_list;
        H->n_blocks = L.n_blocks; H->n_out = n_valid; H->flags = direct ? kTileDirect : (lds_codes ? kTileLdsOffsets : 0);
        H->n_pair_blocks = L.n_pair_blocks; H->pad = 0;
        atomicAdd(&stats[0], (unsigned long long)L.n_pair_blocks * kGroup);
        atomicAdd(&stats[1], (unsigned long long)(direct ? n_list : (uint32_t)(win_n + n_halo)));
        if (direct) atomicAdd(&stats[2], 1ull);
        atomicAdd(&stats[3], (unsigned long long)(sizeof(TileHeader) + sizeof(uint16_t) * kTileT + sizeof(int32_t) * n_list +
                                                  sizeof(uint16_t) * kIdBlockElems * (size_t)L.n_blocks));
    }
    if (tid < kGroupsPerTile) H->group_mask[tid] = L.group_mask[tid];
    if (tid < kTileWaves) { H->wave_mask[tid] = L.wave_mask[tid]; H->wave_block0[tid] = L.wave_block0[tid]; }
    tile_perm[tile * kTileT + tid] = (uint16_t)dealt;
    if (direct) {
        uint32_t pos = S.slot_base[tid];
        for (int kappa = 0; kappa < K3; ++kappa) {
            const int32_t v = L.nb[tid * K3 + kappa];
            if (v == -1) continue;
            my_rows[pos++] = v >= 0 ? v : (v <= -1024 ? S.hash[-1024 - v] : win_lo + (-2 - v));
        }
    }

    FX_KSTAMP(6);
    // ---- id blocks: thread (wave w, voxel column n, share q) fills the entries [voxel n][group
    // slots] of every kQuarters-th block of wave w, so that a block is written as 32 consecutive
    // entries
    {
        constexpr int kQuarters = kPackThreads / (kTileWaves * kGroup);      // threads per (wave, voxel column)
        constexpr int kEntryWords = kGroupsPerWave / 2;                     // 32-bit words per entry
        const int w = tid / (kQuarters * kGroup), q = (tid / kGroup) % kQuarters, n = tid % kGroup;
        int slot[kGroupsPerWave];
        uint32_t smask[kGroupsPerWave], sbase[kGroupsPerWave];
#pragma unroll
        for (int gi = 0; gi < kGroupsPerWave; ++gi) {
            slot[gi] = (int)S.key[tile_group_of(w, gi) * kGroup + n];
            smask[gi] = S.slot_mask[slot[gi]];
            sbase[gi] = direct ? S.slot_base[slot[gi]] : 0u;
        }
        uint32_t wm = L.wave_mask[w];
        size_t blk = (size_t)tile * block_stride + L.wave_block0[w];
        for (int bi = 0; wm; ++bi, ++blk, wm &= wm - 1) {
            if ((bi % kQuarters) != q) continue;
            const int kappa = __ffs(wm) - 1;
            uint32_t ids[kGroupsPerWave];
#pragma unroll
            for (int gi = 0; gi < kGroupsPerWave; ++gi) {
                uint32_t id = kNoRow;
                if ((smask[gi] >> kappa) & 1u) {
                    if (direct) {
                        id = sbase[gi] + __popc(smask[gi] & ((1u << kappa) - 1u));
                    } else {
                        const int32_t v = L.nb[slot[gi] * K3 + kappa];
                        id = v <= -1024 ? (uint32_t)win_n + S.slot_rank[-1024 - v] : (uint32_t)(-2 - v);
                    }
                }
                if (lds_codes) id = lds_row_code(id == kNoRow ? (uint32_t)kRowCap : id);
                ids[gi] = id & 0xFFFFu;
            }
            uint32_t* dst = reinterpret_cast<uint32_t*>(tile_blocks + blk * kIdBlockElems + n * kGroupsPerWave);
#pragma unroll
            for (int e = 0; e < kEntryWords; ++e) dst[e] = ids[2 * e] | (ids[2 * e + 1] << 16);
        }
    }
    FX_KSTAMP(7);
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

#ifdef FX_KMAP_TIMING
extern "C" int fx_debug_kmap_timing(unsigned long long* h_out, size_t bytes) {
    return (int)hipMemcpyFromSymbol(h_out, HIP_SYMBOL(g_kmap_timing), bytes);
}
#endif

extern "C" void fx_kmap_destroy(fx_kmap* km) {
    if (!km) return;
    if (km->refs.fetch_sub(1) != 1) return;
    if (km->d_alloc) dev_free(km->d_alloc, km->stream);
    if (km->d_nbmap) dev_free(km->d_nbmap, km->stream);
    if (km->inverse) fx_kmap_destroy(km->inverse);
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
    FX_HT("(outside)");
    if (stride == 1) { gout = g_in; fx_grid_retain(gout); }
    else FX_TRY(fx_grid_coarsen2(g_in, stream, &gout));
    fx_kmap* km = nullptr;
    FX_TRY(build_map(g_in, gout, K, stride, false, st, &km));     // takes over the reference to gout
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

// The map from the voxels of `gout` (the rows that are produced) to the voxels of `g_in` (the rows that are
// looked up).  Takes over the caller's reference to gout and retains g_in.  inverse: see k_leaf_neighbors.
fx_status fx::build_map(fx_grid* g_in, fx_grid* gout, int K, int stride, bool inverse, hipStream_t st, fx_kmap** out) {
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
    const size_t o_ln = take(tiled ? sizeof(int32_t) * 27 * (size_t)std::max(gout->hdr.n_leaf, 1) : 0);
    const size_t o_tf = take(tiled ? sizeof(int32_t) * (nt + 1) : 0);
    FX_HT("kmap: host setup");
    fx_status rc = dev_alloc(&km->d_alloc, off, st);
    FX_HT("kmap: alloc");
    if (rc != FX_OK) { fx_kmap_destroy(km); return rc; }
    char* p = (char*)km->d_alloc;
    km->d_stats = (int64_t*)(p + o_st);
    km->d_tile_hdr = (TileHeader*)(p + o_th);
    km->d_tile_perm = (uint16_t*)(p + o_tp);
    km->d_tile_rows = (int32_t*)(p + o_tr);
    km->d_tile_blocks = (uint16_t*)(p + o_tb);
    int32_t* d_leaf_nbr = (int32_t*)(p + o_ln);
    int32_t* d_tile_first = (int32_t*)(p + o_tf);

    hipError_t e = hipSuccess;
    if (km->n_tiles == 0) e = hipMemsetAsync(km->d_stats, 0, sizeof(int64_t) * (size_t)(4 + km->K3), st);
    if (e == hipSuccess && km->n_tiles > 0) {
        unsigned long long* stats = (unsigned long long*)km->d_stats;
        const size_t lds = sizeof(PackLds);
        const unsigned ntl = (unsigned)km->n_tiles;
        const TreeView tin = g_in->view(), tout = gout->view();
        {
            ProfScope ps(kProfLeafNeighbors, st);
            const int64_t ne = (int64_t)gout->hdr.n_leaf * 27;
            const unsigned nbk = (unsigned)((ne + 255) / 256);
            if (K == 1) k_leaf_neighbors<1><<<nbk, 256, 0, st>>>(tin, tout, stride, km->n_out, d_leaf_nbr, d_tile_first, stats);
            else if (K == 2) k_leaf_neighbors<2><<<nbk, 256, 0, st>>>(tin, tout, stride, km->n_out, d_leaf_nbr, d_tile_first, stats);
            else if (inverse) k_leaf_neighbors<3, true><<<nbk, 256, 0, st>>>(tin, tout, stride, km->n_out, d_leaf_nbr, d_tile_first, stats);
            else k_leaf_neighbors<3><<<nbk, 256, 0, st>>>(tin, tout, stride, km->n_out, d_leaf_nbr, d_tile_first, stats);
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
                                                                     stats);                                   \
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
    FX_HT("kmap: memset + launches");
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

fx_status fx::kmap_fetch_stats(fx_kmap* km) {
    if (km->stats_valid) return FX_OK;
    hipStream_t st = km->stream;
    unsigned long long* pairs = (unsigned long long*)(km->d_stats + 4);
    FX_HIP_TRY(hipMemsetAsync(pairs, 0, sizeof(int64_t) * (size_t)km->K3, st));
    if (km->n_tiles > 0) {
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
