// Index-grid build on the GPU (Sec. 3.3) and the grid queries (Listing 1).
//
// The paper orders the voxels with two radix sorts (tile key a, then key b) and derives the
// nodes from runs of equal key prefixes.  Here the tree does the ordering itself: every level
// keeps a child bitmask, set bit by bit (the paper's "register ... into its parent" steps
// 11.1-11.4), and a popcount prefix scan over the masks numbers the children in exactly the
// order the sorts would give (bit order of a mask = Listing 2's offset order; node order =
// parent order).  Only the few root tiles are ranked by comparison.  One streaming pass over
// ijk collects the distinct leaves and their voxel masks in a hash table; the levels above are
// built from those leaves (tens of thousands) instead of from the voxels (millions).
#include <cmath>

#include "common.h"
#include "tree_device.h"

#include <string.h>

#include <algorithm>
#include <new>
#include <vector>

namespace fx {

// ---------------------------------------------------------------------------------- helpers
struct GridPtrs {
    GridHeader* hdr;
    int64_t* vox_base;
    uint64_t* root_key;
    int32_t* root_batch;
    uint64_t* upper_mask;
    uint32_t* upper_prefix;
    uint64_t* lower_mask;
    uint32_t* lower_prefix;
    fx_leaf* leaf;
    int32_t cap_upper, cap_lower, cap_leaf, B;
};

// Row ranges of the grids of a batch, as the build's kernels take them: a single grid travels in the kernel
// arguments (no upload, no dependent load per row), more grids in a device array of (begin, end) pairs.
struct BatchRanges {
    const int64_t* d;
    int64_t begin0, end0;
};

// grid that owns row r (ranges sorted, non-overlapping), or -1
__device__ __forceinline__ int find_batch(const BatchRanges& J, int B, int64_t r) {
    if (B == 1) return (r >= J.begin0 && r < J.end0) ? 0 : -1;
    const int64_t* __restrict__ joff = J.d;
    int lo = 0, hi = B;  // last b with start_b <= r
    while (lo < hi) {
        int mid = (lo + hi) >> 1;
        if (joff[2 * mid] <= r) lo = mid + 1; else hi = mid;
    }
    int b = lo - 1;
    if (b < 0 || r >= joff[2 * b + 1]) return -1;
    return b;
}

__device__ __forceinline__ uint32_t mix32(uint32_t h, uint32_t v) {
    h ^= v;
    h *= 0x9E3779B1u;
    h ^= h >> 15;
    return h;
}

// ---------------------------------------------------------------------------------- block scan
constexpr int kScanThreads = 1024;
constexpr int kWordsPerThread = 4;
constexpr int kWordChunk = kScanThreads * kWordsPerThread;  // mask words per block
constexpr int kLeavesPerThread = 1;
constexpr int kLeafChunk = kScanThreads * kLeavesPerThread;

// exclusive scan of one value per thread over a 1024-thread block; returns the block total
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* total) {
    __shared__ uint32_t wave_sums[kScanThreads / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t incl = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t o = __shfl_up(incl, d);
        if (lane >= d) incl += o;
    }
    if (lane == 63) wave_sums[wave] = incl;
    __syncthreads();
    if (wave == 0) {
        uint32_t s = lane < kScanThreads / 64 ? wave_sums[lane] : 0;
#pragma unroll
        for (int d = 1; d < kScanThreads / 64; d <<= 1) {
            uint32_t o = __shfl_up(s, d);
            if (lane >= d) s += o;
        }
        if (lane < kScanThreads / 64) wave_sums[lane] = s;  // inclusive over waves
    }
    __syncthreads();
    const uint32_t wave_base = wave ? wave_sums[wave - 1] : 0;
    *total = wave_sums[kScanThreads / 64 - 1];
    __syncthreads();
    return wave_base + incl - v;
}

// ---------------------------------------------------------------------------------- voxels -> leaves
// The input rows are reduced to the set of distinct (grid, leaf) pairs, each with the 512-bit
// mask of its voxels (step 11.4; duplicates collapse in the bit).  Everything above the leaves
// -- root tiles, upper and lower nodes, the order of the leaves -- is derived afterwards from
// these few leaves instead of from the rows.  Two ways to get there:
//   * partitioned (large inputs): the rows are first scattered into buckets by a hash of their
//     leaf, so that all voxels of a leaf meet in one workgroup, which then builds the masks
//     of its bucket in LDS -- no global atomic per voxel (device-scope atomics run at memory,
//     about 13 G/s on this part, and would cost more than the rest of the build together);
//   * direct (small inputs, or when a bucket holds more leaves than its LDS table): one global
//     open-addressing table, one compare-and-swap per new leaf and one atomic OR per voxel.
struct LeafList {
    int4* key;           // [cap] (leaf i, leaf j, leaf k, grid): leaf coordinates = voxel coordinates >> 3
    int32_t* mask_idx;   // [cap] where the leaf's mask sits in `mask` (units of 8 words)
    uint64_t* mask;
    int32_t cap;
};

__device__ __forceinline__ uint32_t leaf_hash(int b, int li, int lj, int lk) {
    return mix32(mix32(mix32(mix32(0x811C9DC5u, (uint32_t)b), (uint32_t)li), (uint32_t)lj), (uint32_t)lk);
}

// ---- direct path
__global__ void __launch_bounds__(256)
k_voxels_to_leaves(const int32_t* __restrict__ ijk, int64_t n_rows, const BatchRanges joff, int B,
                   int32_t* __restrict__ slots, uint32_t slot_mask, LeafList L, GridHeader* hdr) {
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int b = r < n_rows ? find_batch(joff, B, r) : -1;
    int li = 0, lj = 0, lk = 0;
    uint32_t h = 0;
    bool claimed = false;
    if (b >= 0) {
        const int i = ijk[3 * r], j = ijk[3 * r + 1], k = ijk[3 * r + 2];
        li = i >> 3; lj = j >> 3; lk = k >> 3;
        h = leaf_hash(b, li, lj, lk) & slot_mask;
        bool found = false;
        for (uint32_t probe = 0; probe <= slot_mask; ++probe) {
            // slots hold a representative input row + 1 (0 = empty); device-coherent read: a slot
            // claimed from another XCD must be seen
            int32_t s = __hip_atomic_load(&slots[h], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (s == 0) {
                const int32_t old = atomicCAS(&slots[h], 0, (int32_t)r + 1);
                if (old == 0) { found = claimed = true; break; }
                s = old;
            }
            const int64_t q = s - 1;
            if ((ijk[3 * q] >> 3) == li && (ijk[3 * q + 1] >> 3) == lj && (ijk[3 * q + 2] >> 3) == lk &&
                find_batch(joff, B, q) == b) {
                found = true;
                break;
            }
            h = (h + 1) & slot_mask;
        }
        if (!found) atomicOr(&hdr->overflow, 4 | 32);   // table full: the leaf count is incomplete
        else atomicOr((unsigned long long*)&L.mask[(size_t)h * 8 + (i & 7)], 1ull << (((j & 7) << 3) | (k & 7)));
    }
    // list the newly claimed leaves: one counter update per wave, not per leaf
    const uint64_t cl = __ballot(claimed);
    if (cl) {
        const int lane = threadIdx.x & 63;
        const int leader = __ffsll((long long)cl) - 1;
        int base = 0;
        if (lane == leader) base = atomicAdd(&hdr->n_leaf_raw, __popcll(cl));
        base = __shfl(base, leader);
        if (claimed) {
            const int pos = base + __popcll(cl & ((1ull << lane) - 1));
            if (pos < L.cap) { L.key[pos] = make_int4(li, lj, lk, b); L.mask_idx[pos] = (int32_t)h; }
            else atomicOr(&hdr->overflow, 4);
        }
    }
}

// ---- coarse grid straight from the fine grid's leaves (Sec. 3.6.2: the grid of floor(ijk / 2))
// A fine leaf covers a 4x4x4 block of one coarse leaf: its 512-bit mask folds to 64 bits (a coarse voxel is active
// when any of its 8 children is), 16 bits in each of four words of the coarse leaf's mask.  One thread per fine
// leaf claims the coarse leaf in the table of the direct path (slots hold a representative fine leaf + 1) and ORs
// its four words in -- tens of thousands of items instead of a row per fine voxel through the whole voxel pass.
__global__ void __launch_bounds__(256)
k_coarse_leaves(TreeView fine, int32_t* __restrict__ slots, uint32_t slot_mask, LeafList L, GridHeader* hdr) {
    const int f = (int)((int64_t)blockIdx.x * blockDim.x + threadIdx.x);
    const bool has = f < fine.n_leaf;
    int li = 0, lj = 0, lk = 0, b = 0;
    uint32_t h = 0;
    bool claimed = false;
    if (has) {
        const fx_leaf* lf = fine.leaf + f;
        const int oi = lf->origin[0], oj = lf->origin[1], ok = lf->origin[2];
        b = lf->batch;
        li = oi >> 4; lj = oj >> 4; lk = ok >> 4;                      // coarse leaf coordinate: (origin >> 1) >> 3
        const int bi = (oi >> 1) & 7, bj = (oj >> 1) & 7, bk = (ok >> 1) & 7;   // 0 or 4: the block inside the coarse leaf
        uint64_t word[4];
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            uint64_t m = lf->mask[2 * a] | lf->mask[2 * a + 1];         // pairs along i
            m = (m | (m >> 1)) & 0x5555555555555555ull;                 // pairs along k, kept at the even bits
            m = (m | (m >> 1)) & 0x3333333333333333ull;                 // ... gathered into the low nibble of every byte
            m = (m | (m >> 2)) & 0x0F0F0F0F0F0F0F0Full;
            m = (m | (m >> 8)) & 0x00FF00FF00FF00FFull;                 // pairs along j: bytes 0, 2, 4, 6
            uint64_t r = 0;
#pragma unroll
            for (int cj = 0; cj < 4; ++cj) r |= ((m >> (16 * cj)) & 0xFull) << ((bj + cj) * 8 + bk);
            word[a] = r;
        }
        h = leaf_hash(b, li, lj, lk) & slot_mask;
        bool found = false;
        for (uint32_t probe = 0; probe <= slot_mask; ++probe) {
            int32_t sl = __hip_atomic_load(&slots[h], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (sl == 0) {
                const int32_t old = atomicCAS(&slots[h], 0, f + 1);
                if (old == 0) { found = claimed = true; break; }
                sl = old;
            }
            const fx_leaf* o = fine.leaf + (sl - 1);
            if ((o->origin[0] >> 4) == li && (o->origin[1] >> 4) == lj && (o->origin[2] >> 4) == lk && o->batch == b) {
                found = true;
                break;
            }
            h = (h + 1) & slot_mask;
        }
        if (!found) atomicOr(&hdr->overflow, 4 | 32);
        else {
#pragma unroll
            for (int a = 0; a < 4; ++a)
                if (word[a]) atomicOr((unsigned long long*)&L.mask[(size_t)h * 8 + bi + a], (unsigned long long)word[a]);
        }
    }
    // list the newly claimed coarse leaves: one counter update per wave
    const uint64_t cl = __ballot(claimed);
    if (cl) {
        const int lane = threadIdx.x & 63;
        const int leader = __ffsll((long long)cl) - 1;
        int base = 0;
        if (lane == leader) base = atomicAdd(&hdr->n_leaf_raw, __popcll(cl));
        base = __shfl(base, leader);
        if (claimed) {
            const int pos = base + __popcll(cl & ((1ull << lane) - 1));
            if (pos < L.cap) { L.key[pos] = make_int4(li, lj, lk, b); L.mask_idx[pos] = (int32_t)h; }
            else atomicOr(&hdr->overflow, 4);
        }
    }
}

// ---- padded grid straight from the grid's leaves (Sec. 3.6.2 grid construction by padding; Sec. 3.3's dilation)
// Dilation by r <= 8 moves a leaf's voxels into at most the 27 leaves around it, and a leaf of the padded grid
// takes voxels from at most the 27 source leaves around it.  Two passes, neither with an atomic per voxel or per
// mask word (atomics run at memory; an OR per word of every (leaf, neighbour) pair cost 220 us on a 38 k-leaf grid):
//   k_pad_claim   thread = (source leaf, one of its 27 neighbour positions): the neighbour receives a voxel iff the
//                 leaf has one within r of the shared face, edge or corner -- a mask test; such neighbours are
//                 claimed in the direct path's leaf table (a slot's representative is (source leaf, position) + 1);
//   k_pad_masks   wave = listed leaf of the padded grid: gathers the masks of the 27 source leaves around it into a
//                 24^3 box, dilates axis by axis towards the centre 8^3 and stores the leaf's mask with plain stores.
__device__ __forceinline__ uint32_t reach_bits(int p, int r) {
    // positions 0..7 along one axis whose voxels reach the neighbour at p - 1 (p = 1: the leaf itself) under dilation by r
    return p == 1 ? 0xFFu : (r == 0 ? 0u : (p == 0 ? (0xFFu >> (8 - r)) : ((0xFFu << (8 - r)) & 0xFFu)));
}

constexpr int kPadClaimThreads = 1024;
__global__ void __launch_bounds__(kPadClaimThreads)
k_pad_claim(TreeView src, int r, int32_t* __restrict__ slots, uint32_t slot_mask, LeafList L, GridHeader* hdr,
            int32_t* __restrict__ bad) {
    // Most leaves of the padded grid are leaves of the source grid.  Those are listed by their own thread (position
    // 13, the leaf itself) without the table: their masks sit behind the table's, at slot_mask + 1 + leaf.  A
    // neighbour position first looks its leaf up in the source tree (plain cached loads) and goes to the table only
    // when the leaf is new -- table probes are loads and compare-and-swaps that must see other workgroups' writes,
    // they run at memory, and one per (leaf, position) pair was 800 k of them on a 38 k-leaf grid (40 us).
    // List positions come from one counter; an update per wave would be 19 k updates of one address (150 us, they
    // run one after the other), so a workgroup counts its leaves in LDS and takes its run with one update.
    __shared__ int block_claims, block_base;
    const int lane = threadIdx.x & 63;
    if (threadIdx.x == 0) block_claims = 0;
    __syncthreads();
    const int64_t t = (int64_t)blockIdx.x * kPadClaimThreads + threadIdx.x;
    const int64_t f = t >> 5;
    const int piece = (int)(t & 31);
    int4 my_key = make_int4(0, 0, 0, 0);
    int32_t my_slot = -1;
    if (f < src.n_leaf && piece < 27) {
        const fx_leaf* lf = src.leaf + f;
        const int pa = piece / 9, pb = (piece / 3) % 3, pc = piece % 3;
        const uint32_t ia = reach_bits(pa, r), jb = reach_bits(pb, r), kc = reach_bits(pc, r);
        uint64_t region = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) if ((jb >> j) & 1) region |= (uint64_t)kc << (8 * j);
        uint64_t any = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) if ((ia >> i) & 1) any |= lf->mask[i] & region;
        const int b = lf->batch;
        const int64_t pi = (int64_t)lf->origin[0] + 8 * (pa - 1), pj = (int64_t)lf->origin[1] + 8 * (pb - 1),
                      pk = (int64_t)lf->origin[2] + 8 * (pc - 1);
        const int64_t lo = INT32_MIN, hi = (int64_t)INT32_MAX - 7;
        if (piece == 13) {
            my_slot = (int32_t)(slot_mask + 1 + (uint32_t)f);
            my_key = make_int4((int)(pi >> 3), (int)(pj >> 3), (int)(pk >> 3), b);
        } else if (any) {
            if (pi < lo || pi > hi || pj < lo || pj > hi || pk < lo || pk > hi) {
                atomicAdd(bad, 1);
            } else if (find_leaf<true>(src, b, (int)pi, (int)pj, (int)pk) < 0) {
                const int li = (int)(pi >> 3), lj = (int)(pj >> 3), lk = (int)(pk >> 3);
                uint32_t h = leaf_hash(b, li, lj, lk) & slot_mask;
                bool found = false;
                for (uint32_t probe = 0; probe <= slot_mask; ++probe) {
                    int32_t sl = __hip_atomic_load(&slots[h], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (sl == 0) {
                        const int32_t old = atomicCAS(&slots[h], 0, (int32_t)(f * 27 + piece + 1));
                        if (old == 0) {
                            found = true;
                            my_slot = (int32_t)h;
                            my_key = make_int4(li, lj, lk, b);
                            break;
                        }
                        sl = old;
                    }
                    const int rf = (sl - 1) / 27, rp = (sl - 1) - 27 * rf;
                    const fx_leaf* ro = src.leaf + rf;
                    if ((ro->origin[0] >> 3) + (rp / 9 - 1) == li && (ro->origin[1] >> 3) + ((rp / 3) % 3 - 1) == lj &&
                        (ro->origin[2] >> 3) + (rp % 3 - 1) == lk && ro->batch == b) {
                        found = true;
                        break;
                    }
                    h = (h + 1) & slot_mask;
                }
                if (!found) atomicOr(&hdr->overflow, 4 | 32);     // table full: the leaf count is incomplete
            }
        }
    }
    // positions: rank of the leaf inside the wave, the wave's run inside the workgroup, the workgroup's run
    const uint64_t cl = __ballot(my_slot >= 0);
    int wave_base = 0;
    if (lane == 0 && cl) wave_base = atomicAdd(&block_claims, __popcll(cl));
    wave_base = __shfl(wave_base, 0);
    __syncthreads();
    if (threadIdx.x == 0) block_base = block_claims ? atomicAdd(&hdr->n_leaf_raw, block_claims) : 0;
    __syncthreads();
    if (my_slot >= 0) {
        const int pos = block_base + wave_base + __popcll(cl & ((1ull << lane) - 1));
        if (pos < L.cap) { L.key[pos] = my_key; L.mask_idx[pos] = my_slot; }
        else atomicOr(&hdr->overflow, 4);
    }
}

constexpr int kPadWaves = 4;
__global__ void __launch_bounds__(64 * kPadWaves)
k_pad_masks(TreeView src, int r, LeafList L, const GridHeader* hdr) {
    __shared__ uint32_t box[kPadWaves][24][24];           // [i][j], bit = k: the 27 source leaves, then dilated along k
    __shared__ uint32_t along_j[kPadWaves][24][8];        // [i][centre j], 8 bits of k
    __shared__ unsigned long long centre[kPadWaves][8];   // the leaf's mask, byte (i, j) written by lane (i, j)
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int pos = blockIdx.x * kPadWaves + wave;
    const int n_listed = min(hdr->n_leaf_raw, L.cap);
    if (pos >= n_listed) return;
    auto wave_sync = [] { __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront"); __builtin_amdgcn_wave_barrier(); };
    const int4 key = L.key[pos];
    // the source leaves around the leaf: lane < 27 looks one up
    int around = -1;
    if (lane < 27) {
        const int64_t ni = (int64_t)key.x + (lane / 9 - 1), nj = (int64_t)key.y + ((lane / 3) % 3 - 1), nk = (int64_t)key.z + (lane % 3 - 1);
        const int64_t lo = -(1ll << 28), hi = (1ll << 28) - 1;      // leaf coordinates of int32 voxels
        if (ni >= lo && ni <= hi && nj >= lo && nj <= hi && nk >= lo && nk <= hi)
            around = find_leaf<true>(src, key.w, (int)(ni * 8), (int)(nj * 8), (int)(nk * 8));
    }
    // box rows: task = (pa, pb, i) takes word i of the three leaves (pa, pb, 0..2) and writes rows j = 0..7 of plane
    // 8 pa + i; only the planes and rows within r of the centre are read later
    const int first = 8 - r, last = 15 + r, width = 8 + 2 * r;
    for (int e = lane; e < 128; e += 64) {
        const int pa = e / 24, pb = (e / 8) % 3, i = e & 7;      // e < 72 are tasks
        const int plane = 8 * pa + i;
        const bool wanted = e < 72 && plane >= first && plane <= last && 8 * pb + 7 >= first && 8 * pb <= last;
        uint64_t w[3];
#pragma unroll
        for (int pc = 0; pc < 3; ++pc) {
            const int from = e < 72 ? (pa * 3 + pb) * 3 + pc : 0;
            const int f = __shfl(around, from);
            w[pc] = (wanted && f >= 0) ? src.leaf[f].mask[i] : 0ull;
        }
        if (wanted) {
#pragma unroll
            for (int j = 0; j < 8; ++j)
                box[wave][plane][8 * pb + j] = (uint32_t)((w[0] >> (8 * j)) & 0xFF) | ((uint32_t)((w[1] >> (8 * j)) & 0xFF) << 8) |
                                               ((uint32_t)((w[2] >> (8 * j)) & 0xFF) << 16);
        }
    }
    wave_sync();
    // along k: the centre byte of every row that the later steps read (|i - centre| and |j - centre| within r)
    for (int e = lane; e < width * width; e += 64) {
        const int a = e / width, ii = first + a, jj = first + (e - a * width);
        const uint32_t row = box[wave][ii][jj];
        uint32_t acc = 0;
        for (int sft = 8 - r; sft <= 8 + r; ++sft) acc |= row >> sft;
        box[wave][ii][jj] = acc & 0xFFu;
    }
    wave_sync();
    // along j
    for (int e = lane; e < width * 8; e += 64) {
        const int ii = first + (e >> 3), j = e & 7;
        uint32_t acc = 0;
        for (int d = -r; d <= r; ++d) acc |= box[wave][ii][j + 8 + d];
        along_j[wave][ii][j] = acc;
    }
    wave_sync();
    // along i: lane = (i, j) of the leaf
    {
        const int i = lane >> 3, j = lane & 7;
        uint32_t acc = 0;
        for (int d = -r; d <= r; ++d) acc |= along_j[wave][i + 8 + d][j];
        reinterpret_cast<unsigned char*>(centre[wave])[lane] = (unsigned char)acc;
    }
    wave_sync();
    if (lane < 8) L.mask[(size_t)L.mask_idx[pos] * 8 + lane] = centre[wave][lane];
}

// ---- subdivided grid straight from the grid's leaves (Sec. 3.6.2 grid construction by subdivision)
// A leaf of the fine grid is one octant (4^3 voxels) of a coarse leaf with every voxel doubled along each axis;
// it has exactly one source, so there is no table and no claim: thread = (coarse leaf, octant) expands the octant's
// 64 bits into the fine leaf's 512 (mask slot 8 * leaf + octant) and lists the leaf if the octant is not empty.
constexpr int kSubdivideThreads = 1024;
__global__ void __launch_bounds__(kSubdivideThreads)
k_subdivide_leaves(TreeView coarse, LeafList L, GridHeader* hdr, int32_t* __restrict__ bad) {
    __shared__ int block_count, block_base;
    const int lane = threadIdx.x & 63;
    if (threadIdx.x == 0) block_count = 0;
    __syncthreads();
    const int64_t t = (int64_t)blockIdx.x * kSubdivideThreads + threadIdx.x;
    const int64_t f = t >> 3;
    const int q = (int)(t & 7), bi = q >> 2, bj = (q >> 1) & 1, bk = q & 1;
    bool listed = false;
    int4 key = make_int4(0, 0, 0, 0);
    if (f < coarse.n_leaf) {
        const fx_leaf* lf = coarse.leaf + f;
        uint64_t fine[4];
        uint64_t any = 0;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const uint64_t w = lf->mask[4 * bi + a];
            uint64_t rows = 0;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                uint32_t x = (uint32_t)(w >> (8 * (4 * bj + jj) + 4 * bk)) & 0xFu;     // k = 4 bk .. 4 bk + 3 of row j
                x = (x | (x << 2)) & 0x33u;
                x = (x | (x << 1)) & 0x55u;
                x |= x << 1;                                                           // every bit twice
                rows |= (uint64_t)(x | (x << 8)) << (16 * jj);                         // the row twice
            }
            fine[a] = rows;
            any |= rows;
        }
        if (any) {
            const int o0 = lf->origin[0], o1 = lf->origin[1], o2 = lf->origin[2];
            const int lo = -(1 << 30), hi = (1 << 30) - 8;                             // doubled coordinates stay int32
            if (o0 < lo || o0 > hi || o1 < lo || o1 > hi || o2 < lo || o2 > hi) {
                atomicAdd(bad, 1);
            } else {
                listed = true;
                key = make_int4(2 * (o0 >> 3) + bi, 2 * (o1 >> 3) + bj, 2 * (o2 >> 3) + bk, lf->batch);
                uint64_t* m = L.mask + (size_t)t * 8;
#pragma unroll
                for (int a = 0; a < 4; ++a) { m[2 * a] = fine[a]; m[2 * a + 1] = fine[a]; }      // the plane twice
            }
        }
    }
    const uint64_t li = __ballot(listed);
    int wave_base = 0;
    if (lane == 0 && li) wave_base = atomicAdd(&block_count, __popcll(li));
    wave_base = __shfl(wave_base, 0);
    __syncthreads();
    if (threadIdx.x == 0) block_base = block_count ? atomicAdd(&hdr->n_leaf_raw, block_count) : 0;
    __syncthreads();
    if (listed) {
        const int pos = block_base + wave_base + __popcll(li & ((1ull << lane) - 1));
        if (pos < L.cap) { L.key[pos] = key; L.mask_idx[pos] = (int32_t)t; }
        else atomicOr(&hdr->overflow, 4);
    }
}

// ---- partitioned path
constexpr int kPartThreads = 1024;
constexpr int kPartRowsPerThread = 4;
constexpr int kPartChunk = kPartThreads * kPartRowsPerThread;   // rows per workgroup of the two row passes
constexpr int kMaxBuckets = 2048;
constexpr int kRowsPerBucket = 3072;                             // upper bound of the mean while the bucket count is below its cap
constexpr int kBucketSlots = 1024;                               // LDS leaf table of one bucket

struct PartRow { int i, j, k, b; uint32_t bucket; };

__device__ __forceinline__ PartRow load_part_row(const int32_t* __restrict__ ijk, int64_t n_rows,
                                                 const BatchRanges& joff, int B, int64_t r, uint32_t bucket_mask) {
    PartRow p;
    p.b = r < n_rows ? find_batch(joff, B, r) : -1;
    p.i = p.j = p.k = 0; p.bucket = 0;
    if (p.b >= 0) {
        p.i = ijk[3 * r]; p.j = ijk[3 * r + 1]; p.k = ijk[3 * r + 2];
        p.bucket = leaf_hash(p.b, p.i >> 3, p.j >> 3, p.k >> 3) & bucket_mask;
    }
    return p;
}

// rows per (bucket, workgroup): hist[bucket * n_wg + wg]
// What the first kernel of a build clears besides its own work: the head of the grid buffer (header, bases,
// root table, child masks) and the head of the scratch buffer (scan tickets and block sums, root-tile table).
// Nothing reads or updates either before the next launch.
struct ClearRanges {
    uint4* p[2];
    uint32_t n16[2];   // 16-byte units
};

__global__ void __launch_bounds__(kPartThreads)
k_bucket_count(const int32_t* __restrict__ ijk, int64_t n_rows, const BatchRanges joff, int B,
               uint32_t bucket_mask, uint32_t* __restrict__ hist, ClearRanges clr) {
    __shared__ uint32_t cnt[kMaxBuckets];
#pragma unroll
    for (int c = 0; c < 2; ++c)
        for (uint32_t e = blockIdx.x * kPartThreads + threadIdx.x; e < clr.n16[c]; e += gridDim.x * kPartThreads)
            clr.p[c][e] = make_uint4(0u, 0u, 0u, 0u);
    for (uint32_t e = threadIdx.x; e <= bucket_mask; e += kPartThreads) cnt[e] = 0;
    __syncthreads();
    const int64_t r0 = (int64_t)blockIdx.x * kPartChunk + threadIdx.x;
#pragma unroll
    for (int q = 0; q < kPartRowsPerThread; ++q) {
        const PartRow p = load_part_row(ijk, n_rows, joff, B, r0 + q * kPartThreads, bucket_mask);
        if (p.b >= 0) atomicAdd(&cnt[p.bucket], 1u);
    }
    __syncthreads();
    for (uint32_t e = threadIdx.x; e <= bucket_mask; e += kPartThreads) hist[(size_t)e * gridDim.x + blockIdx.x] = cnt[e];
}

// one wave per bucket: exclusive prefix over the workgroups' counts (in place) and the bucket total
__global__ void __launch_bounds__(256) k_bucket_scan(uint32_t* __restrict__ hist, int n_wg, int n_buckets,
                                                     uint32_t* __restrict__ totals) {
    const int bucket = (int)((blockIdx.x * blockDim.x + threadIdx.x) >> 6), lane = threadIdx.x & 63;
    if (bucket >= n_buckets) return;
    uint32_t* row = hist + (size_t)bucket * n_wg;
    uint32_t carry = 0;
    for (int base = 0; base < n_wg; base += 64) {
        const int e = base + lane;
        const uint32_t v = e < n_wg ? row[e] : 0u;
        uint32_t incl = v;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t o = __shfl_up(incl, d);
            if (lane >= d) incl += o;
        }
        if (e < n_wg) row[e] = carry + incl - v;
        carry += __shfl(incl, 63);
    }
    if (lane == 0) totals[bucket] = carry;
}

// scatter the rows into their buckets as (i, j, k, grid) records; the records of one workgroup
// are ordered by bucket in LDS first so that each bucket receives one contiguous run
__global__ void __launch_bounds__(kPartThreads)
k_bucket_scatter(const int32_t* __restrict__ ijk, int64_t n_rows, const BatchRanges joff, int B,
                 uint32_t bucket_mask, const uint32_t* __restrict__ hist, const uint32_t* __restrict__ totals,
                 uint32_t* __restrict__ bucket_start, int4* __restrict__ records) {
    extern __shared__ __align__(16) unsigned char part_lds[];
    int4* rec = reinterpret_cast<int4*>(part_lds);                          // [kPartChunk]
    uint32_t* dest = reinterpret_cast<uint32_t*>(rec + kPartChunk);         // [kPartChunk]
    uint32_t* cnt = dest + kPartChunk;                                      // [kMaxBuckets] rows of this workgroup
    uint32_t* lstart = cnt + kMaxBuckets;                                   // [kMaxBuckets] first LDS slot
    uint32_t* gbase = lstart + kMaxBuckets;                                 // [kMaxBuckets] first global record
    const uint32_t n_buckets = bucket_mask + 1;
    const int tid = threadIdx.x;
    // bucket starts = exclusive scan of the totals (every workgroup repeats it; the first one publishes it)
    {
        uint32_t v[2], sum = 0;
#pragma unroll
        for (int q = 0; q < 2; ++q) { const uint32_t e = tid * 2 + q; v[q] = e < n_buckets ? totals[e] : 0u; sum += v[q]; }
        uint32_t total;
        uint32_t run = block_exclusive_scan(sum, &total);
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const uint32_t e = tid * 2 + q;
            if (e < n_buckets) {
                gbase[e] = run + hist[(size_t)e * gridDim.x + blockIdx.x];
                if (blockIdx.x == 0) bucket_start[e] = run;
            }
            run += v[q];
        }
        if (blockIdx.x == 0 && tid == 0) bucket_start[n_buckets] = total;
    }
    for (uint32_t e = tid; e < n_buckets; e += kPartThreads) cnt[e] = 0;
    __syncthreads();
    PartRow p[kPartRowsPerThread];
    uint32_t rank[kPartRowsPerThread];
    const int64_t r0 = (int64_t)blockIdx.x * kPartChunk + tid;
#pragma unroll
    for (int q = 0; q < kPartRowsPerThread; ++q) {
        p[q] = load_part_row(ijk, n_rows, joff, B, r0 + q * kPartThreads, bucket_mask);
        rank[q] = p[q].b >= 0 ? atomicAdd(&cnt[p[q].bucket], 1u) : 0u;
    }
    __syncthreads();
    // first LDS slot of every bucket = exclusive scan of this workgroup's counts
    {
        uint32_t v[2], sum = 0;
#pragma unroll
        for (int q = 0; q < 2; ++q) { const uint32_t e = tid * 2 + q; v[q] = e < n_buckets ? cnt[e] : 0u; sum += v[q]; }
        uint32_t total;
        uint32_t run = block_exclusive_scan(sum, &total);
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const uint32_t e = tid * 2 + q;
            if (e < n_buckets) lstart[e] = run;
            run += v[q];
        }
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < kPartRowsPerThread; ++q) {
        if (p[q].b < 0) continue;
        const uint32_t s = lstart[p[q].bucket] + rank[q];
        rec[s] = make_int4(p[q].i, p[q].j, p[q].k, p[q].b);
        dest[s] = gbase[p[q].bucket] + rank[q];
    }
    __syncthreads();
    // number of valid rows of this workgroup = last bucket's start + count
    const uint32_t n_local = lstart[bucket_mask] + cnt[bucket_mask];
    for (uint32_t s = tid; s < n_local; s += kPartThreads) records[dest[s]] = rec[s];
}

// one workgroup per bucket: the bucket's distinct leaves and their masks, built in LDS
constexpr int kBucketThreads = 1024;
__global__ void __launch_bounds__(kBucketThreads)
k_bucket_leaves(const int4* __restrict__ records, const uint32_t* __restrict__ bucket_start, LeafList L, GridHeader* hdr) {
    __shared__ int32_t rep[kBucketSlots];                 // representative record + 1 (0 = empty)
    __shared__ __align__(16) unsigned long long mask[kBucketSlots * 8];
    __shared__ int32_t list_base;
    static_assert(kBucketSlots == kBucketThreads, "one table slot per thread in the listing step");
    const int tid = threadIdx.x;
    rep[tid] = 0;
    for (int e = tid; e < kBucketSlots * 4; e += kBucketThreads) reinterpret_cast<ulonglong2*>(mask)[e] = make_ulonglong2(0ull, 0ull);
    __syncthreads();
    const uint32_t begin = bucket_start[blockIdx.x], end = bucket_start[blockIdx.x + 1];
    bool full = false;
    for (uint32_t r = begin + tid; r < end; r += kBucketThreads) {
        const int4 v = records[r];
        const int li = v.x >> 3, lj = v.y >> 3, lk = v.z >> 3;
        uint32_t h = (leaf_hash(v.w, li, lj, lk) >> 12) & (kBucketSlots - 1);   // other bits than the bucket's
        bool found = false;
        for (int probe = 0; probe < kBucketSlots; ++probe) {
            int32_t s = rep[h];
            if (s == 0) {
                const int32_t old = atomicCAS(&rep[h], 0, (int32_t)(r - begin) + 1);
                if (old == 0) { found = true; break; }
                s = old;
            }
            const int4 o = records[begin + (uint32_t)(s - 1)];
            if ((o.x >> 3) == li && (o.y >> 3) == lj && (o.z >> 3) == lk && o.w == v.w) { found = true; break; }
            h = (h + 1) & (kBucketSlots - 1);
        }
        if (found) atomicOr(&mask[h * 8 + (v.x & 7)], 1ull << (((v.y & 7) << 3) | (v.z & 7)));
        else full = true;
    }
    if (full) atomicOr(&hdr->overflow, 64);   // more leaves than the table holds: the build falls back to the direct path
    __syncthreads();
    // append the bucket's leaves to the global list (thread = table slot)
    const int32_t s = rep[tid];
    uint32_t total;
    const uint32_t before = block_exclusive_scan(s != 0 ? 1u : 0u, &total);
    if (tid == 0) list_base = total ? atomicAdd(&hdr->n_leaf_raw, (int)total) : 0;
    __syncthreads();
    if (s == 0) return;
    const int pos = list_base + (int)before;
    if (pos < L.cap) {
        const int4 v = records[begin + (uint32_t)(s - 1)];
        L.key[pos] = make_int4(v.x >> 3, v.y >> 3, v.z >> 3, v.w);
        L.mask_idx[pos] = pos;
#pragma unroll
        for (int w = 0; w < 8; w += 2)
            *reinterpret_cast<ulonglong2*>(&L.mask[(size_t)pos * 8 + w]) = *reinterpret_cast<const ulonglong2*>(&mask[tid * 8 + w]);
    } else {
        atomicOr(&hdr->overflow, 4);
    }
}

// key of distinct leaf `idx`, or false past the end
__device__ __forceinline__ bool leaf_at(const LeafList& L, const GridHeader* hdr, int64_t idx, int4* key) {
    if (idx >= L.cap) return false;
    *key = L.key[idx];            // fetched together with the count, not after it (entries past the count are unused)
    return idx < hdr->n_leaf_raw;
}

// ---------------------------------------------------------------------------------- root tiles
// Distinct (grid, tile) pairs of the leaves go into a small open-addressing table whose slots
// hold a representative leaf (+1; 0 = empty).  Called by all threads of a workgroup together (`has`:
// this thread holds leaf `idx` with key `key`).
constexpr int kFindTilesThreads = 1024;
constexpr int kTileRounds = 16;
__device__ __forceinline__ void find_tile_item(const LeafList& L, GridHeader* hdr, int idx, bool has, const int4& key,
                                               int32_t* __restrict__ tile_slots, int32_t* __restrict__ rep_leaves) {
    const int4 tile = make_int4(key.x >> 9, key.y >> 9, key.z >> 9, key.w);   // leaf coordinate >> 9 = voxel >> 12
    auto same = [](const int4& a, const int4& b) { return a.x == b.x && a.y == b.y && a.z == b.z && a.w == b.w; };
    // One thread per distinct tile of the WORKGROUP goes to the table: accesses to one address from all over the
    // device queue up at memory (a coherent read of one slot from each of 600 waves took longer than the rest of
    // this launch), and nearly all leaves share one tile.  In rounds, the first thread still waiting proposes its
    // tile (the first waiting lane of every wave bids with an LDS atomic; same-address LDS atomics run lane by lane,
    // so not every lane) and every thread with that tile is done: two barriers and no memory access per distinct tile.
    __shared__ int leader[kTileRounds];
    __shared__ int4 leader_tile[kTileRounds];
    const int tid = (int)threadIdx.x;
    bool waiting = has, speaker = false;
    for (int batch = 0; batch < (int)blockDim.x / kTileRounds + 1; ++batch) {
        if (tid < kTileRounds) leader[tid] = INT32_MAX;
        if (!__syncthreads_or(waiting)) break;
        for (int r = 0; r < kTileRounds; ++r) {
            const uint64_t bids = __ballot(waiting);
            if (bids && (tid & 63) == __ffsll((long long)bids) - 1) atomicMin(&leader[r], tid);
            __syncthreads();
            const int l = leader[r];
            if (l == INT32_MAX) break;
            if (tid == l) { leader_tile[r] = tile; speaker = true; }
            __syncthreads();
            if (waiting && same(tile, leader_tile[r])) waiting = false;
        }
    }
    if (!speaker) return;
    uint32_t h = mix32(mix32(mix32(mix32(0x811C9DC5u, (uint32_t)tile.w), (uint32_t)tile.x), (uint32_t)tile.y), (uint32_t)tile.z);
    h &= (kTileHashSlots - 1);
    for (int probe = 0; probe < kTileHashSlots; ++probe) {
        // device-coherent read: once a tile is in, nobody else reaches the compare-and-swap
        int32_t s = __hip_atomic_load(&tile_slots[h], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (s == 0) {
            if (hdr->n_tiles_raw > kMaxTiles) break;  // over the limit: reported by the ranking step
            const int32_t old = atomicCAS(&tile_slots[h], 0, idx + 1);
            if (old == 0) {
                const int pos = atomicAdd(&hdr->n_tiles_raw, 1);
                if (pos < kMaxTiles) rep_leaves[pos] = idx;
                break;
            }
            s = old;
        }
        const int4 o = L.key[s - 1];
        if (o.w == tile.w && (o.x >> 9) == tile.x && (o.y >> 9) == tile.y && (o.z >> 9) == tile.z) break;
        h = (h + 1) & (kTileHashSlots - 1);
    }
}

__global__ void __launch_bounds__(kFindTilesThreads)
k_find_tiles(LeafList L, int32_t* __restrict__ tile_slots, int32_t* __restrict__ rep_leaves, GridHeader* hdr) {
    if (hdr->overflow) return;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int4 key = make_int4(0, 0, 0, 0);
    const bool has = leaf_at(L, hdr, idx, &key);
    find_tile_item(L, hdr, (int)idx, has, key, tile_slots, rep_leaves);
}

// Rank every tile among all tiles by (grid, signed tile i, j, k): its rank is its upper-node id
// (the run index M of Sec. 3.3 step 5).  O(T^2) comparisons; T is tiny for real scenes.
// `t` = global thread number of the launch.
__device__ __forceinline__ void rank_tile_item(const LeafList& L, const int32_t* __restrict__ rep_leaves, const GridPtrs& g,
                                               int t, int t_stride) {
    const int raw = g.hdr->n_tiles_raw;
    const int T = raw < kMaxTiles ? raw : kMaxTiles;
    if (t == 0) {
        int ov = 0;
        if (raw > kMaxTiles) ov |= 8;
        if (T > g.cap_upper) ov |= 1;
        g.hdr->n_upper = T;
        if (ov) atomicOr(&g.hdr->overflow, ov);
    }
    if (T > g.cap_upper) return;
    for (; t < T; t += t_stride) {
        const int4 me = L.key[rep_leaves[t]];
        const uint64_t key = tile_key(me.x << 3, me.y << 3, me.z << 3);
        int rank = 0;
        for (int o = 0; o < T; ++o) {
            const int4 ot = L.key[rep_leaves[o]];
            const uint64_t ko = tile_key(ot.x << 3, ot.y << 3, ot.z << 3);
            rank += (ot.w < me.w) || (ot.w == me.w && ko < key);
        }
        g.root_key[rank] = key;
        g.root_batch[rank] = me.w;
    }
}

__global__ void k_rank_tiles(LeafList L, const int32_t* __restrict__ rep_leaves, GridPtrs g) {
    if (g.hdr->overflow) return;
    rank_tile_item(L, rep_leaves, g, blockIdx.x * blockDim.x + threadIdx.x, gridDim.x * blockDim.x);
}

// ---------------------------------------------------------------------------------- leaves -> tree
// One thread per distinct leaf.
// LEVEL 0: lower-node bit in the upper node's child mask   (step 11.2)
// LEVEL 1: leaf bit in the lower node's child mask         (step 11.3)
// LEVEL 2: the leaf's final id is known: move its mask into the leaf record
template <int LEVEL>
__device__ __forceinline__ void insert_item(const LeafList& L, const GridPtrs& g, int idx, const int4& key) {
    const int b = key.w;
    const int i = key.x << 3, j = key.y << 3, k = key.z << 3;   // the leaf's origin
    const int u = find_upper_short(g.root_key, g.root_batch, g.hdr->n_upper, b, tile_key(i, j, k));
    if (u < 0) return;
    if (LEVEL == 0) {
        const int off = upper_off(i, j, k);
        uint64_t* word = g.upper_mask + (size_t)u * kUpperWords + (off >> 6);
        const uint64_t bit = 1ull << (off & 63);
        // thousands of leaves share each of these bits: look before the atomic (a stale read only
        // costs a redundant one)
        if (!(*word & bit)) atomicOr((unsigned long long*)word, (unsigned long long)bit);
        return;
    }
    const int l = child_of(g.upper_mask + (size_t)u * kUpperWords, g.upper_prefix + (size_t)u * kUpperWords,
                           upper_off(i, j, k));
    if (l < 0 || l >= g.cap_lower) return;
    if (LEVEL == 1) {
        const int off = lower_off(i, j, k);
        uint64_t* word = g.lower_mask + (size_t)l * kLowerWords + (off >> 6);
        atomicOr((unsigned long long*)word, 1ull << (off & 63));
        return;
    }
    const int f = child_of(g.lower_mask + (size_t)l * kLowerWords, g.lower_prefix + (size_t)l * kLowerWords,
                           lower_off(i, j, k));
    if (f < 0 || f >= g.cap_leaf) return;
    fx_leaf* lf = &g.leaf[f];
    const uint64_t* src = L.mask + (size_t)L.mask_idx[idx] * 8;
#pragma unroll
    for (int w = 0; w < 8; ++w) lf->mask[w] = src[w];
    lf->origin[0] = i;
    lf->origin[1] = j;
    lf->origin[2] = k;
    lf->batch = b;
}

template <int LEVEL>
__global__ void k_insert(LeafList L, GridPtrs g) {
    if (g.hdr->overflow) return;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int4 key;
    if (!leaf_at(L, g.hdr, idx, &key)) return;
    insert_item<LEVEL>(L, g, (int)idx, key);
}

// LEVEL 0 for all leaves: thousands of leaves share every lower node, and atomics on one address queue up at
// memory one after the other.  A workgroup therefore collects the bits of its 1024 leaves in LDS copies of the
// first few upper nodes' masks and sends each touched word to memory once; leaves of further upper nodes (rare)
// update memory directly.
constexpr int kInsertUpperThreads = 1024;
constexpr int kAggUpper = 4;
// With at most kRankInBlock root tiles possible (the capacity of the upper level says so) the launch that ranks the
// tiles is dropped: every workgroup ranks them itself into LDS (a handful of comparisons) and looks its leaves up
// there; the first workgroup also writes the root table and the count for the launches that follow.
constexpr int kRankInBlock = 16;
__global__ void __launch_bounds__(kInsertUpperThreads) k_insert_upper(LeafList L, GridPtrs g,
                                                                       const int32_t* __restrict__ rep_leaves, int rank_here) {
    __shared__ unsigned long long bits[kAggUpper * kUpperWords];
    __shared__ uint64_t tile_keys[kRankInBlock], ranked_key[kRankInBlock];
    __shared__ int32_t tile_batch[kRankInBlock], ranked_batch[kRankInBlock];
    if (g.hdr->overflow) return;
    const uint64_t* root_key = g.root_key;
    const int32_t* root_batch = g.root_batch;
    int n_upper;
    if (rank_here) {
        const int raw = g.hdr->n_tiles_raw;
        const int T = raw < kMaxTiles ? raw : kMaxTiles;
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            int ov = 0;
            if (raw > kMaxTiles) ov |= 8;
            if (T > g.cap_upper) ov |= 1;
            g.hdr->n_upper = T;
            if (ov) atomicOr(&g.hdr->overflow, ov);
        }
        if (T > g.cap_upper) return;              // cap_upper <= kRankInBlock on this path
        if ((int)threadIdx.x < T) {
            const int4 me = L.key[rep_leaves[threadIdx.x]];
            tile_keys[threadIdx.x] = tile_key(me.x << 3, me.y << 3, me.z << 3);
            tile_batch[threadIdx.x] = me.w;
        }
        __syncthreads();
        if ((int)threadIdx.x < T) {
            const uint64_t key = tile_keys[threadIdx.x];
            const int32_t b = tile_batch[threadIdx.x];
            int rank = 0;
            for (int o = 0; o < T; ++o) rank += (tile_batch[o] < b) || (tile_batch[o] == b && tile_keys[o] < key);
            ranked_key[rank] = key;
            ranked_batch[rank] = b;
            if (blockIdx.x == 0) { g.root_key[rank] = key; g.root_batch[rank] = b; }
        }
        n_upper = T;
        root_key = ranked_key;
        root_batch = ranked_batch;
    } else {
        n_upper = g.hdr->n_upper;
    }
    const int n_agg_words = (n_upper < kAggUpper ? n_upper : kAggUpper) * kUpperWords;
    for (int e = threadIdx.x; e < n_agg_words; e += kInsertUpperThreads) bits[e] = 0ull;
    __syncthreads();
    const int64_t idx = (int64_t)blockIdx.x * kInsertUpperThreads + threadIdx.x;
    int4 key;
    if (leaf_at(L, g.hdr, idx, &key)) {
        const int i = key.x << 3, j = key.y << 3, k = key.z << 3;
        const int u = find_upper_short(root_key, root_batch, n_upper, key.w, tile_key(i, j, k));
        if (u >= 0) {
            const int off = upper_off(i, j, k);
            const int word = u * kUpperWords + (off >> 6);
            const unsigned long long bit = 1ull << (off & 63);
            if (word < n_agg_words) atomicOr(&bits[word], bit);
            else atomicOr((unsigned long long*)g.upper_mask + word, bit);
        }
    }
    __syncthreads();
    for (int e = threadIdx.x; e < n_agg_words; e += kInsertUpperThreads) {
        const unsigned long long v = bits[e];
        if (v) atomicOr((unsigned long long*)g.upper_mask + e, v);
    }
}

// ---------------------------------------------------------------------------------- popcount scans
// which level's masks a scan runs over
struct LevelScan {
    const uint64_t* words;
    uint32_t* prefix;
    const int32_t* n_nodes;   // device count of nodes at this level
    int words_per_node;
    int32_t* n_children;      // device count to write (next level)
    int32_t child_cap;
    int32_t overflow_bit;
};

// Single-pass scans over several workgroups.  Each scan has a ticket counter and one word per workgroup (both
// start at zero).  A workgroup takes the next chunk in the order in which workgroups start running, publishes its
// chunk's total as total + 1 in its word with one device-scope store -- the word carries the value, so no fence is
// needed -- and then adds up the words of the chunks before it, waiting for those not yet written.  It only ever
// waits for workgroups that started before it and that publish before they wait themselves, so every wait ends;
// the wait is bounded all the same and an expired one is reported through the overflow word (bit 7).
struct ScanSync {
    uint32_t* ticket;
    uint32_t* sums;
};
constexpr int kScanSpinLimit = 1 << 20;

// the workgroup's chunk, or -1 when an earlier step of the build has failed (one thread decides for all)
__device__ __forceinline__ int ordered_chunk(uint32_t* ticket, const GridHeader* hdr) {
    __shared__ int chunk;
    if (threadIdx.x == 0) chunk = hdr->overflow ? -1 : (int)atomicAdd(ticket, 1u);
    __syncthreads();
    return chunk;
}

// publishes `total` as the sum of chunk `mine`; returns the sum of the chunks before it (to every thread)
__device__ __forceinline__ uint64_t publish_and_sum_before(const ScanSync& y, int mine, uint32_t total, GridHeader* hdr) {
    __shared__ unsigned long long acc;
    if (threadIdx.x == 0) {
        acc = 0ull;
        __hip_atomic_store(&y.sums[mine], total + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    unsigned long long sb = 0;
    for (int i = threadIdx.x; i < mine; i += blockDim.x) {
        uint32_t v = 0;
        for (int spin = 0; spin < kScanSpinLimit; ++spin) {
            v = __hip_atomic_load(&y.sums[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (v) break;
            __builtin_amdgcn_s_sleep(2);
        }
        if (!v) { atomicOr(&hdr->overflow, 128); v = 1u; }
        sb += v - 1u;
    }
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) sb += (unsigned long long)__shfl_xor((long long)sb, d);
    if ((threadIdx.x & 63) == 0 && sb) atomicAdd(&acc, sb);
    __syncthreads();
    const uint64_t before = acc;
    __syncthreads();
    return before;
}

// exclusive popcount prefix per mask word over all nodes of a level; the last chunk writes the number of children
__global__ void __launch_bounds__(kScanThreads) k_scan_words(LevelScan s, GridHeader* hdr, ScanSync y) {
    const int chunk = ordered_chunk(y.ticket, hdr);
    if (chunk < 0) return;
    const int64_t n_words = (int64_t)(*s.n_nodes) * s.words_per_node;
    const int64_t base = (int64_t)chunk * kWordChunk;
    if (base >= n_words && chunk != 0) return;
    const int64_t w0 = base + (int64_t)threadIdx.x * kWordsPerThread;
    uint32_t pc[kWordsPerThread];
    uint32_t sum = 0;
#pragma unroll
    for (int q = 0; q < kWordsPerThread; ++q) {
        pc[q] = (w0 + q < n_words) ? (uint32_t)__popcll(s.words[w0 + q]) : 0u;
        sum += pc[q];
    }
    uint32_t total;
    uint32_t run = block_exclusive_scan(sum, &total);
    const uint64_t before = publish_and_sum_before(y, chunk, total, hdr);
    run += (uint32_t)before;
#pragma unroll
    for (int q = 0; q < kWordsPerThread; ++q) {
        if (w0 + q < n_words) s.prefix[w0 + q] = run;
        run += pc[q];
    }
    if (threadIdx.x == 0 && base + kWordChunk >= n_words) {
        const uint64_t all = before + total;
        *s.n_children = (int32_t)(all < (uint64_t)INT32_MAX ? all : (uint64_t)INT32_MAX);
        if ((int64_t)all > s.child_cap) atomicOr(&hdr->overflow, s.overflow_bit);
    }
}

// First voxel index of every grid of the batch (leaves are ordered by grid): the thread that owns
// the first leaf of a grid writes the entries of that grid and of the empty grids before it; the
// owner of the last leaf writes the entries after it.  (The buffer starts zeroed: no leaves, all 0.)
__device__ __forceinline__ void note_vox_base(const fx_leaf* __restrict__ leaf, int64_t l, int64_t n_leaf, int64_t offset,
                                              int64_t n_voxels, int64_t* __restrict__ vox_base, int B) {
    if (B == 1) {      // a single grid: its bases are 0 (the buffer's initial value) and the voxel count, no record is read
        if (l == n_leaf - 1) vox_base[1] = n_voxels;
        return;
    }
    const int bcur = leaf[l].batch;
    const int bprev = l ? leaf[l - 1].batch : -1;
    for (int b = bprev + 1; b <= bcur; ++b) vox_base[b] = offset;
    if (l == n_leaf - 1)
        for (int b = bcur + 1; b <= B; ++b) vox_base[b] = n_voxels;
}

// Leaf level: mOffset = exclusive scan of the leaves' active-voxel counts; mPrefixSum = the
// seven 9-bit inclusive word prefixes of Listing 1.
__global__ void __launch_bounds__(kScanThreads) k_scan_leaves(fx_leaf* __restrict__ leaf, GridHeader* hdr, ScanSync y,
                                                               int64_t* __restrict__ vox_base, int B) {
    const int chunk = ordered_chunk(y.ticket, hdr);
    if (chunk < 0) return;
    const int64_t n_leaf = hdr->n_leaf;
    const int64_t base = (int64_t)chunk * kLeafChunk;
    if (base >= n_leaf && chunk != 0) return;
    const int64_t l0 = base + (int64_t)threadIdx.x * kLeavesPerThread;
    uint32_t cnt[kLeavesPerThread];
    uint32_t sum = 0;
#pragma unroll
    for (int q = 0; q < kLeavesPerThread; ++q) {
        cnt[q] = 0;
        if (l0 + q < n_leaf) {
            uint64_t pre = 0;
            uint32_t acc = 0;
#pragma unroll
            for (int w = 0; w < 8; ++w) {
                acc += (uint32_t)__popcll(leaf[l0 + q].mask[w]);
                if (w < 7) pre |= (uint64_t)acc << (9 * w);
            }
            leaf[l0 + q].prefix = pre;
            cnt[q] = acc;
        }
        sum += cnt[q];
    }
    {   // voxels that sit in locally dense leaves, summed over the grid
        uint32_t dense = 0;
#pragma unroll
        for (int q = 0; q < kLeavesPerThread; ++q) dense += cnt[q] >= (uint32_t)kDenseLeafVoxels ? cnt[q] : 0u;
#pragma unroll
        for (int d = 32; d > 0; d >>= 1) dense += (uint32_t)__shfl_xor((int)dense, d);
        if ((threadIdx.x & 63) == 0 && dense) atomicAdd((unsigned long long*)&hdr->n_voxels_dense, (unsigned long long)dense);
    }
    uint32_t total;
    const uint32_t local = block_exclusive_scan(sum, &total);
    const uint64_t before = publish_and_sum_before(y, chunk, total, hdr);
    const bool last = base + kLeafChunk >= n_leaf;
    const int64_t all = (int64_t)(before + total);      // the grid's voxel count, in the last chunk
    int64_t run = (int64_t)before + local;
#pragma unroll
    for (int q = 0; q < kLeavesPerThread; ++q) {
        if (l0 + q < n_leaf) {
            leaf[l0 + q].offset = run;
            // only the last chunk holds the last leaf, the one reader of the grand total
            note_vox_base(leaf, l0 + q, n_leaf, run, all, vox_base, B);
        }
        run += cnt[q];
    }
    if (threadIdx.x == 0 && last) {
        hdr->n_voxels = all;
        if (all > (int64_t)INT32_MAX) atomicOr(&hdr->overflow, 16);
    }
}

// The build's one read-back (Sec. 3.3 step 10): counts and per-grid voxel bases, written by the
// device straight into pinned host memory -- one tiny launch instead of two copy-engine transfers.
// The last word written is a ticket the host polls for, which returns sooner than a stream wait.
__global__ void k_publish(const GridHeader* __restrict__ hdr, const int64_t* __restrict__ vox_base, int B,
                          unsigned char* __restrict__ host, int32_t* __restrict__ host_ticket, int32_t ticket) {
    const int t = threadIdx.x;
    constexpr int kHdrWords = (int)(sizeof(GridHeader) / sizeof(int32_t));
    if (t < kHdrWords) reinterpret_cast<int32_t*>(host)[t] = reinterpret_cast<const int32_t*>(hdr)[t];
    for (int b = t; b <= B; b += blockDim.x) reinterpret_cast<int64_t*>(host + sizeof(GridHeader))[b] = vox_base[b];
    __threadfence_system();
    __syncthreads();
    if (t == 0) __hip_atomic_store(host_ticket, ticket, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

// ---------------------------------------------------------------------------------- queries
// One wave per leaf.  The wave first lists the positions of the leaf's active voxels in LDS, in index order (lane =
// bit of the current mask word: every lane tests its bit), then writes the leaf's 3 n coordinates as one contiguous
// run of 4-byte words -- a voxel's three coordinates written by its own lane would be three 4-byte stores 12 bytes
// apart per lane.
__global__ void __launch_bounds__(256) k_grid_ijk(TreeView t, int32_t* __restrict__ ijk_out, int32_t* __restrict__ jidx_out,
                                                   int shift) {
    __shared__ uint16_t active[4][512];
    const int f = (int)(((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6);
    if (f >= t.n_leaf) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const fx_leaf* lf = t.leaf + f;
    const uint64_t lt = (1ull << lane) - 1;
    int n = 0;
#pragma unroll
    for (int w = 0; w < 8; ++w) {
        const uint64_t m = lf->mask[w];
        if ((m >> lane) & 1) active[wave][n + __popcll(m & lt)] = (uint16_t)(w * 64 + lane);
        n += __popcll(m);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    const int64_t first = lf->offset;
    const int o0 = lf->origin[0], o1 = lf->origin[1], o2 = lf->origin[2];
    for (int e = lane; e < 3 * n; e += 64) {
        const int v = e / 3, axis = e - 3 * v;
        const int pos = active[wave][v];
        const int c = axis == 0 ? o0 + (pos >> 6) : axis == 1 ? o1 + ((pos >> 3) & 7) : o2 + (pos & 7);
        ijk_out[3 * first + e] = c >> shift;
    }
    if (jidx_out) {
        const int b = lf->batch;
        for (int e = lane; e < n; e += 64) jidx_out[first + e] = b;
    }
}

__global__ void k_ijk_to_index(TreeView t, const int32_t* __restrict__ ijk, const int32_t* __restrict__ jidx,
                               int64_t n, int32_t* __restrict__ out) {
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= n) return;
    const int b = jidx ? jidx[r] : 0;
    int v = -1;
    if (b >= 0 && b < t.B) v = get_value(t, b, ijk[3 * r], ijk[3 * r + 1], ijk[3 * r + 2]);
    out[r] = v;
}

// ---------------------------------------------------------------------------------- host side
static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

static void layout(fx_grid* g) {
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    const size_t o_hdr = take(sizeof(GridHeader));
    const size_t o_vox = take(sizeof(int64_t) * ((size_t)g->B + 1));
    const size_t o_rk = take(sizeof(uint64_t) * g->cap_upper);
    const size_t o_rb = take(sizeof(int32_t) * g->cap_upper);
    const size_t o_um = take(sizeof(uint64_t) * kUpperWords * (size_t)g->cap_upper);
    const size_t o_up = take(sizeof(uint32_t) * kUpperWords * (size_t)g->cap_upper);
    const size_t o_lm = take(sizeof(uint64_t) * kLowerWords * (size_t)g->cap_lower);
    const size_t o_lp = take(sizeof(uint32_t) * kLowerWords * (size_t)g->cap_lower);
    const size_t o_lf = take(sizeof(fx_leaf) * (size_t)g->cap_leaf);
    g->buf_bytes = off;
    char* p = (char*)g->buf;
    if (!p) return;
    g->d_hdr = (GridHeader*)(p + o_hdr);
    g->d_vox_base = (int64_t*)(p + o_vox);
    g->d_root_key = (uint64_t*)(p + o_rk);
    g->d_root_batch = (int32_t*)(p + o_rb);
    g->d_upper_mask = (uint64_t*)(p + o_um);
    g->d_upper_prefix = (uint32_t*)(p + o_up);
    g->d_lower_mask = (uint64_t*)(p + o_lm);
    g->d_lower_prefix = (uint32_t*)(p + o_lp);
    g->d_leaf = (fx_leaf*)(p + o_lf);
}

static GridPtrs ptrs_of(const fx_grid* g) {
    GridPtrs q;
    q.hdr = g->d_hdr; q.vox_base = g->d_vox_base; q.root_key = g->d_root_key; q.root_batch = g->d_root_batch;
    q.upper_mask = g->d_upper_mask; q.upper_prefix = g->d_upper_prefix;
    q.lower_mask = g->d_lower_mask; q.lower_prefix = g->d_lower_prefix; q.leaf = g->d_leaf;
    q.cap_upper = g->cap_upper; q.cap_lower = g->cap_lower; q.cap_leaf = g->cap_leaf; q.B = g->B;
    return q;
}

static fx_status scan_level(const fx_grid* g, LevelScan s, int cap_nodes, ScanSync y, hipStream_t st) {
    const int64_t cap_words = (int64_t)cap_nodes * s.words_per_node;
    const int n_blocks = (int)std::max<int64_t>(1, (cap_words + kWordChunk - 1) / kWordChunk);
    k_scan_words<<<n_blocks, kScanThreads, 0, st>>>(s, g->d_hdr, y);
    FX_HIP_TRY(hipGetLastError());
    return FX_OK;
}

// One attempt with the given node capacities.  On FX_OK, (*out)->hdr.overflow tells whether a
// capacity was too small (the counts found so far are valid up to the overflowing level).
constexpr int64_t kPartitionMinRows = 65536;   // below this the direct path's few kernels win

// Where the leaves of a grid come from when not from rows of voxel coordinates: the leaves of another grid
// (n_rows of build_attempt is then that grid's leaf count, and the direct path is taken).
struct LeafSource {
    enum Kind { kRows, kCoarsen, kPad, kSubdivide } kind = kRows;
    const fx_grid* grid = nullptr;
    int r = 0;                    // kPad: the padding
    int32_t* d_bad = nullptr;     // kPad, kSubdivide: counter of leaves beyond the int32 coordinate range
    int link_K = 0;               // kCoarsen: the grid becomes the output of a (link_K, 2) kernel map from `grid` (0: no)
};

static fx_status build_attempt(const int32_t* d_ijk, int64_t n_rows, const BatchRanges& d_joff, int32_t B,
                               int cap_upper, int cap_lower, int cap_leaf, bool direct, hipStream_t st, fx_grid** out,
                               const LeafSource& from = LeafSource()) {
    fx_grid* g = new (std::nothrow) fx_grid();
    if (!g) { set_error("host allocation failed"); return FX_ENOMEM; }
    g->B = B; g->stream = st;
    g->cap_upper = std::max(cap_upper, 1); g->cap_lower = std::max(cap_lower, 1); g->cap_leaf = std::max(cap_leaf, 1);
    layout(g);
    fx_status rc = dev_alloc(&g->buf, g->buf_bytes, st);
    if (rc != FX_OK) { delete g; return rc; }
    layout(g);
    g->h_vox_base = (int64_t*)calloc((size_t)B + 1, sizeof(int64_t));

    // Leaf list capacity and the way to it.  Scratch layout:
    //   cleared by both paths:    [scan tickets and block words | tile table]
    //   cleared by the direct one [leaf table slots | leaf masks]
    //   not cleared:              [leaf keys | mask indices | tile representatives |
    //                              partitioned path: leaf masks, bucket records, histogram, totals, bucket starts]
    const int64_t max_items = std::max<int64_t>((int64_t)g->cap_lower * kLowerWords / kWordChunk,
                                                std::max<int64_t>((int64_t)g->cap_upper * kUpperWords / kWordChunk,
                                                                  (int64_t)g->cap_leaf / kLeafChunk)) + 2;
    const bool partition = !direct && n_rows >= kPartitionMinRows;
    size_t n_slots = 0;                       // direct path: table slots, masks indexed by slot
    const bool no_table = from.kind == LeafSource::kSubdivide;       // every leaf has one source: masks by (leaf, octant)
    if (!partition) { n_slots = 1024; while (n_slots < 2 * (size_t)g->cap_leaf) n_slots <<= 1; }
    if (no_table) n_slots = 0;
    // (a padded grid keeps the masks of the source grid's own leaves behind the table's)
    const size_t n_masks = partition ? (size_t)g->cap_leaf
                         : no_table ? 8 * (size_t)n_rows : n_slots + (from.kind == LeafSource::kPad ? (size_t)n_rows : 0);
    if (n_masks > 0x7FFFFFFFull) { fx_grid_destroy(g); set_error("grid build: too many leaves"); return FX_ERANGE; }
    // Buckets of 1500 to 3000 rows: fewer, fuller buckets give the scatter pass longer runs per bucket and the
    // leaf pass fewer workgroups that each clear a 64 KB table (1 M rows: 98 us with ~1000 rows per bucket, 90 with
    // ~2000, 91 with ~4000, 107 with ~8000, which leaves half the compute units without a bucket; four grids of
    // 1.07 M rows: 140 / 123 / 117 / 111 us for ~500 / 1000 / 2000 / 4000).  A bucket's table holds 1024 leaves, so
    // rows that average fewer than three per leaf overflow it and take the path without buckets.
    int n_buckets = 64;
    while (n_buckets < kMaxBuckets && (int64_t)n_buckets * kRowsPerBucket < n_rows) n_buckets <<= 1;
    const int n_part_wg = (int)((n_rows + kPartChunk - 1) / kPartChunk);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    const size_t o_sync = take(sizeof(uint32_t) * 3 * (64 + (size_t)max_items));   // three scans: a ticket, then the words
    const size_t o_tslot = take(sizeof(int32_t) * kTileHashSlots);
    const size_t clear_bytes_head = off;
    const size_t o_slots = take(sizeof(int32_t) * n_slots);
    const size_t clear_bytes_slots = off;
    const size_t o_mask = take(sizeof(uint64_t) * 8 * n_masks);
    // the padded grid's masks are stored whole, the other direct builds OR theirs together
    const bool whole_masks = from.kind == LeafSource::kPad || from.kind == LeafSource::kSubdivide;
    const size_t clear_bytes = partition ? clear_bytes_head : (whole_masks ? clear_bytes_slots : off);
    const size_t o_key = take(sizeof(int4) * (size_t)g->cap_leaf);
    const size_t o_midx = take(sizeof(int32_t) * (size_t)g->cap_leaf);
    const size_t o_rep = take(sizeof(int32_t) * kMaxTiles);
    const size_t o_rec = take(partition ? sizeof(int4) * (size_t)n_rows : 0);
    const size_t o_hist = take(partition ? sizeof(uint32_t) * (size_t)n_buckets * n_part_wg : 0);
    const size_t o_tot = take(partition ? sizeof(uint32_t) * n_buckets : 0);
    const size_t o_bst = take(partition ? sizeof(uint32_t) * (n_buckets + 1) : 0);
    void* scratch = nullptr;
    rc = dev_alloc(&scratch, off, st);
    if (rc != FX_OK) { fx_grid_destroy(g); return rc; }
    char* sp = (char*)scratch;
    LeafList L;
    L.mask = (uint64_t*)(sp + o_mask);
    L.key = (int4*)(sp + o_key);
    L.mask_idx = (int32_t*)(sp + o_midx);
    L.cap = g->cap_leaf;
    int32_t* d_tile_slots = (int32_t*)(sp + o_tslot);
    int32_t* d_slots = (int32_t*)(sp + o_slots);
    int32_t* d_rep = (int32_t*)(sp + o_rep);
    auto scan_sync = [&](int which) {
        uint32_t* base = (uint32_t*)(sp + o_sync) + (size_t)which * (64 + (size_t)max_items);
        return ScanSync{base, base + 64};
    };
    int4* d_records = (int4*)(sp + o_rec);
    uint32_t* d_hist = (uint32_t*)(sp + o_hist);
    uint32_t* d_totals = (uint32_t*)(sp + o_tot);
    uint32_t* d_bucket_start = (uint32_t*)(sp + o_bst);

    auto fail = [&](fx_status s) { dev_free(scratch, st); fx_grid_destroy(g); return s; };
#define FX_TRY_OR_FAIL(expr) do { hipError_t _e = (expr); if (_e != hipSuccess) { \
        set_error("%s failed: %s", #expr, hipGetErrorString(_e)); return fail(FX_EDEVICE); } } while (0)

    // header, bases, root table and the child masks start at zero; the leaf records (most of the buffer) do not
    // need to: every field of every leaf that exists is written by the build.  The partitioned path clears in its
    // first kernel, the direct path (small inputs) with two fills.
    const size_t grid_clear_bytes = (size_t)((char*)g->d_leaf - (char*)g->buf);
    const bool kernel_clears = partition && n_rows > 0 && B > 0;
    if (!kernel_clears) {
        ProfScope ps(kProfMemset, st);
        FX_TRY_OR_FAIL(hipMemsetAsync(g->buf, 0, grid_clear_bytes, st));
        FX_TRY_OR_FAIL(hipMemsetAsync(scratch, 0, clear_bytes, st));
    }
    const GridPtrs q = ptrs_of(g);
    if (n_rows > 0 && B > 0) {
        const unsigned nb_leaf = (unsigned)((g->cap_leaf + 255) / 256);
        if (partition) {
            const uint32_t bucket_mask = (uint32_t)n_buckets - 1;
            const size_t lds = (sizeof(int4) + sizeof(uint32_t)) * kPartChunk + 3 * sizeof(uint32_t) * kMaxBuckets;
            FX_TRY_OR_FAIL(hipFuncSetAttribute((const void*)k_bucket_scatter, hipFuncAttributeMaxDynamicSharedMemorySize,
                                               (int)lds));
            { ProfScope ps(kProfBucketCount, st);
              ClearRanges clr;
              clr.p[0] = (uint4*)g->buf; clr.n16[0] = (uint32_t)(grid_clear_bytes / 16);
              clr.p[1] = (uint4*)scratch; clr.n16[1] = (uint32_t)(clear_bytes / 16);
              k_bucket_count<<<n_part_wg, kPartThreads, 0, st>>>(d_ijk, n_rows, d_joff, B, bucket_mask, d_hist, clr); }
            { ProfScope ps(kProfBucketScan, st);
              k_bucket_scan<<<(n_buckets * 64 + 255) / 256, 256, 0, st>>>(d_hist, n_part_wg, n_buckets, d_totals); }
            { ProfScope ps(kProfBucketScatter, st);
              k_bucket_scatter<<<n_part_wg, kPartThreads, lds, st>>>(d_ijk, n_rows, d_joff, B, bucket_mask, d_hist, d_totals,
                                                                     d_bucket_start, d_records); }
            { ProfScope ps(kProfBucketLeaves, st);
              k_bucket_leaves<<<n_buckets, kBucketThreads, 0, st>>>(d_records, d_bucket_start, L, g->d_hdr); }
        } else {
            const unsigned nb_rows = (unsigned)((n_rows + 255) / 256);
            ProfScope ps(kProfVoxelsToLeaves, st);
            if (from.kind == LeafSource::kCoarsen)
                k_coarse_leaves<<<nb_rows, 256, 0, st>>>(from.grid->view(), d_slots, (uint32_t)(n_slots - 1), L, g->d_hdr);
            else if (from.kind == LeafSource::kPad) {
                k_pad_claim<<<(unsigned)((n_rows * 32 + kPadClaimThreads - 1) / kPadClaimThreads), kPadClaimThreads, 0, st>>>(
                    from.grid->view(), from.r, d_slots, (uint32_t)(n_slots - 1), L, g->d_hdr, from.d_bad);
                k_pad_masks<<<(unsigned)((g->cap_leaf + kPadWaves - 1) / kPadWaves), 64 * kPadWaves, 0, st>>>(from.grid->view(), from.r,
                                                                                                           L, g->d_hdr);
            } else if (from.kind == LeafSource::kSubdivide)
                k_subdivide_leaves<<<(unsigned)((n_rows * 8 + kSubdivideThreads - 1) / kSubdivideThreads), kSubdivideThreads, 0, st>>>(
                    from.grid->view(), L, g->d_hdr, from.d_bad);
            else
                k_voxels_to_leaves<<<nb_rows, 256, 0, st>>>(d_ijk, n_rows, d_joff, B, d_slots, (uint32_t)(n_slots - 1), L, g->d_hdr);
        }
        { ProfScope ps(kProfFindTiles, st); k_find_tiles<<<(unsigned)((g->cap_leaf + kFindTilesThreads - 1) / kFindTilesThreads), kFindTilesThreads, 0, st>>>(L, d_tile_slots, d_rep, g->d_hdr); }
        const bool rank_in_block = g->cap_upper <= kRankInBlock;
        if (!rank_in_block) { ProfScope ps(kProfRankTiles, st); k_rank_tiles<<<kMaxTiles / 256, 256, 0, st>>>(L, d_rep, q); }
        { ProfScope ps(kProfInsertUpper, st);
          k_insert_upper<<<(unsigned)((g->cap_leaf + kInsertUpperThreads - 1) / kInsertUpperThreads), kInsertUpperThreads, 0, st>>>(
              L, q, d_rep, rank_in_block ? 1 : 0); }
        LevelScan su{g->d_upper_mask, g->d_upper_prefix, &g->d_hdr->n_upper, kUpperWords, &g->d_hdr->n_lower,
                     g->cap_lower, 2};
        { ProfScope ps(kProfScanUpper, st); if (scan_level(g, su, g->cap_upper, scan_sync(0), st) != FX_OK) return fail(FX_EDEVICE); }
        { ProfScope ps(kProfInsertLower, st); k_insert<1><<<nb_leaf, 256, 0, st>>>(L, q); }
        LevelScan sl{g->d_lower_mask, g->d_lower_prefix, &g->d_hdr->n_lower, kLowerWords, &g->d_hdr->n_leaf,
                     g->cap_leaf, 4};
        { ProfScope ps(kProfScanLower, st); if (scan_level(g, sl, g->cap_lower, scan_sync(1), st) != FX_OK) return fail(FX_EDEVICE); }
        { ProfScope ps(kProfInsertLeaf, st); k_insert<2><<<nb_leaf, 256, 0, st>>>(L, q); }
        const int lb = std::max(1, (g->cap_leaf + kLeafChunk - 1) / kLeafChunk);
        { ProfScope ps(kProfScanLeaf, st);
          k_scan_leaves<<<lb, kScanThreads, 0, st>>>(g->d_leaf, g->d_hdr, scan_sync(2), g->d_vox_base, B); }
        FX_TRY_OR_FAIL(hipGetLastError());
    }
    // one read-back: counts + per-grid ranges (Sec. 3.3 step 10)
    const size_t hdr_bytes = sizeof(GridHeader);
    const size_t vb_bytes = sizeof(int64_t) * ((size_t)B + 1);
    void* stage = nullptr;
    const size_t ticket_off = align_up(hdr_bytes + vb_bytes, 64);
    rc = host_staging(&stage, ticket_off + 64);
    if (rc != FX_OK) return fail(rc);
    static thread_local int32_t next_ticket = 0;
    const int32_t ticket = ++next_ticket == 0 ? ++next_ticket : next_ticket;   // never 0
    volatile int32_t* h_ticket = reinterpret_cast<volatile int32_t*>((char*)stage + ticket_off);
    *h_ticket = 0;
    k_publish<<<1, 256, 0, st>>>(g->d_hdr, g->d_vox_base, B, (unsigned char*)stage, (int32_t*)h_ticket, ticket);
    FX_TRY_OR_FAIL(hipGetLastError());
    // runs on the device while the host waits for the ticket and returns to its caller
    if (from.kind == LeafSource::kCoarsen && from.link_K) enqueue_leaf_links(g, st, from.grid, from.link_K, 2);
    else enqueue_leaf_links(g, st, nullptr, 3, 1);
    {
        // poll the ticket for a while (a few hundred microseconds at most for the sizes where latency
        // matters), then fall back to waiting for the stream, which also reports any device error
        bool seen = false;
        for (int spin = 0; spin < 200000 && !seen; ++spin) {
            seen = (*h_ticket == ticket);
            if (!seen) __builtin_ia32_pause();
        }
        if (!seen) FX_TRY_OR_FAIL(hipStreamSynchronize(st));
        std::atomic_thread_fence(std::memory_order_acquire);
    }
    memcpy(&g->hdr, stage, hdr_bytes);
    memcpy(g->h_vox_base, (char*)stage + hdr_bytes, vb_bytes);
    dev_free(scratch, st);
#undef FX_TRY_OR_FAIL
    *out = g;
    return FX_OK;
}

static fx_status build_with_ranges(const int32_t* d_ijk, int64_t n_rows, const BatchRanges& d_joff, int32_t B,
                                    hipStream_t st, fx_grid** out) {
    // First attempt with capacities that fit typical occupancy; an attempt that overflows has
    // (almost always) counted the nodes of the overflowing level exactly and is repeated with those.
    int cap_upper = B + 8;
    int cap_lower = (int)std::min<int64_t>(std::max<int64_t>(n_rows, 1), 64 * (int64_t)std::max(B, 1) + n_rows / 256);
    int cap_leaf = (int)std::min<int64_t>(std::max<int64_t>(n_rows, 1), 1024 + n_rows / 8);
    bool direct = option(kOptGridDirect) == 1;
    for (int attempt = 0; attempt < 9; ++attempt) {
        fx_grid* g = nullptr;
        FX_TRY(build_attempt(d_ijk, n_rows, d_joff, B, cap_upper, cap_lower, cap_leaf, direct, st, &g));
        const int ov = g->hdr.overflow;
        if (!ov) { *out = g; return FX_OK; }
        if (ov & 8) {
            fx_grid_destroy(g);
            set_error("more than %d root tiles (4096^3 regions) in the batch", kMaxTiles);
            return FX_ERANGE;
        }
        if (ov & 16) {
            fx_grid_destroy(g);
            set_error("more than 2^31-1 active voxels");
            return FX_ERANGE;
        }
        if (ov & 128) {
            fx_grid_destroy(g);
            set_error("grid build: a workgroup of a scan waited for its predecessors beyond the limit");
            return FX_EDEVICE;
        }
        if (ov & 64) direct = true;   // a bucket held more leaves than its LDS table
        if (ov & 1) cap_upper = g->hdr.n_upper;
        if (ov & 2) { cap_upper = g->hdr.n_upper; cap_lower = g->hdr.n_lower; }
        if (ov & 4) {
            // The voxel pass counts every distinct leaf it can put in its table (twice the
            // capacity); only when the table itself filled up is the count a lower bound, and
            // the capacity grows geometrically instead (at most one leaf per input row exists).
            if ((ov & 32) || (ov & 64)) cap_leaf = (int)std::min<int64_t>(std::max<int64_t>(n_rows, 1), 4 * (int64_t)cap_leaf);
            else cap_leaf = g->hdr.n_leaf_raw;
        }
        fx_grid_destroy(g);
    }
    set_error("grid build did not converge");
    return FX_EDEVICE;
}

// The build from rows already on the device; h_pairs = (begin, end) rows of every grid of the batch, on the host.
// One grid needs no upload at all; more go through pinned staging into a device array that lives until the build
// has synchronised the stream.
fx_status build_index_grid_device(const int32_t* d_ijk, int64_t n_rows, const int64_t* h_pairs, int32_t B,
                                  hipStream_t st, fx_grid** out) {
    BatchRanges J{nullptr, 0, 0};
    int64_t* d_pairs = nullptr;
    if (B >= 1) { J.begin0 = h_pairs[0]; J.end0 = h_pairs[1]; }
    if (B > 1) {
        const size_t jb = sizeof(int64_t) * 2 * (size_t)B;
        FX_TRY(dev_alloc((void**)&d_pairs, jb, st));
        void* stage = nullptr;
        fx_status rc = host_staging(&stage, jb, 1);
        if (rc != FX_OK) { dev_free(d_pairs, st); return rc; }
        memcpy(stage, h_pairs, jb);
        const hipError_t e = hipMemcpyAsync(d_pairs, stage, jb, hipMemcpyHostToDevice, st);
        if (e != hipSuccess) { dev_free(d_pairs, st); set_error("joffsets upload failed: %s", hipGetErrorString(e)); return FX_EDEVICE; }
        J.d = d_pairs;
    }
    const fx_status rc = build_with_ranges(d_ijk, n_rows, J, B, st, out);
    if (d_pairs) dev_free(d_pairs, st);
    return rc;
}

}  // namespace fx

// ====================================================================================== C ABI
using namespace fx;

extern "C" fx_status fx_build_index_grid(const int32_t* d_ijk, int64_t n_rows, const int64_t* h_joffsets,
                                         int32_t B, void* stream, fx_grid** out) {
    if (!out || B < 0 || n_rows < 0 || (B > 0 && !h_joffsets) || (n_rows > 0 && !d_ijk)) {
        set_error("fx_build_index_grid: null pointer or negative size");
        return FX_EINVAL;
    }
    if (n_rows > (int64_t)INT32_MAX) { set_error("more than 2^31-1 input rows"); return FX_ERANGE; }
    int64_t prev_end = 0;
    for (int32_t b = 0; b < B; ++b) {
        const int64_t s = h_joffsets[2 * b], e = h_joffsets[2 * b + 1];
        if (s < prev_end || e < s || e > n_rows) {
            set_error("joffsets[%d] = (%lld, %lld) is out of range, overlapping or out of order", b, (long long)s,
                      (long long)e);
            return FX_EINVAL;
        }
        prev_end = e;
    }
    return build_index_grid_device(d_ijk, n_rows, h_joffsets, B, (hipStream_t)stream, out);
}

extern "C" fx_status fx_grid_info(const fx_grid* g, int64_t* n_voxels, int32_t* B, int64_t* h_voxel_joffsets,
                                  int64_t* h_counts3) {
    if (!g) { set_error("fx_grid_info: null grid"); return FX_EINVAL; }
    if (n_voxels) *n_voxels = g->hdr.n_voxels;
    if (B) *B = g->B;
    if (h_voxel_joffsets)
        for (int b = 0; b < g->B; ++b) {
            h_voxel_joffsets[2 * b] = g->h_vox_base[b];
            h_voxel_joffsets[2 * b + 1] = g->h_vox_base[b + 1];
        }
    if (h_counts3) { h_counts3[0] = g->hdr.n_leaf; h_counts3[1] = g->hdr.n_lower; h_counts3[2] = g->hdr.n_upper; }
    return FX_OK;
}

extern "C" fx_status fx_grid_ijk(const fx_grid* g, int32_t* d_ijk_out, int32_t* d_jidx_out, void* stream) {
    if (!g || (!d_ijk_out && g->hdr.n_voxels > 0)) { set_error("fx_grid_ijk: null pointer"); return FX_EINVAL; }
    if (g->hdr.n_leaf == 0) return FX_OK;
    const int64_t threads = (int64_t)g->hdr.n_leaf * 64;
    k_grid_ijk<<<(unsigned)((threads + 255) / 256), 256, 0, (hipStream_t)stream>>>(g->view(), d_ijk_out, d_jidx_out, 0);
    FX_HIP_TRY(hipGetLastError());
    return FX_OK;
}

extern "C" fx_status fx_grid_ijk_to_index(const fx_grid* g, const int32_t* d_ijk, const int32_t* d_jidx, int64_t n,
                                          int32_t* d_index_out, void* stream) {
    if (!g || n < 0 || (n > 0 && (!d_ijk || !d_index_out))) {
        set_error("fx_grid_ijk_to_index: null pointer or negative size");
        return FX_EINVAL;
    }
    if (n == 0) return FX_OK;
    k_ijk_to_index<<<(unsigned)((n + 255) / 256), 256, 0, (hipStream_t)stream>>>(g->view(), d_ijk, d_jidx, n,
                                                                                  d_index_out);
    FX_HIP_TRY(hipGetLastError());
    return FX_OK;
}

extern "C" fx_status fx_grid_leaf_table(const fx_grid* g, fx_leaf* h_out, size_t bytes, void* stream) {
    if (!g) { set_error("fx_grid_leaf_table: null grid"); return FX_EINVAL; }
    const size_t need = sizeof(fx_leaf) * (size_t)g->hdr.n_leaf;
    if (bytes < need || (need && !h_out)) { set_error("fx_grid_leaf_table: buffer too small"); return FX_EINVAL; }
    if (!need) return FX_OK;
    FX_HIP_TRY(hipMemcpyAsync(h_out, g->d_leaf, need, hipMemcpyDeviceToHost, (hipStream_t)stream));
    FX_HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
    return FX_OK;
}

// Voxel coordinates of points (Sec. 3.6.2: grids from point clouds): element e = 3 * point + axis.
// Subtraction and division are the correctly rounded single-precision ones (no reciprocal, no
// contraction), so that the cell of a point near a face is the same on every implementation.
__global__ void k_points_to_ijk(const float* __restrict__ xyz, int64_t n3, float ox, float oy, float oz, float sx,
                                float sy, float sz, int32_t* __restrict__ ijk, int32_t* __restrict__ n_bad) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n3) return;
    const int axis = (int)(e % 3);
    const float o = axis == 0 ? ox : axis == 1 ? oy : oz;
    const float s = axis == 0 ? sx : axis == 1 ? sy : sz;
    const float t = floorf(__fdiv_rn(__fsub_rn(xyz[e], o), s));
    const bool ok = isfinite(t) && t >= -1073741824.0f && t < 1073741824.0f;
    ijk[e] = ok ? (int32_t)t : 0;
    if (!ok) atomicAdd(n_bad, 1);
}

extern "C" fx_status fx_build_index_grid_from_points(const float* d_xyz, int64_t n_rows, const int64_t* h_joffsets,
                                                     int32_t B, const float* h_origin, const float* h_voxel_size,
                                                     void* stream, fx_grid** out) {
    if (!out || !h_origin || !h_voxel_size || n_rows < 0 || (n_rows > 0 && !d_xyz)) {
        set_error("fx_build_index_grid_from_points: null pointer or negative size");
        return FX_EINVAL;
    }
    for (int a = 0; a < 3; ++a)
        if (!(h_voxel_size[a] > 0.f) || !std::isfinite(h_voxel_size[a]) || !std::isfinite(h_origin[a])) {
            set_error("fx_build_index_grid_from_points: voxel sizes must be positive and finite, the origin finite");
            return FX_EINVAL;
        }
    if (n_rows > (int64_t)INT32_MAX) { set_error("more than 2^31-1 input rows"); return FX_ERANGE; }
    hipStream_t st = (hipStream_t)stream;
    int32_t* d_ijk = nullptr;
    // the counter of invalid points sits behind the coordinates, in the same allocation
    const size_t ijk_bytes = (sizeof(int32_t) * 3 * (size_t)std::max<int64_t>(n_rows, 1) + 15) & ~size_t(15);
    FX_TRY(dev_alloc((void**)&d_ijk, ijk_bytes + 16, st));
    int32_t* d_bad = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(d_ijk) + ijk_bytes);
    hipError_t e = hipMemsetAsync(d_bad, 0, sizeof(int32_t), st);
    if (e == hipSuccess && n_rows > 0) {
        ProfScope ps(kProfPointsToIjk, st);
        const int64_t n3 = 3 * n_rows;
        k_points_to_ijk<<<(unsigned)((n3 + 255) / 256), 256, 0, st>>>(d_xyz, n3, h_origin[0], h_origin[1], h_origin[2],
                                                                    h_voxel_size[0], h_voxel_size[1], h_voxel_size[2],
                                                                    d_ijk, d_bad);
        e = hipGetLastError();
    }
    if (e != hipSuccess) { dev_free(d_ijk, st); set_error("point quantisation failed: %s", hipGetErrorString(e)); return FX_EDEVICE; }
    fx_grid* g = nullptr;
    fx_status rc = fx_build_index_grid(d_ijk, n_rows, h_joffsets, B, stream, &g);    // synchronises the stream
    int32_t bad = 0;
    if (rc == FX_OK) {
        e = hipMemcpy(&bad, d_bad, sizeof(int32_t), hipMemcpyDeviceToHost);
        if (e != hipSuccess) { rc = FX_EDEVICE; set_error("read-back failed: %s", hipGetErrorString(e)); }
    }
    dev_free(d_ijk, st);
    if (rc == FX_OK && bad > 0) {
        set_error("%d point coordinates are not finite or fall outside [-2^30, 2^30) voxels", bad);
        rc = FX_ERANGE;
    }
    if (rc != FX_OK) { if (g) fx_grid_destroy(g); return rc; }
    *out = g;
    return FX_OK;
}

fx_status fx::grid_coarsen2_for_map(const fx_grid* g, int K, hipStream_t st, fx_grid** out) {
    // The coarse grid has at most as many nodes per level as the fine one, so one attempt with the fine grid's
    // counts as capacities always fits; its leaves come from the fine leaves, not from a row per voxel.
    fx_grid* o = nullptr;
    const BatchRanges none{nullptr, 0, 0};
    LeafSource from;
    from.kind = LeafSource::kCoarsen; from.grid = g; from.link_K = K;
    FX_TRY(build_attempt(nullptr, g->hdr.n_leaf, none, g->B, g->hdr.n_upper, g->hdr.n_lower, g->hdr.n_leaf, true, st, &o, from));
    if (o->hdr.overflow) {
        const int ov = o->hdr.overflow;
        fx_grid_destroy(o);
        set_error("fx_grid_coarsen2: the coarse grid did not fit the fine grid's node counts (flags %d)", ov);
        return FX_EDEVICE;
    }
    *out = o;
    return FX_OK;
}

extern "C" fx_status fx_grid_coarsen2(const fx_grid* g, void* stream, fx_grid** out) {
    if (!g || !out) { set_error("fx_grid_coarsen2: null pointer"); return FX_EINVAL; }
    return grid_coarsen2_for_map(g, 0, (hipStream_t)stream, out);
}

extern "C" fx_status fx_grid_subdivide2(const fx_grid* g, void* stream, fx_grid** out) {
    if (!g || !out) { set_error("fx_grid_subdivide2: null pointer"); return FX_EINVAL; }
    hipStream_t st = (hipStream_t)stream;
    const int64_t n = g->hdr.n_voxels;
    if (8 * n > 0x7FFFFFFFll) { set_error("fx_grid_subdivide2: more than 2^31-1 voxels"); return FX_ERANGE; }
    // The fine grid's leaves are the non-empty octants of the coarse leaves (k_subdivide_leaves); a fine node of
    // any level covers an octant of the coarse node of that level, so eight times the coarse counts always fit.
    const int64_t cap_leaf = 8 * (int64_t)g->hdr.n_leaf, cap_lower = 8 * (int64_t)g->hdr.n_lower, cap_upper = 8 * (int64_t)g->hdr.n_upper;
    if (cap_leaf > 0x7FFFFFFFll / 8) { set_error("fx_grid_subdivide2: too many leaves"); return FX_ERANGE; }
    int32_t* d_bad = nullptr;     // octants whose doubled coordinates would leave the int32 range
    FX_TRY(dev_alloc((void**)&d_bad, 16, st));
    if (hipMemsetAsync(d_bad, 0, sizeof(int32_t), st) != hipSuccess) { dev_free(d_bad, st); set_error("fx_grid_subdivide2: fill failed"); return FX_EDEVICE; }
    LeafSource from;
    from.kind = LeafSource::kSubdivide; from.grid = g; from.d_bad = d_bad;
    const BatchRanges none{nullptr, 0, 0};
    fx_grid* o = nullptr;
    fx_status rc = build_attempt(nullptr, g->hdr.n_leaf, none, g->B, (int)cap_upper, (int)cap_lower, (int)cap_leaf, true, st, &o, from);
    int32_t bad = 0;
    if (rc == FX_OK && hipMemcpy(&bad, d_bad, sizeof(int32_t), hipMemcpyDeviceToHost) != hipSuccess) {
        rc = FX_EDEVICE; set_error("fx_grid_subdivide2: read-back failed");
    }
    dev_free(d_bad, st);
    if (rc == FX_OK && bad > 0) {
        set_error("fx_grid_subdivide2: %d leaves hold coordinates beyond +-2^30, whose doubles leave the int32 coordinate limits", bad);
        rc = FX_ERANGE;
    }
    if (rc == FX_OK && o->hdr.overflow) {
        set_error("fx_grid_subdivide2: the fine grid did not fit eight times the coarse grid's node counts (flags %d)", o->hdr.overflow);
        rc = (o->hdr.overflow & 16) ? FX_ERANGE : FX_EDEVICE;
    }
    if (rc != FX_OK) { if (o) fx_grid_destroy(o); return rc; }
    *out = o;
    return FX_OK;
}

extern "C" fx_status fx_grid_pad(const fx_grid* g, int32_t r, void* stream, fx_grid** out) {
    if (!g || !out) { set_error("fx_grid_pad: null pointer"); return FX_EINVAL; }
    if (r < 0) { set_error("fx_grid_pad: negative padding %d", r); return FX_EINVAL; }
    if (r > 8) { set_error("fx_grid_pad: padding %d is above the supported 8 voxels", r); return FX_EUNSUPPORTED; }
    hipStream_t st = (hipStream_t)stream;
    if ((int64_t)g->hdr.n_leaf * 27 > 0x7FFFFFFFll) { set_error("fx_grid_pad: too many leaves"); return FX_ERANGE; }
    int32_t* d_bad = nullptr;     // pieces that would leave the int32 coordinate range
    FX_TRY(dev_alloc((void**)&d_bad, 16, st));
    // The padded grid's leaves come from the source grid's leaves (k_pad_claim, k_pad_masks); every leaf reaches at most the 27
    // leaves around it.  First attempt with room for twice the nodes, then with the counts the attempt found.
    const int64_t nl = g->hdr.n_leaf, nlo = g->hdr.n_lower, nu = g->hdr.n_upper;
    int64_t cap_leaf = std::min<int64_t>(27 * nl, 2 * nl + 4096), cap_lower = std::min<int64_t>(27 * nlo, 2 * nlo + 64),
            cap_upper = std::min<int64_t>(27 * nu, 8 * nu + 8);
    fx_grid* o = nullptr;
    fx_status rc = FX_OK;
    const BatchRanges none{nullptr, 0, 0};
    LeafSource from;
    from.kind = LeafSource::kPad; from.grid = g; from.r = r; from.d_bad = d_bad;
    for (int attempt = 0; attempt < 6; ++attempt) {
        if (hipMemsetAsync(d_bad, 0, sizeof(int32_t), st) != hipSuccess) { rc = FX_EDEVICE; set_error("fx_grid_pad: fill failed"); break; }
        rc = build_attempt(nullptr, nl, none, g->B, (int)cap_upper, (int)cap_lower, (int)cap_leaf, true, st, &o, from);
        if (rc != FX_OK) break;
        const int ov = o->hdr.overflow;
        if (!ov) break;
        if (ov & (8 | 16 | 128) || attempt == 5) {
            fx_grid_destroy(o); o = nullptr;
            if (ov & 8) set_error("more than %d root tiles (4096^3 regions) in the batch", kMaxTiles);
            else if (ov & 16) set_error("fx_grid_pad: the padded grid has more than 2^31-1 active voxels");
            else set_error("fx_grid_pad: the build failed (flags %d)", ov);
            rc = ov & (8 | 16) ? FX_ERANGE : FX_EDEVICE;
            break;
        }
        if (ov & 1) cap_upper = o->hdr.n_upper;
        if (ov & 2) { cap_upper = o->hdr.n_upper; cap_lower = o->hdr.n_lower; }
        if (ov & 4) cap_leaf = (ov & 32) ? std::min<int64_t>(27 * nl, 4 * cap_leaf) : std::max<int64_t>(o->hdr.n_leaf_raw, cap_leaf + 1);
        fx_grid_destroy(o); o = nullptr;
    }
    int32_t bad = 0;
    if (rc == FX_OK) {
        const hipError_t e = hipMemcpy(&bad, d_bad, sizeof(int32_t), hipMemcpyDeviceToHost);
        if (e != hipSuccess) { rc = FX_EDEVICE; set_error("read-back failed: %s", hipGetErrorString(e)); }
    }
    dev_free(d_bad, st);
    if (rc == FX_OK && bad > 0) {
        set_error("fx_grid_pad: %d leaf blocks of the padded grid lie beyond the int32 coordinate limits (a voxel lies within %d of them)", bad, r);
        rc = FX_ERANGE;
    }
    if (rc != FX_OK) { if (o) fx_grid_destroy(o); return rc; }
    *out = o;
    return FX_OK;
}

extern "C" void fx_grid_retain(fx_grid* g) {
    if (g) g->refs.fetch_add(1);
}

extern "C" void fx_grid_destroy(fx_grid* g) {
    if (!g) return;
    if (g->refs.fetch_sub(1) != 1) return;
    if (g->buf) dev_free(g->buf, g->stream);
    if (g->d_leaf_links) dev_free(g->d_leaf_links, g->stream);
    free(g->h_vox_base);
    delete g;
}
