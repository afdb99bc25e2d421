// Kernel-map build (Sec. 3.5): neighbour lookup through the tree for every output voxel and
// stencil offset, then the tiled form the MFMA convolution consumes.
#include "kmap.h"
#include "tree_device.h"

#include <string.h>

#include <algorithm>
#include <new>

namespace fx {

__host__ __device__ constexpr int delta_min(int K) { return (K & 1) ? -(K - 1) / 2 : 0; }

// ---------------------------------------------------------------------------------- dense map
// One wave per OUTPUT leaf (Sec. 3.5 scenario 1: gather offsets come straight from the tree's
// light metadata, amortised over the leaf).  The wave resolves the <= 27 input leaves that the
// leaf's stencil footprint can touch once, keeps their 80-byte records in LDS, lists the leaf's
// active voxels with mask popcounts, and then every lane evaluates Listing 1 for one
// (voxel, offset) entry at a time -- consecutive lanes write consecutive map entries.
constexpr int kNbWavesPerBlock = 4;

struct NbLeafLds {
    uint64_t mask[27][8];
    uint64_t prefix[27];
    int32_t offset[27];   // -1: no such leaf
    uint16_t active[512];
};

template <int K>
__global__ void __launch_bounds__(64 * kNbWavesPerBlock)
k_nbmap(TreeView tin, TreeView tout, int stride, int32_t* __restrict__ nbmap) {
    constexpr int K3 = K * K * K;
    constexpr int D0 = delta_min(K);
    __shared__ NbLeafLds lds_all[kNbWavesPerBlock];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int f_raw = blockIdx.x * kNbWavesPerBlock + wave;
    const bool valid = f_raw < tout.n_leaf;
    const int f = valid ? f_raw : tout.n_leaf - 1;  // surplus waves repeat the last leaf's set-up, write nothing
    NbLeafLds& lds = lds_all[wave];
    const fx_leaf* lf = tout.leaf + f;
    const int b = lf->batch;
    const int oi = lf->origin[0], oj = lf->origin[1], ok = lf->origin[2];
    // leaf coordinates of the first input leaf the footprint touches
    const int bi = (stride * oi + D0) >> 3, bj = (stride * oj + D0) >> 3, bk = (stride * ok + D0) >> 3;
    if (lane < 27) {
        const int a = lane / 9, c = (lane / 3) % 3, d = lane % 3;
        const int li = (bi + a) * 8, lj = (bj + c) * 8, lk = (bk + d) * 8;
        // only slots inside the footprint are looked up
        const int hi_i = (stride * (oi + 7) + D0 + K - 1) >> 3, hi_j = (stride * (oj + 7) + D0 + K - 1) >> 3,
                  hi_k = (stride * (ok + 7) + D0 + K - 1) >> 3;
        int id = -1;
        if (bi + a <= hi_i && bj + c <= hi_j && bk + d <= hi_k) id = find_leaf(tin, b, li, lj, lk);
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
    // active voxels of the output leaf, in index order
    int n_act = 0;
    {
        const uint64_t lt = (1ull << lane) - 1;
#pragma unroll
        for (int w = 0; w < 8; ++w) {
            const uint64_t m = lf->mask[w];
            if ((m >> lane) & 1) lds.active[n_act + __popcll(m & lt)] = (uint16_t)(w * 64 + lane);
            n_act += __popcll(m);
        }
    }
    __syncthreads();
    const int64_t out0 = lf->offset * (int64_t)K3;
    const int total = valid ? n_act * K3 : 0;
    for (int e = lane; e < total; e += 64) {
        const int v = e / K3, kappa = e - v * K3;
        const int loc = lds.active[v];
        const int da = kappa / (K * K), db = (kappa / K) % K, dc = kappa % K;
        const int qi = stride * (oi + (loc >> 6)) + D0 + da;
        const int qj = stride * (oj + ((loc >> 3) & 7)) + D0 + db;
        const int qk = stride * (ok + (loc & 7)) + D0 + dc;
        const int slot = (((qi >> 3) - bi) * 3 + ((qj >> 3) - bj)) * 3 + ((qk >> 3) - bk);
        const int n = qi & 7;
        const uint64_t w = lds.mask[slot][n];
        const uint64_t bit = 1ull << (((qj & 7) << 3) | (qk & 7));
        int idx = -1;
        if (w & bit) {
            const uint64_t sum = n ? (lds.prefix[slot] >> (9 * (n - 1))) & 511 : 0;
            idx = lds.offset[slot] + (int)sum + __popcll(w & (bit - 1));
        }
        nbmap[out0 + e] = idx;
    }
}

// ---------------------------------------------------------------------------------- tiled form
struct PackLds {
    int32_t nb[kTileT * 27];           // the tile's dense map rows (K3 <= 27 on this path)
    uint64_t key[kTileT];              // (mask << 16 | slot), sorted
    int32_t hash[8192];                // open addressing over input rows
    int32_t uniq[8192];                // distinct rows, then sorted
    uint32_t group_mask[kGroupsPerTile];
    uint32_t group_block0[kGroupsPerTile];
    int32_t n_uniq;
    int32_t n_blocks;
};

template <typename T>
__device__ __forceinline__ void lds_bitonic_sort(T* a, int P) {
    // P: power of two >= number of elements (padded with the maximum value)
    for (int k = 2; k <= P; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int t = threadIdx.x; t < P; t += blockDim.x) {
                const int p = t ^ j;
                if (p > t) {
                    const T x = a[t], y = a[p];
                    const bool up = ((t & k) == 0);
                    if ((x > y) == up) { a[t] = y; a[p] = x; }
                }
            }
            __syncthreads();
        }
    }
}

__device__ __forceinline__ uint32_t hash_row(int32_t r) { return ((uint32_t)r * 0x9E3779B1u) >> 19; }  // 13 bits

template <int K3>
__global__ void __launch_bounds__(kTileT)
k_pack_tiles(const int32_t* __restrict__ nbmap, int64_t n_out, TileHeader* __restrict__ tile_hdr,
             uint16_t* __restrict__ tile_perm, int32_t* __restrict__ tile_rows, int row_stride,
             uint16_t* __restrict__ tile_blocks, int block_stride, unsigned long long* __restrict__ stats) {
    static_assert(K3 <= 27, "tiled path supports up to 27 offsets");
    extern __shared__ __align__(16) unsigned char lds_raw[];
    PackLds& L = *reinterpret_cast<PackLds*>(lds_raw);
    const int tid = threadIdx.x;
    const int64_t tile = blockIdx.x;
    const int64_t o0 = tile * kTileT;
    const int n_valid = (int)min((int64_t)kTileT, n_out - o0);

    // stage the tile's map rows (coalesced), clear the hash
    for (int e = tid; e < kTileT * K3; e += kTileT) {
        const int64_t ge = o0 * K3 + e;
        L.nb[e] = (e < n_valid * K3) ? nbmap[ge] : -1;
    }
    for (int e = tid; e < 8192; e += kTileT) { L.hash[e] = -1; L.uniq[e] = INT32_MAX; }
    if (tid == 0) { L.n_uniq = 0; L.n_blocks = 0; }
    __syncthreads();

    // neighbour mask of this thread's output; insert its input rows into the hash
    uint32_t mask = 0;
    for (int kappa = 0; kappa < K3; ++kappa) {
        const int32_t r = L.nb[tid * K3 + kappa];
        if (r < 0) continue;
        mask |= 1u << kappa;
        uint32_t h = hash_row(r);
        for (;;) {
            const int32_t cur = ((volatile int32_t*)L.hash)[h];
            if (cur == r) break;
            if (cur < 0) {
                const int32_t old = atomicCAS(&L.hash[h], -1, r);
                if (old < 0) { L.uniq[atomicAdd(&L.n_uniq, 1)] = r; break; }
                if (old == r) break;
            }
            h = (h + 1) & 8191;
        }
    }
    L.key[tid] = ((uint64_t)mask << 16) | (uint64_t)tid;
    __syncthreads();

    // order outputs by mask so that a group of 16 shares its offsets; order the rows by index
    lds_bitonic_sort(L.key, kTileT);
    const int n_uniq = L.n_uniq;
    int P = 2;
    while (P < n_uniq) P <<= 1;
    lds_bitonic_sort(L.uniq, P);

    if (tid < kGroupsPerTile) {
        uint32_t gm = 0;
        for (int n = 0; n < kGroup; ++n) gm |= (uint32_t)(L.key[tid * kGroup + n] >> 16);
        L.group_mask[tid] = gm;
    }
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        for (int g = 0; g < kGroupsPerTile; ++g) { L.group_block0[g] = run; run += __popc(L.group_mask[g]); }
        L.n_blocks = run;
    }
    __syncthreads();

    // header, permutation, row list
    TileHeader* H = tile_hdr + tile;
    if (tid == 0) {
        H->n_rows = n_uniq; H->n_blocks = L.n_blocks; H->n_out = n_valid; H->pad = 0;
        atomicAdd(&stats[0], (unsigned long long)L.n_blocks * kGroup);
        atomicAdd(&stats[1], (unsigned long long)n_uniq);
    }
    if (tid < kGroupsPerTile) { H->group_mask[tid] = L.group_mask[tid]; H->group_block0[tid] = L.group_block0[tid]; }
    tile_perm[tile * kTileT + tid] = (uint16_t)(L.key[tid] & 0xFFFF);
    for (int e = tid; e < n_uniq; e += kTileT) tile_rows[tile * row_stride + e] = L.uniq[e];

    // blocks: 16 threads write one block of 16 local row ids
    const int n_blocks = L.n_blocks;
    const int sub = tid & 15;
    for (int blk = tid >> 4; blk < n_blocks; blk += kTileT / 16) {
        // group of this block: last g with group_block0[g] <= blk
        int g = 0;
        for (int q = 0; q < kGroupsPerTile; ++q)
            if (L.group_mask[q] != 0 && L.group_block0[q] <= (uint32_t)blk) g = q;
        // kappa: the (blk - block0)-th set bit of the group's mask
        uint32_t gm = L.group_mask[g];
        int skip = blk - (int)L.group_block0[g];
        while (skip-- > 0) gm &= gm - 1;
        const int kappa = __ffs(gm) - 1;
        const int slot = (int)(L.key[g * kGroup + sub] & 0xFFFF);
        const int32_t r = L.nb[slot * K3 + kappa];
        uint16_t id = kNoRow;
        if (r >= 0) {
            int lo = 0, hi = n_uniq - 1;
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (L.uniq[mid] < r) lo = mid + 1; else hi = mid;
            }
            id = (uint16_t)lo;
        }
        tile_blocks[((size_t)tile * block_stride + blk) * kGroup + sub] = id;
    }
}

// decode the tiled form back into the dense table
__global__ void k_tiles_to_dense(const TileHeader* __restrict__ tile_hdr, const uint16_t* __restrict__ tile_perm,
                                 const int32_t* __restrict__ tile_rows, int row_stride,
                                 const uint16_t* __restrict__ tile_blocks, int block_stride, int K3,
                                 int32_t* __restrict__ nbmap) {
    const int64_t tile = blockIdx.x;
    const TileHeader* H = tile_hdr + tile;
    const int n_blocks = H->n_blocks, n_valid = H->n_out;
    const int sub = threadIdx.x & 15;
    for (int blk = threadIdx.x >> 4; blk < n_blocks; blk += blockDim.x / 16) {
        int g = 0;
        for (int q = 0; q < kGroupsPerTile; ++q)
            if (H->group_mask[q] != 0 && H->group_block0[q] <= (uint32_t)blk) g = q;
        uint32_t gm = H->group_mask[g];
        int skip = blk - (int)H->group_block0[g];
        while (skip-- > 0) gm &= gm - 1;
        const int kappa = __ffs(gm) - 1;
        const int local = tile_perm[tile * kTileT + g * kGroup + sub];
        const uint16_t id = tile_blocks[((size_t)tile * block_stride + blk) * kGroup + sub];
        if (id != kNoRow && local < n_valid)
            nbmap[(tile * kTileT + local) * K3 + kappa] = tile_rows[tile * row_stride + id];
    }
}

__global__ void k_fill_i32(int32_t* __restrict__ p, int64_t n, int32_t v) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += stride) p[e] = v;
}

// pairs per offset from the dense table (statistics only)
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

}  // namespace fx

using namespace fx;

extern "C" void fx_kmap_destroy(fx_kmap* km) {
    if (!km) return;
    if (km->refs.fetch_sub(1) != 1) return;
    if (km->d_alloc) dev_free(km->d_alloc, km->stream);
    if (km->gin) fx_grid_destroy(km->gin);
    if (km->gout) fx_grid_destroy(km->gout);
    free(km->h_pairs);
    delete km;
}

extern "C" fx_status fx_build_kernel_map(fx_grid* g_in, int32_t K, int32_t stride, void* stream, fx_grid** g_out,
                                         fx_kmap** out) {
    if (!g_in || !g_out || !out) { set_error("fx_build_kernel_map: null pointer"); return FX_EINVAL; }
    const bool ok = (stride == 1 && (K == 1 || K == 3 || K == 5)) || (stride == 2 && K == 2);
    if (!ok) {
        set_error("fx_build_kernel_map: (kernel_size, stride) = (%d, %d) is not supported", K, stride);
        return (K >= 1 && stride >= 1) ? FX_EUNSUPPORTED : FX_EINVAL;
    }
    hipStream_t st = (hipStream_t)stream;
    fx_grid* gout = nullptr;
    if (stride == 1) { gout = g_in; fx_grid_retain(gout); }
    else FX_TRY(fx_grid_coarsen2(g_in, stream, &gout));

    fx_kmap* km = new (std::nothrow) fx_kmap();
    if (!km) { fx_grid_destroy(gout); set_error("host allocation failed"); return FX_ENOMEM; }
    km->stream = st; km->gin = g_in; fx_grid_retain(g_in); km->gout = gout;
    km->K = K; km->stride = stride; km->K3 = K * K * K;
    km->n_in = g_in->hdr.n_voxels; km->n_out = gout->hdr.n_voxels;
    km->h_pairs = (int64_t*)calloc((size_t)km->K3, sizeof(int64_t));
    const bool tiled = km->K3 <= 27;
    km->n_tiles = tiled ? (km->n_out + kTileT - 1) / kTileT : 0;
    km->row_stride = (int32_t)std::min<int64_t>((int64_t)kTileT * km->K3, std::max<int64_t>(km->n_in, 1));
    km->block_stride = kGroupsPerTile * km->K3;

    // one allocation: dense map | stats | tile headers | perm | rows | blocks
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    const size_t o_nb = take(sizeof(int32_t) * (size_t)std::max<int64_t>(km->n_out * km->K3, 1));
    const size_t o_st = take(sizeof(int64_t) * (size_t)(4 + km->K3));
    const size_t o_th = take(sizeof(TileHeader) * (size_t)std::max<int64_t>(km->n_tiles, 1));
    const size_t o_tp = take(sizeof(uint16_t) * kTileT * (size_t)std::max<int64_t>(km->n_tiles, 1));
    const size_t o_tr = take(sizeof(int32_t) * (size_t)km->row_stride * (size_t)std::max<int64_t>(km->n_tiles, 1));
    const size_t o_tb = take(sizeof(uint16_t) * kGroup * (size_t)km->block_stride *
                             (size_t)std::max<int64_t>(km->n_tiles, 1));
    fx_status rc = dev_alloc(&km->d_alloc, off, st);
    if (rc != FX_OK) { fx_kmap_destroy(km); return rc; }
    char* p = (char*)km->d_alloc;
    km->d_nbmap = (int32_t*)(p + o_nb);
    km->d_stats = (int64_t*)(p + o_st);
    km->d_tile_hdr = (TileHeader*)(p + o_th);
    km->d_tile_perm = (uint16_t*)(p + o_tp);
    km->d_tile_rows = (int32_t*)(p + o_tr);
    km->d_tile_blocks = (uint16_t*)(p + o_tb);

    hipError_t e = hipMemsetAsync(km->d_stats, 0, sizeof(int64_t) * (size_t)(4 + km->K3), st);
    if (e == hipSuccess && gout->hdr.n_leaf > 0) {
        const unsigned nb = (unsigned)((gout->hdr.n_leaf + kNbWavesPerBlock - 1) / kNbWavesPerBlock);
        const TreeView tin = g_in->view(), tout = gout->view();
        ProfScope ps(kProfNbmap, st);
        switch (K) {
            case 1: k_nbmap<1><<<nb, 64 * kNbWavesPerBlock, 0, st>>>(tin, tout, stride, km->d_nbmap); break;
            case 2: k_nbmap<2><<<nb, 64 * kNbWavesPerBlock, 0, st>>>(tin, tout, stride, km->d_nbmap); break;
            case 3: k_nbmap<3><<<nb, 64 * kNbWavesPerBlock, 0, st>>>(tin, tout, stride, km->d_nbmap); break;
            default: k_nbmap<5><<<nb, 64 * kNbWavesPerBlock, 0, st>>>(tin, tout, stride, km->d_nbmap); break;
        }
        e = hipGetLastError();
    }
    if (e == hipSuccess && km->n_tiles > 0) {
        unsigned long long* stats = (unsigned long long*)km->d_stats;
        const size_t lds = sizeof(PackLds);
        const unsigned nt = (unsigned)km->n_tiles;
        ProfScope ps(kProfPackTiles, st);
#define FX_PACK(K3V)                                                                                         \
    do {                                                                                                     \
        e = hipFuncSetAttribute((const void*)k_pack_tiles<K3V>, hipFuncAttributeMaxDynamicSharedMemorySize,  \
                                (int)lds);                                                                   \
        if (e == hipSuccess)                                                                                 \
            k_pack_tiles<K3V><<<nt, kTileT, lds, st>>>(km->d_nbmap, km->n_out, km->d_tile_hdr,               \
                                                       km->d_tile_perm, km->d_tile_rows, km->row_stride,     \
                                                       km->d_tile_blocks, km->block_stride, stats);          \
    } while (0)
        if (km->K3 == 1) FX_PACK(1);
        else if (km->K3 == 8) FX_PACK(8);
        else FX_PACK(27);
#undef FX_PACK
        if (e == hipSuccess) e = hipGetLastError();
    }
    if (e != hipSuccess) {
        set_error("kernel-map build failed: %s", hipGetErrorString(e));
        fx_kmap_destroy(km);
        return FX_EDEVICE;
    }
    *g_out = gout;
    fx_grid_retain(gout);
    *out = km;
    return FX_OK;
}

static fx_status kmap_fetch_stats(fx_kmap* km) {
    if (km->stats_valid) return FX_OK;
    hipStream_t st = km->stream;
    unsigned long long* pairs = (unsigned long long*)(km->d_stats + 4);
    FX_HIP_TRY(hipMemsetAsync(pairs, 0, sizeof(int64_t) * (size_t)km->K3, st));
    if (km->n_out > 0) {
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

extern "C" fx_status fx_kmap_dense(const fx_kmap* km, int32_t* d_nbmap, void* stream) {
    if (!km || (!d_nbmap && km->n_out > 0)) { set_error("fx_kmap_dense: null pointer"); return FX_EINVAL; }
    if (km->n_out == 0) return FX_OK;
    hipStream_t st = (hipStream_t)stream;
    const int64_t total = km->n_out * km->K3;
    if (km->n_tiles > 0) {
        const unsigned nb = (unsigned)std::min<int64_t>((total + 256 * 8 - 1) / (256 * 8), 8192);
        k_fill_i32<<<nb, 256, 0, st>>>(d_nbmap, total, -1);
        k_tiles_to_dense<<<(unsigned)km->n_tiles, 256, 0, st>>>(km->d_tile_hdr, km->d_tile_perm, km->d_tile_rows,
                                                               km->row_stride, km->d_tile_blocks, km->block_stride,
                                                               km->K3, d_nbmap);
        FX_HIP_TRY(hipGetLastError());
    } else {
        FX_HIP_TRY(hipMemcpyAsync(d_nbmap, km->d_nbmap, sizeof(int32_t) * (size_t)total, hipMemcpyDeviceToDevice, st));
    }
    return FX_OK;
}
