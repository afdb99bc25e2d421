// Kernel-map handle shared by the map builder and the convolution kernels.
#pragma once
#include "common.h"

namespace fx {

// Tiled form of the map, the input of the MFMA convolution (Sec. 3.5 scenario 3 (a)-(c):
// blocks of consecutive output indices, per-offset packed pairs, staged input rows).
//
// Outputs are cut into tiles of kTileT consecutive indices.  Inside a tile the outputs are
// reordered so that voxels with equal neighbour masks sit together, then cut into groups of
// 32 (one MFMA column block).  The 16 groups are dealt to the 4 waves of the convolution
// workgroup (tile_group_of), 4 per wave.  For every (wave, offset) where at least one of the
// wave's 4 groups has an active pair, an "id block" of 32 x 4 local row ids is stored
// ([voxel n of the group][group slot of the wave], so one 8-byte read gives a lane the ids of
// its voxel column in all 4 groups).  A local id r addresses the tile's input rows:
//     r <  win_n            -> global row win_lo + r          (a contiguous window; for a
//                              submanifold map the tile's own index range, which the centre
//                              tap needs anyway)
//     r >= win_n            -> global row rows[r - win_n]     (the halo: distinct rows outside
//                              the window, ascending)
//     r == kNoRow           -> no input (multiplies a zero row, or the block is skipped)
// When all rows of a tile fit the convolution's LDS budget (flag kTileLdsOffsets) the id blocks
// hold lds_row_code(r) instead of r (kNoRow -> the zero row), so the multiply loop needs no
// address arithmetic beyond one XOR.
// A tile flagged kTileDirect keeps no window and lists one row per active pair (no
// de-duplication): used for strided maps, where every input row is used exactly once, and as
// the fallback when a tile's halo exceeds the builder's table.
constexpr int kTileT = 512;                 // outputs per tile
constexpr int kGroup = 32;                  // outputs per MFMA column block (32x32x16 MFMA)
constexpr int kGroupsPerTile = kTileT / kGroup;
#ifndef FX_TILE_WAVES
#define FX_TILE_WAVES 4
#endif
constexpr int kTileWaves = FX_TILE_WAVES;   // consumer waves of the convolution workgroup (4 or 8)
constexpr int kTileWavesLog2 = kTileWaves == 8 ? 3 : 2;
static_assert(kTileWaves == (1 << kTileWavesLog2), "4 or 8 consumer waves");
constexpr int kGroupsPerWave = kGroupsPerTile / kTileWaves;
constexpr int kDealShift = 0;               // runs of 2^kDealShift adjacent groups go to the same wave
constexpr int kMaxK3Tiled = 27;             // offsets supported by the tiled form
constexpr int kMaxHalo = 1024;              // distinct halo rows a tile may de-duplicate
constexpr uint16_t kNoRow = 0xFFFF;
constexpr int32_t kTileDirect = 1;
constexpr int32_t kTileLdsOffsets = 2;       // id blocks hold LDS byte offsets instead of row ids
constexpr int32_t kTilePartial = 4;          // some outputs of the tile are left to another kernel (permutation entry 0xFFFF): never stored

// LDS row layout of the convolution (shared with the builder, which pre-computes offsets):
// rows of kCinChunk bf16/fp16 values (64 bytes); the 16-byte piece q of row r sits at
// r*64 + ((q ^ ((r >> 2) & 3)) << 4); row kRowCap is all zeros.
constexpr int kCinChunk = 32;               // input channels staged in LDS at a time (one MFMA k-step)
constexpr int kRowBytes = kCinChunk * 2;
constexpr int kRowCap = 792;                // LDS rows per tile
__host__ __device__ constexpr uint32_t lds_row_code(uint32_t row) { return row * kRowBytes | (((row >> 2) & 3u) << 4); }
constexpr int kIdBlockElems = kGroup * kGroupsPerWave;   // ids of one block (2 bytes each)

// group (in mask-sorted order) that wave `w` handles in its slot `gi`
__host__ __device__ constexpr int tile_group_of(int w, int gi) {
    return ((gi >> kDealShift) << (kDealShift + kTileWavesLog2)) | (w << kDealShift) | (gi & ((1 << kDealShift) - 1));
}
// and back: the wave and the wave's slot of group g
__host__ __device__ constexpr int tile_wave_of(int g) { return (g >> kDealShift) & (kTileWaves - 1); }
__host__ __device__ constexpr int tile_slot_of(int g) {
    return ((g >> (kDealShift + kTileWavesLog2)) << kDealShift) | (g & ((1 << kDealShift) - 1));
}

struct TileHeader {
    int32_t win_lo;                         // first global row of the window
    int32_t win_n;                          // rows in the window
    int32_t n_list;                         // entries in the tile's row list (halo or direct)
    int32_t n_blocks;                       // id blocks = sum over waves of popcount(wave_mask)
    int32_t n_out;                          // valid outputs in the tile (<= kTileT)
    int32_t flags;                          // kTileDirect
    int32_t n_pair_blocks;                  // non-empty (group, offset) pairs (kGroup MFMA columns each)
    int32_t pad;
    uint32_t group_mask[kGroupsPerTile];    // per group (sorted order): bit kappa set = some voxel has that tap
    uint32_t wave_mask[kTileWaves];         // union of the wave's group masks
    uint32_t wave_block0[kTileWaves];       // first id block of each wave
};

}  // namespace fx

struct fx_kmap {
    std::atomic<int> refs{1};
    hipStream_t stream = nullptr;
    fx_grid* gin = nullptr;
    fx_grid* gout = nullptr;
    int32_t K = 0, stride = 0, K3 = 0;
    int64_t n_in = 0, n_out = 0;
    int32_t* d_nbmap = nullptr;             // dense [n_out, K3]; only when the map is not tiled
    fx_kmap* inverse = nullptr;             // 3x3x3 stride 2: the inverse as a tiled map (produced rows = this map's inputs); built on demand
    bool is_inverse = false;
    // Per-leaf dispatch (Sec. 5 names it as future work; Sec. 3.5's scenarios are its regimes): the same map with the
    // outputs of locally dense leaves left out, and the list of those leaves for the leaf-window kernel.  Built on
    // the first convolution that splits the grid; `mixed` owns the list.
    fx_kmap* mixed = nullptr;
    int32_t* d_dense_leaves = nullptr;      // [n_leaf] leaf ids with at least kDenseLeafVoxels voxels (first *d_n_dense entries)
    int32_t* d_n_dense = nullptr;
    // tiled form
    int64_t n_tiles = 0;
    fx::TileHeader* d_tile_hdr = nullptr;   // [n_tiles]
    uint16_t* d_tile_perm = nullptr;        // [n_tiles][kTileT] output slot -> local output (0..T-1)
    int32_t* d_tile_rows = nullptr;         // [n_tiles][row_stride] global input rows (halo / direct)
    uint16_t* d_tile_blocks = nullptr;      // [n_tiles][block_stride][16][8] local row ids (id blocks)
    int32_t row_stride = 0, block_stride = 0;
    int64_t* d_stats = nullptr;             // [4 + K3]: MFMA rows issued, staged rows, direct tiles, tiled bytes, pairs per offset
    void* d_alloc = nullptr;                // single allocation backing all of the above
    // Tiles whose rows are not all staged in LDS (no kTileLdsOffsets): their number (-1: not counted yet) and the
    // first kMaxListedTiles of them in ascending order; counted on the first weight gradient over the map.
    int32_t h_n_unstaged = -1;
    int32_t* d_unstaged_list = nullptr;
    bool stats_valid = false;
    int64_t h_stats[4] = {0, 0, 0, 0};
    int64_t* h_pairs = nullptr;             // [K3]
    int64_t h_n_pairs = 0;
    int64_t h_tiled_bytes = 0;              // bytes of the tiled form the builder wrote
};

namespace fx {
// whether the tiles of a stride-1 map stage shared input rows (the LDS-staged convolution kernel) or list one row
// per pair (the gather kernels): the submanifold map, a map onto a grid at least twice the size of its input, and
// the inverse of the 3x3x3 stride-2 map
inline bool map_shares_rows(const fx_kmap* km) {
    if (km->is_inverse) return true;       // fine voxels looking up their coarse voxels: neighbours share them
    return km->stride == 1 && (km->gin == km->gout || km->n_out >= 2 * km->n_in);
}
// dense [n_out, K3] table for the scalar convolution path, built on first use (not thread-safe)
fx_status kmap_ensure_dense(fx_kmap* km, hipStream_t st);
// the inverse of a 3x3x3 stride-2 map in tiled form (km->inverse), built on first use (not thread-safe)
fx_status kmap_ensure_inverse(fx_kmap* km, hipStream_t st);
// gout_made_for_map: gout was made by grid_coarsen2_for_map(g_in, K) for this very map (its prepared table applies)
fx_status build_map(fx_grid* g_in, fx_grid* gout, int K, int stride, bool inverse, hipStream_t st, fx_kmap** out, int dense_min = 0,
                    bool gout_made_for_map = false);
// the submanifold 3x3x3 map without the outputs of locally dense leaves + the list of those leaves (km->mixed),
// built on first use (not thread-safe)
fx_status kmap_ensure_mixed(fx_kmap* km, hipStream_t st);
// host copies of the map's statistics (pairs per offset, tiling figures); synchronises the build stream once
fx_status kmap_fetch_stats(fx_kmap* km);
constexpr int kMaxListedTiles = 16;
// km->h_n_unstaged / d_unstaged_list, counting (one small kernel and a wait for its result) on first use
fx_status kmap_unstaged_tiles(fx_kmap* km, hipStream_t st);
}
