// Kernel-map handle shared by the map builder and the convolution kernels.
#pragma once
#include "common.h"

namespace fx {

// Tiled form of the map, the input of the MFMA convolution (Sec. 3.5 scenario 3 (a)-(c):
// blocks of consecutive output indices, per-offset packed pairs, staged input rows).
//
// Outputs are cut into tiles of kTileT consecutive indices.  Inside a tile the outputs are
// reordered so that voxels with equal neighbour masks sit together, then cut into groups of
// 16 (one MFMA column block).  For every (group, offset) with at least one active pair a
// "block" of 16 local row ids is stored; id r < n_rows points into the tile's list of distinct
// input rows (staged once in LDS), kNoRow means "no input" (multiplies a zero row).
constexpr int kTileT = 256;                 // outputs per tile
constexpr int kGroup = 16;                  // outputs per MFMA column block
constexpr int kGroupsPerTile = kTileT / kGroup;
constexpr int kMaxStagedRows = 768;         // LDS rows per tile; further rows are read from global
constexpr uint16_t kNoRow = 0xFFFF;

struct TileHeader {                         // 64 + 16*4 bytes
    int32_t n_rows;                         // distinct input rows of the tile
    int32_t n_blocks;                       // non-empty (group, offset) blocks
    int32_t n_out;                          // valid outputs in the tile (<= kTileT)
    int32_t pad;
    uint32_t group_mask[kGroupsPerTile];    // per group: bit kappa set = block present
    uint32_t group_block0[kGroupsPerTile];  // first block of each group
};

}  // namespace fx

struct fx_kmap {
    std::atomic<int> refs{1};
    hipStream_t stream = nullptr;
    fx_grid* gin = nullptr;
    fx_grid* gout = nullptr;
    int32_t K = 0, stride = 0, K3 = 0;
    int64_t n_in = 0, n_out = 0;
    int32_t* d_nbmap = nullptr;        // dense [n_out, K3] (scalar path, export)
    // tiled form
    int64_t n_tiles = 0;
    fx::TileHeader* d_tile_hdr = nullptr;   // [n_tiles]
    uint16_t* d_tile_perm = nullptr;        // [n_tiles][kTileT] output slot -> local output (0..T-1)
    int32_t* d_tile_rows = nullptr;         // [n_tiles][row_stride] global input rows
    uint16_t* d_tile_blocks = nullptr;      // [n_tiles][block_stride][16] local row ids
    int32_t row_stride = 0, block_stride = 0;
    int64_t* d_stats = nullptr;             // [4 + K3]: rows issued, staged rows, spare, pairs, pairs per offset
    void* d_alloc = nullptr;                // single allocation backing all of the above
    bool stats_valid = false;
    int64_t h_stats[4] = {0, 0, 0, 0};
    int64_t* h_pairs = nullptr;             // [K3]
    int64_t h_n_pairs = 0;
};
