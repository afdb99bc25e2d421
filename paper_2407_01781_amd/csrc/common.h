// Shared host/device declarations of the fVDB hot-path library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <atomic>
#include <string>

#include "../../include/fvdb_hotpath.h"

namespace fx {

// ------------------------------------------------------------------ errors
void set_error(const char* fmt, ...);

#define FX_HIP_TRY(expr)                                                                   \
    do {                                                                                   \
        hipError_t _e = (expr);                                                            \
        if (_e != hipSuccess) {                                                            \
            fx::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(_e), __FILE__, \
                          __LINE__);                                                       \
            return FX_EDEVICE;                                                             \
        }                                                                                  \
    } while (0)

#define FX_TRY(expr)                   \
    do {                               \
        fx_status _s = (expr);         \
        if (_s != FX_OK) return _s;    \
    } while (0)

// ------------------------------------------------------------------ options (fx_set_option)
// -1 = automatic: the library decides; any other value is what the caller set.
enum Option {
    kOptForceScalar = 0, kOptLeafDispatch, kOptFp32Tiles, kOptConvGather, kOptGatherLds, kOptScalarLds, kOptGridDirect,
    kOptLeafLinks, kOptCacheMb, kOptSyncAlloc, kOptCount
};
int option(Option o);

// ------------------------------------------------------------------ device memory
// From the caller's allocator when one is set (fx_set_allocator), else from the library's own cache of blocks.
fx_status dev_alloc(void** p, size_t bytes, hipStream_t s);
void dev_free(void* p, hipStream_t s);

// Pinned host staging owned by the library (per thread), at least `bytes` large.  Area 0 is
// for read-backs (the caller synchronises before using the data), area 1 for uploads that stay
// in flight until the caller's next synchronisation on the same stream.
fx_status host_staging(void** p, size_t bytes, int area = 0);

// compute units of the current device (256 on an MI355X; 256 if the query fails)
int compute_units();

// ------------------------------------------------------------------ per-kernel timing
// When enabled (fx_profile_enable), every kernel launch of the library is bracketed by a pair
// of hipEvents on the launch stream; fx_profile_read sums the elapsed times per slot.
enum ProfSlot {
    kProfBucketCount = 0, kProfBucketScan, kProfBucketScatter, kProfBucketLeaves, kProfVoxelsToLeaves, kProfFindTiles, kProfRankTiles, kProfInsertUpper, kProfScanUpper, kProfInsertLower, kProfScanLower,
    kProfInsertLeaf, kProfScanLeaf, kProfGridIjk, kProfNbmap, kProfLeafNeighbors, kProfBuildTiles,
    kProfPackWeights, kProfConvMfma, kProfConvGather, kProfConvScalar, kProfMemset,
    kProfDgradStrided, kProfWgrad, kProfWgradReduce, kProfPool, kProfUpsample, kProfConvLeaf, kProfPointsToIjk, kProfSlotCount
};
bool prof_enabled();
void prof_begin(int slot, hipStream_t s);
void prof_end(int slot, hipStream_t s);
struct ProfScope {
    int slot; hipStream_t s; bool on;
    ProfScope(int slot_, hipStream_t s_) : slot(slot_), s(s_), on(prof_enabled()) { if (on) prof_begin(slot, s); }
    ~ProfScope() { if (on) prof_end(slot, s); }
};


// ------------------------------------------------------------------ tree layout
// Node fan-outs of the VDB tree (Sec. 3.1): upper 32^3 children, lower 16^3, leaf 8^3 voxels.
constexpr int kUpperWords = 32 * 32 * 32 / 64;  // 512 child-mask words per upper node
constexpr int kLowerWords = 16 * 16 * 16 / 64;  // 64 child-mask words per lower node
// a leaf counts as locally dense from 40 % occupancy on (Sec. 3.5: the dense-window operators win from there)
constexpr int kDenseLeafVoxels = 205;
constexpr int kMaxTiles = 65536;                // root tiles per batch (documented limit)
constexpr int kTileHashSlots = 1 << 17;

// counts kept at the head of the grid buffer (device) and mirrored on the host
struct GridHeader {
    int32_t n_tiles_raw;  // distinct root tiles found (may exceed capacity)
    int32_t n_upper;
    int32_t n_lower;
    int32_t n_leaf;
    int32_t overflow;     // bit0: upper capacity, bit1: lower, bit2: leaf, bit3: tile limit, bit4: voxel count, bit5: leaf table full, bit6: a bucket's LDS table full, bit7: a scan's bounded wait expired
    int32_t n_leaf_raw;   // distinct leaves found by the voxel pass (may exceed capacity)
    int32_t pad[2];
    int64_t n_voxels;
    int64_t n_voxels_dense;   // voxels in leaves that hold at least kDenseLeafVoxels of them (what the convolution's per-leaf dispatch goes by)
};

// Device view of one GridBatch.  Internal nodes keep only a child bitmask and, per mask
// word, the global id of the first child in that word: child id = prefix[w] +
// popcount(mask[w] & (bit-1)) -- the indexing of Listing 1 applied at every level.
struct TreeView {
    const uint64_t* root_key;      // [n_upper] biased tile key, sorted by (root_batch, root_key)
    const int32_t*  root_batch;    // [n_upper]
    const uint64_t* upper_mask;    // [n_upper][512]
    const uint32_t* upper_prefix;  // [n_upper][512]
    const uint64_t* lower_mask;    // [n_lower][64]
    const uint32_t* lower_prefix;  // [n_lower][64]
    const fx_leaf*  leaf;          // [n_leaf]
    int32_t n_upper, n_lower, n_leaf, B;
};

}  // namespace fx

struct fx_grid {
    std::atomic<int> refs{1};
    hipStream_t stream = nullptr;
    void* buf = nullptr;          // the one flat device buffer
    size_t buf_bytes = 0;
    int32_t B = 0;
    int32_t cap_upper = 0, cap_lower = 0, cap_leaf = 0;
    fx::GridHeader hdr{};         // host mirror
    int64_t* h_vox_base = nullptr;  // [B+1] host copy of per-grid first indices
    // device section pointers inside buf
    fx::GridHeader* d_hdr = nullptr;
    int64_t* d_vox_base = nullptr;  // [B+1]
    uint64_t* d_root_key = nullptr;
    int32_t* d_root_batch = nullptr;
    uint64_t* d_upper_mask = nullptr;
    uint32_t* d_upper_prefix = nullptr;
    uint64_t* d_lower_mask = nullptr;
    uint32_t* d_lower_prefix = nullptr;
    fx_leaf* d_leaf = nullptr;
    // Prepared by the grid build behind its last step, while the host waits for the counts (see enqueue_leaf_links):
    // [27 * cap_leaf] the leaves of the input grid around every leaf (-1: none) -- the table a kernel map onto this
    // grid starts from: by default the 3x3x3 stride-1 map of the grid onto itself; for the coarse grid that a strided
    // map makes for itself, that map's (links_K, links_stride; its input grid is the one the map is being built from)
    // -- then [cap_leaf + 2] the leaf that holds the first voxel of every run of 512 voxels.
    // Valid for work on `stream` only.  Null when not prepared.
    int32_t* d_leaf_links = nullptr;
    int32_t* d_tile_first_leaf = nullptr;
    int32_t links_K = 0, links_stride = 0;
    fx::TreeView view() const {
        fx::TreeView v;
        v.root_key = d_root_key; v.root_batch = d_root_batch;
        v.upper_mask = d_upper_mask; v.upper_prefix = d_upper_prefix;
        v.lower_mask = d_lower_mask; v.lower_prefix = d_lower_prefix;
        v.leaf = d_leaf;
        v.n_upper = hdr.n_upper; v.n_lower = hdr.n_lower; v.n_leaf = hdr.n_leaf; v.B = B;
        return v;
    }
};

namespace fx {
// Called by the grid build right after its last kernel: allocates g->d_leaf_links / d_tile_first_leaf and enqueues
// the kernel that fills them from the finished tree, reading the counts from the device header (the host does not
// know them yet).  The kernel runs while the host waits for the counts and returns to its caller, a stretch in
// which the device would otherwise idle; the kernel map that comes next then starts with its tile builder.
// g_in = nullptr: the table of the 3x3x3 stride-1 map of the grid onto itself (the common next call); otherwise
// that of the (K, stride) map from g_in onto g, for the coarse grid a strided map build makes for itself.
// A grid whose build overflowed a capacity is skipped by the kernel.  Failure to allocate is not an error: the map
// build then makes the table itself.
void enqueue_leaf_links(fx_grid* g, hipStream_t st, const fx_grid* g_in, int K, int stride);
// fx_grid_coarsen2 for the output grid of a (K, 2) kernel map from g: prepares that map's table (see above)
fx_status grid_coarsen2_for_map(const fx_grid* g, int K, hipStream_t st, fx_grid** out);
}  // namespace fx

