/*
 * fvdb_hotpath.h -- C ABI of the MI355X (gfx950) sparse-convolution hot path of fVDB
 * (arXiv 2407.01781): index-grid build, kernel-map build, sparse convolution forward.
 *
 * Conventions that hold for every call
 *   - Pointers named d_* are DEVICE pointers (HIP, current device); h_* are HOST pointers.
 *   - Inputs are borrowed for the duration of the stream-ordered work; outputs named d_*
 *     are caller-allocated.  Handles (fx_grid, fx_kmap) are library-owned, reference
 *     counted and released with the matching *_destroy.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All device
 *     work is enqueued on it.  Calls that must read a count back (documented below)
 *     synchronise that stream internally.
 *   - Every call returns an fx_status.  Out-parameters are written only on FX_OK.  No C++
 *     exception and no abort crosses this boundary.  fx_last_error() gives a thread-local
 *     message for the last non-OK status.
 *   - Voxel indices are 0-based row numbers of the side-car feature arrays (jdata);
 *     -1 means "no active voxel" (Sec. 3.2: only active voxels get an index).
 *   - A batch of grids is described as a JaggedTensor (Sec. 3.6.1): jdata rows of all
 *     grids back to back plus joffsets [B,2] = (start,end) row of each grid.
 */
#ifndef FVDB_HOTPATH_H
#define FVDB_HOTPATH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fx_grid fx_grid; /* one GridBatch: B IndexGrids in one flat device buffer (Sec. 3.6) */
typedef struct fx_kmap fx_kmap; /* kernel map of one (g_in, kernel_size, stride); holds refs on its grids */

typedef enum {
    FX_OK = 0,
    FX_EINVAL = -1,       /* bad argument (null pointer, negative size, malformed joffsets, ...) */
    FX_EUNSUPPORTED = -2, /* valid request this build does not implement                       */
    FX_ENOMEM = -3,       /* device or host allocation failed                                  */
    FX_EDEVICE = -4,      /* a HIP call failed; fx_last_error() carries hipGetErrorString      */
    FX_ERANGE = -5        /* input exceeds a documented limit                                  */
} fx_status;

typedef enum { FX_F32 = 0, FX_F16 = 1, FX_BF16 = 2 } fx_dtype;

/* One leaf node as exported by fx_grid_leaf_table: the 80-byte record of Listing 1
 * (mOffset, mPrefixSum, mBitMask[8]) followed by the leaf's origin and grid id.
 *   offset : index of the leaf's first active voxel (0-based, global over the batch)
 *   prefix : bits 9w..9w+8 (w = 0..6) = popcount of mask words 0..w
 *   mask   : word = i&7, bit = (j&7)<<3 | (k&7)   (Listing 1's `off`)
 *   origin : 8*(i>>3), 8*(j>>3), 8*(k>>3)                                              */
typedef struct {
    int64_t  offset;
    uint64_t prefix;
    uint64_t mask[8];
    int32_t  origin[3];
    int32_t  batch;
} fx_leaf;

/* Library version string; fx_init checks that a HIP device is present (FX_EDEVICE otherwise) and does the
 * per-device set-up of the current device ahead of time (optional: every entry point does its own on first use). */
const char* fx_version(void);
fx_status   fx_init(void);
const char* fx_last_error(void);

/* Device memory that the library needs beyond the caller's buffers (grid and map handles, scratch).
 *
 * fx_set_allocator hands that to the caller's allocator -- PyTorch's caching allocator, say (the Python binding
 * offers exactly that) -- so that one allocator owns the device's memory:
 *     alloc(bytes, stream, ctx)   -> device pointer usable by work enqueued on `stream` (NULL: out of memory)
 *     release(ptr, stream, ctx)    the block is no longer needed by work enqueued on `stream` after this call
 * Both NULL restores the default.  Set it before handles exist: a block goes back to the allocator that is set
 * when it is released.
 *
 * By default the library keeps the blocks its calls release and hands them to later requests of a similar size
 * (hipMalloc / hipFree cost more than the kernels of a stage); at most option "cache_mb" MiB are kept (default
 * 2048).  fx_release_cached_memory returns all cached blocks to the driver; it waits for the device first. */
typedef void* (*fx_alloc_fn)(size_t bytes, void* stream, void* ctx);
typedef void  (*fx_free_fn)(void* ptr, void* stream, void* ctx);
fx_status fx_set_allocator(fx_alloc_fn alloc, fx_free_fn release, void* ctx);
void fx_release_cached_memory(void);

/* Process-wide switches (atomic; -1 = automatic, the default: the library decides).  They exist so that tests and
 * measurements can send a call to every kernel that is able to serve it; results are the same within the stated
 * tolerances.  Unknown names and values below -1 return FX_EINVAL.
 *   "force_scalar"   1: convolution and both gradients on the scalar kernels (no matrix units)
 *   "leaf_dispatch"  3x3x3 stride-1 maps: 0 never / 1 always (when the shape allows) hand the call to the
 *                    leaf-window kernels, 2 always split it per leaf; automatic: by mean leaf occupancy and the
 *                    share of voxels in dense leaves (see fx_sparse_conv_fwd)
 *   "fp32_tiles"     1: FX_F32 takes the matrix-unit tile kernel at any grid size (automatic: from ~128 tiles on)
 *   "conv_gather"    0 / 1: the LDS-staged / the gather kernel on every tiled map (automatic: by the kind of map)
 *   "gather_lds"     0: the gather kernels fetch their weights per step instead of keeping them in LDS; 1: the
 *                    forward gather kernel keeps one 64-channel output slice's weights in LDS (automatic: two
 *                    slices when both fit, so that a gathered row serves 128 output channels)
 *   "scalar_lds"     0: the scalar kernel reads its weights through L1 instead of LDS
 *   "grid_direct"    1: the grid build skips the bucket pass (one global leaf table)
 *   "leaf_links"     0: the grid build does not prepare the table of the leaves around every leaf behind its last
 *                    step (automatic: it does, and the kernel map of a 3x3x3 convolution of the grid onto itself on
 *                    the grid's stream starts from it)
 *   "cache_mb"       MiB of released device blocks kept for reuse (automatic: 2048)
 *   "sync_alloc"     1: plain hipMalloc / hipFree, no cache                                                     */
fx_status fx_set_option(const char* name, int32_t value);
fx_status fx_get_option(const char* name, int32_t* value);

/* ---------------------------------------------------------------------------------------
 * Index-grid build (Sec. 3.3: build an IndexGrid from N signed voxel coordinates; Sec. 3.2
 * and Listings 1-2: the leaf / lower / upper node layout and offsets; Sec. 3.6: batches).
 *
 *   d_ijk      device [n_rows,3] int32, row-major (i,j,k); any order, duplicates allowed
 *   h_joffsets host   [B,2] int64: grid b owns rows [start_b,end_b); ranges must lie in
 *              [0,n_rows], be non-overlapping and in increasing order; empty ranges and
 *              B == 0 are valid
 *   out        new grid handle.  Active voxels of grid b are ordered by (root tile signed
 *              i,j,k; upper offset; lower offset; leaf offset) -- the order produced by the
 *              two sorts of Sec. 3.3 -- and numbered base_b + rank, base_b = number of
 *              voxels in grids 0..b-1.
 * Synchronises `stream` internally (node counts are read back to size the tree: step 10).
 * Limits: at most 65536 root tiles (4096^3 regions) per batch, 2^31-1 voxels -> FX_ERANGE.
 * FX_EDEVICE when a launch fails or a workgroup of the build's single-pass scans waited for its
 * predecessors beyond the bound (no grid is returned; fx_last_error says which).
 */
fx_status fx_build_index_grid(const int32_t* d_ijk, int64_t n_rows, const int64_t* h_joffsets,
                              int32_t B, void* stream, fx_grid** out);

/* The same grid from point coordinates (Sec. 3.6.2: grids are also built from point clouds; Sec. 4.1.1
 * times the build from ijk or xyz lists).  The paper prints no formula; here voxel (i,j,k) is the
 * half-open cell [origin + i*s, origin + (i+1)*s) per axis:
 *     ijk = floor((xyz - origin) / voxel_size)
 * evaluated in IEEE single precision (rounded subtraction, rounded division, floor), then
 * fx_build_index_grid on those coordinates (a caller who wants voxel centres at integer
 * coordinates passes origin - voxel_size / 2).
 *
 *   d_xyz         device [n_rows,3] float32, row-major
 *   h_joffsets, B as fx_build_index_grid
 *   h_origin      host [3] float32, finite
 *   h_voxel_size  host [3] float32, finite and > 0
 * FX_ERANGE if any coordinate is not finite or its cell lies outside [-2^30, 2^30) (no grid is
 * returned).  Allocates n_rows * 12 bytes of temporary device memory; synchronises `stream`.
 */
fx_status fx_build_index_grid_from_points(const float* d_xyz, int64_t n_rows, const int64_t* h_joffsets,
                                          int32_t B, const float* h_origin, const float* h_voxel_size,
                                          void* stream, fx_grid** out);

/* Sizes of a grid: total active voxels, batch size, per-grid voxel ranges [B,2] (host, may
 * be NULL) and node counts {leaf, lower, upper} (host, may be NULL). */
fx_status fx_grid_info(const fx_grid* g, int64_t* n_voxels, int32_t* B,
                       int64_t* h_voxel_joffsets, int64_t* h_counts3);

/* Coordinates of all active voxels in index order: d_ijk_out [N,3] int32, and the grid id
 * of each (d_jidx_out [N] int32, may be NULL) -- the jidx of Sec. 3.6.1. */
fx_status fx_grid_ijk(const fx_grid* g, int32_t* d_ijk_out, int32_t* d_jidx_out, void* stream);

/* Listing 1's getValue for n query coordinates: d_index_out[r] = index of voxel d_ijk[r] in
 * grid d_jidx[r] (NULL = grid 0), or -1 if inactive / grid id out of range. */
fx_status fx_grid_ijk_to_index(const fx_grid* g, const int32_t* d_ijk, const int32_t* d_jidx,
                               int64_t n, int32_t* d_index_out, void* stream);

/* Copy the leaf table (n_leaf records of fx_leaf, index order) to HOST memory.
 * `bytes` must be >= n_leaf * sizeof(fx_leaf).  Synchronises `stream`. */
fx_status fx_grid_leaf_table(const fx_grid* g, fx_leaf* h_out, size_t bytes, void* stream);

/* Output grid of a stride-2 operator: active set = distinct floor(ijk/2) per grid (the
 * coarsening of Sec. 3.6.2 "Grid Construction Operators").  Synchronises `stream`. */
fx_status fx_grid_coarsen2(const fx_grid* g, void* stream, fx_grid** out);

/* The subdivided grid of Sec. 3.6.2 (the grid that upsampling produces): active set =
 * all eight children 2*ijk + {0,1}^3 of every active voxel, per grid of the batch.  The kernel map
 * fx_build_kernel_map(*out, 2, 2) then has g as its output grid (same voxels, same order).
 * FX_ERANGE beyond 2^31-1 voxels, or if a leaf of g holds coordinates outside [-2^30, 2^30) (their doubles
 * leave the int32 coordinate limits).  The caller owns *out.  Synchronises `stream`. */
fx_status fx_grid_subdivide2(const fx_grid* g, void* stream, fx_grid** out);

/* The padded grid of Sec. 3.6.2 (a grid made from another by padding; the dilation that Sec. 3.3 names as
 * the case that changes topology): active set = every voxel within Chebyshev distance r of an active one,
 * { p + d : p active, d in {-r..r}^3 }, per grid of the batch.  r = 0 gives a copy; r = 1 is the set of sites
 * a 3x3x3 stencil reaches the grid from.  0 <= r <= 8 (FX_EINVAL below, FX_EUNSUPPORTED above);
 * FX_ERANGE if the padded grid has more than 2^31-1 voxels or a voxel lies within r of the int32 coordinate limits.
 * The caller owns *out.  Synchronises `stream`. */
fx_status fx_grid_pad(const fx_grid* g, int32_t r, void* stream, fx_grid** out);

void fx_grid_retain(fx_grid* g);
void fx_grid_destroy(fx_grid* g);

/* ---------------------------------------------------------------------------------------
 * Kernel map (Sec. 3.5: for every output voxel and stencil offset, the input voxel linked
 * by that offset, found through the tree's index lookup; scenario 3 (a)-(c): blocks of
 * consecutive output indices with per-offset packed pairs).
 *
 *   kernel_size K, stride s: supported (K,s) = (1,1), (3,1), (5,1), (2,2), (3,2).
 *   Offsets: K odd -> delta in {-(K-1)/2..(K-1)/2}^3; K even -> {0..K-1}^3;
 *            kappa = (di-dmin)*K*K + (dj-dmin)*K + (dk-dmin)   (i slowest).
 *   Output grid: s == 1 -> g_in itself (submanifold; *g_out = g_in with one more reference);
 *                s == 2 -> fx_grid_coarsen2(g_in) for K = 2 and for K = 3 alike (the paper leaves the
 *                          output set of a strided 3x3x3 convolution open; this reading keeps the
 *                          coarse grid of the 2x2x2 case, and output p reads the inputs 2p + {-1,0,1}^3).
 *   map(o,kappa) = index in g_in of voxel  s*p_o + delta_kappa  (same grid of the batch), or -1.
 * Both handles must be destroyed by the caller.  Synchronises `stream` when s == 2.
 */
fx_status fx_build_kernel_map(fx_grid* g_in, int32_t kernel_size, int32_t stride, void* stream,
                              fx_grid** g_out, fx_kmap** out);

/* The stride-1 map onto a caller-given output grid: map(o,kappa) = index in g_in of voxel p_o + delta_kappa
 * for the voxels p_o of g_out (same offsets and kappa order as above).  With g_out = fx_grid_pad(g_in, 1) and
 * K = 3 this is the map of a convolution that is not restricted to the input's voxels: every (input, offset)
 * pair occurs once, so no product of the dense cross-correlation is dropped (Sec. 3.5 describes the operator
 * for any pair of input and output index spaces; Sec. 3.6.2 makes the output grid by padding).
 *   K in {1, 3, 5}; the grids must hold the same number of batch members (FX_EINVAL otherwise); g_out may be
 *   g_in itself (the submanifold map of fx_build_kernel_map).  The map keeps references to both grids.
 * All operators that take a stride-1 map accept it: fx_sparse_conv_fwd, fx_sparse_conv_bwd_data,
 * fx_sparse_conv_bwd_weight, fx_sparse_conv_transpose_fwd.  Between two different grids the tiles hold one row
 * per pair (no staging of shared rows), and the input gradient and the transposed convolution run over the
 * map from g_in's voxels into g_out, built on their first call and kept with the map. */
fx_status fx_build_kernel_map_onto(fx_grid* g_in, fx_grid* g_out, int32_t kernel_size, void* stream, fx_kmap** out);

/* n_out, K^3, number of active (output, offset) pairs and pairs per offset (host [K^3], may
 * be NULL).  Synchronises the stream the map was built on. */
fx_status fx_kmap_info(const fx_kmap* km, int64_t* n_out, int32_t* k3, int64_t* n_pairs,
                       int64_t* h_pairs_per_offset);

/* The map as a dense table d_nbmap [N_out, K^3] int32 (-1 = none), decoded from the tiled
 * form the convolution kernels consume. */
fx_status fx_kmap_dense(const fx_kmap* km, int32_t* d_nbmap, void* stream);

/* Tiling statistics (host): h_stats[0] = MFMA rows issued by the tiled convolution (16 per
 * non-empty (group, offset) block), [1] = number of tiles, [2] = staged input rows summed
 * over tiles, [3] = tile size T.  Synchronises the build stream. */
fx_status fx_kmap_tile_stats(const fx_kmap* km, int64_t* h_stats4);

/* Bytes of the tiled form that the map build wrote to device memory (tile headers, output
 * permutations, row lists, id blocks): the figure the map build's bandwidth is quoted on.
 * 0 for maps that are kept as a dense table only (K = 5).  Synchronises the build stream. */
fx_status fx_kmap_tiled_bytes(const fx_kmap* km, int64_t* h_bytes);

void fx_kmap_destroy(fx_kmap* km);

/* ---------------------------------------------------------------------------------------
 * Sparse convolution forward (Sec. 3.6.2: G_in, kernel, Z_in -> Z_out on G_out; Sec. 3.5
 * scenario 3: gather, per-offset GEMM, accumulate, sequential write-back; Sec. 4.1.3:
 * only taps with an active input voxel contribute):
 *     out[o,:] = sum_{kappa : map(o,kappa) >= 0}  feat[map(o,kappa),:] . W[kappa]
 *
 *   d_feat  device [N_in, C_in]  row-major, dtype in_dt
 *   d_w     device [K^3, C_in, C_out] row-major, dtype in_dt
 *   d_out   device [N_out, C_out] row-major, dtype out_dt (= in_dt or FX_F32); every row is
 *           written (rows without any active tap become 0)
 * Products are exact in the input precision's product format and accumulated in fp32; the result is
 * rounded to out_dt with round-to-nearest-even.  C_in, C_out >= 1.
 * Which kernel runs (all give the same sum within the stated tolerance):
 *   - the matrix units (v_mfma_f32_32x32x16 for FX_F16 / FX_BF16; v_mfma_f32_32x32x2_f32, true fp32 products, for
 *     FX_F32) when the map is tiled (K^3 <= 27), C_in * sizeof(element) is a multiple of 64 bytes (32 channels of
 *     a 16-bit type, 16 of fp32) and C_out is even (padded to 64 with zero weights); FX_F32 only from about 128
 *     tiles on (smaller grids are served faster by the scalar kernel spread over the chip);
 *   - on a 3x3x3 stride-1 submanifold map whose grid is locally dense (mean leaf occupancy >= 0.40, or >= 0.08
 *     for FX_F32 with C_in not a multiple of 16) and whose shape fx_sparse_conv_leaf_fwd serves: the
 *     leaf-window kernels;
 *   - per-leaf dispatch (16-bit types, shapes of the leaf-window kernel): a sparser grid of which at least 10 % of
 *     the voxels sit in locally dense leaves (>= 205 of 512 voxels) is split inside the call -- those leaves go to
 *     the leaf-window kernel, all other outputs to the tile kernel over a second copy of the map, built on the
 *     first such call and kept with the map;
 *   - everything else: a scalar kernel (fp32 FMA in offset-then-channel order).
 */
fx_status fx_sparse_conv_fwd(const fx_kmap* km, const void* d_feat, fx_dtype in_dt, const void* d_w,
                             int32_t C_in, int32_t C_out, void* d_out, fx_dtype out_dt, void* stream);

/* fx_sparse_conv_fwd for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same result bits; the memory
 * the kernels need beyond inputs and outputs (the packed weights and eight work-list counters) is a static
 * device array of FX_NOALLOC_MAX_WEIGHT_BYTES + 256 bytes that each GPU the library runs on holds until the
 * process ends.  The call allocates and frees nothing, on the device or through any library.
 *   Serves the matrix-unit kernels only: a tiled map (K^3 <= 27), C_in * sizeof(element) a multiple of 64,
 *   C_out even; anything else returns FX_EUNSUPPORTED (use fx_sparse_conv_fwd).  Packed weights
 *   (K^3 * C_in * roundup(C_out, 64) elements) beyond the static buffer return FX_ERANGE; 3x3x3 at 256 -> 256
 *   channels of a 16-bit type fits.
 *   All calls on one GPU share that GPU's array: calls that overlap on one GPU (different streams or threads)
 *   race on it and give undefined outputs; calls on one stream are ordered and safe.  Every call rewrites what
 *   it reads from the array (weights and counters), so nothing carries over from the previous call. */
#define FX_NOALLOC_MAX_WEIGHT_BYTES (4u << 20)
fx_status fx_sparse_conv_fwd_noalloc(const fx_kmap* km, const void* d_feat, fx_dtype in_dt, const void* d_w,
                                     int32_t C_in, int32_t C_out, void* d_out, fx_dtype out_dt, void* stream);

/* ---------------------------------------------------------------------------------------
 * Sparse convolution backward (Sec. 3.6 / 3.6.2: the operators are differentiable; Sec. 4.1.3
 * names the gradient with respect to the filter coefficients).  The paper prints no formula;
 * these are the derivatives of the forward sum above.  With gout = dL/dout:
 *
 *   fx_sparse_conv_bwd_data:    gin[i,:] = sum over pairs (o,kappa) with map(o,kappa) = i of
 *                                          W[kappa] . gout[o,:]
 *   fx_sparse_conv_bwd_weight:  gw[kappa,:,:] = sum over o with map(o,kappa) >= 0 of
 *                                          feat[map(o,kappa),:]^T  gout[o,:]
 *
 *   d_gout  device [N_out, C_out] row-major, dtype dt
 *   d_w     device [K^3, C_in, C_out], dtype dt          (bwd_data)
 *   d_feat  device [N_in, C_in], dtype dt                (bwd_weight)
 *   d_gin   device [N_in, C_in], dtype out_dt (= dt or FX_F32); every row is written
 *   d_gw    device [K^3, C_in, C_out], dtype out_dt (= dt or FX_F32); every element is written
 * Products are exact and accumulated in fp32, one rounding (RNE) to out_dt at the end.  The
 * weight gradient is summed in a fixed order (per-workgroup partial sums over contiguous tile
 * ranges, then one ordered reduction): repeated calls give identical bits.  The first bwd_weight call
 * over a sparse stride-1 map counts the map's tiles whose rows do not fit the kernel's LDS stage (one small
 * kernel whose result the host waits for; kept with km) and picks its launches by that count.
 * bwd_data on a stride-1 map is the forward kernel run on the same map with the offsets
 * mirrored and W[kappa] transposed (the map of a submanifold convolution is symmetric); on a
 * K = stride map every input has exactly one pair and its row is written once; on the 3x3x3 stride-2
 * map an input is shared by up to 8 outputs and the sum is gathered per input through the inverse map
 * (a tiled map of its own, built on the first such call and kept with km; no atomics, fixed order).
 * MFMA paths: FX_F16 / FX_BF16 with C_in % 64 == 0 and C_out % 64 == 0 (bwd_data: C_in % 64 == 0
 * and C_out % 32 == 0; bwd_weight: C_in % 32 == 0 and C_out % 64 == 0) on tiled maps; everything
 * else takes scalar kernels.  In the MFMA weight-gradient kernel a tile whose input rows do not all
 * fit the kernel's local memory has its operand transposed by a multiplication with the identity; on
 * such a tile a non-finite value in feat makes the whole 32-channel block of gw that it touches NaN
 * rather than only its own row.  On the (3,1) map of one grid bwd_weight follows the forward pass's rule for
 * the leaf-window kernels: at those shapes a locally dense grid (mean leaf occupancy >= 0.40) is summed leaf by
 * leaf without the map (fx_sparse_conv_leaf_bwd_weight), and a grid that mixes dense and sparse leaves is split per
 * leaf between that kernel and the tile kernel inside the call (option leaf_dispatch as for the forward pass).
 */
fx_status fx_sparse_conv_bwd_data(const fx_kmap* km, const void* d_gout, fx_dtype dt, const void* d_w,
                                  int32_t C_in, int32_t C_out, void* d_gin, fx_dtype out_dt, void* stream);
fx_status fx_sparse_conv_bwd_weight(const fx_kmap* km, const void* d_feat, const void* d_gout, fx_dtype dt,
                                    int32_t C_in, int32_t C_out, void* d_gw, fx_dtype out_dt, void* stream);

/* ---------------------------------------------------------------------------------------
 * Transposed convolution, pooling, upsampling (Sec. 3.6.2 lists max and average pooling of a grid and
 * its features, and upsampling by subdivision with nearest-neighbour sampling; Sec. 4.1.4's network
 * needs them and the transposed convolution in its decoder half).  The
 * paper prints no formulas; with km the kernel map of a convolution from grid g_in (inputs i) to
 * g_out (outputs o):
 *
 *   fx_sparse_conv_transpose_fwd   out[i,:] = sum over pairs (o,kappa) with map(o,kappa) = i of
 *                                             feat[o,:] . W[kappa]
 *        d_feat [N_out, C_in] lives on g_out, d_out [N_in, C_out] on g_in, d_w [K^3, C_in, C_out];
 *        supported maps: K = stride (one pair per input, every row of d_out is written), stride 1
 *        (symmetric map: the forward kernels over the mirrored offsets) and 3x3x3 stride 2 (gathered per
 *        input through the inverse map, built on first use).  Types, accumulation and
 *        rounding as fx_sparse_conv_fwd; MFMA path for K = stride: FX_F16 / FX_BF16, C_in % 32 == 0,
 *        C_out % 64 == 0.
 *   fx_pool2       km must be a (2,2) map.  out[o,c] = max (FX_POOL_MAX) or mean (FX_POOL_AVG) over the
 *                  ACTIVE children i = map(o,kappa) of feat[i,c]; the mean is the fp32 sum in offset
 *                  order divided by the number of active children (not by 8), rounded once to dt.
 *        d_feat [N_in, C], d_out [N_out, C], both dtype dt.
 *   fx_upsample2   km must be a (2,2) map.  out[i,:] = feat[o,:] for the pair with map(o,kappa) = i
 *                  (nearest neighbour: every fine voxel copies its parent's row, bit for bit).
 *        d_feat [N_out, C], d_out [N_in, C], both dtype dt.  To upsample onto all children of a grid
 *        g: fine = fx_grid_subdivide2(g), km = fx_build_kernel_map(fine, 2, 2).
 * All device pointers are borrowed for the stream-ordered work; outputs are caller-allocated.
 */
typedef enum { FX_POOL_MAX = 0, FX_POOL_AVG = 1 } fx_pool_mode;

fx_status fx_sparse_conv_transpose_fwd(const fx_kmap* km, const void* d_feat, fx_dtype dt, const void* d_w,
                                       int32_t C_in, int32_t C_out, void* d_out, fx_dtype out_dt, void* stream);
fx_status fx_pool2(const fx_kmap* km, int32_t mode, const void* d_feat, fx_dtype dt, int32_t C, void* d_out,
                   void* stream);
fx_status fx_upsample2(const fx_kmap* km, const void* d_feat, fx_dtype dt, int32_t C, void* d_out, void* stream);

/* Gradients of fx_pool2 and fx_upsample2 (Sec. 3.6: the operators are differentiable); km a (2,2) map,
 * i its inputs (fine voxels), o its outputs (coarse voxels), n(o) the number of active children of o:
 *   fx_pool2_bwd      FX_POOL_AVG: gin[i,c] = gout[o,c] / n(o) for the parent o of i (fp32 division, one
 *                     rounding to dt); d_feat is not read and may be NULL.
 *                     FX_POOL_MAX: gin[i,c] = gout[o,c] if i is the child whose feat[i,c] is the maximum --
 *                     the first in offset order among equals, the one fx_pool2 keeps -- else 0 (exact);
 *                     d_feat is the input of the forward call.
 *        d_feat [N_in, C], d_gout [N_out, C], d_gin [N_in, C], all dtype dt; every row of d_gin is written.
 *   fx_upsample2_bwd  gin[o,c] = sum over the active children i of o of gout[i,c] (fp32 sum in offset order,
 *                     one rounding to dt).  d_gout [N_in, C], d_gin [N_out, C]. */
fx_status fx_pool2_bwd(const fx_kmap* km, int32_t mode, const void* d_feat, const void* d_gout, fx_dtype dt, int32_t C,
                       void* d_gin, void* stream);
fx_status fx_upsample2_bwd(const fx_kmap* km, const void* d_gout, fx_dtype dt, int32_t C, void* d_gin, void* stream);

/* ---------------------------------------------------------------------------------------
 * 3x3x3 submanifold convolution straight from the grid, without a kernel map (Sec. 3.5 scenario 1,
 * the "Leaf" operator: the 10^3 window of input rows around each 8^3 leaf is densified in on-chip
 * memory, the gather offsets come from the tree itself, and each leaf's outputs are written as one
 * contiguous range; the same window serves the locally dense, deeper regime that scenario 2 targets).
 * Same result as fx_sparse_conv_fwd on the (3,1) map of g:
 *     out[o,:] = sum over the 27 offsets kappa whose neighbour i of voxel o is active of
 *                feat[i,:] . W[kappa]
 *
 *   g       the grid; inputs and outputs both live on it (N = its voxel count)
 *   d_feat  device [N, C_in]  row-major, dtype dt, 16-byte aligned
 *   d_w     device [27, C_in, C_out] row-major, dtype dt, kappa = (di+1)*9 + (dj+1)*3 + (dk+1)
 *   d_out   device [N, C_out] row-major, dtype out_dt (= dt or FX_F32), 16-byte aligned; every row is written
 * Supported shapes:
 *   FX_F32            C_in in {4, 8, 12, 16}, C_out a multiple of 4 up to 32, out_dt = FX_F32 (true fp32 products on the
 *                     matrix units, fp32 sums; order differs from fx_sparse_conv_fwd, same tolerance)
 *   FX_F16 / FX_BF16  C_in % 32 == 0, C_out % 64 == 0 (exact products, fp32 sums, one RNE rounding to out_dt);
 *                     allocates the packed weights (27 * C_in * C_out * 2 bytes) for the call
 * anything else returns FX_EUNSUPPORTED (build a kernel map and call fx_sparse_conv_fwd).  Unlike the
 * paper's kernel, (column tile, offset) pairs without any active neighbour are skipped: at these shapes
 * the operator is bound by arithmetic on gfx950, not by memory.  Meant for leaf occupancy above ~20 %
 * (volumetric and dense grids); on sparse grids the kernel-map path is several times faster.
 * Does not synchronise; pointers are borrowed for the stream-ordered work.
 */
fx_status fx_sparse_conv_leaf_fwd(const fx_grid* g, const void* d_feat, fx_dtype dt, const void* d_w,
                                  int32_t C_in, int32_t C_out, void* d_out, fx_dtype out_dt, void* stream);

/* Input gradient of the convolution above (Sec. 3.6: the operators are differentiable), again without a
 * kernel map:  gin[i,:] = sum over pairs (o,kappa) with neighbour(o,kappa) = i of  W[kappa] . gout[o,:].
 * The map of a submanifold convolution is symmetric, so this is the forward kernel on gout with the
 * offsets reflected (kappa -> 26 - kappa) and every W[kappa] transposed; same result as
 * fx_sparse_conv_bwd_data on the (3,1) map of g.
 *   d_gout [N, C_out] dtype dt, d_w [27, C_in, C_out] (the forward layout), d_gin [N, C_in] dtype out_dt.
 * Supported shapes: the forward's with the roles of C_in and C_out exchanged (fp32: C_out in
 * {4, 8, 12, 16}, C_in a multiple of 4 up to 32; FX_F16 / FX_BF16: C_out % 32 == 0, C_in % 64 == 0); others
 * FX_EUNSUPPORTED. */
fx_status fx_sparse_conv_leaf_bwd_data(const fx_grid* g, const void* d_gout, fx_dtype dt, const void* d_w,
                                       int32_t C_in, int32_t C_out, void* d_gin, fx_dtype out_dt, void* stream);

/* Weight gradient of the same convolution without a kernel map (fp32 at low depth; f16 / bf16 at depth >= 32):
 *     gw[kappa,:,:] = sum over voxels o whose neighbour i at offset kappa is active of  feat[i,:]^T gout[o,:]
 * with the voxels as the contracted dimension of the matrix instructions, straight from the leaf window; same
 * result as fx_sparse_conv_bwd_weight on the (3,1) map of g.
 *   d_feat [N, C_in] and d_gout [N, C_out] device, dtype dt, 16-byte aligned; d_gw [27, C_in, C_out] device,
 *   dtype out_dt; every element is written (zeros for an empty grid).
 * Supported: dt = FX_F32 with C_in in {4, 8, 12, 16} and C_out a multiple of 4 up to 32 (the forward's shapes; C_in
 * of 12 or 16 with more than 16 output channels takes two launches), out_dt = FX_F32; dt = FX_F16 / FX_BF16 with
 * C_in % 32 == 0 and C_out % 64 == 0, out_dt = dt or FX_F32 (exact products, one rounding of the result); others
 * FX_EUNSUPPORTED.  fp32 sums in a
 * fixed order (leaves in fixed ranges per workgroup, the workgroups' partial sums added in index order): repeated
 * calls give identical bits.  Allocates the partial sums (one [27, C_in, C_out] fp32 block per workgroup, at
 * most a few thousand) for the call.  Does not synchronise. */
fx_status fx_sparse_conv_leaf_bwd_weight(const fx_grid* g, const void* d_feat, const void* d_gout, fx_dtype dt,
                                         int32_t C_in, int32_t C_out, void* d_gw, fx_dtype out_dt, void* stream);

/* ---------------------------------------------------------------------------------------
 * Measurement support (the paper's protocol, Sec. 4.1: per-operator times).  While enabled,
 * every kernel launch of the library is bracketed by hipEvents on its launch stream;
 * fx_profile_read waits for the recorded events and returns the summed time and launch count
 * of one slot (slot names: fx_profile_slot_name, e.g. "k_conv_mfma", "k_build_tiles").
 */
void        fx_profile_enable(int on);
void        fx_profile_reset(void);
int         fx_profile_slot_count(void);
const char* fx_profile_slot_name(int slot);
fx_status   fx_profile_read(int slot, double* total_ms, int64_t* count);

#ifdef __cplusplus
}
#endif
#endif /* FVDB_HOTPATH_H */
