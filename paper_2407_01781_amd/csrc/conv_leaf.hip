// Low-depth 3x3x3 submanifold convolution computed leaf by leaf, straight from the tree, with no
// kernel map (Sec. 3.5 scenario 1, "Leaf": local densification of the 10^3 window around an 8^3
// leaf in on-chip memory, gather offsets taken from the tree's own metadata, sequential
// write-back of the leaf's outputs).
//
// What is kept from the paper's design: one workgroup per leaf; the window of input rows
// densified in LDS (inactive cells hold zeros) so that the 27 taps become fixed address
// offsets; the leaf's outputs leave as one contiguous range.  What differs, and why: the
// paper's kernel multiplies all 512 cells of the leaf by all 27 taps because on its hardware a
// dense 8 -> 16 convolution at fp32 is bound by memory.  On gfx950 it is not: 6912 flop per
// 96 bytes is 72 flop/byte against a ridge of 157.3 TFLOP/s / 8 TB/s = 20 flop/byte, so wasted
// multiplies cost time.  This kernel therefore packs the leaf's ACTIVE voxels into column tiles
// of 16 and skips every (tile, tap) in which no voxel of the tile has an active neighbour.
// The contraction runs on v_mfma_f32_16x16x4_f32 (gfx950 has no TF32-class format): output
// channels are the rows, voxels the columns, so a lane ends up holding four adjacent channels
// of one voxel and a tile of 16 output rows leaves as one 16-byte store per lane.
#include <algorithm>

#include "common.h"
#include "conv_common.h"
#include "tree_device.h"

namespace fx {
namespace {

typedef __attribute__((ext_vector_type(2))) float f32x2;

constexpr int kLeafWaves = 4;                // one wave per SIMD, so that workgroups pack evenly onto a compute unit
constexpr int kLeafThreads = 64 * kLeafWaves;
constexpr int kWinCells = 1000;              // 10 x 10 x 10 cells: the leaf plus a one-voxel halo
constexpr int kVoxTile = 16;                 // active voxels per MFMA column tile

struct LeafLds {
    uint64_t mask[27][8];                    // records of the 27 leaves around (and including) this one
    uint64_t prefix[27];
    int32_t offset[27];                      // first index of the leaf; masks are zero when the leaf is absent
    uint32_t act_row[100];                   // per (x, y) of the window: bit z = cell (x, y, z) is active
    uint16_t cell_of_rank[512];              // window cell of the leaf's r-th active voxel
    uint32_t tile_taps[512 / kVoxTile];      // per column tile: bit kappa = some voxel has that neighbour
    int32_t next_tile;                       // column tiles handed out so far
    int32_t range[2];                        // this workgroup's leaves [range[0], range[1])
};

__device__ __forceinline__ int window_cell(int x, int y, int z) { return (x * 10 + y) * 10 + z; }

// index of the voxel at leaf-local (lx,ly,lz) of staged record `slot`, or -1 (Listing 1)
template <typename LDS>
__device__ __forceinline__ int staged_value(const LDS& L, int slot, int lx, int ly, int lz) {
    const uint64_t w = L.mask[slot][lx];
    const uint64_t bit = 1ull << ((ly << 3) | lz);
    if (!(w & bit)) return -1;
    const uint64_t pre = lx ? (L.prefix[slot] >> (9 * (lx - 1))) & 511 : 0;
    return L.offset[slot] + (int)pre + __popcll(w & (bit - 1));
}

// J consecutive floats from LDS (p is J*4-byte aligned for J = 1, 2, 4)
template <int J> struct Floats { float v[J]; };
template <int J>
__device__ __forceinline__ Floats<J> lds_floats(const float* p) {
    Floats<J> r;
    if (J == 2) {
        const f32x2 t = *reinterpret_cast<const f32x2*>(p);
        r.v[0] = t[0]; r.v[1] = t[1];
    } else if (J == 4) {
        const f32x4 t = *reinterpret_cast<const f32x4*>(p);
#pragma unroll
        for (int j = 0; j < J; ++j) r.v[j] = t[j];
    } else {
#pragma unroll
        for (int j = 0; j < J; ++j) r.v[j] = p[j];
    }
    return r;
}


// Records of the 27 leaves around (and including) leaf f into LDS: one tree descent per lane.
template <typename LDS>
__device__ __forceinline__ void stage_records(const TreeView& t, LDS& L, int f, int lane) {
    if (lane >= 27) return;
    const fx_leaf* lf = t.leaf + f;
    const int a = lane / 9, b = (lane / 3) % 3, c = lane % 3;
    const int id = lane == 13 ? f
                              : find_leaf(t, lf->batch, lf->origin[0] + 8 * (a - 1), lf->origin[1] + 8 * (b - 1),
                                          lf->origin[2] + 8 * (c - 1));
    if (id >= 0) {
        const fx_leaf* nl = t.leaf + id;
#pragma unroll
        for (int x = 0; x < 8; ++x) L.mask[lane][x] = nl->mask[x];
        L.prefix[lane] = nl->prefix;
        L.offset[lane] = (int32_t)nl->offset;
    } else {
#pragma unroll
        for (int x = 0; x < 8; ++x) L.mask[lane][x] = 0;
        L.prefix[lane] = 0;
        L.offset[lane] = -1;
    }
}

// Leaves are dealt to the persistent workgroups as contiguous ranges of equal estimated cost: a
// leaf costs kLeafFixedCost (staging, densifying 1000 cells) plus one unit per active voxel, so the
// cost of leaves [0, f) is kLeafFixedCost * f + offset of leaf f, which grows with f.  Returns the
// first leaf whose prefix cost reaches `target` (wave-wide 64-ary search; every lane gets the result).
constexpr int64_t kLeafFixedCost = 220;
template <int64_t FIXED>
__device__ __forceinline__ int first_leaf_at_cost(const TreeView& t, int64_t first_index, int64_t target, int lane) {
    int lo = 0, hi = t.n_leaf;               // answer in [lo, hi]; prefix cost of leaf n_leaf counts as infinite
    while (hi - lo > 0) {
        const int span = hi - lo;
        const int step = (span + 63) / 64;
        const int f = lo + lane * step;      // probes lo, lo + step, ...
        bool below = false;                  // prefix cost of f < target
        if (f < hi) below = FIXED * f + (t.leaf[f].offset - first_index) < target;
        const int n_below = __popcll(__ballot(below));     // probes are ascending in cost: a prefix of them is below
        if (n_below == 0) { hi = lo; break; }
        const int last_below = lo + (n_below - 1) * step;
        lo = last_below + 1;
        hi = min(hi, last_below + step);
    }
    return lo;
}

// window-cell distance of tap kappa
__device__ __forceinline__ int tap_delta(int kappa) { return (kappa / 9) * 100 + ((kappa / 3) % 3) * 10 + kappa % 3 - 111; }

// Element of the caller's weights that multiplies contracted channel c into produced channel p at tap
// kappa.  Forward: W[kappa][c][p].  Mirrored (the input gradient on the symmetric submanifold map): the
// caller's array is W[27][p-count][c-count] and the tap is reflected: W[26 - kappa][p][c].
__device__ __forceinline__ int leaf_weight_index(int kappa, int c, int p, int n_contract, int n_produce, int mirrored) {
    return mirrored ? ((26 - kappa) * n_produce + p) * n_contract + c : (kappa * n_contract + c) * n_produce + p;
}

// J = C_in / 4 MFMA k-steps per tap, NT row tiles of 16 produced channels (n_produce <= 16 NT of them exist,
// a multiple of 4: the others multiply zero weights and are not stored), WREG: every lane keeps its share of
// the weights (27 * J * NT values) in registers instead of LDS.
// Workgroups are persistent: each keeps the weights and takes leaves blockIdx.x, blockIdx.x +
// gridDim.x, ...  All four waves densify; in the multiply phase the waves claim column tiles from a
// counter in LDS, and the last wave first walks the tree for the NEXT leaf's 27 records (they are not
// read during the multiply, so one copy of them is enough) and joins the others afterwards.  The
// multiply is bound by the matrix pipes, which all workgroups of a compute unit share; the other
// phases of one workgroup overlap with the multiplies of the others.
// Lane l of a wave works on voxel column v = l % 16 and k-quarter q = l / 16: it holds the J
// input channels J*q .. J*q + J-1 of its voxel's neighbour (k-step j contracts channels {J*q + j})
// and, per row tile, the same channels of output channel 16*nt + v of the weights.
template <int J, int NT, bool WREG, bool FULLP>     // FULLP: all 16 NT produced channels exist
__global__ __launch_bounds__(kLeafThreads, 4) void k_conv_leaf(TreeView t, const float* __restrict__ feat,
                                                            const float* __restrict__ w, float* __restrict__ out,
                                                            int64_t n_voxels, int mirrored, int n_produce_arg) {
    constexpr int C_in = 4 * J, C_out = 16 * NT;
    const int n_produce = FULLP ? C_out : n_produce_arg;
    extern __shared__ __align__(16) unsigned char smem[];
    LeafLds& L = *reinterpret_cast<LeafLds*>(smem);
    float* win = reinterpret_cast<float*>(smem + ((sizeof(LeafLds) + 15) & ~size_t(15)));   // [cell][C_in]
    float* wl = win + kWinCells * C_in;                                  // [kappa][q][cout][j], unless WREG
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int v = lane & 15, q = lane >> 4;

    float wr[WREG ? 27 : 1][NT][J];
    if (WREG) {
#pragma unroll
        for (int kappa = 0; kappa < 27; ++kappa)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int j = 0; j < J; ++j)
                    wr[WREG ? kappa : 0][nt][j] =
                        FULLP || 16 * nt + v < n_produce ? w[leaf_weight_index(kappa, J * q + j, 16 * nt + v, C_in, n_produce, mirrored)] : 0.f;
    } else {
        for (int e = tid; e < 27 * C_in * C_out; e += kLeafThreads) {
            const int cout = e % C_out, ci = (e / C_out) % C_in, kappa = e / (C_out * C_in);
            wl[((kappa * 4 + ci / J) * C_out + cout) * J + ci % J] =
                FULLP || cout < n_produce ? w[leaf_weight_index(kappa, ci, cout, C_in, n_produce, mirrored)] : 0.f;
        }
    }
    if (wave < 2) {
        const int64_t first_index = t.leaf[0].offset;
        const int64_t total = kLeafFixedCost * t.n_leaf + n_voxels;
        const int b = blockIdx.x + wave;
        const int f = b >= (int)gridDim.x ? t.n_leaf
                                          : first_leaf_at_cost<kLeafFixedCost>(t, first_index, total * b / (int64_t)gridDim.x, lane);
        if (lane == 0) L.range[wave] = f;
    }
    __syncthreads();
    const int f_begin = L.range[0], f_end = L.range[1];
    if (wave == kLeafWaves - 1 && f_begin < f_end) stage_records(t, L, f_begin, lane);
    __syncthreads();

    for (int f = f_begin; f < f_end; ++f) {
        // ---- densify: row of every window cell, its channels into LDS (zeros where inactive)
        {
            if (tid < 512 / kVoxTile) L.tile_taps[tid] = 0;
            if (tid == 64) L.next_tile = 0;
            if (tid >= 128 && tid < 228) {       // activity bits of window row (x, y): z = 0 and 9 from the leaves beside
                int xy = tid - 128;
                asm volatile("" : "+v"(xy));
                const int x = xy / 10, y = xy % 10;
                const int s9 = ((x + 7) >> 3) * 9 + ((y + 7) >> 3) * 3, lx = (x - 1) & 7, sh = ((y - 1) & 7) * 8;
                L.act_row[xy] = (uint32_t)((L.mask[s9][lx] >> (sh + 7)) & 1) | (uint32_t)((L.mask[s9 + 1][lx] >> sh) & 0xff) << 1 |
                                (uint32_t)((L.mask[s9 + 2][lx] >> sh) & 1) << 9;
            }
            // loads of all passes are issued before the first is stored: an inactive cell reads row 0 and drops it
            f32x4 val[(kWinCells + kLeafThreads - 1) / kLeafThreads][J];
            bool on[(kWinCells + kLeafThreads - 1) / kLeafThreads];
#pragma unroll
            for (int it = 0; it < (kWinCells + kLeafThreads - 1) / kLeafThreads; ++it) {
                int cell = min(tid + it * kLeafThreads, kWinCells - 1);
                asm volatile("" : "+v"(cell));      // recompute the cell's addresses per leaf: registers are scarce
                const int x = cell / 100, y = (cell / 10) % 10, z = cell % 10;
                const int slot = ((x + 7) >> 3) * 9 + ((y + 7) >> 3) * 3 + ((z + 7) >> 3);
                const int row = staged_value(L, slot, (x - 1) & 7, (y - 1) & 7, (z - 1) & 7);
                on[it] = row >= 0;
                const f32x4* src = reinterpret_cast<const f32x4*>(feat + (int64_t)max(row, 0) * C_in);
#pragma unroll
                for (int c4 = 0; c4 < J; ++c4) val[it][c4] = src[c4];
            }
#pragma unroll
            for (int it = 0; it < (kWinCells + kLeafThreads - 1) / kLeafThreads; ++it) {
                const int cell = tid + it * kLeafThreads;
                if (cell < kWinCells) {
                    f32x4* dst = reinterpret_cast<f32x4*>(win + cell * C_in);
#pragma unroll
                    for (int c4 = 0; c4 < J; ++c4) dst[c4] = on[it] ? val[it][c4] : f32x4{0.f, 0.f, 0.f, 0.f};
                }
            }
        }
        __syncthreads();

        // ---- the leaf's active voxels in index order, and which taps each column tile needs
        const int n_act = (int)((L.prefix[13] >> 54) & 511) + __popcll(L.mask[13][7]);
        const int64_t base = L.offset[13];
        {
#pragma unroll
            for (int it = 0; it < 512 / kLeafThreads; ++it) {
                int m = tid + it * kLeafThreads;
                asm volatile("" : "+v"(m));
                const int lx = m >> 6, ly = (m >> 3) & 7, lz = m & 7;
                const int row = staged_value(L, 13, lx, ly, lz);
                if (row >= 0) {
                    const int r = row - (int)base;
                    const int cell = window_cell(lx + 1, ly + 1, lz + 1);
                    L.cell_of_rank[r] = (uint16_t)cell;
                    uint32_t taps = 0;       // three taps (dz = -1, 0, 1) per window row: bits lz .. lz + 2 of it
#pragma unroll
                    for (int ab = 0; ab < 9; ++ab)
                        taps |= ((L.act_row[(lx + ab / 3) * 10 + ly + ab % 3] >> lz) & 7u) << (3 * ab);
                    atomicOr(&L.tile_taps[r / kVoxTile], taps);
                }
            }
        }
        __syncthreads();

        if (wave == kLeafWaves - 1 && f + 1 < f_end) stage_records(t, L, f + 1, lane);
        {
            // ---- multiply: per column tile of 16 active voxels, the taps that tile needs.  The window
            // rows of nine taps are fetched together (any cell of the window may be read), then the
            // multiplies of the taps the tile needs are issued.
            const int n_tiles = (n_act + kVoxTile - 1) / kVoxTile;
            int claimed = uni(lane == 0 ? atomicAdd(&L.next_tile, 1) : 0);
            while (claimed < n_tiles) {
                const int tile = claimed;
                claimed = uni(lane == 0 ? atomicAdd(&L.next_tile, 1) : 0);     // in flight during this tile's multiplies
                const int r = tile * kVoxTile + v;
                const int cell = L.cell_of_rank[min(r, n_act - 1)];
                const float* fp = win + cell * C_in + J * q;
                const float* wp = wl + (q * C_out + v) * J;
                f32x4 acc[NT];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
                const uint32_t taps = (uint32_t)uni((int)L.tile_taps[tile]);
#pragma unroll
                for (int a = 0; a < 3; ++a) {
                    __builtin_amdgcn_sched_barrier(0);       // keeps the fetches of one plane of taps together
                    Floats<J> x[9];
#pragma unroll
                    for (int bc = 0; bc < 9; ++bc) x[bc] = lds_floats<J>(fp + tap_delta(a * 9 + bc) * C_in);
#pragma unroll
                    for (int bc = 0; bc < 9; ++bc) {
                        const int kappa = a * 9 + bc;
                        if (taps & (1u << kappa)) {
#pragma unroll
                            for (int nt = 0; nt < NT; ++nt) {
                                Floats<J> wv;
                                if (WREG) {
#pragma unroll
                                    for (int j = 0; j < J; ++j) wv.v[j] = wr[WREG ? kappa : 0][nt][j];
                                } else {
                                    wv = lds_floats<J>(wp + (kappa * 4 * C_out + 16 * nt) * J);
                                }
#pragma unroll
                                for (int j = 0; j < J; ++j)
                                    acc[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.v[j], x[bc].v[j], acc[nt], 0, 0, 0);
                            }
                        }
                    }
                }
                if (r < n_act) {
                    float* o = out + (base + r) * n_produce + 4 * q;      // n_produce is a multiple of 4
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        if (FULLP || 16 * nt + 4 * q < n_produce) *reinterpret_cast<f32x4*>(o + 16 * nt) = acc[nt];
                }
            }
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------------- weight gradient, fp32, low depth
// gw[kappa][ci][co] = sum over active voxels o with an active neighbour at tap kappa of
// feat[nb(o,kappa)][ci] * gout[o][co] (the derivative of the forward sum in the weights), from the same leaf
// window: the voxels are the contracted dimension of v_mfma_f32_16x16x4_f32, four per instruction.  Lane
// (v = l % 16, q = l / 16) supplies, for the q-th voxel of a quad, one window value as A (row v) and one gout
// value as B (column v = output channel).  The 16 rows hold 16 / C_in taps side by side (C_in = 8: two taps,
// C_in = 4: four), so the 27 taps take ceil(27 / taps-per-instruction) multiplies per quad and as many
// accumulator tiles, which a wave keeps in registers over all its leaves.  An inactive neighbour is a zero
// window cell and adds nothing.  Quads are dealt to the four waves round-robin and leaves to workgroups in
// fixed ranges; the waves' sums are added in wave order, the workgroups' partial sums in index order by the
// ordered reduction that the other weight-gradient kernels use: repeated calls give identical bits.
template <int C_IN> struct WgLeafShape {
    static constexpr int kTapsPer = C_IN <= 4 ? 4 : (C_IN <= 8 ? 2 : 1);
    static constexpr int kGroups = (27 + kTapsPer - 1) / kTapsPer;
    // waves per SIMD the register budget is set for: the accumulators take 4 * kGroups * NT registers
    static constexpr int waves_per_simd(int NT) { return 4 * kGroups * NT <= 32 ? 4 : (4 * kGroups * NT <= 64 ? 3 : 2); }
};

template <int C_IN, int NT>
__global__ __launch_bounds__(kLeafThreads, WgLeafShape<C_IN>::waves_per_simd(NT)) void k_wgrad_leaf(TreeView t, const float* __restrict__ feat,
                                                             const float* __restrict__ gout, int C_out, int co_base,
                                                             int64_t n_voxels, float* __restrict__ part) {
    // serves the output channels co_base .. co_base + 16 NT - 1 (those below C_out) of gout and of gw
    constexpr int J = C_IN / 4, TPI = WgLeafShape<C_IN>::kTapsPer, NG = WgLeafShape<C_IN>::kGroups;
    extern __shared__ __align__(16) unsigned char smem[];
    LeafLds& L = *reinterpret_cast<LeafLds*>(smem);
    float* win = reinterpret_cast<float*>(smem + ((sizeof(LeafLds) + 15) & ~size_t(15)));   // [cell][C_IN]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int v = lane & 15, q = lane >> 4;
    const int sub = v / C_IN, ci = v % C_IN;                 // the lane's tap within a group, its input channel
    const bool row_ok = v < TPI * C_IN;                      // C_IN = 12: rows 12..15 stay zero

    f32x4 acc[NG][NT];
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[g][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    if (wave < 2) {
        const int64_t first_index = t.leaf[0].offset;
        const int64_t total = kLeafFixedCost * t.n_leaf + n_voxels;
        const int b = blockIdx.x + wave;
        const int f = b >= (int)gridDim.x ? t.n_leaf
                                          : first_leaf_at_cost<kLeafFixedCost>(t, first_index, total * b / (int64_t)gridDim.x, lane);
        if (lane == 0) L.range[wave] = f;
    }
    __syncthreads();
    const int f_begin = L.range[0], f_end = L.range[1];
    if (wave == kLeafWaves - 1 && f_begin < f_end) stage_records(t, L, f_begin, lane);
    __syncthreads();

    for (int f = f_begin; f < f_end; ++f) {
        // ---- densify: as in k_conv_leaf
        {
            f32x4 val[(kWinCells + kLeafThreads - 1) / kLeafThreads][J];
            bool on[(kWinCells + kLeafThreads - 1) / kLeafThreads];
#pragma unroll
            for (int it = 0; it < (kWinCells + kLeafThreads - 1) / kLeafThreads; ++it) {
                int cell = min(tid + it * kLeafThreads, kWinCells - 1);
                asm volatile("" : "+v"(cell));
                const int x = cell / 100, y = (cell / 10) % 10, z = cell % 10;
                const int slot = ((x + 7) >> 3) * 9 + ((y + 7) >> 3) * 3 + ((z + 7) >> 3);
                const int row = staged_value(L, slot, (x - 1) & 7, (y - 1) & 7, (z - 1) & 7);
                on[it] = row >= 0;
                const f32x4* src = reinterpret_cast<const f32x4*>(feat + (int64_t)max(row, 0) * C_IN);
#pragma unroll
                for (int c4 = 0; c4 < J; ++c4) val[it][c4] = src[c4];
            }
#pragma unroll
            for (int it = 0; it < (kWinCells + kLeafThreads - 1) / kLeafThreads; ++it) {
                const int cell = tid + it * kLeafThreads;
                if (cell < kWinCells) {
                    f32x4* dst = reinterpret_cast<f32x4*>(win + cell * C_IN);
#pragma unroll
                    for (int c4 = 0; c4 < J; ++c4) dst[c4] = on[it] ? val[it][c4] : f32x4{0.f, 0.f, 0.f, 0.f};
                }
            }
            // the leaf's active voxels in index order (reads the centre record only)
#pragma unroll
            for (int it = 0; it < 512 / kLeafThreads; ++it) {
                int m = tid + it * kLeafThreads;
                asm volatile("" : "+v"(m));
                const int lx = m >> 6, ly = (m >> 3) & 7, lz = m & 7;
                const int row = staged_value(L, 13, lx, ly, lz);
                if (row >= 0) L.cell_of_rank[row - L.offset[13]] = (uint16_t)window_cell(lx + 1, ly + 1, lz + 1);
            }
        }
        const int n_act = uni((int)((L.prefix[13] >> 54) & 511) + __popcll(L.mask[13][7]));
        const int64_t base = uni(L.offset[13]);
        __syncthreads();

        if (wave == kLeafWaves - 1 && f + 1 < f_end) stage_records(t, L, f + 1, lane);
        {
            const int n_quads = (n_act + 3) >> 2;
            const float* gp = gout + base * C_out + co_base + v;
            // the next quad's cell and gout values are requested before the current quad's multiplies
            int cell_n = 0;
            float b_n[NT];
            auto fetch = [&](int qd) {
                const int r = qd * 4 + q;
                cell_n = L.cell_of_rank[min(r, n_act - 1)];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    b_n[nt] = (r < n_act && co_base + 16 * nt + v < C_out) ? gp[(int64_t)r * C_out + 16 * nt] : 0.f;
            };
            if (wave < n_quads) fetch(wave);
            for (int qd = wave; qd < n_quads; qd += kLeafWaves) {
                const float* fp = win + cell_n * C_IN + ci;
                float b[NT];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) b[nt] = b_n[nt];
                if (qd + kLeafWaves < n_quads) fetch(qd + kLeafWaves);
#pragma unroll
                for (int g = 0; g < NG; ++g) {
                    const int kappa = g * TPI + sub;                   // < 27 + TPI
                    const bool ok = row_ok && kappa < 27;
                    const float a = ok ? fp[tap_delta(min(kappa, 26)) * C_IN] : 0.f;
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        acc[g][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b[nt], acc[g][nt], 0, 0, 0);
                }
            }
        }
        __syncthreads();                 // the window and the records are rewritten for the next leaf
    }

    // ---- the four waves' sums, added in wave order through LDS (the window is free now)
    float* red = win;                    // [NG][NT][64 lanes][4]
    for (int w = 1; w < kLeafWaves; ++w) {
        if (wave == w) {
#pragma unroll
            for (int g = 0; g < NG; ++g)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) *reinterpret_cast<f32x4*>(red + ((g * NT + nt) * 64 + lane) * 4) = acc[g][nt];
        }
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int g = 0; g < NG; ++g)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const f32x4 o = *reinterpret_cast<const f32x4*>(red + ((g * NT + nt) * 64 + lane) * 4);
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[g][nt][e] += o[e];
                }
        }
        __syncthreads();
    }
    if (wave == 0) {
        // accumulator register e of lane (v, q) is row 4 q + e (tap sub-slot and input channel), column v
        float* dst = part + (int64_t)blockIdx.x * 27 * C_IN * C_out;
#pragma unroll
        for (int g = 0; g < NG; ++g)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int row = 4 * q + e;
                const int kappa = g * TPI + row / C_IN, c = row % C_IN;
                if (row < TPI * C_IN && kappa < 27) {
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        if (co_base + 16 * nt + v < C_out) dst[(kappa * C_IN + c) * C_out + co_base + 16 * nt + v] = acc[g][nt][e];
                }
            }
    }
}

template <int C_IN, int NT>
fx_status launch_wgrad_leaf(const fx_grid* g, const float* feat, const float* gout, int C_out, void* gw, fx_dtype out_dt,
                            hipStream_t st) {
    constexpr int NG = WgLeafShape<C_IN>::kGroups;
    static_assert((size_t)NG * NT * 64 * 4 <= (size_t)kWinCells * C_IN, "the waves' sums are exchanged through the window");
    const size_t lds = ((sizeof(LeafLds) + 15) & ~size_t(15)) + sizeof(float) * (size_t)kWinCells * C_IN;
    static int per_cu = 0;
    if (per_cu == 0) {
        FX_HIP_TRY(hipFuncSetAttribute((const void*)k_wgrad_leaf<C_IN, NT>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        int n = 0;
        FX_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k_wgrad_leaf<C_IN, NT>, kLeafThreads, lds));
        per_cu = std::max(1, n);
    }
    const int n_wg = (int)std::min<int64_t>(g->hdr.n_leaf, (int64_t)per_cu * compute_units());
    const int64_t total = (int64_t)27 * C_IN * C_out;
    float* part = nullptr;
    FX_TRY(dev_alloc((void**)&part, sizeof(float) * (size_t)total * n_wg, st));
    {
        // wider gradients than one launch's accumulators hold take one launch per 16 NT output channels; the
        // launches write disjoint columns of the same partial sums
        ProfScope ps(kProfWgrad, st);
        for (int co_base = 0; co_base < C_out; co_base += 16 * NT)
            k_wgrad_leaf<C_IN, NT><<<n_wg, kLeafThreads, lds, st>>>(g->view(), feat, gout, C_out, co_base, g->hdr.n_voxels, part);
    }
    fx_status rc = FX_OK;
    if (hipGetLastError() != hipSuccess) { set_error("leaf-window weight gradient: launch failed"); rc = FX_EDEVICE; }
    if (rc == FX_OK) rc = wgrad_reduce_ranges(part, n_wg, total, gw, out_dt, st);
    dev_free(part, st);
    return rc;
}

// ---------------------------------------------------------------------------------- 16-bit types, depth >= 32
// The same leaf window for f16 / bf16 at C_in % 32 == 0, C_out % 64 == 0: the regime of locally dense
// grids at moderate depth (Sec. 3.5 scenario 2 serves it with dense 4x2x2 bricks; here the window stays
// the leaf's, the columns are the leaf's ACTIVE voxels in tiles of 32, and taps a tile does not need
// are skipped).  The window holds one 32-channel chunk of every cell (64-byte rows, 16-byte pieces
// XOR-swizzled by (row >> 2) & 3 like the tile kernel's rows); a tap is an address offset, so neither
// row lists nor id blocks exist and a full leaf with all its neighbours needs 64 KB where the
// kernel-map tiles of a dense region exceed their LDS budget.  Each wave owns up to four column tiles
// (128 voxels x 64 output channels in 128 accumulator registers), fetches a tap's packed weights
// once for all of them (same packing as the tile kernel: features A, weights B, channels
// interleaved so that a half-wave stores whole output rows) and prefetches the next tap's.
constexpr int kLeaf16Threads = 256;
constexpr int kLeaf16Waves = kLeaf16Threads / 64;
constexpr int kLeaf16Groups = 4;             // column tiles of 32 voxels per wave: 4 waves x 4 x 32 = 512

constexpr int kWinSlabs = (kWinCells + 15) / 16;     // direct-to-LDS loads fill 16 rows (1 KB) per wave instruction
typedef __attribute__((address_space(3))) void* leaf_lds_ptr;

struct Leaf16Lds {
    uint64_t mask[27][8];
    uint64_t prefix[27];
    int32_t offset[27];
    uint32_t act_row[100];
    int32_t cell_row[kWinCells];             // input row of each window cell, -1 = inactive
    uint16_t cell_of_rank[512];
    uint32_t tile_taps[16];                  // per column tile of 32 voxels
    int32_t range[2];
    unsigned char win[kWinSlabs * 1024] __attribute__((aligned(16)));   // 64-byte rows, in slabs of 16
};

__device__ __forceinline__ uint32_t win_piece_offset(int row, int piece) {
    return (uint32_t)row * 64u + (uint32_t)((piece ^ ((row >> 2) & 3)) << 4);
}

template <typename T, bool OUT_F32>
__global__ __launch_bounds__(kLeaf16Threads, 2) void k_conv_leaf16(TreeView t, const unsigned char* __restrict__ feat,
                                                                  const unsigned char* __restrict__ wp,
                                                                  unsigned char* __restrict__ out, int C_in, int C_out,
                                                                  int32_t* __restrict__ work_counter,
                                                                  const unsigned char* __restrict__ zero_row,
                                                                  const int32_t* __restrict__ leaf_list,
                                                                  const int32_t* __restrict__ n_list) {
    typedef typename Elem<T>::vec8 vec8;
    extern __shared__ __align__(16) unsigned char smem[];
    Leaf16Lds& L = *reinterpret_cast<Leaf16Lds*>(smem);
    const int tid0 = threadIdx.x, wave = tid0 >> 6;
    const int nchunk = C_in / 32, nslice = C_out / 64;
    const int64_t pitch = (int64_t)C_in * 2;

    // Leaves are claimed one at a time from a counter in global memory, in index order: workgroups that run
    // together then work on neighbouring leaves (whose windows overlap, so their rows meet in L2), and the
    // tail is one leaf long.  The next claim is made while the current leaf is processed.
    // With a leaf list (per-leaf dispatch) the claimed numbers index the list: only those leaves are worked on.
    const int n_work = leaf_list ? uni(*n_list) : t.n_leaf;
    if (tid0 == 0) L.range[0] = atomicAdd(work_counter, 1);
    __syncthreads();
    int fi = uni(L.range[0]);
    int parity = 0;

    while (fi < n_work) {
        const int f = leaf_list ? uni(leaf_list[fi]) : fi;
        parity ^= 1;
        if (tid0 == 64) L.range[parity] = atomicAdd(work_counter, 1);    // by the second wave (the first walks the tree); read after this leaf's barriers
        // everything a thread derives from its number is recomputed per leaf (registers are needed
        // for the accumulators, not for loop-invariant addresses)
        int tid = tid0;
        asm volatile("" : "+v"(tid));
        const int lane = tid & 63, n = lane & 31, h = lane >> 5;
        // ---- the leaf's 27 records, then per cell its input row; activity bits per window row
        if (wave == 0) stage_records(t, L, f, lane);
        __syncthreads();
        if (tid < 16) L.tile_taps[tid] = 0;
        if (tid >= 128 && tid < 228) {
            const int xy = tid - 128;
            const int x = xy / 10, y = xy % 10;
            const int s9 = ((x + 7) >> 3) * 9 + ((y + 7) >> 3) * 3, lx = (x - 1) & 7, sh = ((y - 1) & 7) * 8;
            L.act_row[xy] = (uint32_t)((L.mask[s9][lx] >> (sh + 7)) & 1) | (uint32_t)((L.mask[s9 + 1][lx] >> sh) & 0xff) << 1 |
                            (uint32_t)((L.mask[s9 + 2][lx] >> sh) & 1) << 9;
        }
        for (int cell = tid; cell < kWinCells; cell += kLeaf16Threads) {
            const int x = cell / 100, y = (cell / 10) % 10, z = cell % 10;
            const int slot = ((x + 7) >> 3) * 9 + ((y + 7) >> 3) * 3 + ((z + 7) >> 3);
            L.cell_row[cell] = staged_value(L, slot, (x - 1) & 7, (y - 1) & 7, (z - 1) & 7);
        }
        __syncthreads();
        const int n_act = uni((int)((L.prefix[13] >> 54) & 511) + __popcll(L.mask[13][7]));
        const int64_t base = uni(L.offset[13]);
        for (int m = tid; m < 512; m += kLeaf16Threads) {
            const int lx = m >> 6, ly = (m >> 3) & 7, lz = m & 7;
            const int row = L.cell_row[window_cell(lx + 1, ly + 1, lz + 1)];
            if (row >= 0) {
                const int r = row - (int)base;
                L.cell_of_rank[r] = (uint16_t)window_cell(lx + 1, ly + 1, lz + 1);
                uint32_t taps = 0;
#pragma unroll
                for (int ab = 0; ab < 9; ++ab)
                    taps |= ((L.act_row[(lx + ab / 3) * 10 + ly + ab % 3] >> lz) & 7u) << (3 * ab);
                atomicOr(&L.tile_taps[r >> 5], taps);
            }
        }
        __syncthreads();

        // this wave's column tiles: tile gi * 4 + wave, voxel n of it in lanes n and n + 32
        const int n_tiles = (n_act + 31) >> 5;
        uint32_t gtaps[kLeaf16Groups];
        uint32_t gcell[kLeaf16Groups];          // byte offset of the voxel's own window row
        uint32_t wtaps = 0;
#pragma unroll
        for (int gi = 0; gi < kLeaf16Groups; ++gi) {
            const int tile = gi * kLeaf16Waves + wave;
            gtaps[gi] = (uint32_t)uni((int)(tile < n_tiles ? L.tile_taps[tile] : 0u));
            wtaps |= gtaps[gi];
            gcell[gi] = L.cell_of_rank[min(tile * 32 + n, n_act - 1)];
        }

        for (int s = 0; s < nslice; ++s) {
            f32x16 acc[kLeaf16Groups][2];
#pragma unroll
            for (int gi = 0; gi < kLeaf16Groups; ++gi)
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[gi][mt][v] = 0.f;
            for (int c = 0; c < nchunk; ++c) {
                // ---- densify chunk c: direct-to-LDS loads, one 1 KB slab of 16 rows per wave instruction; lane l
                // of a slab writes the 16 bytes at slab + 16 l, i.e. stored piece l & 3 of row l / 4, which is
                // piece (l & 3) ^ ((row >> 2) & 3) of the cell's chunk; inactive cells load from a zero row
                __syncthreads();                 // the previous multiply has finished with the window
                {
                    const int piece = (lane & 3) ^ ((lane >> 4) & 3);
                    // all row numbers first: a read of LDS after an asynchronous write to LDS has been issued
                    // would wait for that write
                    constexpr int kSlabsPerWave = (kWinSlabs + kLeaf16Waves - 1) / kLeaf16Waves;
                    int rows[kSlabsPerWave];
#pragma unroll
                    for (int j = 0; j < kSlabsPerWave; ++j) {
                        const int cell = 16 * (wave + j * kLeaf16Waves) + (lane >> 2);
                        rows[j] = cell < kWinCells ? L.cell_row[cell] : -1;
                    }
#pragma unroll
                    for (int j = 0; j < kSlabsPerWave; ++j) {
                        const int sl = wave + j * kLeaf16Waves;
                        if (sl < kWinSlabs) {
                            const unsigned char* src = rows[j] >= 0 ? feat + (int64_t)rows[j] * pitch + c * 64 + piece * 16
                                                                    : zero_row + piece * 16;
                            __builtin_amdgcn_global_load_lds(src, (leaf_lds_ptr)(L.win + sl * 1024), 16, 0, 0);
                        }
                    }
                    __builtin_amdgcn_s_waitcnt(0);
                }
                __syncthreads();

                // ---- multiply: the taps this wave's tiles need; the next tap's weights are in flight
                const unsigned char* wq = wp + ((int64_t)c * nslice + s) * 4096 + lane * 16;
                const int64_t wstep = (int64_t)nchunk * nslice * 4096;
                uint32_t taps = (uint32_t)uni((int)wtaps);
                if (taps) {
                    // one tap: request the weights of the tap after it into the other register set, fetch the
                    // four tiles' fragments of this tap from the window, multiply.  Two register sets take turns
                    // (the loop is unrolled by two), so a set is first touched a whole tap after its request.
                    auto fetch_w = [&](vec8 (&wset)[4], int k) {
#pragma unroll
                        for (int q4 = 0; q4 < 4; ++q4) wset[q4] = *reinterpret_cast<const vec8*>(wq + k * wstep + q4 * 1024);
                    };
                    auto tap = [&](const vec8 (&wcur)[4], vec8 (&wnext)[4], int kappa, int knext) {
                        fetch_w(wnext, knext);
                        const int d = tap_delta(kappa);
                        vec8 bf[kLeaf16Groups][2];
#pragma unroll
                        for (int gi = 0; gi < kLeaf16Groups; ++gi) {
                            const int row = (int)gcell[gi] + d;
                            const uint32_t a0 = win_piece_offset(row, h);
                            bf[gi][0] = *reinterpret_cast<const vec8*>(L.win + a0);
                            bf[gi][1] = *reinterpret_cast<const vec8*>(L.win + (a0 ^ 32u));
                        }
#pragma unroll
                        for (int gi = 0; gi < kLeaf16Groups; ++gi) {
                            if ((gtaps[gi] >> kappa) & 1u) {
#pragma unroll
                                for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                                    for (int mt = 0; mt < 2; ++mt)
                                        acc[gi][mt] = Elem<T>::mma(bf[gi][ks], wcur[mt * 2 + ks], acc[gi][mt]);
                            }
                        }
                    };
                    auto pop = [&]() { const int k = taps ? __builtin_ctz(taps) : -1; taps &= taps - 1; return k; };
                    vec8 wa[4], wb[4];
                    int k0 = pop(), k1 = pop();
                    fetch_w(wa, k0);
                    while (true) {
                        tap(wa, wb, k0, k1 >= 0 ? k1 : k0);
                        if (k1 < 0) break;
                        k0 = pop();
                        tap(wb, wa, k1, k0 >= 0 ? k0 : k1);
                        if (k0 < 0) break;
                        k1 = pop();
                    }
                }
            }
            // ---- write-back: register v of tile mt in lane (n, h) is channel 64 s + 2 n + mt of the
            // tile's voxel 8 (v / 4) + 4 h + v % 4; the leaf's outputs are consecutive rows
            const uint32_t esize = OUT_F32 ? 4u : 2u;
            int lane_w = lane;
            asm volatile("" : "+v"(lane_w));      // offsets and bounds of the stores are computed here, per slice
            const int n_w = lane_w & 31, h_w = lane_w >> 5;
            const uint32_t row_bytes = (uint32_t)C_out * esize, lane_off = 2u * (uint32_t)n_w * esize;
            // wave-uniform 64-bit base, 32-bit lane offsets: the stores take the base as their scalar operand
            const uint64_t bits = reinterpret_cast<uint64_t>(out) + (uint64_t)((base * C_out + 64 * s) * (int64_t)esize);
            typedef __attribute__((address_space(1))) unsigned char gbyte;
            gbyte* ob = (gbyte*)(((uint64_t)(uint32_t)uni((int)(uint32_t)(bits >> 32)) << 32) | (uint32_t)uni((int)(uint32_t)bits));
#pragma unroll
            for (int gi = 0; gi < kLeaf16Groups; ++gi) {
                const int tile = gi * kLeaf16Waves + wave;
                if (tile >= n_tiles) continue;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int r = tile * 32 + 8 * (v >> 2) + 4 * h_w + (v & 3);
                    if (r >= n_act) continue;
                    gbyte* dst = ob + ((uint32_t)r * row_bytes + lane_off);
                    if (OUT_F32) *reinterpret_cast<__attribute__((address_space(1))) f32x2*>(dst) = f32x2{acc[gi][0][v], acc[gi][1][v]};
                    else *reinterpret_cast<__attribute__((address_space(1))) uint32_t*>(dst) = Elem<T>::pack2(acc[gi][0][v], acc[gi][1][v]);
                }
            }
        }
        __syncthreads();                         // records and lists are rewritten for the next leaf
        fi = uni(L.range[parity]);
    }
}

template <typename T, bool OUT_F32>
fx_status launch_leaf16(const fx_grid* g, const void* feat, const void* wpacked, void* out, int C_in, int C_out,
                        void* work_counter, const void* zero_row, const int32_t* leaf_list, const int32_t* n_list, hipStream_t st) {
    const size_t lds = sizeof(Leaf16Lds);
    static int per_cu = 0;
    if (per_cu == 0) {
        FX_HIP_TRY(hipFuncSetAttribute((const void*)k_conv_leaf16<T, OUT_F32>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)lds));
        int nb = 0;
        FX_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, k_conv_leaf16<T, OUT_F32>, kLeaf16Threads, lds));
        per_cu = std::max(1, nb);
    }
    const unsigned n_wg = (unsigned)std::min<int64_t>(g->hdr.n_leaf, (int64_t)per_cu * compute_units());
    ProfScope ps(kProfConvLeaf, st);
    k_conv_leaf16<T, OUT_F32><<<n_wg, kLeaf16Threads, lds, st>>>(g->view(), (const unsigned char*)feat,
                                                                 (const unsigned char*)wpacked, (unsigned char*)out, C_in,
                                                                 C_out, (int32_t*)work_counter, (const unsigned char*)zero_row, leaf_list, n_list);
    FX_HIP_TRY(hipGetLastError());
    return FX_OK;
}

// ---------------------------------------------------------------------------------- weight gradient, 16-bit types, depth >= 32
// gw[kappa][ci][co] = sum over the active voxels o with an active neighbour at tap kappa of
// feat[nb(o, kappa)][ci] * gout[o][co], leaf by leaf from the same window as k_conv_leaf16: no kernel map, a tap is an
// address offset.  A workgroup owns a block of 32 input x 64 output channels of every gw[kappa] and a range of leaves
// of equal estimated cost; its 8 waves split the taps (wave w: kappa = w, w + 8, w + 16 and, for w < 3, w + 24) and keep
// their accumulator tiles over the whole range (128 registers; two waves per SIMD).  Measured with 4, 12 and 16
// waves as well: 408, 329 and 335 us on a dense 96^3 grid against 298 -- fewer waves read every gout fragment for
// more taps, but one wave per SIMD no longer covers its own waits.  Per leaf it stages the window (one 32-channel chunk of every cell, inactive cells
// zero) and the gout rows of the leaf's active voxels (consecutive rows of the tensor; 128 bytes per voxel, 16-byte
// pieces swizzled by the voxel's rank), both straight from global memory to LDS.  The voxels are the contracted
// dimension, so both operands are read with the transposing LDS read (tr_read4): per column tile of 32 voxels a wave
// reads the gout fragments once for its taps and, per tap, the window rows of the voxels' neighbours.
// A (tile, tap) in which no voxel has that neighbour is skipped; ranks past the leaf's last voxel contribute
// zeros on both sides.  Partial sums go to part[range][kappa][ci][co]; the ordered reduction adds the ranges.
constexpr int kWg16Waves = 8;
constexpr int kWg16Threads = 64 * kWg16Waves;
constexpr int kWg16Offsets = (27 + kWg16Waves - 1) / kWg16Waves;
constexpr int kWg16GoutRow = 128;            // 64 output channels of a 16-bit type

struct Wg16Lds {
    uint64_t mask[27][8];
    uint64_t prefix[27];
    int32_t offset[27];
    uint32_t act_row[100];
    int32_t cell_row[kWinCells];
    uint16_t cell_of_rank[512];
    uint32_t tile_taps[16];                  // per column tile of 32 voxels
    int32_t range[2];
    unsigned char win[kWinSlabs * 1024] __attribute__((aligned(16)));   // 64-byte rows, in slabs of 16, as in k_conv_leaf16
    unsigned char gt[512 * kWg16GoutRow] __attribute__((aligned(16)));  // gout row of rank r at r * 128, piece p at p ^ 4 * ((r >> 1) & 1)
};
static_assert(sizeof(Wg16Lds) <= 160 * 1024, "LDS budget of one compute unit");

template <typename T>
__global__ __launch_bounds__(kWg16Threads, 1) void k_wgrad_leaf16(TreeView t, const uint16_t* __restrict__ feat,
                                                                  const uint16_t* __restrict__ gout, int C_in, int C_out,
                                                                  int n_ranges, int64_t n_voxels, float* __restrict__ part,
                                                                  const int32_t* __restrict__ leaf_list,
                                                                  const int32_t* __restrict__ n_list) {
    typedef typename Elem<T>::vec8 vec8;
    extern __shared__ __align__(16) unsigned char smem[];
    Wg16Lds& L = *reinterpret_cast<Wg16Lds*>(smem);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, h = lane >> 5;
    const int n_cib = C_in / 32, n_cblk = n_cib * (C_out / 64);
    // workgroup b runs on XCD b % 8: the channel blocks of one range of leaves share an XCD and its L2
    int blk = blockIdx.x % n_cblk, range = blockIdx.x / n_cblk;
    if (n_ranges % 8 == 0) {
        blk = (blockIdx.x >> 3) % n_cblk;
        range = (int)(blockIdx.x / (8 * n_cblk)) * 8 + (blockIdx.x & 7);
    }
    const int cib = blk % n_cib, cob = blk / n_cib;

    // With a leaf list (per-leaf dispatch: the locally dense leaves of a mixed grid) the ranges are equal shares of the
    // list and the numbers below index it; without one they are ranges of leaves of equal estimated cost.
    if (wave < 2) {
        const int b = range + wave;
        int f;
        if (leaf_list) {
            f = (int)((int64_t)uni(*n_list) * min(b, n_ranges) / n_ranges);
        } else {
            const int64_t first_index = t.leaf[0].offset;
            const int64_t total = kLeafFixedCost * t.n_leaf + n_voxels;
            f = b >= n_ranges ? t.n_leaf : first_leaf_at_cost<kLeafFixedCost>(t, first_index, total * b / (int64_t)n_ranges, lane);
        }
        if (lane == 0) L.range[wave] = f;
    }
    __syncthreads();
    const int f_begin = uni(L.range[0]), f_end = uni(L.range[1]);
    auto leaf_of = [&](int i) { return leaf_list ? uni(leaf_list[i]) : i; };

    f32x16 acc[kWg16Offsets][2];
#pragma unroll
    for (int j = 0; j < kWg16Offsets; ++j)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][cb][v] = 0.f;

    // what this lane's address contributes to a transposing read: voxel jv of four, channels 16*g1 + 4*q .. + 3
    const int q = lane & 3, jv = (lane >> 2) & 3, g1 = (lane >> 4) & 1;
    const int a_piece = 2 * g1 + (q >> 1);
    const uint32_t half8 = (uint32_t)(q & 1) << 3;

    if (wave == kWg16Waves - 1 && f_begin < f_end) stage_records(t, L, leaf_of(f_begin), lane);
    __syncthreads();
    for (int f = f_begin; f < f_end; ++f) {
        // ---- from the leaf's 27 records (fetched while the leaf before was multiplied): per cell its input row,
        // activity bits per window row (as in k_conv_leaf16)
        if (tid < 16) L.tile_taps[tid] = 0;
        if (tid >= 128 && tid < 228) {
            const int xy = tid - 128;
            const int x = xy / 10, y = xy % 10;
            const int s9 = ((x + 7) >> 3) * 9 + ((y + 7) >> 3) * 3, lx = (x - 1) & 7, sh = ((y - 1) & 7) * 8;
            L.act_row[xy] = (uint32_t)((L.mask[s9][lx] >> (sh + 7)) & 1) | (uint32_t)((L.mask[s9 + 1][lx] >> sh) & 0xff) << 1 |
                            (uint32_t)((L.mask[s9 + 2][lx] >> sh) & 1) << 9;
        }
        for (int cell = tid; cell < kWinCells; cell += kWg16Threads) {
            const int x = cell / 100, y = (cell / 10) % 10, z = cell % 10;
            const int slot = ((x + 7) >> 3) * 9 + ((y + 7) >> 3) * 3 + ((z + 7) >> 3);
            L.cell_row[cell] = staged_value(L, slot, (x - 1) & 7, (y - 1) & 7, (z - 1) & 7);
        }
        __syncthreads();
        const int n_act = uni((int)((L.prefix[13] >> 54) & 511) + __popcll(L.mask[13][7]));
        const int64_t base = uni(L.offset[13]);
        for (int m = tid; m < 512; m += kWg16Threads) {
            const int lx = m >> 6, ly = (m >> 3) & 7, lz = m & 7;
            const int row = L.cell_row[window_cell(lx + 1, ly + 1, lz + 1)];
            if (row >= 0) {
                const int r = row - (int)base;
                L.cell_of_rank[r] = (uint16_t)window_cell(lx + 1, ly + 1, lz + 1);
                uint32_t taps = 0;
#pragma unroll
                for (int ab = 0; ab < 9; ++ab)
                    taps |= ((L.act_row[(lx + ab / 3) * 10 + ly + ab % 3] >> lz) & 7u) << (3 * ab);
                atomicOr(&L.tile_taps[r >> 5], taps);
            }
        }
        __syncthreads();

        // ---- stage the window (chunk cib of every cell) and the gout rows of the leaf's voxels.  All reads of LDS
        // and all plain stores come before the first asynchronous load is issued.
        {
            constexpr int kSlabsPerWave = (kWinSlabs + kWg16Waves - 1) / kWg16Waves;
            constexpr int kGoutSlabs = 512 * kWg16GoutRow / 1024, kGoutSlabsPerWave = (kGoutSlabs + kWg16Waves - 1) / kWg16Waves;
            int rows[kSlabsPerWave];
#pragma unroll
            for (int j = 0; j < kSlabsPerWave; ++j) {
                const int sl = wave + j * kWg16Waves, cell = 16 * sl + (lane >> 2);
                rows[j] = (sl < kWinSlabs && cell < kWinCells) ? L.cell_row[cell] : -1;
            }
#pragma unroll
            for (int j = 0; j < kSlabsPerWave; ++j) {
                const int sl = wave + j * kWg16Waves;
                if (sl < kWinSlabs && rows[j] < 0) *reinterpret_cast<u32x4*>(L.win + sl * 1024 + lane * 16) = u32x4{0, 0, 0, 0};
            }
#pragma unroll
            for (int j = 0; j < kGoutSlabsPerWave; ++j) {
                const int slab = wave + j * kWg16Waves, r = 8 * slab + (lane >> 3);
                if (slab < kGoutSlabs && r >= n_act) *reinterpret_cast<u32x4*>(L.gt + slab * 1024 + lane * 16) = u32x4{0, 0, 0, 0};
            }
            const int piece = (lane & 3) ^ ((lane >> 4) & 3);
#pragma unroll
            for (int j = 0; j < kSlabsPerWave; ++j) {
                const int sl = wave + j * kWg16Waves;
                if (sl < kWinSlabs && rows[j] >= 0)
                    __builtin_amdgcn_global_load_lds(feat + (int64_t)rows[j] * C_in + cib * 32 + piece * 8, (leaf_lds_ptr)(L.win + sl * 1024), 16, 0, 0);
            }
#pragma unroll
            for (int j = 0; j < kGoutSlabsPerWave; ++j) {
                const int slab = wave + j * kWg16Waves, r = 8 * slab + (lane >> 3);
                const int gpiece = (lane & 7) ^ (((r >> 1) & 1) << 2);
                if (slab < kGoutSlabs && r < n_act)
                    __builtin_amdgcn_global_load_lds(gout + (base + r) * (int64_t)C_out + cob * 64 + gpiece * 8, (leaf_lds_ptr)(L.gt + slab * 1024), 16, 0, 0);
            }
            __builtin_amdgcn_s_waitcnt(0);
        }
        __syncthreads();

        // ---- multiply; the last wave (three taps, not four) first walks the tree for the next leaf's records, which nobody reads meanwhile
        if (wave == kWg16Waves - 1 && f + 1 < f_end) stage_records(t, L, leaf_of(f + 1), lane);
        const int n_tiles = (n_act + 31) >> 5;
        for (int g = 0; g < n_tiles; ++g) {
            const uint32_t taps = (uint32_t)uni((int)L.tile_taps[g]);
            bool on[kWg16Offsets];
            bool any = false;
#pragma unroll
            for (int j = 0; j < kWg16Offsets; ++j) {
                const int kappa = wave + kWg16Waves * j;
                on[j] = kappa < 27 && ((taps >> kappa) & 1u);
                any = any || on[j];
            }
            if (!any) continue;
            // the voxels whose rows this lane's addresses contribute: ranks 32g + 16ks + 8h + 4tt + jv
            int cell[2][2];
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int tt = 0; tt < 2; ++tt) cell[ks][tt] = L.cell_of_rank[min(32 * g + 16 * ks + 8 * h + 4 * tt + jv, n_act - 1)];
            vec8 bfr[2][2];
#pragma unroll
            for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
                    const int r = 32 * g + 16 * ks + 8 * h + jv;
                    const uint32_t pos = (uint32_t)((4 * cb + 2 * g1 + (q >> 1)) ^ (((r >> 1) & 1) << 2)) << 4;
                    const unsigned char* src = L.gt + r * kWg16GoutRow + pos + half8;
                    const u32x2 lo = tr_read4(src);
                    const u32x2 hi = tr_read4(src + 4 * kWg16GoutRow);
                    bfr[cb][ks] = vec8_from_words<T>(u32x4{lo[0], lo[1], hi[0], hi[1]});
                }
            const bool tail = 32 * g + 32 > n_act;       // ranks past the last voxel: their A elements are cleared too
#pragma unroll
            for (int j = 0; j < kWg16Offsets; ++j) {
                if (!on[j]) continue;
                const int d = tap_delta(wave + kWg16Waves * j);
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
                    u32x2 w[2];
#pragma unroll
                    for (int tt = 0; tt < 2; ++tt) {
                        w[tt] = tr_read4(L.win + win_piece_offset(cell[ks][tt] + d, a_piece) + half8);
                        if (tail) {      // element e of this read is the voxel of rank 32g + 16ks + 8h + 4tt + e
                            const int left = n_act - (32 * g + 16 * ks + 8 * h + 4 * tt);
                            w[tt][0] &= left >= 2 ? 0xFFFFFFFFu : (left == 1 ? 0x0000FFFFu : 0u);
                            w[tt][1] &= left >= 4 ? 0xFFFFFFFFu : (left == 3 ? 0x0000FFFFu : 0u);
                        }
                    }
                    const vec8 fT = vec8_from_words<T>(u32x4{w[0][0], w[0][1], w[1][0], w[1][1]});
#pragma unroll
                    for (int cb = 0; cb < 2; ++cb) acc[j][cb] = Elem<T>::mfma(fT, bfr[cb][ks], acc[j][cb]);
                }
            }
        }
        __syncthreads();                 // window, gout rows and records are rewritten for the next leaf
    }

    // ---- partial sums of this range: lane (co = n, h), register 4b + r  ->  ci = 8b + 4h + r
#pragma unroll
    for (int j = 0; j < kWg16Offsets; ++j) {
        const int kappa = wave + kWg16Waves * j;
        if (kappa >= 27) continue;
        float* dst = part + (((int64_t)range * 27 + kappa) * C_in + cib * 32) * C_out + cob * 64 + n;
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int v = 0; v < 16; ++v) dst[(int64_t)(8 * (v >> 2) + 4 * h + (v & 3)) * C_out + cb * 32] = acc[j][cb][v];
    }
}

// ranges (= partial sums) of the 16-bit leaf-window weight gradient on grid g
int wgrad_leaf16_ranges(const fx_grid* g, int C_in, int C_out) {
    const int n_cblk = (C_in / 32) * (C_out / 64);
    int n_ranges = (int)std::max<int64_t>(1, std::min<int64_t>(g->hdr.n_leaf, compute_units() / std::max(1, n_cblk)));
    if (n_ranges > 8) n_ranges -= n_ranges % 8;   // see the block-to-XCD mapping in the kernel
    return n_ranges;
}

template <typename T>
fx_status launch_wgrad_leaf16(const fx_grid* g, const void* feat, const void* gout, int C_in, int C_out, const int32_t* leaf_list,
                              const int32_t* n_list, float* part, int n_ranges, hipStream_t st) {
    const size_t lds = sizeof(Wg16Lds);
    static bool attr_set = false;
    if (!attr_set) {
        FX_HIP_TRY(hipFuncSetAttribute((const void*)k_wgrad_leaf16<T>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        attr_set = true;
    }
    const int n_cblk = (C_in / 32) * (C_out / 64);
    ProfScope ps(kProfWgrad, st);
    k_wgrad_leaf16<T><<<(unsigned)(n_cblk * n_ranges), kWg16Threads, lds, st>>>(g->view(), (const uint16_t*)feat, (const uint16_t*)gout,
                                                                                C_in, C_out, n_ranges, g->hdr.n_voxels, part, leaf_list, n_list);
    if (hipGetLastError() != hipSuccess) { set_error("leaf-window weight gradient: launch failed"); return FX_EDEVICE; }
    return FX_OK;
}

}  // namespace

int leaf_wgrad16_ranges(const fx_grid* g, int C_in, int C_out) { return wgrad_leaf16_ranges(g, C_in, C_out); }

fx_status leaf_wgrad16_partial(const fx_grid* g, const void* d_feat, const void* d_gout, fx_dtype dt, int32_t C_in, int32_t C_out,
                               const int32_t* leaf_list, const int32_t* n_list, float* part, int n_ranges, hipStream_t st) {
    if (dt == FX_BF16) return launch_wgrad_leaf16<__bf16>(g, d_feat, d_gout, C_in, C_out, leaf_list, n_list, part, n_ranges, st);
    return launch_wgrad_leaf16<_Float16>(g, d_feat, d_gout, C_in, C_out, leaf_list, n_list, part, n_ranges, st);
}

namespace {

constexpr bool leaf_weights_in_registers(int J, int NT) { return 27 * J * NT <= 64; }

size_t leaf_lds_bytes(int J, int NT) {
    const int C_in = 4 * J, C_out = 16 * NT;
    return ((sizeof(LeafLds) + 15) & ~size_t(15)) +
           sizeof(float) * ((size_t)kWinCells * C_in + (leaf_weights_in_registers(J, NT) ? 0 : (size_t)27 * C_in * C_out));
}

template <int J, int NT, bool FULLP>
fx_status launch_leaf_full(const fx_grid* g, const float* feat, const float* w, float* out, int mirrored, int n_produce,
                           hipStream_t st) {
    constexpr bool WREG = leaf_weights_in_registers(J, NT);
    const size_t lds = leaf_lds_bytes(J, NT);
    static int per_cu = 0;                    // resident workgroups per compute unit (registers, LDS, wave slots)
    if (per_cu == 0) {
        FX_HIP_TRY(hipFuncSetAttribute((const void*)k_conv_leaf<J, NT, WREG, FULLP>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)lds));
        int n = 0;
        FX_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k_conv_leaf<J, NT, WREG, FULLP>, kLeafThreads, lds));
        per_cu = std::max(1, n);
    }
    const unsigned n_wg = (unsigned)std::min<int64_t>(g->hdr.n_leaf, (int64_t)per_cu * compute_units());
    ProfScope ps(kProfConvLeaf, st);
    k_conv_leaf<J, NT, WREG, FULLP><<<n_wg, kLeafThreads, lds, st>>>(g->view(), feat, w, out, g->hdr.n_voxels, mirrored, n_produce);
    FX_HIP_TRY(hipGetLastError());
    return FX_OK;
}

template <int J, int NT>
fx_status launch_leaf(const fx_grid* g, const float* feat, const float* w, float* out, int mirrored, int n_produce,
                      hipStream_t st) {
    return n_produce == 16 * NT ? launch_leaf_full<J, NT, true>(g, feat, w, out, mirrored, n_produce, st)
                                : launch_leaf_full<J, NT, false>(g, feat, w, out, mirrored, n_produce, st);
}

}  // namespace
}  // namespace fx

using namespace fx;


// The leaf-window convolution of `src` [N, C_contract] into `dst` [N, C_produce]; `mode` says how the
// caller's weights are read (kWeightsForward, or kWeightsMirrored for the input gradient).
fx_status fx::leaf_apply(const char* who, const fx_grid* g, const void* d_src, fx_dtype dt, const void* d_w,
                            int32_t C_contract, int32_t C_produce, void* d_dst, fx_dtype out_dt, hipStream_t st, int mode,
                            const int32_t* leaf_list, const int32_t* n_list) {
    if (!g || !d_w || C_contract < 1 || C_produce < 1 || (g->hdr.n_voxels > 0 && (!d_src || !d_dst))) {
        set_error("%s: null pointer or non-positive channel count", who);
        return FX_EINVAL;
    }
    if (dt != FX_F32 && dt != FX_F16 && dt != FX_BF16) { set_error("unknown input dtype"); return FX_EINVAL; }
    if (out_dt != dt && out_dt != FX_F32) {
        set_error("output dtype must equal the input dtype or be fp32");
        return FX_EUNSUPPORTED;
    }
    if (dt != FX_F32) {
        if (C_contract % 32 || C_produce % 64) {
            set_error("%s: 16-bit types need a multiple of 32 contracted and of 64 produced channels (got %d -> %d); "
                      "use the kernel-map path", who, C_contract, C_produce);
            return FX_EUNSUPPORTED;
        }
        if (g->hdr.n_voxels == 0) return FX_OK;
        void* wpk = nullptr;
        const size_t wbytes = packed_weight_bytes(27, C_contract, C_produce, 2);
        // behind the packed weights: 32 bytes that the memset and the packing kernel clear (the first four are the
        // leaf kernel's work counter), then a 64-byte row of zeros
        FX_TRY(dev_alloc(&wpk, wbytes + 96, st));
        const void* zero_row = (const char*)wpk + wbytes + 32;
        if (hipMemsetAsync((char*)wpk + wbytes, 0, 96, st) != hipSuccess) {
            dev_free(wpk, st);
            set_error("%s: memset failed", who);
            return FX_EDEVICE;
        }
        launch_pack_weights(d_w, wpk, 27, C_contract, C_produce, 2, reinterpret_cast<int32_t*>((char*)wpk + wbytes), mode, st);
        fx_status rc;
        if (dt == FX_BF16)
            rc = out_dt == FX_F32 ? launch_leaf16<__bf16, true>(g, d_src, wpk, d_dst, C_contract, C_produce, (char*)wpk + wbytes, zero_row, leaf_list, n_list, st)
                                  : launch_leaf16<__bf16, false>(g, d_src, wpk, d_dst, C_contract, C_produce, (char*)wpk + wbytes, zero_row, leaf_list, n_list, st);
        else
            rc = out_dt == FX_F32 ? launch_leaf16<_Float16, true>(g, d_src, wpk, d_dst, C_contract, C_produce, (char*)wpk + wbytes, zero_row, leaf_list, n_list, st)
                                  : launch_leaf16<_Float16, false>(g, d_src, wpk, d_dst, C_contract, C_produce, (char*)wpk + wbytes, zero_row, leaf_list, n_list, st);
        dev_free(wpk, st);
        return rc;
    }
    if (!leaf_shape_supported(dt, C_contract, C_produce)) {
        set_error("%s: fp32 needs 4, 8, 12 or 16 contracted and a multiple of 4 up to 32 produced channels (got %d -> %d); "
                  "use the kernel-map path", who, C_contract, C_produce);
        return FX_EUNSUPPORTED;
    }
    if (g->hdr.n_voxels == 0) return FX_OK;
    const float* src = (const float*)d_src;
    const float* w = (const float*)d_w;
    float* dst = (float*)d_dst;
    const int mirrored = mode == kWeightsMirrored;
#define FX_LEAF(JV)                                                                                  \
    case JV:                                                                                         \
        return C_produce <= 16 ? launch_leaf<JV, 1>(g, src, w, dst, mirrored, C_produce, st)                \
                               : launch_leaf<JV, 2>(g, src, w, dst, mirrored, C_produce, st)
    switch (C_contract / 4) {
        FX_LEAF(1);
        FX_LEAF(2);
        FX_LEAF(3);
        FX_LEAF(4);
    }
#undef FX_LEAF
    return FX_EINVAL;
}

fx_status fx::leaf_wgrad(const char* who, const fx_grid* g, const void* d_feat, const void* d_gout, fx_dtype dt, int32_t C_in,
                         int32_t C_out, void* d_gw, fx_dtype out_dt, hipStream_t st) {
    if (!g || !d_gw || C_in < 1 || C_out < 1 || (g->hdr.n_voxels > 0 && (!d_feat || !d_gout))) {
        set_error("%s: null pointer or non-positive channel count", who);
        return FX_EINVAL;
    }
    if (dt != FX_F32 && dt != FX_F16 && dt != FX_BF16) { set_error("unknown input dtype"); return FX_EINVAL; }
    if (out_dt != dt && out_dt != FX_F32) {
        set_error("output dtype must equal the input dtype or be fp32");
        return FX_EUNSUPPORTED;
    }
    if (!leaf_wgrad_shape_supported(dt, C_in, C_out)) {
        set_error("%s: serves fp32 with 4, 8, 12 or 16 input channels and a multiple of 4 up to 32 output channels, f16 / bf16 "
                  "with a multiple of 32 input and of 64 output channels (got %d -> %d); use the kernel-map path", who, C_in, C_out);
        return FX_EUNSUPPORTED;
    }
    const float* x = (const float*)d_feat;
    const float* gy = (const float*)d_gout;
    if (g->hdr.n_voxels == 0) return wgrad_reduce_ranges(nullptr, 0, (int64_t)27 * C_in * C_out, d_gw, out_dt, st);
    if (dt != FX_F32) {
        const int n_ranges = leaf_wgrad16_ranges(g, C_in, C_out);
        const int64_t total = (int64_t)27 * C_in * C_out;
        float* part = nullptr;
        FX_TRY(dev_alloc((void**)&part, sizeof(float) * (size_t)total * n_ranges, st));
        fx_status rc = leaf_wgrad16_partial(g, d_feat, d_gout, dt, C_in, C_out, nullptr, nullptr, part, n_ranges, st);
        if (rc == FX_OK) rc = wgrad_reduce_ranges(part, n_ranges, total, d_gw, out_dt, st);
        dev_free(part, st);
        return rc;
    }
    const bool wide = C_out > 16;
    switch (C_in) {
        case 4: return wide ? launch_wgrad_leaf<4, 2>(g, x, gy, C_out, d_gw, out_dt, st) : launch_wgrad_leaf<4, 1>(g, x, gy, C_out, d_gw, out_dt, st);
        case 8: return wide ? launch_wgrad_leaf<8, 2>(g, x, gy, C_out, d_gw, out_dt, st) : launch_wgrad_leaf<8, 1>(g, x, gy, C_out, d_gw, out_dt, st);
        case 12: return launch_wgrad_leaf<12, 1>(g, x, gy, C_out, d_gw, out_dt, st);
        case 16: return launch_wgrad_leaf<16, 1>(g, x, gy, C_out, d_gw, out_dt, st);
    }
    return FX_EINVAL;
}

extern "C" fx_status fx_sparse_conv_leaf_bwd_weight(const fx_grid* g, const void* d_feat, const void* d_gout, fx_dtype dt,
                                                    int32_t C_in, int32_t C_out, void* d_gw, fx_dtype out_dt, void* stream) {
    return leaf_wgrad("fx_sparse_conv_leaf_bwd_weight", g, d_feat, d_gout, dt, C_in, C_out, d_gw, out_dt, (hipStream_t)stream);
}

extern "C" fx_status fx_sparse_conv_leaf_fwd(const fx_grid* g, const void* d_feat, fx_dtype dt, const void* d_w,
                                             int32_t C_in, int32_t C_out, void* d_out, fx_dtype out_dt, void* stream) {
    return leaf_apply("fx_sparse_conv_leaf_fwd", g, d_feat, dt, d_w, C_in, C_out, d_out, out_dt, (hipStream_t)stream,
                      kWeightsForward);
}

extern "C" fx_status fx_sparse_conv_leaf_bwd_data(const fx_grid* g, const void* d_gout, fx_dtype dt, const void* d_w,
                                                  int32_t C_in, int32_t C_out, void* d_gin, fx_dtype out_dt, void* stream) {
    return leaf_apply("fx_sparse_conv_leaf_bwd_data", g, d_gout, dt, d_w, C_out, C_in, d_gin, out_dt, (hipStream_t)stream,
                      kWeightsMirrored);
}
