// Backward pass of the sparse convolution (Sec. 3.6 / 3.6.2: differentiable operators; Sec. 4.1.3
// names the gradient with respect to the filter coefficients).  The paper gives no formula; these
// are the derivatives of  out[o,:] = sum_kappa feat[map(o,kappa),:] . W[kappa]:
//
//   input gradient    gin[i,:]      = sum over pairs (o,kappa) with map(o,kappa) = i of W[kappa] . gout[o,:]
//   weight gradient   gw[kappa,:,:] = sum over o with map(o,kappa) >= 0 of feat[map(o,kappa),:]^T gout[o,:]
//
// Input gradient: a submanifold map is symmetric (map(o,kappa) = i  <=>  map(i,K^3-1-kappa) = o), so
// the forward kernels run unchanged on gout with the offsets mirrored and every W[kappa] transposed
// (conv_apply, kWeightsMirrored).  On a K = stride map no two outputs share an input: one wave per
// column block multiplies the block's gout rows with each W[kappa]^T and stores the product rows
// straight to the inputs the map names (k_dgrad_strided).
//
// Weight gradient: a contraction over voxels, so both MFMA operands must hold 8 consecutive
// *voxels* per lane while the rows in memory hold consecutive *channels*.  Both operands are staged
// in LDS as rows and read with the transposing LDS read of this hardware (ds_read_b64_tr_b16: four
// lanes that each address four channels of a different voxel's row receive four voxels of one
// channel each), see k_wgrad_mfma.
#include "conv_common.h"

namespace fx {

// ---------------------------------------------------------------------------------- helpers
// bit pattern of 1.0 in the storage type
template <typename T> __device__ __forceinline__ uint16_t one_bits();
template <> __device__ __forceinline__ uint16_t one_bits<__bf16>() { return 0x3F80; }
template <> __device__ __forceinline__ uint16_t one_bits<_Float16>() { return 0x3C00; }

// eight fp32 values that are exactly representable in T -> one operand fragment
template <typename T>
__device__ __forceinline__ typename Elem<T>::vec8 pack8(const f32x16& t, int first) {
    u32x4 w;
#pragma unroll
    for (int e = 0; e < 4; ++e) w[e] = Elem<T>::pack2(t[first + 2 * e], t[first + 2 * e + 1]);
    return vec8_from_words<T>(w);
}

// Global input row behind a local row id of a tile (-1: none).
__device__ __forceinline__ int32_t tile_row_of(uint32_t id, int flags, int win_lo, int win_n,
                                               const int32_t* __restrict__ rows) {
    if (flags & kTileLdsOffsets) id = (id / kRowBytes == (uint32_t)kRowCap) ? kNoRow : id / kRowBytes;
    if (id == kNoRow) return -1;
    return id < (uint32_t)win_n ? win_lo + (int32_t)id : rows[id - (uint32_t)win_n];
}

// ---------------------------------------------------------------------------------- input gradient, K = stride
// One wave per (tile, column block of 32 outputs, 64 produced channels).  The A operand of every
// offset is the same: the gout rows of the block's outputs (re-read per offset, they stay in L1);
// the B operand is W[kappa]^T in the packed fragment order (interleaved channels).  After the chunks
// of one offset the accumulators hold gin rows of the 32 inputs map(o, kappa), the rows along the
// registers and the channels across the lanes: a half-wave stores one row's 64-channel slice in one
// piece, and the accumulators start again from zero.
constexpr int kDgradWaves = 4;

template <typename T, bool OUT_F32>
__global__ void __launch_bounds__(64 * kDgradWaves)
k_dgrad_strided(const TileHeader* __restrict__ tile_hdr, const uint16_t* __restrict__ tile_perm,
                const int32_t* __restrict__ tile_rows, int row_stride, const uint16_t* __restrict__ tile_blocks,
                int block_stride, int64_t n_items, const uint16_t* __restrict__ gout, const uint16_t* __restrict__ wp,
                int C_contract, int C_produce, void* __restrict__ gin) {
    typedef typename Elem<T>::vec8 vec8;
    __shared__ __align__(16) int32_t row_of[kDgradWaves][kMaxK3Tiled][kGroup];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t item = (int64_t)blockIdx.x * kDgradWaves + wave;
    if (item >= n_items) return;
    const int nchunk = C_contract / kCinChunk, nslice = C_produce / kCoutSlice;
    const int slice = (int)(item % nslice);
    const int64_t tg = item / nslice;
    const int g = (int)(tg % kGroupsPerTile);
    const int64_t tile = tg / kGroupsPerTile;
    const TileHeader* H = tile_hdr + tile;
    const int w = tile_wave_of(g), gi = tile_slot_of(g);
    const uint32_t gm = (uint32_t)uni((int)H->group_mask[g]);
    const uint32_t wm = (uint32_t)uni((int)H->wave_mask[w]);
    const int n = lane & 31, h = lane >> 5;
    const int n_valid = uni(H->n_out);
    {
        const int flags = uni(H->flags), win_lo = uni(H->win_lo), win_n = uni(H->win_n);
        const size_t blk0 = (size_t)tile * block_stride + (uint32_t)uni((int)H->wave_block0[w]);
        const int32_t* rows = tile_rows + tile * (int64_t)row_stride;
        int rank = 0;
        for (uint32_t m = gm; m; m &= m - 1, ++rank) {
            if ((rank & 1) != h) continue;
            const int kappa = __ffs(m) - 1;
            const size_t blk = blk0 + __popc(wm & ((1u << kappa) - 1u));
            const uint32_t id = tile_blocks[blk * kIdBlockElems + n * kGroupsPerWave + gi];
            row_of[wave][rank][n] = tile_row_of(id, flags, win_lo, win_n, rows);
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();

    const int local = tile_perm[tile * kTileT + g * kGroup + n];
    const bool valid = local < n_valid;
    const uint16_t* grow = gout + (tile * kTileT + (valid ? local : 0)) * (int64_t)C_contract + h * 8;
    const int w_kappa_stride = nchunk * nslice * 4 * 64;
    const vec8* wl = reinterpret_cast<const vec8*>(wp) + lane;
    vec8 zero;
#pragma unroll
    for (int e = 0; e < 8; ++e) zero[e] = 0;

    int rank = 0;
    for (uint32_t m = gm; m; m &= m - 1, ++rank) {
        const int kappa = __ffs(m) - 1;
        f32x16 acc[2];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mt][v] = 0.f;
        for (int c = 0; c < nchunk; ++c) {
            vec8 b[2] = {zero, zero}, wf[4];
            if (valid) {
                b[0] = *reinterpret_cast<const vec8*>(grow + c * kCinChunk);
                b[1] = *reinterpret_cast<const vec8*>(grow + c * kCinChunk + 16);
            }
            const vec8* ws = wl + ((c * nslice + slice) * 4) * 64 + kappa * w_kappa_stride;
#pragma unroll
            for (int f = 0; f < 4; ++f) wf[f] = ws[f * 64];
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int nt = 0; nt < 2; ++nt) acc[nt] = Elem<T>::mfma(b[ks], wf[nt * 2 + ks], acc[nt]);
        }
        // accumulator register v of lane (n, h) is voxel 8 * (v / 4) + 4 * h + v % 4 of the block, channels 2n and
        // 2n + 1 of the slice (one per n-tile)
        const int64_t col = (int64_t)slice * kCoutSlice + 2 * n;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const i32x4 r4 = *reinterpret_cast<const i32x4*>(&row_of[wave][rank][8 * q + 4 * h]);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int32_t r = r4[j];
                if (r < 0) continue;
                if (OUT_F32)
                    *reinterpret_cast<f32x2*>(reinterpret_cast<float*>(gin) + (int64_t)r * C_produce + col) =
                        f32x2{acc[0][4 * q + j], acc[1][4 * q + j]};
                else
                    *reinterpret_cast<uint32_t*>(reinterpret_cast<uint16_t*>(gin) + (int64_t)r * C_produce + col) =
                        Elem<T>::pack2(acc[0][4 * q + j], acc[1][4 * q + j]);
            }
        }
    }
}

// The same product with the packed weights of one produced slice kept in LDS and the block's B
// fragments kept in registers for all offsets (at most kDgradMaxChunks 32-channel chunks): the
// offset loop then issues no vector loads at all.  Persistent workgroups of W waves; workgroup b
// serves produced slice b % nslice and walks column blocks with a stride.
//
// What a block needs before its first multiply hangs on chains of dependent loads (tile header ->
// id block -> row list; output permutation -> gout rows), and a wave that walked them block by block
// spent most of its time waiting.  The chains are therefore cut into stages that run one or two
// blocks ahead: the header and permutation entry of block i + 2 are requested while block i
// multiplies, the ids and the gout fragments of block i + 1 are requested before block i's offset
// loop (into a second fragment set) and turned into the row table after it.  R = offset ranks a lane
// half resolves (ceil(K^3 / 2)).
//
// Operand roles: A = gout rows (32 voxels x 16 contracted channels), B = packed weights in the
// interleaved layout (column n of n-tile t = produced channel 2n + t), so the produced rows lie along
// the accumulator registers and the channels across the lanes: a half-wave stores one produced row's
// 64-channel slice as one contiguous 128-byte (bf16) piece, where the other assignment wrote sixteen
// bytes per lane to 64 different rows per instruction.
constexpr int kDgradLdsWaves = 12;
constexpr int kDgradMaxChunks = 4;

template <typename T, bool OUT_F32, int W, int R>
__global__ void __launch_bounds__(64 * W, 1)
k_dgrad_strided_ldsw(const TileHeader* __restrict__ tile_hdr, const uint16_t* __restrict__ tile_perm,
                     const int32_t* __restrict__ tile_rows, int row_stride, const uint16_t* __restrict__ tile_blocks,
                     int block_stride, int64_t n_blocks_total, int K3, const uint16_t* __restrict__ gout,
                     const uint16_t* __restrict__ wp, int C_contract, int C_produce, void* __restrict__ gin) {
    typedef typename Elem<T>::vec8 vec8;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const int lane = threadIdx.x & 63, wave = uni((int)(threadIdx.x >> 6));
    const int nchunk = C_contract / kCinChunk, nslice = C_produce / kCoutSlice;
    const int slice = blockIdx.x % nslice;
    const int wg = blockIdx.x / nslice, n_wg = gridDim.x / nslice;
    unsigned char* wlds = lds_raw;                                       // [kappa][chunk][4 fragments][64 lanes][16 bytes]
    const int w_bytes = K3 * nchunk * 4096;
    int32_t* tab = reinterpret_cast<int32_t*>(lds_raw + w_bytes) + wave * K3 * kGroup;   // [rank][voxel]
    for (int sl = wave; sl * 1024 < w_bytes; sl += W) {
        const int kc = sl >> 2, f = sl & 3;
        const unsigned char* src = reinterpret_cast<const unsigned char*>(wp) + ((size_t)(kc * nslice + slice) * 4 + f) * 1024 + lane * 16;
        __builtin_amdgcn_global_load_lds(src, (lds_ptr_t)(wlds + sl * 1024), 16, 0, 0);
    }

    const int n = lane & 31, h = lane >> 5;
    vec8 zero;
#pragma unroll
    for (int e = 0; e < 8; ++e) zero[e] = 0;
    const int64_t tg_stride = (int64_t)n_wg * W;
    const int64_t tg0 = (int64_t)wg * W + wave;

    struct Hdr { uint32_t gm, wm, blk0; int flags, win_lo, win_n, n_out; };
    // the header fields of block tg (uniform addresses: scalar loads)
    auto load_hdr = [&](int64_t tg) -> Hdr {
        Hdr d = {0u, 0u, 0u, 0, 0, 0, 0};
        if (tg < n_blocks_total) {
            const int g = (int)(tg % kGroupsPerTile);
            const TileHeader* H = tile_hdr + tg / kGroupsPerTile;
            const int w = tile_wave_of(g);
            d.gm = H->group_mask[g]; d.wm = H->wave_mask[w]; d.blk0 = H->wave_block0[w];
            d.flags = H->flags; d.win_lo = H->win_lo; d.win_n = H->win_n; d.n_out = H->n_out;
        }
        return d;
    };
    auto load_perm = [&](int64_t tg) -> int {
        return tg < n_blocks_total ? (int)tile_perm[tg / kGroupsPerTile * kTileT + (tg % kGroupsPerTile) * kGroup + n] : 0;
    };
    // requests the local row ids of block tg: lane (n, h) takes the offset ranks of parity h, slot j = rank / 2
    auto issue_ids = [&](int64_t tg, const Hdr& d, uint32_t (&idv)[R]) {
        const int g = (int)(tg % kGroupsPerTile);
        const int gi = tile_slot_of(g);
        const size_t blk0 = (size_t)(tg / kGroupsPerTile) * block_stride + d.blk0;
        uint32_t m = d.gm;
#pragma unroll
        for (int j = 0; j < 2 * R; ++j) {
            if (m) {
                const int kappa = __ffs(m) - 1;
                m &= m - 1;
                if ((j & 1) == h)
                    idv[j >> 1] = tile_blocks[(blk0 + __popc(d.wm & ((1u << kappa) - 1u))) * kIdBlockElems + n * kGroupsPerWave + gi];
            }
        }
    };
    // requests the block's rows of the contracted side, all chunks
    auto issue_rows = [&](int64_t tg, const Hdr& d, int local, vec8 (&b)[kDgradMaxChunks][2]) {
        const bool valid = local < d.n_out;
        const uint16_t* grow = gout + (tg / kGroupsPerTile * kTileT + (valid ? local : 0)) * (int64_t)C_contract + h * 8;
#pragma unroll
        for (int c = 0; c < kDgradMaxChunks; ++c) {
            b[c][0] = zero; b[c][1] = zero;
            if (valid && c < nchunk) {
                b[c][0] = *reinterpret_cast<const vec8*>(grow + c * kCinChunk);
                b[c][1] = *reinterpret_cast<const vec8*>(grow + c * kCinChunk + 16);
            }
        }
    };
    // ids -> global produced rows (a second load for ids outside the tile's window), into the wave's table
    auto finish_table = [&](int64_t tg, const Hdr& d, const uint32_t (&idv)[R]) {
        const int32_t* rows = tile_rows + tg / kGroupsPerTile * (int64_t)row_stride;
        const int n_k = __popc(d.gm);
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const int rank = 2 * j + h;
            if (rank < n_k) tab[rank * kGroup + n] = tile_row_of(idv[j], d.flags, d.win_lo, d.win_n, rows);
        }
    };

    Hdr h0 = load_hdr(tg0), h1 = load_hdr(tg0 + tg_stride);
    int p0 = load_perm(tg0), p1 = load_perm(tg0 + tg_stride);
    uint32_t idv[R];
#pragma unroll
    for (int j = 0; j < R; ++j) idv[j] = kNoRow;
    vec8 bc[kDgradMaxChunks][2], bn[kDgradMaxChunks][2];
#pragma unroll
    for (int c = 0; c < kDgradMaxChunks; ++c) { bc[c][0] = zero; bc[c][1] = zero; bn[c][0] = zero; bn[c][1] = zero; }
    if (tg0 < n_blocks_total) {
        issue_ids(tg0, h0, idv);
        issue_rows(tg0, h0, p0, bc);
        finish_table(tg0, h0, idv);
    }
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();                       // the weights are in LDS

#pragma unroll 1
    for (int64_t tg = tg0; tg < n_blocks_total; tg += tg_stride) {
        const Hdr h2 = load_hdr(tg + 2 * tg_stride);
        const int p2 = load_perm(tg + 2 * tg_stride);
        const bool more = tg + tg_stride < n_blocks_total;
        if (more) {
            issue_ids(tg + tg_stride, h1, idv);
            issue_rows(tg + tg_stride, h1, p1, bn);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // a wave's LDS accesses are processed in order
        __builtin_amdgcn_wave_barrier();

        int rank = 0;
#pragma unroll 1
        for (uint32_t m = h0.gm; m; m &= m - 1, ++rank) {
            const int kappa = __ffs(m) - 1;
            f32x16 acc[2];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[mt][v] = 0.f;
#pragma unroll
            for (int c = 0; c < kDgradMaxChunks; ++c) {
                if (c < nchunk) {
                    const unsigned char* ws = wlds + (kappa * nchunk + c) * 4096 + lane * 16;
                    vec8 wf[4];
#pragma unroll
                    for (int f = 0; f < 4; ++f) wf[f] = *reinterpret_cast<const vec8*>(ws + f * 1024);
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                        for (int nt = 0; nt < 2; ++nt) acc[nt] = Elem<T>::mfma(bc[c][ks], wf[nt * 2 + ks], acc[nt]);
                }
            }
            // accumulator register v of lane (n, h) is voxel 8 * (v / 4) + 4 * h + v % 4 of the block, channels 2n and
            // 2n + 1 of the slice (one per n-tile): the 32 lanes of a half-wave store one whole 64-channel row slice
            const int64_t col = (int64_t)slice * kCoutSlice + 2 * n;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const i32x4 r4 = *reinterpret_cast<const i32x4*>(tab + rank * kGroup + 8 * q + 4 * h);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int32_t r = r4[j];
                    if (r < 0) continue;
                    if (OUT_F32)
                        *reinterpret_cast<f32x2*>(reinterpret_cast<float*>(gin) + (int64_t)r * C_produce + col) =
                            f32x2{acc[0][4 * q + j], acc[1][4 * q + j]};
                    else
                        *reinterpret_cast<uint32_t*>(reinterpret_cast<uint16_t*>(gin) + (int64_t)r * C_produce + col) =
                            Elem<T>::pack2(acc[0][4 * q + j], acc[1][4 * q + j]);
                }
            }
        }
        __builtin_amdgcn_wave_barrier();     // the row table is rewritten for the next block
        if (more) finish_table(tg + tg_stride, h1, idv);
        h0 = h1; h1 = h2; p0 = p1; p1 = p2;
#pragma unroll
        for (int c = 0; c < kDgradMaxChunks; ++c) { bc[c][0] = bn[c][0]; bc[c][1] = bn[c][1]; }
    }
}

// One thread per (pair, input channel) of a K = stride map (each input row has exactly one pair):
// gin[map(o,kappa), ci] = sum_co W[kappa][ci][co] * gout[o][co], fp32 FMA in channel order.
template <int DT, bool OUT_F32>
__global__ void k_dgrad_strided_scalar(const int32_t* __restrict__ nbmap, int64_t n_out, int K3,
                                       const void* __restrict__ gout, const void* __restrict__ w, int C_in, int C_out,
                                       void* __restrict__ gin) {
    const int64_t total = n_out * K3 * C_in;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const int64_t pair = e / C_in;
        const int ci = (int)(e - pair * C_in);
        const int32_t in = nbmap[pair];
        if (in < 0) continue;
        const int64_t o = pair / K3;
        const int kappa = (int)(pair - o * K3);
        const int64_t wb = ((int64_t)kappa * C_in + ci) * C_out, gb = o * C_out;
        float acc = 0.f;
        for (int co = 0; co < C_out; ++co) acc = fmaf(load_as_float<DT>(w, wb + co), load_as_float<DT>(gout, gb + co), acc);
        const int64_t dst = (int64_t)in * C_in + ci;
        if (OUT_F32) reinterpret_cast<float*>(gin)[dst] = acc;
        else if (DT == FX_F16) reinterpret_cast<uint16_t*>(gin)[dst] = Elem<_Float16>::from_float(acc);
        else reinterpret_cast<uint16_t*>(gin)[dst] = Elem<__bf16>::from_float(acc);
    }
}

// The same product with the weights read forward, W[kappa][contracted][produced] (transposed
// convolution): one thread per (pair, produced channel).
template <int DT, bool OUT_F32>
__global__ void k_conv_transpose_scalar(const int32_t* __restrict__ nbmap, int64_t n_out, int K3, const void* __restrict__ z,
                                        const void* __restrict__ w, int C_in, int C_out, void* __restrict__ out) {
    const int64_t total = n_out * K3 * C_out;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const int64_t pair = e / C_out;
        const int co = (int)(e - pair * C_out);
        const int32_t in = nbmap[pair];
        if (in < 0) continue;
        const int64_t o = pair / K3;
        const int kappa = (int)(pair - o * K3);
        const int64_t wb = (int64_t)kappa * C_in * C_out + co, zb = o * C_in;
        float acc = 0.f;
        for (int ci = 0; ci < C_in; ++ci)
            acc = fmaf(load_as_float<DT>(z, zb + ci), load_as_float<DT>(w, wb + (int64_t)ci * C_out), acc);
        const int64_t dst = (int64_t)in * C_out + co;
        if (OUT_F32) reinterpret_cast<float*>(out)[dst] = acc;
        else if (DT == FX_F16) reinterpret_cast<uint16_t*>(out)[dst] = Elem<_Float16>::from_float(acc);
        else reinterpret_cast<uint16_t*>(out)[dst] = Elem<__bf16>::from_float(acc);
    }
}

// ---------------------------------------------------------------------------------- weight gradient, MFMA
// A workgroup owns a block of 32 input channels x 64 output channels of every gw[kappa] and a
// contiguous range of tiles; its 8 waves split the offsets (wave w: kappa = w, w+8, w+16, w+24), so a wave
// keeps up to 4 offsets x 2 accumulator tiles (32 ci x 32 co) in registers over the whole range, and two
// waves per SIMD hide each other's LDS and matrix latencies (16 waves with two offsets each have 128 registers
// per wave, which the loop does not fit without spilling: 261 us against 208 on a 1 M-voxel LiDAR grid; 4 waves 279).  Per tile the workgroup stages,
// single-buffered and all with loads that go straight from global memory to LDS: the tile's input rows
// (32 channels, the forward kernel's LDS row layout, so the map's precomputed LDS offsets apply), its id
// blocks, and the gout rows of its 512 output slots (64 channels = 128 bytes per slot; 16-byte piece p of
// slot s sits at position p ^ 4*((s >> 1) & 1), which spreads a fragment read over all banks).
//
// Transposing read (tr_read4): in every group of 16 lanes, lane 4q+e receives, as element j, element e of
// the 8 bytes that lane 4j+q addresses.  With lane 4j+q pointing at channels 4q..4q+3 of voxel j's row,
// lane c of the group ends up with channel c of voxels 0..3: rows in, operand columns out.
//
// For one (column block g, offset kappa) a wave:
//   1. takes, per k-step ks and half t, the id of voxel 16ks + 8h + 4t + j of the block (h = lane / 32,
//      j = (lane / 4) % 4) -- the row its address contributes -- and reads the A fragment
//      [channel lane % 32][voxels 16ks + 8h .. + 7] of the gathered rows with two transposing reads;
//   2. reads the B fragments [voxel][co] of the gout slots 32g + 16ks + 8h .. + 7 the same way
//      (channels 32cb + lane % 32) and accumulates
//      gw[kappa][ci][co] += sum_voxel feat[voxel][ci] * gout[voxel][co].
// A voxel of the block without that tap reads the zero row and adds nothing; a slot past the end
// of the last tile has a zero gout row.  Tiles whose rows are not all staged in LDS keep the older form
// of step 1: the lane reads the row of voxel lane % 32 (from LDS or from global memory), and a product with
// the identity on the matrix unit leaves the block in the accumulator layout, which is the operand layout
// with voxels along k; rounding back to the storage type is exact.
// Partial sums go to part[range][kappa][ci][co] (fp32); k_wgrad_reduce adds the ranges in
// ascending order, so the result does not depend on scheduling.
constexpr int kWgCi = kCinChunk;            // 32: the row chunk staged in LDS
constexpr int kWgCo = 64;
constexpr int kGoutRowBytes = kWgCo * 2;    // one slot of the staged gout tile
constexpr int kGoutSlabs = kTileT * kGoutRowBytes / 1024;     // 1 KB slabs: 8 slots each

struct WgradLds {
    unsigned char rows[kRowBufBytes];
    unsigned char blocks[kBlockBufBytes];
    unsigned char gt[kTileT * kGoutRowBytes];
};
static_assert(sizeof(WgradLds) <= 160 * 1024, "LDS budget of one compute unit");
static_assert(kGroupsPerWave == 4 && kTileWaves == 4, "id blocks of four column blocks, 8 bytes per voxel");

// Which tiles a launch takes.  Tiles whose rows are all staged in LDS (kTileLdsOffsets; all but one or two of a
// sparse grid's) need neither the identity fragments nor the fallback loads of the older form: without that code the
// kernel fits 128 registers, runs sixteen waves with two offsets each -- four waves per SIMD to cover each other's
// LDS latencies -- and took 150 us where the eight-wave kernel with both forms took 204 (1 M-voxel LiDAR grid,
// 64 -> 64); 30 us of those 204 were one workgroup's single tile of the other kind, which costs as much as four
// staged ones.  When the map has at most kMaxListedTiles such tiles (counted once per map), kWgStaged (16 waves)
// takes the staged tiles of the ranges, and kWgOthers (8 waves, both forms) takes the listed tiles with one
// workgroup per column block of a tile, so that no workgroup carries a whole one: workgroup s sums column block s
// of every listed tile into partial sum n_ranges + s.  Other maps (strided, between two grids, dense grids, whose
// tiles mostly list one row per pair) take one launch of kWgAll (8 waves, both forms, every tile of the range).
// Either way a partial sum is made of the same terms in a fixed order.
enum WgradMode { kWgAll = 0, kWgStaged = 1, kWgOthers = 2 };

template <typename T, int W, int MODE>
__global__ void __launch_bounds__(64 * W, 1)
k_wgrad_mfma(const TileHeader* __restrict__ tile_hdr, const uint16_t* __restrict__ tile_perm,
             const int32_t* __restrict__ tile_rows, int row_stride, const uint16_t* __restrict__ tile_blocks,
             int block_stride, int64_t n_tiles, int n_ranges, const uint16_t* __restrict__ feat,
             const uint16_t* __restrict__ gout, int C_in, int C_out, int K3, float* __restrict__ part,
             const int32_t* __restrict__ tile_list, int n_listed) {
    constexpr int kWgWaves = W;
    constexpr int kGoutSlabsPerWave = kGoutSlabs / kWgWaves;
    constexpr int kWgOffsetsPerWave = (kMaxK3Tiled + kWgWaves - 1) / kWgWaves;
    static_assert(kGoutSlabs % kWgWaves == 0, "gout slabs per wave");
    typedef typename Elem<T>::vec8 vec8;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    WgradLds& L = *reinterpret_cast<WgradLds*>(lds_raw);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, h = lane >> 5;
    const int n_cib = C_in / kWgCi, n_cblk = n_cib * (C_out / kWgCo);
    // Workgroup b runs on XCD b % 8.  The channel blocks of one tile range read the same gout tiles and
    // id blocks: with the number of ranges a multiple of 8 they get block indices 8 apart, so they share
    // an XCD and its L2 and run side by side.
    int blk = blockIdx.x % n_cblk, range = blockIdx.x / n_cblk;      // kWgOthers: range = the column block it sums
    if (MODE != kWgOthers && n_ranges % 8 == 0) {
        blk = (blockIdx.x >> 3) % n_cblk;
        range = (int)(blockIdx.x / (8 * n_cblk)) * 8 + (blockIdx.x & 7);
    }
    const int cib = blk % n_cib, cob = blk / n_cib;
    const int64_t t0 = MODE == kWgOthers ? 0 : n_tiles * range / n_ranges, t1 = MODE == kWgOthers ? n_listed : n_tiles * (range + 1) / n_ranges;

    if (tid < kRowBytes / 16) reinterpret_cast<u32x4*>(L.rows + kRowCap * kRowBytes)[tid] = u32x4{0, 0, 0, 0};

    // identity fragments: element e of lane (n, h) in k-step ks is row k = 8h + e, column n of [I16 at columns 16ks..]
    vec8 ident[2];
    {
        u32x4 wds[2];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) {
                const uint32_t lo = (n == 16 * ks + 8 * h + 2 * e2) ? one_bits<T>() : 0u;
                const uint32_t hi = (n == 16 * ks + 8 * h + 2 * e2 + 1) ? one_bits<T>() : 0u;
                wds[ks][e2] = lo | (hi << 16);
            }
        ident[0] = vec8_from_words<T>(wds[0]);
        ident[1] = vec8_from_words<T>(wds[1]);
    }

    f32x16 acc[kWgOffsetsPerWave][2];
#pragma unroll
    for (int j = 0; j < kWgOffsetsPerWave; ++j)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][cb][v] = 0.f;

    // what this lane's address contributes to a transposing read: voxel jv of four, channels 16*g1 + 4*q .. + 3
    const int q = lane & 3, jv = (lane >> 2) & 3, g1 = (lane >> 4) & 1;
    const uint32_t a_piece = (uint32_t)(2 * g1 + (q >> 1)) << 4, half8 = (uint32_t)(q & 1) << 3;
    constexpr int kWgSlabs = ((kRowCap + 15) / 16 + kWgWaves - 1) / kWgWaves;   // 1 KB row slabs per wave
    int32_t nx_gr[kWgSlabs];
    int nx_local[kGoutSlabsPerWave];      // output row (inside the tile) of the slot this lane stages in each of its slabs
    auto resolve = [&](int64_t t) {
        const TileHeader* Ht = tile_hdr + t;
        const int fl = uni(Ht->flags), wl = uni(Ht->win_lo), wn = uni(Ht->win_n), nl = uni(Ht->n_list);
        const int ns = (fl & kTileDirect) ? 0 : min(wn + nl, kRowCap);
        const int32_t* rows_t = tile_rows + t * (int64_t)row_stride;
#pragma unroll
        for (int j = 0; j < kWgSlabs; ++j) {
            const int r = 16 * (wave + kWgWaves * j) + (lane >> 2);
            nx_gr[j] = -1;
            if (r < ns) nx_gr[j] = r < wn ? wl + r : rows_t[r - wn];
        }
#pragma unroll
        for (int j = 0; j < kGoutSlabsPerWave; ++j) nx_local[j] = tile_perm[t * kTileT + 8 * (wave + kWgWaves * j) + (lane >> 3)];
    };
    // the tiles that this workgroup takes, in order: positions t0 .. t1 of its range (kWgStaged: the staged ones
    // among them) or of the list
    auto tile_of = [&](int64_t c) -> int64_t { return MODE == kWgOthers ? (int64_t)uni(tile_list[c]) : c; };
    auto next_mine = [&](int64_t c) {
        if (MODE == kWgStaged)
            while (c < t1 && !(uni(tile_hdr[c].flags) & kTileLdsOffsets)) ++c;
        return c;
    };
    int64_t cur = next_mine(t0);
    if (cur < t1) resolve(tile_of(cur));
    while (cur < t1) {
        const int64_t cur_next = next_mine(cur + 1);
        const int64_t tile = tile_of(cur);
        const TileHeader* H = tile_hdr + tile;
        const int flags = uni(H->flags), win_lo = uni(H->win_lo), win_n = uni(H->win_n), n_list = uni(H->n_list);
        const int n_blocks = uni(H->n_blocks), n_valid = uni(H->n_out);
        const int n_staged = (flags & kTileDirect) ? 0 : min(win_n + n_list, kRowCap);
        const bool general = MODE == kWgStaged ? false : MODE == kWgOthers ? true : !(flags & kTileLdsOffsets);
        const int32_t* my_rows = tile_rows + tile * (int64_t)row_stride;
        uint32_t wmask[kTileWaves], gmask[kGroupsPerTile];
        int block0[kTileWaves];
#pragma unroll
        for (int fw = 0; fw < kTileWaves; ++fw) {
            wmask[fw] = (uint32_t)uni((int)H->wave_mask[fw]);
            block0[fw] = uni((int)H->wave_block0[fw]);
        }
#pragma unroll
        for (int g = 0; g < kGroupsPerTile; ++g) gmask[g] = (uint32_t)uni((int)H->group_mask[g]);

        // ---- stage: input rows (32 channels of this block), id blocks, gout rows.  The global
        // row of every slab piece and the output rows of the lane's slots were resolved while the
        // previous tile was staged, so all of this tile's loads leave at once.
        {
            const int piece = (lane & 3) ^ ((lane >> 4) & 3);
            int32_t gr[kWgSlabs];
#pragma unroll
            for (int j = 0; j < kWgSlabs; ++j) gr[j] = nx_gr[j];
            int local[kGoutSlabsPerWave];
#pragma unroll
            for (int j = 0; j < kGoutSlabsPerWave; ++j) local[j] = nx_local[j];
#pragma unroll
            for (int j = 0; j < kWgSlabs; ++j) {
                if (gr[j] >= 0) {
                    const uint16_t* src = feat + (int64_t)gr[j] * C_in + cib * kWgCi + piece * 8;
                    __builtin_amdgcn_global_load_lds(src, (lds_ptr_t)(L.rows + (wave + kWgWaves * j) * 1024), 16, 0, 0);
                }
            }
#pragma unroll
            for (int j = 0; j < kGoutSlabsPerWave; ++j) {
                const int slab = wave + kWgWaves * j, slot = 8 * slab + (lane >> 3);
                if (MODE == kWgOthers && slab / (kGroup / 8) != range) continue;   // only the slots of this workgroup's column block
                const int gpiece = (lane & 7) ^ (((slot >> 1) & 1) << 2);        // the piece stored at position lane & 7
                if (local[j] < n_valid) {
                    const uint16_t* src = gout + (tile * kTileT + local[j]) * (int64_t)C_out + cob * kWgCo + gpiece * 8;
                    __builtin_amdgcn_global_load_lds(src, (lds_ptr_t)(L.gt + slab * 1024), 16, 0, 0);
                } else {
                    *reinterpret_cast<u32x4*>(L.gt + slab * 1024 + lane * 16) = u32x4{0, 0, 0, 0};
                }
            }
            const unsigned char* bsrc =
                reinterpret_cast<const unsigned char*>(tile_blocks + (size_t)tile * block_stride * kIdBlockElems);
            const int bytes = n_blocks * kIdBlockElems * 2;
            for (int s = wave; s * 1024 < bytes; s += kWgWaves) {
                const int off = s * 1024 + lane * 16;
                if (off < bytes) __builtin_amdgcn_global_load_lds(bsrc + off, (lds_ptr_t)(L.blocks + s * 1024), 16, 0, 0);
            }
            if (cur_next < t1) resolve(tile_of(cur_next));
        }
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();

        // ---- multiply
#pragma unroll
        for (int j = 0; j < kWgOffsetsPerWave; ++j) {
            const int kappa = wave + kWgWaves * j;
            if (kappa >= K3) continue;
#pragma unroll
            for (int fw = 0; fw < kTileWaves; ++fw) {
                if (MODE == kWgOthers && fw != tile_wave_of(range)) continue;     // the column block this workgroup sums
                const uint32_t wm = wmask[fw];
                if (!((wm >> kappa) & 1u)) continue;
                const int b = block0[fw] + __popc(wm & ((1u << kappa) - 1u));
                const unsigned char* blk = L.blocks + (size_t)b * kGroup * 8;
                u32x2 ids = u32x2{0, 0}, idv[2][2];
                vec8 ga[2][2];
                if (general) {
                    ids = *reinterpret_cast<const u32x2*>(blk + n * 8);
                } else {
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                        for (int t = 0; t < 2; ++t) idv[ks][t] = *reinterpret_cast<const u32x2*>(blk + (16 * ks + 8 * h + 4 * t + jv) * 8);
                }
#pragma unroll
                for (int gi = 0; gi < kGroupsPerWave; ++gi) {
                    // general tiles: the rows of voxel lane % 32 in two groups are requested before the first of their
                    // products, so that the two latencies overlap (all four at once do not fit the registers)
                    if (general && (gi & 1) == 0) {
#pragma unroll
                        for (int gj = gi; gj < gi + 2; ++gj) {
                            if (MODE == kWgOthers && tile_group_of(fw, gj) != range) continue;
                            if (!((gmask[tile_group_of(fw, gj)] >> kappa) & 1u)) continue;
                            const uint32_t id = (ids[gj >> 1] >> (16 * (gj & 1))) & 0xFFFFu;
                            const bool staged = id < (uint32_t)n_staged;
                            const int row = staged ? (int)id : kRowCap;
                            ga[gj & 1][0] = *reinterpret_cast<const vec8*>(L.rows + lds_row_offset(row, h));
                            ga[gj & 1][1] = *reinterpret_cast<const vec8*>(L.rows + lds_row_offset(row, h + 2));
                            if (!staged && id != kNoRow) {
                                const int64_t gr = id < (uint32_t)win_n ? (int64_t)win_lo + id : (int64_t)my_rows[id - win_n];
                                const uint16_t* src = feat + gr * C_in + cib * kWgCi + h * 8;
                                ga[gj & 1][0] = *reinterpret_cast<const vec8*>(src);
                                ga[gj & 1][1] = *reinterpret_cast<const vec8*>(src + 16);
                            }
                        }
                    }
                    const int g = tile_group_of(fw, gi);
                    if (MODE == kWgOthers && g != range) continue;
                    if (!((gmask[g] >> kappa) & 1u)) continue;
                    vec8 fT[2];
                    if (!general) {
#pragma unroll
                        for (int ks = 0; ks < 2; ++ks) {
                            u32x2 w[2];
#pragma unroll
                            for (int t = 0; t < 2; ++t) {
                                const uint32_t id = (idv[ks][t][gi >> 1] >> (16 * (gi & 1))) & 0xFFFFu;
                                w[t] = tr_read4(L.rows + ((id ^ a_piece) + half8));
                            }
                            fT[ks] = vec8_from_words<T>(u32x4{w[0][0], w[0][1], w[1][0], w[1][1]});
                        }
                    } else {
                        f32x16 t;
#pragma unroll
                        for (int v = 0; v < 16; ++v) t[v] = 0.f;
                        t = Elem<T>::mfma(ga[gi & 1][0], ident[0], t);
                        t = Elem<T>::mfma(ga[gi & 1][1], ident[1], t);
                        fT[0] = pack8<T>(t, 0);
                        fT[1] = pack8<T>(t, 8);
                    }
#pragma unroll
                    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                        for (int ks = 0; ks < 2; ++ks) {
                            // slots 32g + 16ks + 8h + jv (+ 4), channels 32cb + 16g1 + 4q .. + 3: piece 4cb + 2g1 + q/2
                            // (after the identity product the A fragment holds voxels 4h .. 4h + 3 and 8 + 4h .. 8 + 4h + 3 instead)
                            const int slot = g * kGroup + 16 * ks + (general ? 4 : 8) * h + jv;
                            const uint32_t pos = (uint32_t)((4 * cb + 2 * g1 + (q >> 1)) ^ (((slot >> 1) & 1) << 2)) << 4;
                            const unsigned char* src = L.gt + slot * kGoutRowBytes + pos + half8;
                            const u32x2 lo = tr_read4(src);
                            const u32x2 hi = tr_read4(src + (general ? 8 : 4) * kGoutRowBytes);
                            acc[j][cb] = Elem<T>::mfma(fT[ks], vec8_from_words<T>(u32x4{lo[0], lo[1], hi[0], hi[1]}), acc[j][cb]);
                        }
                }
            }
        }
        __syncthreads();
        cur = cur_next;
    }

    // ---- partial sums of this range: lane (co = n, h), register 4b + r  ->  ci = 8b + 4h + r
    const int range_out = MODE == kWgOthers ? n_ranges + range : range;
#pragma unroll
    for (int j = 0; j < kWgOffsetsPerWave; ++j) {
        const int kappa = wave + kWgWaves * j;
        if (kappa >= K3) continue;
        float* dst = part + (((int64_t)range_out * K3 + kappa) * C_in + cib * kWgCi) * C_out + cob * kWgCo + n;
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int v = 0; v < 16; ++v) dst[(int64_t)(8 * (v >> 2) + 4 * h + (v & 3)) * C_out + cb * 32] = acc[j][cb][v];
    }
}

// gw[e] = part[0][e] + part[1][e] + ... in ascending order, rounded once to the output type.  One
// thread per four consecutive elements when the element count is a multiple of 4 (both channel counts
// even), one per element otherwise.
template <int OUT_DT>
__global__ void k_wgrad_reduce(const float* __restrict__ part, int n_ranges, int64_t total, void* __restrict__ gw) {
    const int64_t n4 = (total & 3) ? 0 : total / 4;    // the vector path needs every range 16-byte aligned
    for (int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < n4; q += (int64_t)gridDim.x * blockDim.x) {
        f32x4 s = {0.f, 0.f, 0.f, 0.f};
        int r = 0;
        for (; r + 8 <= n_ranges; r += 8) {   // eight loads in flight, added in ascending order
            f32x4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const f32x4*>(part + (int64_t)(r + u) * total + 4 * q);
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int e = 0; e < 4; ++e) s[e] += v[u][e];
        }
        for (; r + 4 <= n_ranges; r += 4) {   // four loads in flight, added in ascending order
            const f32x4 a = *reinterpret_cast<const f32x4*>(part + (int64_t)r * total + 4 * q);
            const f32x4 b = *reinterpret_cast<const f32x4*>(part + (int64_t)(r + 1) * total + 4 * q);
            const f32x4 c = *reinterpret_cast<const f32x4*>(part + (int64_t)(r + 2) * total + 4 * q);
            const f32x4 d = *reinterpret_cast<const f32x4*>(part + (int64_t)(r + 3) * total + 4 * q);
#pragma unroll
            for (int e = 0; e < 4; ++e) s[e] = (((s[e] + a[e]) + b[e]) + c[e]) + d[e];
        }
        for (; r < n_ranges; ++r) {
            const f32x4 a = *reinterpret_cast<const f32x4*>(part + (int64_t)r * total + 4 * q);
#pragma unroll
            for (int e = 0; e < 4; ++e) s[e] += a[e];
        }
        if (OUT_DT == FX_F32) *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(gw) + 4 * q) = s;
        else if (OUT_DT == FX_F16)
            *reinterpret_cast<u32x2*>(reinterpret_cast<uint16_t*>(gw) + 4 * q) =
                u32x2{Elem<_Float16>::pack2(s[0], s[1]), Elem<_Float16>::pack2(s[2], s[3])};
        else
            *reinterpret_cast<u32x2*>(reinterpret_cast<uint16_t*>(gw) + 4 * q) =
                u32x2{Elem<__bf16>::pack2(s[0], s[1]), Elem<__bf16>::pack2(s[2], s[3])};
    }
    for (int64_t e = 4 * n4 + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        float s = 0.f;
        for (int r = 0; r < n_ranges; ++r) s += part[(int64_t)r * total + e];
        if (OUT_DT == FX_F32) reinterpret_cast<float*>(gw)[e] = s;
        else if (OUT_DT == FX_F16) reinterpret_cast<uint16_t*>(gw)[e] = Elem<_Float16>::from_float(s);
        else reinterpret_cast<uint16_t*>(gw)[e] = Elem<__bf16>::from_float(s);
    }
}

// Scalar weight gradient: one thread per element of gw and per range of outputs, fp32 FMA in
// output order; the ranges are added by k_wgrad_reduce.
template <int DT>
__global__ void k_wgrad_scalar(const int32_t* __restrict__ nbmap, int64_t n_out, int K3, const void* __restrict__ feat,
                               const void* __restrict__ gout, int C_in, int C_out, int n_ranges,
                               float* __restrict__ part) {
    const int64_t total = (int64_t)K3 * C_in * C_out;
    const int range = blockIdx.y;
    const int64_t o0 = n_out * range / n_ranges, o1 = n_out * (range + 1) / n_ranges;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const int kappa = (int)(e / ((int64_t)C_in * C_out));
        const int rem = (int)(e - (int64_t)kappa * C_in * C_out);
        const int ci = rem / C_out, co = rem - ci * C_out;
        float acc = 0.f;
        int64_t o = o0;
        for (; o + 8 <= o1; o += 8) {      // eight map entries, then eight row pairs in flight; added in output order
            int32_t in[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) in[u] = nbmap[(o + u) * K3 + kappa];
            float f[8], g[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                f[u] = load_as_float<DT>(feat, (int64_t)max(in[u], 0) * C_in + ci);
                g[u] = load_as_float<DT>(gout, (o + u) * C_out + co);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) acc = in[u] >= 0 ? fmaf(f[u], g[u], acc) : acc;
        }
        for (; o < o1; ++o) {
            const int32_t in = nbmap[o * K3 + kappa];
            if (in < 0) continue;
            acc = fmaf(load_as_float<DT>(feat, (int64_t)in * C_in + ci), load_as_float<DT>(gout, o * C_out + co), acc);
        }
        part[(int64_t)range * total + e] = acc;
    }
}

// First level of a two-level ordered reduction: group blockIdx.y adds its `group` consecutive ranges in
// ascending order into part2[group index]; the final reduction then adds the groups in order.  The
// bracketing is fixed by (n_ranges, group), so repeated calls still give identical bits.
__global__ void k_wgrad_reduce_groups(const float* __restrict__ part, int n_ranges, int64_t total, int group,
                                      float* __restrict__ part2) {
    const int r0 = blockIdx.y * group, r1 = min(n_ranges, r0 + group);
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        float s = 0.f;
        int r = r0;
        for (; r + 4 <= r1; r += 4) {
            const float a = part[(int64_t)r * total + e], b = part[(int64_t)(r + 1) * total + e],
                        c = part[(int64_t)(r + 2) * total + e], d = part[(int64_t)(r + 3) * total + e];
            s = (((s + a) + b) + c) + d;
        }
        for (; r < r1; ++r) s += part[(int64_t)r * total + e];
        part2[(int64_t)blockIdx.y * total + e] = s;
    }
}

static hipError_t launch_reduce(const float* part, int n_ranges, int64_t total, void* gw, fx_dtype out_dt, hipStream_t st) {
    // small weight tensors (27 x 64 x 64 / 4 = 27 648 threads) in workgroups of one wave: 108 workgroups of 256 left
    // more than half the compute units without one (13.6 -> 11 us); large ones keep 256 (one wave each was slower)
    const unsigned bs = total / 4 <= 65536 ? 64u : 256u;
    const unsigned nb = (unsigned)std::max<int64_t>(1, std::min<int64_t>((total / 4 + bs - 1) / bs, 1 << 16));
    ProfScope ps(kProfWgradReduce, st);
    if (out_dt == FX_F32) k_wgrad_reduce<FX_F32><<<nb, bs, 0, st>>>(part, n_ranges, total, gw);
    else if (out_dt == FX_F16) k_wgrad_reduce<FX_F16><<<nb, bs, 0, st>>>(part, n_ranges, total, gw);
    else k_wgrad_reduce<FX_BF16><<<nb, bs, 0, st>>>(part, n_ranges, total, gw);
    return hipGetLastError();
}

// dst[map(o,kappa), :] = W'[kappa] applied to src[o, :] for every pair of a K = stride map (each input
// row has exactly one pair, so every row of dst is written once).  C_contract channels of src are
// contracted, C_produce channels produced; mode kWeightsTransposed reads W[kappa][produced][contracted]
// (the input gradient), kWeightsForward reads W[kappa][contracted][produced] (transposed convolution).
fx_status strided_pair_product(const fx_kmap* km, const void* d_src, fx_dtype dt, const void* d_w, int32_t C_contract,
                               int32_t C_produce, void* d_dst, fx_dtype out_dt, hipStream_t st, int mode) {
    const bool out_f32 = out_dt == FX_F32;
    const bool mfma = dt != FX_F32 && km->n_tiles > 0 && C_contract % kCinChunk == 0 && C_produce % kCoutSlice == 0 &&
                      option(kOptForceScalar) != 1;
    if (mfma) {
        void* wp = nullptr;
        const size_t wbytes = packed_weight_bytes(km->K3, C_contract, C_produce, 2);
        FX_TRY(dev_alloc(&wp, wbytes + 8 * sizeof(int32_t), st));
        int32_t* counters = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(wp) + wbytes);
        const int nslice = C_produce / kCoutSlice, nchunk = C_contract / kCinChunk;
        const size_t lds = (size_t)km->K3 * nchunk * 4096 + (size_t)kDgradLdsWaves * km->K3 * kGroup * sizeof(int32_t);
        const bool lds_weights = lds <= 160 * 1024 && nchunk <= kDgradMaxChunks && km->K3 <= 27 && option(kOptGatherLds) != 0;
        launch_pack_weights(d_w, wp, km->K3, C_contract, C_produce, 2, counters, mode, st);
        hipError_t e = hipGetLastError();
        if (e == hipSuccess && lds_weights) {
            const int64_t n_blocks_total = km->n_tiles * (int64_t)kGroupsPerTile;
            int64_t grid = std::max(nslice, compute_units() / nslice * nslice);
            grid = std::min<int64_t>(grid, (n_blocks_total + kDgradLdsWaves - 1) / kDgradLdsWaves * nslice);
            ProfScope ps(kProfDgradStrided, st);
#define FX_DGRAD_R(T, F32, R)                                                                                         \
    do {                                                                                                              \
        e = hipFuncSetAttribute((const void*)k_dgrad_strided_ldsw<T, F32, kDgradLdsWaves, R>,                         \
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                                \
        if (e == hipSuccess)                                                                                          \
            k_dgrad_strided_ldsw<T, F32, kDgradLdsWaves, R><<<(unsigned)grid, 64 * kDgradLdsWaves, lds, st>>>(         \
                km->d_tile_hdr, km->d_tile_perm, km->d_tile_rows, km->row_stride, km->d_tile_blocks, km->block_stride, \
                n_blocks_total, km->K3, (const uint16_t*)d_src, (const uint16_t*)wp, C_contract, C_produce, d_dst);    \
    } while (0)
#define FX_DGRAD(T, F32)                                                                                              \
    do { if (km->K3 <= 8) FX_DGRAD_R(T, F32, 4); else FX_DGRAD_R(T, F32, 14); } while (0)
            if (dt == FX_BF16) { if (out_f32) FX_DGRAD(__bf16, true); else FX_DGRAD(__bf16, false); }
            else { if (out_f32) FX_DGRAD(_Float16, true); else FX_DGRAD(_Float16, false); }
#undef FX_DGRAD
#undef FX_DGRAD_R
            if (e == hipSuccess) e = hipGetLastError();
        } else if (e == hipSuccess) {
            const int64_t n_items = km->n_tiles * (int64_t)kGroupsPerTile * (C_produce / kCoutSlice);
            const unsigned grid = (unsigned)((n_items + kDgradWaves - 1) / kDgradWaves);
            ProfScope ps(kProfDgradStrided, st);
#define FX_DGRAD(T, F32)                                                                                             \
    k_dgrad_strided<T, F32><<<grid, 64 * kDgradWaves, 0, st>>>(km->d_tile_hdr, km->d_tile_perm, km->d_tile_rows,      \
                                                               km->row_stride, km->d_tile_blocks, km->block_stride,  \
                                                               n_items, (const uint16_t*)d_src, (const uint16_t*)wp, \
                                                               C_contract, C_produce, d_dst)
            if (dt == FX_BF16) { if (out_f32) FX_DGRAD(__bf16, true); else FX_DGRAD(__bf16, false); }
            else { if (out_f32) FX_DGRAD(_Float16, true); else FX_DGRAD(_Float16, false); }
#undef FX_DGRAD
            e = hipGetLastError();
        }
        dev_free(wp, st);
        if (e != hipSuccess) { set_error("strided pair product launch failed: %s", hipGetErrorString(e)); return FX_EDEVICE; }
        return FX_OK;
    }
    FX_TRY(kmap_ensure_dense(const_cast<fx_kmap*>(km), st));
    const int64_t total = km->n_out * km->K3 * C_produce;
    const unsigned nb = (unsigned)std::max<int64_t>(1, std::min<int64_t>((total + 255) / 256, 1 << 20));
    ProfScope ps(kProfDgradStrided, st);
    // k_dgrad_strided_scalar takes W[kappa][produced][contracted], k_conv_transpose_scalar W[kappa][contracted][produced]
#define FX_SCALAR(DT)                                                                                                    \
    do {                                                                                                                 \
        if (mode == kWeightsTransposed) {                                                                                \
            if (out_f32) k_dgrad_strided_scalar<DT, true><<<nb, 256, 0, st>>>(km->d_nbmap, km->n_out, km->K3, d_src, d_w, \
                                                                              C_produce, C_contract, d_dst);             \
            else k_dgrad_strided_scalar<DT, false><<<nb, 256, 0, st>>>(km->d_nbmap, km->n_out, km->K3, d_src, d_w,        \
                                                                       C_produce, C_contract, d_dst);                    \
        } else {                                                                                                         \
            if (out_f32) k_conv_transpose_scalar<DT, true><<<nb, 256, 0, st>>>(km->d_nbmap, km->n_out, km->K3, d_src, d_w, \
                                                                               C_contract, C_produce, d_dst);            \
            else k_conv_transpose_scalar<DT, false><<<nb, 256, 0, st>>>(km->d_nbmap, km->n_out, km->K3, d_src, d_w,       \
                                                                        C_contract, C_produce, d_dst);                   \
        }                                                                                                                \
    } while (0)
    if (dt == FX_F32) FX_SCALAR(FX_F32);
    else if (dt == FX_F16) FX_SCALAR(FX_F16);
    else FX_SCALAR(FX_BF16);
#undef FX_SCALAR
    FX_HIP_TRY(hipGetLastError());
    return FX_OK;
}

}  // namespace fx

using namespace fx;

static fx_status check_bwd_types(const char* who, fx_dtype dt, fx_dtype out_dt) {
    if (dt != FX_F32 && dt != FX_F16 && dt != FX_BF16) { set_error("%s: unknown dtype", who); return FX_EINVAL; }
    if (out_dt != dt && out_dt != FX_F32) {
        set_error("%s: output dtype must equal the input dtype or be fp32", who);
        return FX_EUNSUPPORTED;
    }
    return FX_OK;
}

static bool force_scalar() {
    return option(kOptForceScalar) == 1;
}

extern "C" fx_status fx_sparse_conv_bwd_data(const fx_kmap* km, const void* d_gout, fx_dtype dt, const void* d_w,
                                             int32_t C_in, int32_t C_out, void* d_gin, fx_dtype out_dt, void* stream) {
    if (!km || !d_w || C_in < 1 || C_out < 1 || (km->n_out > 0 && !d_gout) || (km->n_in > 0 && !d_gin)) {
        set_error("fx_sparse_conv_bwd_data: null pointer or non-positive channel count");
        return FX_EINVAL;
    }
    FX_TRY(check_bwd_types("fx_sparse_conv_bwd_data", dt, out_dt));
    if (km->n_in == 0) return FX_OK;
    hipStream_t st = (hipStream_t)stream;
    if (km->stride == 1) {
        // symmetric map, same grid on both sides: the forward multiply on gout with mirrored offsets
        // and transposed weights (C_out channels are contracted, C_in produced); between two grids the
        // same over the map the other way round
        const fx_kmap* back = km;
        if (km->gin != km->gout) {
            FX_TRY(kmap_ensure_inverse(const_cast<fx_kmap*>(km), st));
            back = km->inverse;
        }
        return conv_apply(back, d_gout, dt, d_w, C_out, C_in, d_gin, out_dt, st, kWeightsMirrored);
    }
    if (km->K != km->stride) {
        // 3x3x3 stride 2: an input is shared by up to 8 outputs.  Gather per input through the inverse map
        // (a tiled map of its own, built on first use): gin[i,:] = sum over kappa with inv(i, kappa) = o of
        // W[kappa] . gout[o,:], i.e. the forward kernels of strided maps with W[kappa] transposed
        FX_TRY(kmap_ensure_inverse(const_cast<fx_kmap*>(km), st));
        return conv_apply(km->inverse, d_gout, dt, d_w, C_out, C_in, d_gin, out_dt, st, kWeightsTransposed);
    }
    return strided_pair_product(km, d_gout, dt, d_w, C_out, C_in, d_gin, out_dt, st, kWeightsTransposed);
}

// Adds the ranges of part[n_ranges][total] in ascending order into gw; above 192 ranges in two levels (groups of
// 64, then the groups), so that the first level runs at full occupancy.  The bracketing depends on n_ranges only.
fx_status fx::wgrad_reduce_ranges(const float* part, int n_ranges, int64_t total, void* gw, fx_dtype out_dt, hipStream_t st) {
    constexpr int kReduceGroup = 64;
    hipError_t e;
    if (n_ranges > 3 * kReduceGroup) {
        float* part2 = nullptr;
        const int n_groups = (n_ranges + kReduceGroup - 1) / kReduceGroup;
        FX_TRY(dev_alloc((void**)&part2, sizeof(float) * (size_t)total * n_groups, st));
        const dim3 grid((unsigned)std::min<int64_t>((total + 255) / 256, 1 << 16), (unsigned)n_groups);
        {
            ProfScope ps(kProfWgradReduce, st);
            k_wgrad_reduce_groups<<<grid, 256, 0, st>>>(part, n_ranges, total, kReduceGroup, part2);
            e = hipGetLastError();
        }
        if (e == hipSuccess) e = launch_reduce(part2, n_groups, total, gw, out_dt, st);
        dev_free(part2, st);
    } else {
        e = launch_reduce(part, n_ranges, total, gw, out_dt, st);
    }
    if (e != hipSuccess) { set_error("weight-gradient reduction failed: %s", hipGetErrorString(e)); return FX_EDEVICE; }
    return FX_OK;
}

extern "C" fx_status fx_sparse_conv_bwd_weight(const fx_kmap* km, const void* d_feat, const void* d_gout, fx_dtype dt,
                                               int32_t C_in, int32_t C_out, void* d_gw, fx_dtype out_dt, void* stream) {
    if (!km || !d_gw || C_in < 1 || C_out < 1 || (km->n_in > 0 && !d_feat) || (km->n_out > 0 && !d_gout)) {
        set_error("fx_sparse_conv_bwd_weight: null pointer or non-positive channel count");
        return FX_EINVAL;
    }
    FX_TRY(check_bwd_types("fx_sparse_conv_bwd_weight", dt, out_dt));
    hipStream_t st = (hipStream_t)stream;
    const int64_t total = (int64_t)km->K3 * C_in * C_out;
    if (km->n_out == 0) {   // no pairs: the gradient is zero
        FX_HIP_TRY(launch_reduce(nullptr, 0, total, d_gw, out_dt, st));
        return FX_OK;
    }
    // fp32 at low depth on a 3x3x3 submanifold map: the leaf-window kernel sums on the matrix units straight from
    // the grid, where everything below would take the scalar kernel (option leaf_dispatch = 0 keeps that one)
    // The 16-bit types at depth >= 32 take it on locally dense grids only (mean leaf occupancy of 0.40 and above, the
    // forward pass's rule): there the tiles of the map need more rows than the tile kernel's LDS holds
    // (option leaf_dispatch = 1 takes it on any grid).
    if (km->K == 3 && km->stride == 1 && km->gin == km->gout && leaf_wgrad_shape_supported(dt, C_in, C_out) &&
        !force_scalar()) {
        const int ld = option(kOptLeafDispatch);
        const double occupancy = (double)km->n_in / (512.0 * (double)std::max<int64_t>(1, km->gin->hdr.n_leaf));
        const bool take = dt == FX_F32 ? ld != 0 : (ld >= 0 ? ld == 1 : occupancy >= 0.40);
        if (take)
            return leaf_wgrad("sparse convolution weight gradient (leaf-window kernel)", km->gin, d_feat, d_gout, dt, C_in,
                              C_out, d_gw, out_dt, st);
    }
    bool mfma = dt != FX_F32 && km->n_tiles > 0 && C_in % kWgCi == 0 && C_out % kWgCo == 0 && !force_scalar();
    // Per-leaf dispatch, as in the forward pass: on a grid that mixes locally dense leaves with sparse ones the pairs
    // of the dense leaves' outputs are summed by the leaf-window kernel (over the list of those leaves) and all
    // others by the tile kernel over the copy of the map that leaves those outputs out; both write partial sums of
    // the same form and one ordered reduction adds them.  leaf_dispatch = 2 forces it.
    int leaf_ranges = 0;
    if (mfma && km->K == 3 && km->stride == 1 && km->gin == km->gout && !km->is_inverse && leaf_wgrad_shape_supported(dt, C_in, C_out)) {
        const int ld = option(kOptLeafDispatch);
        const double occupancy = (double)km->n_in / (512.0 * (double)std::max<int64_t>(1, km->gin->hdr.n_leaf));
        const double dense = (double)km->gin->hdr.n_voxels_dense / (double)std::max<int64_t>(1, km->n_in);
        if (ld == 2 || (ld < 0 && occupancy < 0.40 && dense >= 0.10)) {
            FX_TRY(kmap_ensure_mixed(const_cast<fx_kmap*>(km), st));
            leaf_ranges = leaf_wgrad16_ranges(km->gin, C_in, C_out);
        }
    }
    const fx_kmap* kmt = leaf_ranges ? km->mixed : km;      // the map whose tiles are walked
    mfma = mfma && kmt->n_tiles > 0;
    float* part = nullptr;
    hipError_t e = hipSuccess;
    int n_ranges = 1;
    if (mfma) {
        const fx_kmap* km_all = km;
        km = kmt;
        const int n_cblk = (C_in / kWgCi) * (C_out / kWgCo);
        n_ranges = (int)std::max<int64_t>(1, std::min<int64_t>(km->n_tiles, compute_units() / n_cblk));
        if (n_ranges > 8) n_ranges -= n_ranges % 8;   // see the block-to-XCD mapping in the kernel
        // Sparse submanifold maps with at most a few tiles that are not staged in LDS: the sixteen-wave launch for the
        // staged tiles and, if there are others, the launch that spreads those over one workgroup per column block
        // (see WgradMode).  Strided maps, maps between two grids and dense grids: one launch that
        // takes every tile.  (With a per-leaf split the tiles walked are those of the map without the dense leaves.)
        const double occ = (double)km->n_in / (512.0 * (double)std::max<int64_t>(1, km->gin->hdr.n_leaf));
        bool split = km->stride == 1 && km->gin == km->gout && !km->is_inverse && occ < 0.20;
        if (split) {
            FX_TRY(kmap_unstaged_tiles(const_cast<fx_kmap*>(km), st));
            split = km->h_n_unstaged <= kMaxListedTiles;
        }
        const int n_listed = split ? km->h_n_unstaged : 0;
        const int list_ranges = n_listed > 0 ? kGroupsPerTile : 0;       // one partial sum per column block of the listed tiles
        FX_TRY(dev_alloc((void**)&part, sizeof(float) * (size_t)total * (n_ranges + list_ranges + leaf_ranges), st));
        if (leaf_ranges) {
            const fx_status rl = leaf_wgrad16_partial(km_all->gin, d_feat, d_gout, dt, C_in, C_out, km->d_dense_leaves, km->d_n_dense,
                                                      part + (size_t)total * (n_ranges + list_ranges), leaf_ranges, st);
            if (rl != FX_OK) { dev_free(part, st); return rl; }
        }
        const size_t lds = sizeof(WgradLds);
        ProfScope ps(kProfWgrad, st);
#define FX_WGRAD_ONE(T, W, MODE, NWG)                                                                                  \
    do {                                                                                                               \
        if (e == hipSuccess)                                                                                           \
            e = hipFuncSetAttribute((const void*)k_wgrad_mfma<T, W, MODE>, hipFuncAttributeMaxDynamicSharedMemorySize, \
                                    (int)lds);                                                                         \
        if (e == hipSuccess) {                                                                                         \
            k_wgrad_mfma<T, W, MODE><<<(unsigned)(n_cblk * (NWG)), 64 * W, lds, st>>>(                                 \
                km->d_tile_hdr, km->d_tile_perm, km->d_tile_rows, km->row_stride, km->d_tile_blocks, km->block_stride, \
                km->n_tiles, n_ranges, (const uint16_t*)d_feat, (const uint16_t*)d_gout, C_in, C_out, km->K3, part,    \
                km->d_unstaged_list, n_listed);                                                                        \
            e = hipGetLastError();                                                                                     \
        }                                                                                                              \
    } while (0)
#define FX_WGRAD(T)                                                                                                    \
    do {                                                                                                               \
        if (split) {                                                                                                   \
            FX_WGRAD_ONE(T, 16, kWgStaged, n_ranges);                                                                  \
            if (n_listed > 0) FX_WGRAD_ONE(T, 8, kWgOthers, kGroupsPerTile);                                           \
        } else FX_WGRAD_ONE(T, 8, kWgAll, n_ranges);                                                                   \
    } while (0)
        if (dt == FX_BF16) FX_WGRAD(__bf16); else FX_WGRAD(_Float16);
        n_ranges += list_ranges;      // what the reduction adds up
#undef FX_WGRAD
#undef FX_WGRAD_ONE
        if (e == hipSuccess) e = hipGetLastError();
    } else {
        fx_status rc = kmap_ensure_dense(const_cast<fx_kmap*>(km), st);
        if (rc != FX_OK) return rc;
        // one thread per (element of gw, range of outputs): small weight tensors (low depth) get many short
        // ranges so that the chip is full -- up to 64 MB of partial sums -- and a two-level ordered reduction
        const int64_t cap = std::max<int64_t>(64, std::min<int64_t>(4096, ((int64_t)64 << 20) / (total * 4)));
        n_ranges = (int)std::max<int64_t>(1, std::min<int64_t>(cap, km->n_out / 256));
        FX_TRY(dev_alloc((void**)&part, sizeof(float) * (size_t)total * n_ranges, st));
        const dim3 grid((unsigned)std::min<int64_t>((total + 255) / 256, 1 << 16), (unsigned)n_ranges);
        ProfScope ps(kProfWgrad, st);
        if (dt == FX_F32) k_wgrad_scalar<FX_F32><<<grid, 256, 0, st>>>(km->d_nbmap, km->n_out, km->K3, d_feat, d_gout, C_in, C_out, n_ranges, part);
        else if (dt == FX_F16) k_wgrad_scalar<FX_F16><<<grid, 256, 0, st>>>(km->d_nbmap, km->n_out, km->K3, d_feat, d_gout, C_in, C_out, n_ranges, part);
        else k_wgrad_scalar<FX_BF16><<<grid, 256, 0, st>>>(km->d_nbmap, km->n_out, km->K3, d_feat, d_gout, C_in, C_out, n_ranges, part);
        e = hipGetLastError();
    }
    fx_status rc_red = FX_OK;
    if (e == hipSuccess) rc_red = wgrad_reduce_ranges(part, n_ranges + (mfma ? leaf_ranges : 0), total, d_gw, out_dt, st);
    dev_free(part, st);
    if (e != hipSuccess) { set_error("weight-gradient launch failed: %s", hipGetErrorString(e)); return FX_EDEVICE; }
    return rc_red;
}
