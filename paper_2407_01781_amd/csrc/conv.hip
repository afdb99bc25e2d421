// Sparse convolution forward (Sec. 3.5 scenario 3, re-designed for CDNA4).
//
// MFMA path.  A workgroup owns one tile of 512 consecutive output voxels.  The tile's distinct
// input rows are staged once in LDS (the paper's per-offset gathers become LDS reads), the
// per-offset products run on v_mfma_f32_32x32x16_{bf16,f16}, and -- unlike the paper's shared-
// memory scatter buffer -- every output voxel keeps its accumulators in registers for all
// offsets: a column block of 32 outputs is fixed for the whole tile, and an offset contributes
// a block only if one of the 32 has a neighbour there (missing neighbours read a zero row).
// Nothing is scattered; the write-back is one sequential range per tile.
//
// Operand roles in the tile kernel: A = gathered features (32 voxels x 16 input channels per
// instruction), B = packed weights (16 input channels x 32 output channels), D = 32 voxels x 32
// channels with the channels across lanes; the two weight tiles of a 64-channel slice interleave
// the channels (column n of tile t = channel 2n + t), so lane n holds two adjacent channels of
// every voxel and the 32 lanes of a half-wave store one whole output row at a time.  The gather
// kernels for strided maps keep the same roles with their A fragments read straight from global memory.
#include "conv_common.h"
#include "dev_timing.h"

#include <mutex>

namespace fx {

// ---------------------------------------------------------------------------------- weight packing
// Wp[kappa][cin chunk][cout slice][ntile 0..1][kstep 0..1][lane 0..63][8]: the 16-byte B-operand
// fragment of each lane for one (offset, 32 input channels, 64 output channels): lane (n, kq) holds
// the eight input channels 16 * kstep + 8 * kq .. + 7 of column n.  Column n of n-tile t is output
// channel 2n + t of the slice, so that lane n of an accumulator row (32x32 accumulator layout: lane
// half h, register v -> voxel row 8*(v/4) + 4*h + v%4) holds two adjacent channels, one per n-tile,
// and the 32 lanes of a half-wave store one whole output row.
template <typename E>   // uint16_t or uint32_t: the bits of one element
__global__ void k_pack_weights(const E* __restrict__ w, E* __restrict__ wp, int K3, int C_in, int C_out,
                               int32_t* __restrict__ counters, int mode) {
    if (blockIdx.x == 0 && threadIdx.x < 8) counters[threadIdx.x] = 0;   // the convolution's work-list counters
    constexpr int EPL = 16 / (int)sizeof(E);     // elements per lane fragment
    constexpr int kChunk = 4 * EPL;              // input channels per 64-byte row chunk
    const int nchunk = C_in / kChunk, nslice = (C_out + kCoutSlice - 1) / kCoutSlice;
    const int64_t total = (int64_t)K3 * C_in * nslice * kCoutSlice;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        int64_t r = e;
        const int el = (int)(r % EPL); r /= EPL;
        const int lane = (int)(r & 63); r >>= 6;
        const int ks = (int)(r & 1); r >>= 1;
        const int nt = (int)(r & 1); r >>= 1;
        const int s = (int)(r % nslice); r /= nslice;
        const int c = (int)(r % nchunk); r /= nchunk;
        const int kappa = (int)r;
        const int m = lane & 31, kq = lane >> 5;
        const int cin = c * kChunk + ks * 2 * EPL + kq * EPL + el;
        const int cout = s * kCoutSlice + 2 * m + nt;
        E v = 0;
        if (cout < C_out) {
            const int64_t kw = (mode & kWeightsFlipped) ? K3 - 1 - kappa : kappa;
            if (mode & kWeightsTransposed) v = w[(kw * C_out + cout) * C_in + cin];
            else v = w[(kw * C_in + cin) * C_out + cout];
        }
        wp[e] = v;
    }
}

size_t packed_weight_bytes(int K3, int C_in, int C_out, int elem_bytes) {
    return (size_t)elem_bytes * K3 * C_in * ((C_out + kCoutSlice - 1) / kCoutSlice) * kCoutSlice;
}

void launch_pack_weights(const void* d_w, void* wp, int K3, int C_in, int C_out, int elem_bytes, int32_t* counters,
                         int mode, hipStream_t st) {
    const int64_t total = (int64_t)(packed_weight_bytes(K3, C_in, C_out, elem_bytes) / elem_bytes);
    const unsigned nb = (unsigned)std::min<int64_t>((total + 255) / 256, 4096);
    ProfScope ps(kProfPackWeights, st);
    if (elem_bytes == 2)
        k_pack_weights<uint16_t><<<nb, 256, 0, st>>>((const uint16_t*)d_w, (uint16_t*)wp, K3, C_in, C_out, counters, mode);
    else
        k_pack_weights<uint32_t><<<nb, 256, 0, st>>>((const uint32_t*)d_w, (uint32_t*)wp, K3, C_in, C_out, counters, mode);
}

// Write-back of one column block computed with the features as the A operand: register v of
// accumulator tile t in lane (n, h) is output channel 2n + t of the slice for the block's slot
// 8*(v/4) + 4*h + v%4.  perm_g points at the block's 32 entries of the tile permutation in LDS
// (slot -> local output number).  Each store instruction covers two whole output rows.
typedef __attribute__((address_space(1))) unsigned char global_byte;

template <typename T, bool OUT_F32, bool FULL>
__device__ __forceinline__ void store_block_rows_impl(const f32x16 (&acc)[2], const uint16_t* perm_g, global_byte* tile_out,
                                                      uint32_t row_bytes, uint32_t lane_off, int n_valid, bool lane_ok, int h) {
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const u32x2 lp = *reinterpret_cast<const u32x2*>(perm_g + 8 * b + 4 * h);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const uint32_t local = (lp[r >> 1] >> (16 * (r & 1))) & 0xFFFFu;
            if (!FULL && ((int)local >= n_valid || !lane_ok)) continue;
            global_byte* dst = tile_out + (uint32_t)(__umul24(local, row_bytes) + lane_off);   // 32-bit offset from a wave-uniform base
            const int v = 4 * b + r;
            if (OUT_F32) {
                typedef __attribute__((ext_vector_type(2))) float f32x2;
                *reinterpret_cast<__attribute__((address_space(1))) f32x2*>(dst) = f32x2{acc[0][v], acc[1][v]};
            } else {
                *reinterpret_cast<__attribute__((address_space(1))) uint32_t*>(dst) = Elem<T>::pack2(acc[0][v], acc[1][v]);
            }
        }
    }
}

// tile_out: first byte of the tile's first output row at the slice's first channel (wave-uniform);
// cols: channels of the slice that exist (64, or fewer in the last slice of a padded channel count).
// The same with the weights held in LDS as fp32 in forward order W'[kappa][ci][co] (read through `mode` once per
// workgroup): at low depth the weight reads are most of the kernel's loads, and all lanes of a wave that work
// on the same four produced channels read the same 16 bytes, which LDS serves as a broadcast.  Few, fat
// workgroups walk the outputs so that the copy of the weights is paid a few thousand times, not per 256 outputs.
// QV: groups of four produced channels per thread.  1 is what runs: with 4 (one thread per voxel and 16 channels)
// the 64 lanes of a wave walk 64 different map rows and input rows, and the kernel took twice as long.
template <int DT, bool OUT_F32, int QV>
__global__ void __launch_bounds__(256)
k_conv_scalar4_ldsw(const int32_t* __restrict__ nbmap, int64_t n_out, int K3, const void* __restrict__ feat,
                    const void* __restrict__ w, int C_in, int C_out, void* __restrict__ out, int mode) {
    extern __shared__ __align__(16) unsigned char lds_w_raw[];
    float* wl = reinterpret_cast<float*>(lds_w_raw);
    const int n_w = K3 * C_in * C_out;
    for (int e = threadIdx.x; e < n_w; e += blockDim.x) {
        const int co = e % C_out, ci = (e / C_out) % C_in, kappa = e / (C_out * C_in);
        const int64_t kw = (mode & kWeightsFlipped) ? K3 - 1 - kappa : kappa;
        const int64_t src = (mode & kWeightsTransposed) ? (kw * C_out + co) * C_in + ci : (kw * C_in + ci) * C_out + co;
        wl[e] = load_as_float<DT>(w, src);
    }
    __syncthreads();
    const int q_out = C_out / (4 * QV);
    const int64_t total = n_out * q_out;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const int64_t o = e / q_out;
        const int co = (int)(e - o * q_out) * 4 * QV;
        f32x4 acc[QV];
#pragma unroll
        for (int g = 0; g < QV; ++g) acc[g] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int kappa = 0; kappa < K3; ++kappa) {
            const int32_t in = nbmap[o * K3 + kappa];
            if (in < 0) continue;
            const int64_t fb = (int64_t)in * C_in;
            const float* wk = wl + kappa * C_in * C_out + co;
            for (int ci = 0; ci < C_in; ci += 4) {
                const f32x4 x = load4_as_float<DT>(feat, fb + ci);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
#pragma unroll
                    for (int g = 0; g < QV; ++g) {
                        const f32x4 wr = *reinterpret_cast<const f32x4*>(wk + (ci + j) * C_out + 4 * g);
#pragma unroll
                        for (int v = 0; v < 4; ++v) acc[g][v] = fmaf(x[j], wr[v], acc[g][v]);
                    }
                }
            }
        }
#pragma unroll
        for (int g = 0; g < QV; ++g) {
            const int64_t at = o * C_out + co + 4 * g;
            if (OUT_F32) {
                *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(out) + at) = acc[g];
            } else if (DT == FX_F16) {
                *reinterpret_cast<u32x2*>(reinterpret_cast<uint16_t*>(out) + at) =
                    u32x2{Elem<_Float16>::pack2(acc[g][0], acc[g][1]), Elem<_Float16>::pack2(acc[g][2], acc[g][3])};
            } else {
                *reinterpret_cast<u32x2*>(reinterpret_cast<uint16_t*>(out) + at) =
                    u32x2{Elem<__bf16>::pack2(acc[g][0], acc[g][1]), Elem<__bf16>::pack2(acc[g][2], acc[g][3])};
            }
        }
    }
}

template <typename T, bool OUT_F32>
__device__ __forceinline__ void store_block_rows(const f32x16 (&acc)[2], const uint16_t* perm_g, unsigned char* tile_out,
                                                 int C_out, int cols, int n_valid, int n, int h, bool all_rows) {
    const uint32_t esize = OUT_F32 ? 4u : 2u;
    const uint32_t row_bytes = (uint32_t)C_out * esize, lane_off = 2u * (uint32_t)n * esize;
    // keep the base in scalar registers: the stores then take it as their scalar address operand
    const uint64_t bits = reinterpret_cast<uint64_t>(tile_out);
    const uint32_t lo = (uint32_t)uni((int)(uint32_t)bits), hi = (uint32_t)uni((int)(uint32_t)(bits >> 32));
    global_byte* base = (global_byte*)(((uint64_t)hi << 32) | lo);
    if (all_rows && n_valid == kTileT && cols == kCoutSlice)      // otherwise: rows beyond the tile's end or left to another kernel (0xFFFF)
        store_block_rows_impl<T, OUT_F32, true>(acc, perm_g, base, row_bytes, lane_off, n_valid, true, h);
    else
        store_block_rows_impl<T, OUT_F32, false>(acc, perm_g, base, row_bytes, lane_off, n_valid, 2 * n < cols, h);
}


// ---------------------------------------------------------------------------------- MFMA kernel
constexpr int kMetaSlots = 3;

// A work item (tile x 64-channel output slice) as the workgroup sees it: its number in the work
// list (-1: the list is exhausted) and a copy of the tile header.
struct MetaSlot {
    int64_t work;
    int64_t pad;
    TileHeader hdr;
};

// Rows and id blocks are double-buffered: while the consumer waves multiply out of one half, the
// producer waves fill the other half straight from global memory.  The work items themselves are
// announced two steps ahead in a ring of three slots.
struct ConvLds {
    unsigned char rows[2][kRowBufBytes];     // 64-byte rows; 16-byte piece p stored at p ^ ((row >> 2) & 3)
    unsigned char blocks[2][kBlockBufBytes]; // id blocks [block][voxel n][group slot], u16
    uint16_t perm[3][kTileT];                // a ring of three: the write-back of item i reads its entry while item i+1 multiplies
    MetaSlot meta[kMetaSlots];
};
static_assert(sizeof(ConvLds) <= 160 * 1024, "LDS budget of one compute unit");


// What a wave needs to know about one work item; all fields are wave-uniform.
struct Item {
    int64_t tile;
    int slice;
    int win_lo, win_n, n_list, n_blocks, n_valid, n_staged;
    bool general, all_rows;
};

__device__ __forceinline__ int64_t slot_work(const MetaSlot& M) {
    const int lo = uni((int)(uint32_t)(M.work & 0xFFFFFFFFll)), hi = uni((int)(M.work >> 32));
    return ((int64_t)hi << 32) | (uint32_t)lo;
}

__device__ __forceinline__ Item item_of(const MetaSlot& M, int64_t work, int nslice) {
    Item I;
    I.tile = work / nslice;
    I.slice = (int)(work - I.tile * nslice);
    I.win_lo = uni(M.hdr.win_lo); I.win_n = uni(M.hdr.win_n); I.n_list = uni(M.hdr.n_list);
    I.n_blocks = uni(M.hdr.n_blocks); I.n_valid = uni(M.hdr.n_out);
    const int flags = uni(M.hdr.flags);
    I.n_staged = (flags & kTileDirect) ? 0 : min(I.win_n + I.n_list, kRowCap);
    I.general = !(flags & kTileLdsOffsets);
    I.all_rows = !(flags & kTilePartial);
    return I;
}

// word e of a lane's id entry (a scalar when a wave has two groups, a vector otherwise)
__device__ __forceinline__ uint32_t id_word(uint32_t v, int) { return v; }
template <typename V>
__device__ __forceinline__ uint32_t id_word(const V& v, int e) { return v[e]; }

// Loop over the stencil offsets a wave needs for one 32-channel chunk.  Software pipeline per
// offset step i: the weights of step i+2, the B fragments of step i+1 and the ids of step i+2
// are fetched while the MFMAs of step i are issued (2 m-tiles x 2 k-steps per present column
// block).  The weights come from L2, whose latency exceeds one step, hence two steps of lead and
// three register sets; the sets are rotated by unrolling, never copied, and steps run in triples
// (the surplus steps multiply nothing) so that the rotation is the same at every exit.  Weight
// fragments are addressed as wbase0 (the packed array) + a wave-uniform offset + the lane's 16 bytes.
// The pipeline runs across calls: the last two steps fetch the fragments at offsets w_after0 and
// w_after1 -- the first two offsets of whatever this wave multiplies next -- into wa and wb, and
// wa_at / wb_at record what the two sets hold, so that a call normally starts with both in
// flight (and fetches them itself if a call in between was skipped).  GENERAL adds the fallback
// for rows that are not staged in LDS.
template <typename T, bool GENERAL>
__device__ __forceinline__ void offsets_loop(const unsigned char* lds_rows, const unsigned char* lds_blocks,
                                             f32x16 (&acc)[kGroupsPerWave][2],
                                             const uint32_t (&gmask)[kGroupsPerWave], uint32_t wave_mask,
                                             int wave_block0, const typename Elem<T>::vec8* __restrict__ wbase0,
                                             uint32_t lane_off, int w_base, int w_kappa_stride, typename Elem<T>::vec8 (&wa)[4],
                                             typename Elem<T>::vec8 (&wb)[4], int& wa_at, int& wb_at, int w_after0,
                                             int w_after1, int n, int h, int n_staged, int win_lo, int win_n,
                                             const int32_t* __restrict__ my_rows, const unsigned char* __restrict__ feat,
                                             int64_t pitch, int c) {
    typedef typename Elem<T>::vec8 vec8;
    constexpr int NG = kGroupsPerWave;
    const int n_off = __popc(wave_mask);
    const int n_steps = (n_off + 2) / 3 * 3;
    typedef __attribute__((ext_vector_type(NG / 2))) uint32_t IdVec;    // a lane's ids of one block: NG x u16
    const IdVec* idp = reinterpret_cast<const IdVec*>(lds_blocks) + (size_t)wave_block0 * kGroup + n;
    uint32_t rest = wave_mask;            // offsets not yet fetched; 31 (which no group has) once exhausted
    auto pop_kappa = [&]() {               // branch-free: 31 once the mask is exhausted
        const int k = __builtin_ctz(rest | 0x80000000u);
        rest &= rest - 1;
        return k;
    };
    // wave-uniform offset of the weights that step t multiplies (t may lie past this call's end);
    // written with masks so that it stays a handful of scalar instructions without branches
    auto w_offset = [&](int t, int k) {
        const int in = -(int)(t < n_off), last = -(int)(t == n_steps + 1);
        const int past = (w_after1 & last) | (w_after0 & ~last);
        return ((w_base + k * w_kappa_stride) & in) | (past & ~in);
    };
    auto fetch_w = [&](vec8 (&w)[4], int off) {   // [mtile*2 + kstep]; uniform base + 32-bit lane offset
        const unsigned char* ws = reinterpret_cast<const unsigned char*>(wbase0 + off);
#pragma unroll
        for (int f = 0; f < 4; ++f) w[f] = *reinterpret_cast<const vec8*>(ws + lane_off + f * 1024);
    };
    const uint32_t hsel = (uint32_t)h << 4;
    // B fragments (16 channels x 32 voxels, two k-steps) of column block gi for offset kappa
    auto fetch_b = [&](vec8 (&bf)[2], const IdVec& ids, int gi, int kappa) {
        // In the LDS-only variant the reads are issued for every group: an absent group's ids all
        // point at the zero row (one broadcast address).  With the reads unconditional every path
        // issues the same number of LDS instructions and the compiler waits for exactly the
        // fragments it needs; behind uniform branches it assumed the worst and drained the freshly
        // issued prefetch before every multiply.
        if (GENERAL && !((gmask[gi] >> kappa) & 1u)) return;
        const uint32_t id = (id_word(ids, gi >> 1) >> (16 * (gi & 1))) & 0xFFFFu;
        if (GENERAL) {
            const bool staged = id < (uint32_t)n_staged;
            const int row = staged ? (int)id : kRowCap;
            bf[0] = *reinterpret_cast<const vec8*>(lds_rows + lds_row_offset(row, h));
            bf[1] = *reinterpret_cast<const vec8*>(lds_rows + lds_row_offset(row, h + 2));
            const bool from_global = !staged && id != kNoRow;
            if (__any(from_global)) {
                if (from_global) {
                    const int64_t gr = id < (uint32_t)win_n ? (int64_t)win_lo + id : (int64_t)my_rows[id - win_n];
                    const unsigned char* src = feat + gr * pitch + c * kRowBytes + h * 16;
                    bf[0] = *reinterpret_cast<const vec8*>(src);
                    bf[1] = *reinterpret_cast<const vec8*>(src + 32);
                }
            }
        } else {   // id = lds_row_code(row): 16-byte piece p of the row sits at id ^ (p << 4); pieces h and h + 2
            const uint32_t a0 = id ^ hsel;
            bf[0] = *reinterpret_cast<const vec8*>(lds_rows + a0);
            bf[1] = *reinterpret_cast<const vec8*>(lds_rows + (a0 ^ 32u));
        }
    };
    vec8 wc[4];
    vec8 bf[NG][2];   // one set: a group's fragments for the next offset are fetched right after its multiplies
    int q0 = pop_kappa(), q1 = pop_kappa(), q2 = pop_kappa(), it = 0;   // offsets of steps it, it+1, it+2
    if (wa_at != w_offset(0, q0)) fetch_w(wa, w_offset(0, q0));          // only after a call was skipped
    if (wb_at != w_offset(1, q1)) fetch_w(wb, w_offset(1, q1));
    wa_at = w_after0;
    wb_at = w_after1;
    // Both sets were requested at least two steps ago (or, rarely, just now).  Waiting for them here
    // costs nothing in the common case and tells the compiler so: without it the loop's wait counts
    // are computed for the rare case and every step also waits for the weights of the next one.
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0), other counters untouched
    IdVec idn = idp[min(1, n_off - 1) * kGroup];   // ids of step 1
    {
        const IdVec id0 = idp[0];
#pragma unroll
        for (int gi = 0; gi < NG; ++gi) fetch_b(bf[gi], id0, gi, q0);
    }
    // one step: fetch the weights of step it+2 and the ids of step it+2, then, group by group,
    // multiply the current offset and fetch the group's fragments for the next one
    auto step = [&](const vec8 (&wcur)[4], vec8 (&wload)[4]) {
        fetch_w(wload, w_offset(it + 2, q2));
        const IdVec ids_next = idn;
        idn = idp[min(it + 2, n_off - 1) * kGroup];
#pragma unroll
        for (int gi = 0; gi < NG; ++gi) {
            if ((gmask[gi] >> q0) & 1u) {
#pragma unroll
                for (int ks = 0; ks < 2; ++ks)      // k-step outermost: consecutive MFMAs never share an accumulator
#pragma unroll
                    for (int mt = 0; mt < 2; ++mt) acc[gi][mt] = Elem<T>::mma(bf[gi][ks], wcur[mt * 2 + ks], acc[gi][mt]);
            }
            fetch_b(bf[gi], ids_next, gi, q1);
        }
        ++it;
        q0 = q1; q1 = q2; q2 = pop_kappa();
    };
    while (it < n_off) {
        step(wa, wc);
        step(wb, wa);
        step(wc, wb);
    }
}

// Producer side: one wave copies 1 KB slabs (16 rows of 64 bytes, or 4 id blocks) from global
// memory straight into LDS; lane l of a slab load writes the 16 bytes at slab + 16*l.
__device__ __forceinline__ void produce_rows(unsigned char* lds_rows, const Item& I, int pwave, int lane,
                                             const int32_t* __restrict__ tile_rows, int row_stride,
                                             const unsigned char* __restrict__ feat, int64_t pitch, int c) {
    const int32_t* my_rows = tile_rows + I.tile * (int64_t)row_stride;
    const int n_slabs = (I.n_staged + 15) >> 4;
    const int piece = (lane & 3) ^ ((lane >> 4) & 3);   // stored position lane&3 holds piece (lane&3) ^ ((row >> 2) & 3)
    for (int s = pwave; s < n_slabs; s += kProducerWaves) {
        const int r = 16 * s + (lane >> 2);
        if (r < I.n_staged) {
            const int64_t gr = r < I.win_n ? (int64_t)I.win_lo + r : (int64_t)my_rows[r - I.win_n];
            const unsigned char* src = feat + gr * pitch + c * kRowBytes + piece * 16;
            __builtin_amdgcn_global_load_lds(src, (lds_ptr_t)(lds_rows + s * 1024), 16, 0, 0);
        }
    }
}

// The same with the global row of every slab a lane serves kept in registers: the rows of a tile
// are the same for all its chunks, so only the first chunk pays the dependent load of the halo list.
constexpr int kSlabsPerProducer = ((kRowCap + 15) / 16 + kProducerWaves - 1) / kProducerWaves;

__device__ __forceinline__ void resolve_rows(int32_t (&gr)[kSlabsPerProducer], const Item& I, int pwave, int lane,
                                             const int32_t* __restrict__ tile_rows, int row_stride) {
    const int32_t* my_rows = tile_rows + I.tile * (int64_t)row_stride;
#pragma unroll
    for (int j = 0; j < kSlabsPerProducer; ++j) {
        const int r = 16 * (pwave + kProducerWaves * j) + (lane >> 2);
        gr[j] = -1;
        if (r < I.n_staged) gr[j] = r < I.win_n ? I.win_lo + r : my_rows[r - I.win_n];
    }
}

__device__ __forceinline__ void produce_rows_resolved(unsigned char* lds_rows, const int32_t (&gr)[kSlabsPerProducer],
                                                      int pwave, int lane, const unsigned char* __restrict__ feat,
                                                      int64_t pitch, int c) {
    const int piece = (lane & 3) ^ ((lane >> 4) & 3);
#pragma unroll
    for (int j = 0; j < kSlabsPerProducer; ++j) {
        if (gr[j] >= 0) {
            const unsigned char* src = feat + (int64_t)gr[j] * pitch + c * kRowBytes + piece * 16;
            __builtin_amdgcn_global_load_lds(src, (lds_ptr_t)(lds_rows + (pwave + kProducerWaves * j) * 1024), 16, 0, 0);
        }
    }
}

__device__ __forceinline__ void produce_meta(unsigned char* lds_blocks, uint16_t* lds_perm, const Item& I, int pwave, int lane,
                                             const uint16_t* __restrict__ tile_perm,
                                             const uint16_t* __restrict__ tile_blocks, int block_stride) {
    const unsigned char* src = reinterpret_cast<const unsigned char*>(tile_blocks + (size_t)I.tile * block_stride * kIdBlockElems);
    const int bytes = I.n_blocks * kIdBlockElems * 2;
    for (int s = pwave; s * 1024 < bytes; s += kProducerWaves) {
        const int off = s * 1024 + lane * 16;
        if (off < bytes) __builtin_amdgcn_global_load_lds(src + off, (lds_ptr_t)(lds_blocks + s * 1024), 16, 0, 0);
    }
    if (pwave == 0)
        __builtin_amdgcn_global_load_lds(reinterpret_cast<const unsigned char*>(tile_perm + I.tile * kTileT) + lane * 16,
                                         (lds_ptr_t)lds_perm, 16, 0, 0);
}

// Next unclaimed work item: first from the list of the workgroup's own XCD, then from the others'.
// The first wg_per_xcd items of every list are taken statically by that XCD's workgroups.
__device__ __forceinline__ int64_t take_work(int32_t* __restrict__ counters, int xcd, int per_xcd, int wg_per_xcd,
                                             int64_t n_work) {
    for (int v = 0; v < 8; ++v) {
        const int x = (xcd + v) & 7;
        const int64_t begin = (int64_t)x * per_xcd;
        const int64_t end = min(n_work, begin + per_xcd);
        if (begin + wg_per_xcd >= end) continue;
        const int64_t w = begin + wg_per_xcd + atomicAdd(&counters[x], 1);
        if (w < end) return w;
    }
    return -1;
}

// One wave announces work item `work` (or the end of the list) in a slot of the ring.
__device__ __forceinline__ void announce(MetaSlot& M, int64_t work, int nslice, const TileHeader* __restrict__ tile_hdr,
                                         int lane) {
    if (work >= 0) {
        const int32_t* src = reinterpret_cast<const int32_t*>(tile_hdr + work / nslice);
        if (lane < (int)(sizeof(TileHeader) / 4)) reinterpret_cast<int32_t*>(&M.hdr)[lane] = src[lane];
    }
    if (lane == 0) M.work = work;
}

// offset (in 16-byte fragments, wave-uniform) of the first weight fragment for (slice, chunk, offset)
// (the packed weights of one call stay far below 2^31 fragments)
__device__ __forceinline__ int w_frag(int nslice, int w_kappa_stride, int slice, int c, int kappa) {
    return ((c * nslice + slice) * 4) * 64 + kappa * w_kappa_stride;
}

__device__ __forceinline__ int first_offset(uint32_t mask) { return mask ? __ffs(mask) - 1 : 0; }

// Consumer side of one work item: multiply all chunks (one barrier after each, matching the
// producers' barriers), then write the tile's outputs back (lane (n, h) holds channels
// slice*64 + 32h .. +31 of output slot g*32 + n).  `phase` counts chunks since kernel start and
// selects the LDS half; `mb` selects the half that holds this tile's id blocks.
// The weight pipeline (wa, wb and their tags) runs across chunks and, in the LDS-only variant,
// across items: the last steps of an item already fetch the first weights of the next one (MN
// is its slot), ahead of the write-back stores -- loads and stores retire in order, and weights
// requested after the stores would have to wait for them.
template <typename T, bool OUT_F32, bool GENERAL>
__device__ __forceinline__ void consume_item(ConvLds& L, const MetaSlot& M, const MetaSlot& MN, const Item& I, int phase,
                                             int mb, int pb, int nchunk, int nslice, int wave, int lane,
                                             const int32_t* __restrict__ tile_rows, int row_stride,
                                             const unsigned char* __restrict__ feat, const unsigned char* __restrict__ wp,
                                             int64_t pitch, int C_out, void* __restrict__ out, typename Elem<T>::vec8 (&wa)[4],
                                             typename Elem<T>::vec8 (&wb)[4], int& wa_at, int& wb_at,
                                             unsigned long long (&tm)[4]) {
    typedef typename Elem<T>::vec8 vec8;
    constexpr int NG = kGroupsPerWave;
    const int n = lane & 31, h = lane >> 5;
    uint32_t gmask[NG];
#pragma unroll
    for (int gi = 0; gi < NG; ++gi) gmask[gi] = (uint32_t)uni((int)M.hdr.group_mask[tile_group_of(wave, gi)]);
    const uint32_t wave_mask = (uint32_t)uni((int)M.hdr.wave_mask[wave]);
    const int wave_block0 = uni((int)M.hdr.wave_block0[wave]);
    const int32_t* my_rows = tile_rows + I.tile * (int64_t)row_stride;
    const int w_kappa_stride = nchunk * nslice * 4 * 64;

    f32x16 acc[NG][2];
#pragma unroll
    for (int gi = 0; gi < NG; ++gi)
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[gi][mt][v] = 0.f;

    for (int c = 0; c < nchunk; ++c) {
        // where this wave's weights come from after this chunk
        int w_after0, w_after1;
        {
            int nsl = I.slice, nc = c + 1;
            uint32_t nmask = wave_mask;
            if (nc == nchunk) {      // the next item (if it is not one for this variant, the fetches go unused)
                const int64_t nwork = slot_work(MN);
                nc = 0;
                nsl = nwork >= 0 ? (int)(nwork % nslice) : I.slice;
                nmask = nwork >= 0 ? (uint32_t)uni((int)MN.hdr.wave_mask[wave]) : 0u;
            }
            w_after0 = w_frag(nslice, w_kappa_stride, nsl, nc, first_offset(nmask));
            const uint32_t more = nmask & (nmask - 1);
            w_after1 = more ? w_frag(nslice, w_kappa_stride, nsl, nc, first_offset(more)) : w_after0;
        }
        if (wave_mask) {
            FX_CYCLES_BEGIN();
            offsets_loop<T, GENERAL>(L.rows[(phase + c) & 1], L.blocks[mb], acc, gmask, wave_mask, wave_block0,
                                     reinterpret_cast<const vec8*>(wp), (uint32_t)lane * 16u,
                                     w_frag(nslice, w_kappa_stride, I.slice, c, 0), w_kappa_stride, wa, wb, wa_at, wb_at,
                                     w_after0, w_after1, n, h, I.n_staged, I.win_lo, I.win_n, my_rows, feat, pitch, c);
            FX_CYCLES_ADD(tm[0]);
        }
        { FX_CYCLES_BEGIN(); __syncthreads(); FX_CYCLES_ADD(tm[1]); }
    }
    FX_CYCLES_BEGIN();
    unsigned char* tile_out = reinterpret_cast<unsigned char*>(out) +
                              ((I.tile * kTileT) * C_out + (int64_t)I.slice * kCoutSlice) * (OUT_F32 ? 4 : 2);
#pragma unroll
    for (int gi = 0; gi < NG; ++gi)
        store_block_rows<T, OUT_F32>(acc[gi], L.perm[pb] + tile_group_of(wave, gi) * kGroup, tile_out, C_out,
                                     min(kCoutSlice, C_out - I.slice * kCoutSlice), I.n_valid, n, h, I.all_rows);
    FX_CYCLES_ADD(tm[2]);
}

// Items whose rows are not all staged in LDS take this path: a real call, so that its registers
// are allocated apart from the main loop's.
template <typename T, bool OUT_F32>
__device__ __noinline__ void consume_item_general(int slot, int phase, int mb, int pb, int nchunk, int nslice, int wave, int lane,
                                                  const int32_t* __restrict__ tile_rows, int row_stride,
                                                  const unsigned char* __restrict__ feat, const unsigned char* __restrict__ wp,
                                                  int64_t pitch, int C_out, void* __restrict__ out) {
    typedef typename Elem<T>::vec8 vec8;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    ConvLds& L = *reinterpret_cast<ConvLds*>(lds_raw);
    const MetaSlot& M = L.meta[slot];
    const Item I = item_of(M, slot_work(M), nslice);
    vec8 wa[4], wb[4];
    int wa_at = -1, wb_at = -1;
    unsigned long long tm[4] = {0, 0, 0, 0};
    consume_item<T, OUT_F32, true>(L, M, L.meta[(slot + 1) % kMetaSlots], I, phase, mb, pb, nchunk, nslice, wave, lane, tile_rows,
                                   row_stride, feat, wp, pitch, C_out, out, wa, wb, wa_at, wb_at, tm);
}

// Persistent workgroups, one per compute unit.  Work items (tile of 512 consecutive outputs x
// slice of 64 output channels) are cut into eight contiguous lists, one per XCD, so that
// neighbouring tiles, which share halo rows, meet in the same L2; a workgroup starts with a fixed
// item of its XCD's list and then claims items through per-list counters (its own list first),
// which evens out tiles of different cost.  Time advances in phases of one 32-channel chunk.
// Waves 0-3 are consumers: wave w owns 4 of the tile's 16 column blocks (128 outputs, 4 x 2
// accumulator tiles of 32x32) and multiplies out of one half of LDS.  Waves 4-7 are producers:
// meanwhile they copy the rows of the next phase (and, at a tile change, its id blocks) from
// global memory straight into the other half, and the first of them announces the item that
// starts two phases later (claim + tile header) in a ring of three slots.  One barrier per phase
// hands everything over; both roles walk the same ring and execute the same barriers.
// Producers and consumers are separate waves because a wave's loads complete in order: the
// consumer's short weight fetches must not queue behind the long HBM reads.
template <typename T, bool OUT_F32>
__global__ void __launch_bounds__(kConvThreads, 1)
k_conv_mfma(const TileHeader* __restrict__ tile_hdr, const uint16_t* __restrict__ tile_perm,
            const int32_t* __restrict__ tile_rows, int row_stride, const uint16_t* __restrict__ tile_blocks,
            int block_stride, int64_t n_work, int per_xcd, int32_t* __restrict__ counters,
            const unsigned char* __restrict__ feat, const unsigned char* __restrict__ wp, int C_in, int C_out,
            void* __restrict__ out) {
    typedef typename Elem<T>::vec8 vec8;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    ConvLds& L = *reinterpret_cast<ConvLds*>(lds_raw);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t pitch = (int64_t)C_in * Elem<T>::kBytes;                      // bytes per feature row
    const int nchunk = (int)(pitch / kRowBytes), nslice = (C_out + kCoutSlice - 1) / kCoutSlice;

    // workgroup b runs on XCD b % 8 (round-robin dispatch)
    const int xcd = blockIdx.x & 7, in_xcd = blockIdx.x >> 3, wg_per_xcd = gridDim.x >> 3;
    const int64_t first = (int64_t)xcd * per_xcd + in_xcd;
    if (in_xcd >= per_xcd || first >= n_work) return;

    if (tid < 2 * (kRowBytes / 16))   // the zero row of both halves
        reinterpret_cast<u32x4*>(L.rows[tid >> 2] + kRowCap * kRowBytes)[tid & 3] = u32x4{0, 0, 0, 0};

    if (wave >= kTileWaves) {
        // ---------------- producers
        const int pwave = wave - kTileWaves;
        if (pwave == 0) {   // items that start in phases 0 and 1
            announce(L.meta[0], first, nslice, tile_hdr, lane);
            if (nchunk == 1) {
                int64_t w = 0;
                if (lane == 0) w = take_work(counters, xcd, per_xcd, wg_per_xcd, n_work);
                w = __shfl(w, 0);
                announce(L.meta[1], w, nslice, tile_hdr, lane);
            }
        }
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        int32_t gr[kSlabsPerProducer];
        {
            const Item cur = item_of(L.meta[0], first, nslice);
            produce_meta(L.blocks[0], L.perm[0], cur, pwave, lane, tile_perm, tile_blocks, block_stride);
            resolve_rows(gr, cur, pwave, lane, tile_rows, row_stride);
            produce_rows_resolved(L.rows[0], gr, pwave, lane, feat, pitch, 0);
        }
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        int phase = 0;
        for (int item_no = 0;; ++item_no) {
            const MetaSlot& M = L.meta[item_no % kMetaSlots];
            const int64_t work = slot_work(M);
            if (work < 0) break;
            const Item cur = item_of(M, work, nslice);
            for (int c = 0; c < nchunk; ++c, ++phase) {
                const int rb = (phase + 1) & 1;
                if (c != nchunk - 1) {
                    produce_rows_resolved(L.rows[rb], gr, pwave, lane, feat, pitch, c + 1);
                } else {
                    const MetaSlot& MN = L.meta[(item_no + 1) % kMetaSlots];
                    const int64_t nwork = slot_work(MN);
                    if (nwork >= 0) {
                        const Item nxt = item_of(MN, nwork, nslice);
                        const int nb = (item_no + 1) & 1;
                        produce_meta(L.blocks[nb], L.perm[(item_no + 1) % 3], nxt, pwave, lane, tile_perm, tile_blocks, block_stride);
                        resolve_rows(gr, nxt, pwave, lane, tile_rows, row_stride);
                        produce_rows_resolved(L.rows[rb], gr, pwave, lane, feat, pitch, 0);
                    }
                }
                if (pwave == 0 && (phase + 2) % nchunk == 0) {   // an item starts two phases from now
                    int64_t w = 0;
                    if (lane == 0) w = take_work(counters, xcd, per_xcd, wg_per_xcd, n_work);
                    w = __shfl(w, 0);
                    announce(L.meta[((phase + 2) / nchunk) % kMetaSlots], w, nslice, tile_hdr, lane);
                }
                __builtin_amdgcn_s_waitcnt(0);
                __syncthreads();
            }
        }
    } else {
        // ---------------- consumers
        unsigned long long tm[4] = {0, 0, 0, 0};
        const unsigned long long t_start = FX_CYCLES_NOW();
        __syncthreads();
        vec8 wa[4], wb[4];
        int wa_at, wb_at;
        {   // weights of the first two offsets of the first item
            const int w_kappa_stride = nchunk * nslice * 4 * 64;
            const uint32_t m0 = (uint32_t)uni((int)L.meta[0].hdr.wave_mask[wave]);
            const uint32_t m1 = m0 & (m0 - 1);
            wa_at = w_frag(nslice, w_kappa_stride, (int)(first % nslice), 0, first_offset(m0));
            wb_at = m1 ? w_frag(nslice, w_kappa_stride, (int)(first % nslice), 0, first_offset(m1)) : wa_at;
            const vec8* w0 = reinterpret_cast<const vec8*>(wp) + lane;
#pragma unroll
            for (int f = 0; f < 4; ++f) { wa[f] = (w0 + wa_at)[f * 64]; wb[f] = (w0 + wb_at)[f * 64]; }
        }
        __syncthreads();
        int phase = 0, n_items = 0;
        for (int item_no = 0;; ++item_no, phase += nchunk) {
            const int slot = item_no % kMetaSlots;
            const MetaSlot& M = L.meta[slot];
            const int64_t work = slot_work(M);
            if (work < 0) break;
            const Item cur = item_of(M, work, nslice);
            if (cur.general) {
                consume_item_general<T, OUT_F32>(slot, phase, item_no & 1, item_no % 3, nchunk, nslice, wave, lane, tile_rows, row_stride,
                                                 feat, wp, pitch, C_out, out);
                wa_at = wb_at = -1;       // nothing is handed over a call
#pragma unroll
                for (int f = 0; f < 4; ++f) { wa[f] = vec8{}; wb[f] = vec8{}; }
            } else {
                consume_item<T, OUT_F32, false>(L, M, L.meta[(item_no + 1) % kMetaSlots], cur, phase, item_no & 1, item_no % 3, nchunk, nslice,
                                                wave, lane, tile_rows, row_stride, feat, wp, pitch, C_out, out, wa, wb, wa_at,
                                                wb_at, tm);
            }
            ++n_items;
        }
        // development builds: per-workgroup cycles of the first consumer wave (multiply, barrier waits, write-back, items)
        if (tid == 0) {
            FX_STAMP_VALUE(blockIdx.x, 0, tm[0]); FX_STAMP_VALUE(blockIdx.x, 1, tm[1]); FX_STAMP_VALUE(blockIdx.x, 2, tm[2]);
            FX_STAMP_VALUE(blockIdx.x, 3, FX_CYCLES_NOW() - t_start); FX_STAMP_VALUE(blockIdx.x, 4, (unsigned long long)n_items);
        }
        (void)t_start;
    }
}

// ---------------------------------------------------------------------------------- gather kernel
// For maps whose input rows are used (almost) once -- strided maps, where staging rows in LDS buys no
// reuse.  One wave owns one column block (32 outputs) x one 64-channel output slice for all
// offsets: it first resolves the block's (offset, voxel) -> input row table into LDS with independent
// loads, then walks the offsets, reading each lane's 16-byte A fragments straight from the feature
// rows (one step ahead) and the packed weights (the B operand, interleaved channels) from L2; a
// half-wave stores one output row's 64-channel slice in one piece.  No barriers, ~100 registers, so
// several waves per SIMD hide the gather latency.
constexpr int kGatherWaves = 4;

template <typename T, bool OUT_F32>
__global__ void __launch_bounds__(64 * kGatherWaves)
k_conv_gather(const TileHeader* __restrict__ tile_hdr, const uint16_t* __restrict__ tile_perm,
              const int32_t* __restrict__ tile_rows, int row_stride, const uint16_t* __restrict__ tile_blocks,
              int block_stride, int64_t n_items, const uint16_t* __restrict__ feat, const uint16_t* __restrict__ wp,
              int C_in, int C_out, void* __restrict__ out) {
    typedef typename Elem<T>::vec8 vec8;
    __shared__ int32_t row_of[kGatherWaves][kMaxK3Tiled][kGroup];
    __shared__ __align__(16) int32_t out_of[kGatherWaves][kGroup];      // the block's output rows within the tile (-1: none)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t item = (int64_t)blockIdx.x * kGatherWaves + wave;
    if (item >= n_items) return;
    const int nchunk = C_in / kCinChunk, nslice = C_out / kCoutSlice;
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
    if (h == 0) {
        const int local = tile_perm[tile * kTileT + g * kGroup + n];
        out_of[wave][n] = local < n_valid ? local : -1;
    }

    // (offset, voxel) -> global input row (-1: none); lane (n, h) resolves every second offset
    {
        const int flags = uni(H->flags), win_lo = uni(H->win_lo), win_n = uni(H->win_n);
        const size_t blk0 = (size_t)tile * block_stride + (uint32_t)uni((int)H->wave_block0[w]);
        const int32_t* rows = tile_rows + tile * (int64_t)row_stride;
        int rank = 0;
        for (uint32_t m = gm; m; m &= m - 1, ++rank) {
            if ((rank & 1) != h) continue;
            const int kappa = __ffs(m) - 1;
            const size_t blk = blk0 + __popc(wm & ((1u << kappa) - 1u));
            uint32_t id = tile_blocks[blk * kIdBlockElems + n * kGroupsPerWave + gi];
            if (flags & kTileLdsOffsets) id = (id / kRowBytes == (uint32_t)kRowCap) ? kNoRow : id / kRowBytes;
            int32_t r = -1;
            if (id != kNoRow) r = id < (uint32_t)win_n ? win_lo + (int32_t)id : rows[id - (uint32_t)win_n];
            row_of[wave][rank][n] = r;
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // a wave's LDS accesses are processed in order
    __builtin_amdgcn_wave_barrier();

    f32x16 acc[2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[mt][v] = 0.f;

    const int w_kappa_stride = nchunk * nslice * 4 * 64;
    const vec8* wl = reinterpret_cast<const vec8*>(wp) + lane;
    const int n_k = __popc(gm);
    const int n_steps = n_k * nchunk;            // step = (offset rank, chunk), chunk fastest
    vec8 zero;
#pragma unroll
    for (int e = 0; e < 8; ++e) zero[e] = 0;
    auto fetch = [&](vec8 (&b)[2], vec8 (&wf)[4], int step, uint32_t& rest, int& kappa) {
        const int rank = step / nchunk, c = step - rank * nchunk;
        if (c == 0) { kappa = __ffs(rest) - 1; rest &= rest - 1; }
        const int32_t r = row_of[wave][rank][n];
        b[0] = zero; b[1] = zero;
        if (r >= 0) {
            const uint16_t* src = feat + (int64_t)r * C_in + c * kCinChunk + h * 8;
            b[0] = *reinterpret_cast<const vec8*>(src);
            b[1] = *reinterpret_cast<const vec8*>(src + 16);
        }
        const vec8* ws = wl + w_frag(nslice, w_kappa_stride, slice, c, kappa);
#pragma unroll
        for (int f = 0; f < 4; ++f) wf[f] = ws[f * 64];
    };
    vec8 ba[2], bb[2], wa[4], wb[4];
    uint32_t rest = gm;
    int kappa = 0;
    if (n_steps > 0) fetch(ba, wa, 0, rest, kappa);
    for (int step = 0; step < n_steps; step += 2) {
        if (step + 1 < n_steps) fetch(bb, wb, step + 1, rest, kappa);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) acc[nt] = Elem<T>::mfma(ba[ks], wa[nt * 2 + ks], acc[nt]);
        if (step + 2 < n_steps) fetch(ba, wa, step + 2, rest, kappa);
        if (step + 1 < n_steps) {       // a guard, not an early exit: one loop exit keeps one copy of the accumulators
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int nt = 0; nt < 2; ++nt) acc[nt] = Elem<T>::mfma(bb[ks], wb[nt * 2 + ks], acc[nt]);
        }
    }

    // accumulator register v of lane (n, h) is voxel 8 * (v / 4) + 4 * h + v % 4 of the block, channels 2n and 2n + 1
    // of the slice (one per n-tile): the 32 lanes of a half-wave store one whole 64-channel row slice
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const i32x4 o4 = *reinterpret_cast<const i32x4*>(&out_of[wave][8 * q + 4 * h]);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (o4[j] < 0) continue;
            const int64_t at = (tile * kTileT + o4[j]) * C_out + (int64_t)slice * kCoutSlice + 2 * n;
            if (OUT_F32)
                *reinterpret_cast<f32x2*>(reinterpret_cast<float*>(out) + at) = f32x2{acc[0][4 * q + j], acc[1][4 * q + j]};
            else
                *reinterpret_cast<uint32_t*>(reinterpret_cast<uint16_t*>(out) + at) = Elem<T>::pack2(acc[0][4 * q + j], acc[1][4 * q + j]);
        }
    }
}

// ---------------------------------------------------------------------------------- gather kernel, weights in LDS
// k_conv_gather issues six vector loads per four multiplies, four of them for the weights, and
// is bound by the load path of the compute unit (one wave-wide 16-byte load occupies it for at
// least 16 cycles).  When the packed weights of one 64-channel output slice fit in LDS next to
// the row tables (K^3 * C_in * 128 bytes; 64 KB for a 2x2x2 kernel with 64 input channels), a
// persistent workgroup copies them there once, and each wave then walks column blocks with its
// weight fragments read from LDS: two vector loads per four multiplies.
// * When the weights of two adjacent slices fit together (NS = 2) a gathered fragment feeds the
//   multiplies of both and the gather is issued once per 128 output channels; that form runs twelve
//   waves with a third more registers (64 more accumulators).  With CP = 2 a step covers two
//   32-channel chunks, so its four loads use the whole 128-byte line of a 64-channel row while it
//   is in L1 instead of coming back for the second half a step later.
// * Operand roles: A = gathered rows (32 voxels x 16 input channels), B = packed weights in the
//   interleaved layout (column n of n-tile t = output channel 2n + t), so the output rows lie along
//   the accumulator registers and the channels across the lanes: a half-wave stores one output row's
//   64-channel slice as one contiguous piece.
// * What a block needs before its first gather hangs on a chain of dependent loads (tile header ->
//   id block -> row list), and so does its write-back (output permutation).  The chain is cut into
//   stages that run ahead: the header and permutation entry of block i + 2 are requested while block
//   i multiplies, the ids of block i + 1 before block i's step loop, and they are turned into the
//   row table after it.
// Workgroup b serves slice set b % (nslice / NS).  NS = output slices per workgroup, CP = 32-channel
// chunks per step, W = waves per workgroup, D = fragment sets in flight, R = offset ranks a lane half
// resolves (ceil(K^3 / 2)).
constexpr int kGatherLdsWaves = 16;
constexpr int kGatherPairWaves = 12;

template <typename T, bool OUT_F32, int NS, int CP, int W, int D, int R>
__global__ void __launch_bounds__(64 * W, 1)
k_conv_gather_ldsw(const TileHeader* __restrict__ tile_hdr, const uint16_t* __restrict__ tile_perm,
                   const int32_t* __restrict__ tile_rows, int row_stride, const uint16_t* __restrict__ tile_blocks,
                   int block_stride, int64_t n_blocks_total, int K3, const uint16_t* __restrict__ feat,
                   const uint16_t* __restrict__ wp, int C_in, int C_out, void* __restrict__ out) {
    typedef typename Elem<T>::vec8 vec8;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const int lane = threadIdx.x & 63, wave = uni((int)(threadIdx.x >> 6));
    const int nchunk = C_in / kCinChunk, nslice = C_out / kCoutSlice, nset = nslice / NS;
    const int npair = nchunk / CP;                                       // steps per offset (the launch checks CP | nchunk)
    const int slice = (blockIdx.x % nset) * NS;                          // first slice of this workgroup's set
    const int wg = blockIdx.x / nset, n_wg = gridDim.x / nset;           // the launch makes gridDim a multiple of nset
    unsigned char* wlds = lds_raw;                                       // [kappa][chunk][slice of the set][4 fragments][64 lanes][16 bytes]
    const int w_bytes = K3 * nchunk * NS * 4096;
    // per wave: [rank][voxel] global input rows of the current block, then [voxel] its output rows within the tile (-1: none)
    int32_t* tab = reinterpret_cast<int32_t*>(lds_raw + w_bytes) + wave * (K3 + 1) * kGroup;
    int32_t* out_of = tab + K3 * kGroup;

    for (int sl = wave; sl * 1024 < w_bytes; sl += W) {                  // 1 KB = one fragment of all lanes
        const int kc = sl / (4 * NS), sn = (sl >> 2) % NS, f = sl & 3;   // (kappa * nchunk + chunk), slice of the set, fragment
        const unsigned char* src = reinterpret_cast<const unsigned char*>(wp) + ((size_t)(kc * nslice + slice + sn) * 4 + f) * 1024 + lane * 16;
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
    // ids -> global input rows (a second load for ids outside the tile's window) and the voxels' output rows, into the
    // wave's table
    auto finish_table = [&](int64_t tg, const Hdr& d, const uint32_t (&idv)[R], int local) {
        const int32_t* rows = tile_rows + tg / kGroupsPerTile * (int64_t)row_stride;
        const int n_k = __popc(d.gm);
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const int rank = 2 * j + h;
            if (rank < n_k) {
                uint32_t id = idv[j];
                if (d.flags & kTileLdsOffsets) id = (id / kRowBytes == (uint32_t)kRowCap) ? kNoRow : id / kRowBytes;
                int32_t r = -1;
                if (id != kNoRow) r = id < (uint32_t)d.win_n ? d.win_lo + (int32_t)id : rows[id - (uint32_t)d.win_n];
                tab[rank * kGroup + n] = r;
            }
        }
        if (h == 0) out_of[n] = local < d.n_out ? local : -1;
    };

    Hdr h0 = load_hdr(tg0), h1 = load_hdr(tg0 + tg_stride);
    int p0 = load_perm(tg0), p1 = load_perm(tg0 + tg_stride);
    uint32_t idv[R];
#pragma unroll
    for (int j = 0; j < R; ++j) idv[j] = kNoRow;
    if (tg0 < n_blocks_total) {
        issue_ids(tg0, h0, idv);
        finish_table(tg0, h0, idv, p0);
    }
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();                       // the weights are in LDS

#pragma unroll 1
    for (int64_t tg = tg0; tg < n_blocks_total; tg += tg_stride) {
        const Hdr h2 = load_hdr(tg + 2 * tg_stride);
        const int p2 = load_perm(tg + 2 * tg_stride);
        const bool more = tg + tg_stride < n_blocks_total;
        if (more) issue_ids(tg + tg_stride, h1, idv);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // a wave's LDS accesses are processed in order
        __builtin_amdgcn_wave_barrier();

        const uint32_t gm = h0.gm;
        f32x16 acc[2 * NS];
#pragma unroll
        for (int t = 0; t < 2 * NS; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
        const int n_steps = __popc(gm) * npair;         // step = (offset rank, CP chunks), chunks fastest
        // A fragments of step `step` into b; returns where the step's B fragments start in LDS
        // fetches come in step order: (offset rank, chunk pair) advance with them
        int f_rank = -1, f_c = npair - 1;
        auto fetch = [&](vec8 (&b)[2 * CP], int step, uint32_t& rest, int& kappa) {
            if (++f_c == npair) { f_c = 0; ++f_rank; kappa = __ffs(rest | 0x80000000u) - 1; rest &= rest - 1; }
            const int32_t r = step < n_steps ? tab[f_rank * kGroup + n] : -1;
#pragma unroll
            for (int j = 0; j < 2 * CP; ++j) b[j] = zero;
            if (r >= 0) {
                const uint16_t* src = feat + (int64_t)r * C_in + f_c * (CP * kCinChunk) + h * 8;
#pragma unroll
                for (int j = 0; j < 2 * CP; ++j) b[j] = *reinterpret_cast<const vec8*>(src + 16 * j);
            }
            return (kappa * nchunk + f_c * CP) * NS * 4096 + lane * 16;
        };
        auto multiply = [&](const vec8 (&b)[2 * CP], int w_at) {
#pragma unroll
            for (int c = 0; c < CP; ++c)
#pragma unroll
                for (int sn = 0; sn < NS; ++sn) {
                    vec8 wf[4];
#pragma unroll
                    for (int f = 0; f < 4; ++f)
                        wf[f] = *reinterpret_cast<const vec8*>(wlds + w_at + (c * NS + sn) * 4096 + f * 1024);
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                        for (int nt = 0; nt < 2; ++nt)
                            acc[2 * sn + nt] = Elem<T>::mfma(b[2 * c + ks], wf[nt * 2 + ks], acc[2 * sn + nt]);
                }
        };
        // D fragment sets: the gathers of the next D - 1 steps are in flight while one multiplies.  The loop has one
        // exit and guards instead of breaks: with early exits between the multiplies the compiler kept a second
        // copy of the accumulators (80 registers more).
        vec8 ring[D][2 * CP];
        int w_at[D];
        uint32_t rest = gm;
        int kappa = 0;
#pragma unroll
        for (int d = 0; d < D - 1; ++d) { w_at[d] = 0; if (d < n_steps) w_at[d] = fetch(ring[d], d, rest, kappa); }
        w_at[D - 1] = 0;
#pragma unroll 1
        for (int step = 0; step < n_steps; step += D) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                if (step + d + D - 1 < n_steps) w_at[(d + D - 1) % D] = fetch(ring[(d + D - 1) % D], step + d + D - 1, rest, kappa);
                if (step + d < n_steps) multiply(ring[d], w_at[d]);
            }
        }

        // accumulator register v of lane (n, h) is voxel 8 * (v / 4) + 4 * h + v % 4 of the block, channels 2n and
        // 2n + 1 of a slice (one per n-tile): the 32 lanes of a half-wave store one whole 64-channel row slice
        const int64_t row0 = tg / kGroupsPerTile * kTileT;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const i32x4 o4 = *reinterpret_cast<const i32x4*>(out_of + 8 * q + 4 * h);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (o4[j] < 0) continue;
                const int64_t at = (row0 + o4[j]) * C_out + (int64_t)slice * kCoutSlice + 2 * n;
#pragma unroll
                for (int sn = 0; sn < NS; ++sn) {
                    if (OUT_F32)
                        *reinterpret_cast<f32x2*>(reinterpret_cast<float*>(out) + at + sn * kCoutSlice) =
                            f32x2{acc[2 * sn][4 * q + j], acc[2 * sn + 1][4 * q + j]};
                    else
                        *reinterpret_cast<uint32_t*>(reinterpret_cast<uint16_t*>(out) + at + sn * kCoutSlice) =
                            Elem<T>::pack2(acc[2 * sn][4 * q + j], acc[2 * sn + 1][4 * q + j]);
                }
            }
        }
        __builtin_amdgcn_wave_barrier();     // the table is rewritten for the next block
        if (more) finish_table(tg + tg_stride, h1, idv, p1);
        h0 = h1; h1 = h2; p0 = p1; p1 = p2;
    }
}

// ---------------------------------------------------------------------------------- scalar path
// One thread per (output voxel, output channel); fp32 FMA in offset-then-channel order.  Used
// for fp32 data (true fp32 products) and for channel counts the MFMA tiling does not cover.
template <int DT, bool OUT_F32>
__global__ void k_conv_scalar(const int32_t* __restrict__ nbmap, int64_t n_out, int K3, const void* __restrict__ feat,
                              const void* __restrict__ w, int C_in, int C_out, void* __restrict__ out, int mode) {
    const int64_t total = n_out * C_out;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const int64_t o = e / C_out;
        const int co = (int)(e - o * C_out);
        float acc = 0.f;
        for (int kappa = 0; kappa < K3; ++kappa) {
            const int32_t in = nbmap[o * K3 + kappa];
            if (in < 0) continue;
            const int64_t fb = (int64_t)in * C_in;
            // plain: W[kw][ci][co]; transposed (e.g. the input gradient on a symmetric map): W[kw][co][ci]
            const int64_t kw = (mode & kWeightsFlipped) ? K3 - 1 - kappa : kappa;
            const int64_t wb = (mode & kWeightsTransposed) ? (kw * C_out + co) * C_in : kw * C_in * C_out + co;
            const int64_t ws = (mode & kWeightsTransposed) ? 1 : C_out;
            for (int ci = 0; ci < C_in; ++ci)
                acc = fmaf(load_as_float<DT>(feat, fb + ci), load_as_float<DT>(w, wb + (int64_t)ci * ws), acc);
        }
        if (OUT_F32) reinterpret_cast<float*>(out)[e] = acc;
        else if (DT == FX_F16) reinterpret_cast<uint16_t*>(out)[e] = Elem<_Float16>::from_float(acc);
        else reinterpret_cast<uint16_t*>(out)[e] = Elem<__bf16>::from_float(acc);
    }
}

// The same sum with four output channels per thread and four input channels per load (channel
// counts that are multiples of 4): one 16-byte feature load and four 16-byte
// weight loads feed 16 multiply-adds, a sixth of the loads of the kernel above.  The sum over the
// input channels of one offset keeps the order ci = 0, 1, 2, ... of the one-channel kernel.
template <int DT, bool OUT_F32>
__global__ void k_conv_scalar4(const int32_t* __restrict__ nbmap, int64_t n_out, int K3, const void* __restrict__ feat,
                               const void* __restrict__ w, int C_in, int C_out, void* __restrict__ out, int mode) {
    const int q_out = C_out / 4;
    const int64_t total = n_out * q_out;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const int64_t o = e / q_out;
        const int co = (int)(e - o * q_out) * 4;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        for (int kappa = 0; kappa < K3; ++kappa) {
            const int32_t in = nbmap[o * K3 + kappa];
            if (in < 0) continue;
            const int64_t fb = (int64_t)in * C_in;
            const int64_t kw = (mode & kWeightsFlipped) ? K3 - 1 - kappa : kappa;
            if (!(mode & kWeightsTransposed)) {
                const int64_t wb = kw * C_in * C_out + co;
                for (int ci = 0; ci < C_in; ci += 4) {
                    const f32x4 x = load4_as_float<DT>(feat, fb + ci);
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const f32x4 wr = load4_as_float<DT>(w, wb + (int64_t)(ci + j) * C_out);
#pragma unroll
                        for (int v = 0; v < 4; ++v) acc[v] = fmaf(x[j], wr[v], acc[v]);
                    }
                }
            } else {   // W[kw][co][ci]: the four contracted channels of a produced channel are adjacent
                const int64_t wb = (kw * C_out + co) * C_in;
                for (int ci = 0; ci < C_in; ci += 4) {
                    const f32x4 x = load4_as_float<DT>(feat, fb + ci);
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const f32x4 wr = load4_as_float<DT>(w, wb + (int64_t)v * C_in + ci);
#pragma unroll
                        for (int j = 0; j < 4; ++j) acc[v] = fmaf(x[j], wr[j], acc[v]);
                    }
                }
            }
        }
        const int64_t at = o * C_out + co;
        if (OUT_F32) {
            *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(out) + at) = acc;
        } else if (DT == FX_F16) {
            *reinterpret_cast<u32x2*>(reinterpret_cast<uint16_t*>(out) + at) =
                u32x2{Elem<_Float16>::pack2(acc[0], acc[1]), Elem<_Float16>::pack2(acc[2], acc[3])};
        } else {
            *reinterpret_cast<u32x2*>(reinterpret_cast<uint16_t*>(out) + at) =
                u32x2{Elem<__bf16>::pack2(acc[0], acc[1]), Elem<__bf16>::pack2(acc[2], acc[3])};
        }
    }
}

template <typename T, bool OUT_F32>
static hipError_t launch_mfma(const fx_kmap* km, const void* feat, const void* wp, int32_t* counters, int C_in, int C_out,
                              void* out, hipStream_t st) {
    const size_t lds = sizeof(ConvLds);
    hipError_t e = hipFuncSetAttribute((const void*)k_conv_mfma<T, OUT_F32>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const int n_cu = compute_units();
    const int64_t n_work = km->n_tiles * (int64_t)((C_out + kCoutSlice - 1) / kCoutSlice);
    const int per_xcd = (int)((n_work + 7) / 8);
    // one workgroup per compute unit, a multiple of 8 (one share per XCD), no more than the work needs
    int grid = std::max(8, (n_cu / 8) * 8);
    grid = (int)std::min<int64_t>(grid, (int64_t)8 * per_xcd);
    k_conv_mfma<T, OUT_F32><<<grid, kConvThreads, lds, st>>>(km->d_tile_hdr, km->d_tile_perm, km->d_tile_rows,
                                                             km->row_stride, km->d_tile_blocks, km->block_stride, n_work,
                                                             per_xcd, counters, (const unsigned char*)feat,
                                                             (const unsigned char*)wp, C_in, C_out, out);
    return hipGetLastError();
}

// How the gather kernel with its weights in LDS would serve a map and shape: ns = 0 if it cannot (the weights of
// one 64-channel output slice and the waves' tables exceed 160 KB, or option gather_lds = 0), else the slices per
// workgroup (two when their weights fit together and option gather_lds is not 1), chunks per step, waves and the
// dynamic LDS bytes.  Maps with more than eight offsets take twelve waves (their tables are larger).
struct GatherLdsPlan { int ns, cp, waves; size_t lds; };
static GatherLdsPlan gather_lds_plan(const fx_kmap* km, int C_in, int C_out) {
    const int nslice = C_out / kCoutSlice, nchunk = C_in / kCinChunk;
    const size_t w_slice = (size_t)km->K3 * nchunk * 4096;                   // packed weights of one output slice
    auto tables = [&](int waves) { return (size_t)waves * (km->K3 + 1) * kGroup * sizeof(int32_t); };
    GatherLdsPlan p = {0, 1, 0, 0};
    if (option(kOptGatherLds) == 0 || km->K3 > 27) return p;
    if (km->K3 <= 8 && nslice % 2 == 0 && 2 * w_slice + tables(kGatherPairWaves) <= 160 * 1024 && option(kOptGatherLds) != 1) {
        p.ns = 2; p.cp = nchunk % 2 == 0 ? 2 : 1; p.waves = kGatherPairWaves;
    } else if (km->K3 <= 8 && w_slice + tables(kGatherLdsWaves) <= 160 * 1024) {
        p.ns = 1; p.waves = kGatherLdsWaves;
    } else if (km->K3 > 8 && w_slice + tables(kGatherPairWaves) <= 160 * 1024) {
        p.ns = 1; p.waves = kGatherPairWaves;
    }
    p.lds = p.ns * w_slice + tables(p.waves);
    return p;
}

template <typename T, bool OUT_F32>
static hipError_t launch_gather(const fx_kmap* km, const void* feat, const void* wp, int C_in, int C_out, void* out,
                                hipStream_t st) {
    const GatherLdsPlan plan = gather_lds_plan(km, C_in, C_out);
    if (plan.ns) {
        const int ns = plan.ns, cp = plan.cp, waves = plan.waves;
        const int nslice = C_out / kCoutSlice;
        const bool few = km->K3 <= 8;            // ranks per lane half: 4, else 14
        const int64_t n_blocks_total = km->n_tiles * (int64_t)kGroupsPerTile;
        // one workgroup per compute unit, a multiple of the number of slice sets, no more than there is work for
        const int nset = nslice / ns;
        int64_t grid = std::max(nset, compute_units() / nset * nset);
        grid = std::min<int64_t>(grid, (n_blocks_total + waves - 1) / waves * nset);
#define FX_GATHER_LDSW(NS_, CP_, W_, D_, R_)                                                                             \
        if (ns == NS_ && cp == CP_ && waves == W_ && few == (R_ == 4)) {                                                 \
            hipError_t e = hipFuncSetAttribute((const void*)k_conv_gather_ldsw<T, OUT_F32, NS_, CP_, W_, D_, R_>,        \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)plan.lds);              \
            if (e != hipSuccess) return e;                                                                               \
            k_conv_gather_ldsw<T, OUT_F32, NS_, CP_, W_, D_, R_><<<(unsigned)grid, 64 * W_, plan.lds, st>>>(             \
                km->d_tile_hdr, km->d_tile_perm, km->d_tile_rows, km->row_stride, km->d_tile_blocks, km->block_stride,   \
                n_blocks_total, km->K3, (const uint16_t*)feat, (const uint16_t*)wp, C_in, C_out, out);                   \
            return hipGetLastError();                                                                                    \
        }
        // measured at config 4 (64 -> 128) before the staged look-ahead: 58 us for (2, 2, 12 waves, 3 sets), 58-59
        // for 8 waves with 2 to 4 sets, 63-64 for one chunk per step, 79-81 for one slice per workgroup
        FX_GATHER_LDSW(1, 1, kGatherLdsWaves, 4, 4) FX_GATHER_LDSW(1, 1, kGatherPairWaves, 2, 14)
        FX_GATHER_LDSW(2, 1, kGatherPairWaves, 4, 4) FX_GATHER_LDSW(2, 2, kGatherPairWaves, 3, 4)
#undef FX_GATHER_LDSW
        return hipErrorInvalidValue;
    }
    const int64_t n_items = km->n_tiles * (int64_t)kGroupsPerTile * (C_out / kCoutSlice);
    const unsigned grid = (unsigned)((n_items + kGatherWaves - 1) / kGatherWaves);
    k_conv_gather<T, OUT_F32><<<grid, 64 * kGatherWaves, 0, st>>>(km->d_tile_hdr, km->d_tile_perm, km->d_tile_rows,
                                                                 km->row_stride, km->d_tile_blocks, km->block_stride,
                                                                 n_items, (const uint16_t*)feat, (const uint16_t*)wp,
                                                                 C_in, C_out, out);
    return hipGetLastError();
}

}  // namespace fx

using namespace fx;

FX_DEV_TIMING_EXPORT(fx_debug_conv_timing)



// Device memory the matrix-unit kernels need beyond inputs and outputs: the packed weights and, behind them, the
// eight work-list counters of the persistent kernel.
static size_t conv_scratch_bytes(int K3, int C_in, int C_out, int esize) {
    return packed_weight_bytes(K3, C_in, C_out, esize) + 8 * sizeof(int32_t);    // the packed part is a multiple of 64 bytes
}

// The tiled map's convolution on the matrix units with that memory supplied by the caller (`scratch`, at least
// conv_scratch_bytes, 16-byte aligned): pack the weights (which also clears the counters), then the LDS-staged
// kernel or, for maps whose tiles list one row per pair, the gather kernel.  Allocates nothing.
static fx_status conv_tiles_with_scratch(const fx_kmap* km, const void* d_feat, fx_dtype in_dt, const void* d_w, int32_t C_in,
                                         int32_t C_out, void* d_out, fx_dtype out_dt, hipStream_t st, int mode, void* scratch) {
    const bool out_f32 = (out_dt == FX_F32);
    const int esize = in_dt == FX_F32 ? 4 : 2;
    void* wp = scratch;
    const size_t wbytes = packed_weight_bytes(km->K3, C_in, C_out, esize);
    int32_t* counters = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(wp) + wbytes);
    // maps whose tiles list one row per pair (strided; stride 1 back from a larger grid): the gather kernel;
    // others: the LDS-staged kernel
    const int fg = option(kOptConvGather);          // 0 / 1: the LDS-staged / the gather kernel on every map
    const bool gather = (fg >= 0 ? fg == 1 : !map_shares_rows(km)) && in_dt != FX_F32 && C_out % kCoutSlice == 0;
    launch_pack_weights(d_w, wp, km->K3, C_in, C_out, esize, counters, mode, st);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && gather) {
        ProfScope ps(kProfConvGather, st);
        if (in_dt == FX_BF16)
            e = out_f32 ? launch_gather<__bf16, true>(km, d_feat, wp, C_in, C_out, d_out, st)
                        : launch_gather<__bf16, false>(km, d_feat, wp, C_in, C_out, d_out, st);
        else
            e = out_f32 ? launch_gather<_Float16, true>(km, d_feat, wp, C_in, C_out, d_out, st)
                        : launch_gather<_Float16, false>(km, d_feat, wp, C_in, C_out, d_out, st);
    } else if (e == hipSuccess) {
        ProfScope ps(kProfConvMfma, st);
        if (in_dt == FX_F32)
            e = launch_mfma<float, true>(km, d_feat, wp, counters, C_in, C_out, d_out, st);
        else if (in_dt == FX_BF16)
            e = out_f32 ? launch_mfma<__bf16, true>(km, d_feat, wp, counters, C_in, C_out, d_out, st)
                        : launch_mfma<__bf16, false>(km, d_feat, wp, counters, C_in, C_out, d_out, st);
        else
            e = out_f32 ? launch_mfma<_Float16, true>(km, d_feat, wp, counters, C_in, C_out, d_out, st)
                        : launch_mfma<_Float16, false>(km, d_feat, wp, counters, C_in, C_out, d_out, st);
    }
    if (e != hipSuccess) { set_error("convolution launch failed: %s", hipGetErrorString(e)); return FX_EDEVICE; }
    return FX_OK;
}

// whether the matrix-unit kernels take this map and shape at all (the size heuristics of conv_apply aside)
static bool conv_tiles_shape_ok(const fx_kmap* km, fx_dtype in_dt, int C_in, int C_out) {
    const int esize = in_dt == FX_F32 ? 4 : 2;
    return km->n_tiles > 0 && ((int64_t)C_in * esize) % kRowBytes == 0 && C_out % 2 == 0;
}

fx_status fx::conv_apply(const fx_kmap* km, const void* d_feat, fx_dtype in_dt, const void* d_w, int32_t C_in,
                         int32_t C_out, void* d_out, fx_dtype out_dt, hipStream_t st, int mode) {
    const bool out_f32 = (out_dt == FX_F32);
    const bool force_scalar = option(kOptForceScalar) == 1;
    // Locally dense grids (Sec. 3.5 scenarios 1-2): on a 3x3x3 stride-1 map the leaf-window kernels compute the same
    // sum from the grid alone and are faster once the leaves are full enough -- the tiles of such a map need more
    // rows than the tile kernel's LDS holds -- and, at fp32 depths that the tile kernel does not take, almost
    // everywhere.  Option leaf_dispatch = 0 keeps the kernel-map kernels, = 1 takes the leaf kernels whenever
    // they serve the shape.
    if (km->K == 3 && km->stride == 1 && km->gin == km->gout && (mode == kWeightsForward || mode == kWeightsMirrored) &&
        leaf_shape_supported(in_dt, C_in, C_out) && !force_scalar) {
        const int ld = option(kOptLeafDispatch);
        const double occupancy = (double)km->n_in / (512.0 * (double)std::max<int64_t>(1, km->gin->hdr.n_leaf));
        // Per-leaf dispatch: a grid that mixes locally dense leaves (solid bodies) with sparse ones (thin surfaces,
        // scan lines) is split inside this one call -- the leaves with at least kDenseLeafVoxels voxels go to the
        // leaf-window kernel, the outputs of all other leaves to the tile kernel over a copy of the map that leaves
        // the dense leaves' outputs out.  Taken when the grid as a whole is too sparse for the leaf-window kernel
        // (mean occupancy below 0.40) but at least 10 % of its voxels sit in dense leaves; leaf_dispatch = 2 forces it.
        if (in_dt != FX_F32 && !km->is_inverse) {
            const double dense = (double)km->gin->hdr.n_voxels_dense / (double)std::max<int64_t>(1, km->n_in);
            if (ld == 2 || (ld < 0 && occupancy < 0.40 && dense >= 0.10)) {
                fx_kmap* kmw = const_cast<fx_kmap*>(km);
                FX_TRY(kmap_ensure_mixed(kmw, st));
                void* wp = nullptr;
                FX_TRY(dev_alloc(&wp, conv_scratch_bytes(27, C_in, C_out, 2), st));
                fx_status rc = conv_tiles_with_scratch(km->mixed, d_feat, in_dt, d_w, C_in, C_out, d_out, out_dt, st, mode, wp);
                dev_free(wp, st);
                if (rc != FX_OK) return rc;
                return leaf_apply("sparse convolution (per-leaf dispatch)", km->gin, d_feat, in_dt, d_w, C_in, C_out, d_out, out_dt, st,
                                  mode, km->mixed->d_dense_leaves, km->mixed->d_n_dense);
            }
        }
        const bool scalar_otherwise = in_dt == FX_F32 && C_in % 16 != 0;
        const bool take = ld >= 0 ? ld >= 1 : occupancy >= (scalar_otherwise ? 0.08 : 0.40);
        if (take)
            return leaf_apply("sparse convolution (leaf-window kernels)", km->gin, d_feat, in_dt, d_w, C_in, C_out, d_out, out_dt,
                              st, mode);
    }
    const int esize = in_dt == FX_F32 ? 4 : 2;
    // The tile kernel takes input rows in 64-byte chunks (32 channels of a 16-bit type, 16 of fp32) and
    // pads the produced channels to 64 with zero weights; the gather kernel for strided maps needs whole
    // 64-channel slices of a 16-bit type.  Everything else is left to the scalar kernel.
    // fp32 multiplies at 1/16 of the 16-bit rate on the matrix units, so a grid of few tiles (one
    // workgroup each) is served faster by the scalar kernel spread over the whole chip
    const int64_t n_items = km->n_tiles * (int64_t)((C_out + kCoutSlice - 1) / kCoutSlice);
    const bool mfma = conv_tiles_shape_ok(km, in_dt, C_in, C_out) &&
                      (in_dt != FX_F32 || n_items >= compute_units() / 2 || option(kOptFp32Tiles) == 1) &&   // fp32_tiles = 1: at any size
                      !force_scalar;
    if (mfma) {
        void* wp = nullptr;
        FX_TRY(dev_alloc(&wp, conv_scratch_bytes(km->K3, C_in, C_out, esize), st));
        const fx_status rc = conv_tiles_with_scratch(km, d_feat, in_dt, d_w, C_in, C_out, d_out, out_dt, st, mode, wp);
        dev_free(wp, st);
        return rc;
    }
    FX_TRY(kmap_ensure_dense(const_cast<fx_kmap*>(km), st));
    return conv_scalar_on_table(km->d_nbmap, km->n_out, km->K3, d_feat, in_dt, d_w, C_in, C_out, d_out, out_dt, st, mode);
}

fx_status fx::conv_scalar_on_table(const int32_t* d_table, int64_t n_rows, int K3, const void* d_feat, fx_dtype in_dt,
                                   const void* d_w, int32_t C_in, int32_t C_out, void* d_out, fx_dtype out_dt, hipStream_t st,
                                   int mode) {
    const bool out_f32 = (out_dt == FX_F32);
    const bool four = C_in % 4 == 0 && C_out % 4 == 0;
    const int64_t total = n_rows * (four ? C_out / 4 : C_out);
    const size_t w_lds = sizeof(float) * (size_t)K3 * C_in * C_out;
    const bool lds_w = four && w_lds <= 32 * 1024 && total >= 8 * 1024 && option(kOptScalarLds) != 0;   // scalar_lds = 0: weights from L1
    const unsigned nb = lds_w ? (unsigned)std::max<int64_t>(1, std::min<int64_t>((total + 255) / 256, (int64_t)compute_units() * 8))
                              : (unsigned)std::max<int64_t>(1, std::min<int64_t>((total + 255) / 256, 1 << 20));
#define FX_SCALAR(DT)                                                                                            \
    do {                                                                                                         \
        if (lds_w && out_f32) k_conv_scalar4_ldsw<DT, true, 1><<<nb, 256, w_lds, st>>>(d_table, n_rows, K3, d_feat, \
                                                                                       d_w, C_in, C_out, d_out, mode); \
        else if (lds_w) k_conv_scalar4_ldsw<DT, false, 1><<<nb, 256, w_lds, st>>>(d_table, n_rows, K3, d_feat, d_w, \
                                                                                  C_in, C_out, d_out, mode);     \
        else if (four && out_f32) k_conv_scalar4<DT, true><<<nb, 256, 0, st>>>(d_table, n_rows, K3, d_feat,      \
                                                                          d_w, C_in, C_out, d_out, mode);        \
        else if (four) k_conv_scalar4<DT, false><<<nb, 256, 0, st>>>(d_table, n_rows, K3, d_feat, d_w,           \
                                                                     C_in, C_out, d_out, mode);                  \
        else if (out_f32) k_conv_scalar<DT, true><<<nb, 256, 0, st>>>(d_table, n_rows, K3, d_feat, d_w,          \
                                                                      C_in, C_out, d_out, mode);                 \
        else k_conv_scalar<DT, false><<<nb, 256, 0, st>>>(d_table, n_rows, K3, d_feat, d_w, C_in,                \
                                                          C_out, d_out, mode);                                   \
    } while (0)
    ProfScope ps(kProfConvScalar, st);
    if (in_dt == FX_F32) FX_SCALAR(FX_F32);
    else if (in_dt == FX_F16) FX_SCALAR(FX_F16);
    else FX_SCALAR(FX_BF16);
#undef FX_SCALAR
    FX_HIP_TRY(hipGetLastError());
    return FX_OK;
}

extern "C" fx_status fx_sparse_conv_fwd(const fx_kmap* km, const void* d_feat, fx_dtype in_dt, const void* d_w,
                                        int32_t C_in, int32_t C_out, void* d_out, fx_dtype out_dt, void* stream) {
    if (!km || !d_w || C_in < 1 || C_out < 1 || (km->n_in > 0 && !d_feat) || (km->n_out > 0 && !d_out)) {
        set_error("fx_sparse_conv_fwd: null pointer or non-positive channel count");
        return FX_EINVAL;
    }
    if (in_dt != FX_F32 && in_dt != FX_F16 && in_dt != FX_BF16) { set_error("unknown input dtype"); return FX_EINVAL; }
    if (out_dt != in_dt && out_dt != FX_F32) {
        set_error("output dtype must equal the input dtype or be fp32");
        return FX_EUNSUPPORTED;
    }
    if (km->n_out == 0) return FX_OK;
    return conv_apply(km, d_feat, in_dt, d_w, C_in, C_out, d_out, out_dt, (hipStream_t)stream, kWeightsForward);
}

// ---------------------------------------------------------------------------------- no allocation
// fx_sparse_conv_fwd for callers that cannot allocate device memory (under graph capture, in tight serving loops):
// the packed weights and the work-list counters live in a file-scope device array instead of an allocation.
// The array's name stands for the symbol in host code; its device address is looked up once per device and only
// that address is ever handed to kernels.
namespace {
constexpr size_t kNoAllocScratchBytes = FX_NOALLOC_MAX_WEIGHT_BYTES + 256;
__device__ __align__(256) unsigned char scratch[kNoAllocScratchBytes];
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];
std::atomic<bool> g_scratch_ready[kMaxDevices];
std::mutex g_scratch_mu;
}  // namespace

// Device address of the scratch array on the current device (looked up on first use per device).
fx_status fx::conv_noalloc_setup(void** out_ptr) {
    int dev = 0;
    FX_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) { set_error("device ordinal %d out of range", dev); return FX_EDEVICE; }
    if (!g_scratch_ready[dev].load(std::memory_order_acquire)) {
        std::lock_guard<std::mutex> lock(g_scratch_mu);
        if (!g_scratch_ready[dev].load(std::memory_order_relaxed)) {
            void* ptr = nullptr;
            FX_HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
            if (!ptr) { set_error("hipGetSymbolAddress returned a null address"); return FX_EDEVICE; }
            g_scratch_ptr[dev] = ptr;
            g_scratch_ready[dev].store(true, std::memory_order_release);
        }
    }
    if (out_ptr) *out_ptr = g_scratch_ptr[dev];
    return FX_OK;
}

extern "C" fx_status fx_sparse_conv_fwd_noalloc(const fx_kmap* km, const void* d_feat, fx_dtype in_dt, const void* d_w,
                                                int32_t C_in, int32_t C_out, void* d_out, fx_dtype out_dt, void* stream) {
    if (!km || !d_w || C_in < 1 || C_out < 1 || (km->n_in > 0 && !d_feat) || (km->n_out > 0 && !d_out)) {
        set_error("fx_sparse_conv_fwd_noalloc: null pointer or non-positive channel count");
        return FX_EINVAL;
    }
    if (in_dt != FX_F32 && in_dt != FX_F16 && in_dt != FX_BF16) { set_error("unknown input dtype"); return FX_EINVAL; }
    if (out_dt != in_dt && out_dt != FX_F32) {
        set_error("output dtype must equal the input dtype or be fp32");
        return FX_EUNSUPPORTED;
    }
    if (km->n_out == 0) return FX_OK;
    if (!conv_tiles_shape_ok(km, in_dt, C_in, C_out)) {
        set_error("fx_sparse_conv_fwd_noalloc: only maps and shapes of the matrix-unit kernels (a tiled map, input rows in whole "
                  "64-byte chunks, an even number of output channels); K = %d, C_in = %d, C_out = %d is not", km->K, C_in, C_out);
        return FX_EUNSUPPORTED;
    }
    const size_t need = conv_scratch_bytes(km->K3, C_in, C_out, in_dt == FX_F32 ? 4 : 2);
    if (need > kNoAllocScratchBytes) {
        set_error("fx_sparse_conv_fwd_noalloc: the packed weights need %zu bytes, the static buffer holds %zu "
                  "(FX_NOALLOC_MAX_WEIGHT_BYTES)", need, kNoAllocScratchBytes);
        return FX_ERANGE;
    }
    void* ptr = nullptr;
    FX_TRY(conv_noalloc_setup(&ptr));
    return conv_tiles_with_scratch(km, d_feat, in_dt, d_w, C_in, C_out, d_out, out_dt, (hipStream_t)stream, kWeightsForward, ptr);
}
