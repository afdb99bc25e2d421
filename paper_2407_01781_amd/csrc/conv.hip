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
// Operand roles: A = packed weights (32 output channels x 16 input channels per instruction),
// B = gathered features (16 input channels x 32 voxels), D = 32 channels x 32 voxels; the
// weight rows are permuted so that each lane ends up with 32 consecutive output channels of
// one voxel.
#include "kmap.h"

#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include <algorithm>

namespace fx {

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kCoutSlice = 64;      // output channels per wave
constexpr int kConvThreads = 64 * kTileWaves;
constexpr int kMaxIdBlocks = kTileWaves * kMaxK3Tiled;

// ---------------------------------------------------------------------------------- element types
template <typename T> struct Elem;
template <> struct Elem<__bf16> {
    typedef bf16x8 vec8;
    static __device__ __forceinline__ f32x16 mfma(vec8 a, vec8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ float to_float(uint16_t bits) { return __uint_as_float((uint32_t)bits << 16); }
    static __device__ __forceinline__ uint16_t from_float(float f) {  // round to nearest even
        uint32_t u = __float_as_uint(f);
        if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40);
        u += 0x7FFFu + ((u >> 16) & 1u);
        return (uint16_t)(u >> 16);
    }
    static __device__ __forceinline__ uint32_t pack2(float a, float b) {  // two RNE conversions, a in the low half
        typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
        typedef __attribute__((ext_vector_type(2))) float f32x2;
        const bf16x2 h = __builtin_convertvector(f32x2{a, b}, bf16x2);
        uint32_t bits;
        __builtin_memcpy(&bits, &h, 4);
        return bits;
    }
};
template <> struct Elem<_Float16> {
    typedef f16x8 vec8;
    static __device__ __forceinline__ f32x16 mfma(vec8 a, vec8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ float to_float(uint16_t bits) {
        _Float16 h;
        __builtin_memcpy(&h, &bits, 2);
        return (float)h;
    }
    static __device__ __forceinline__ uint16_t from_float(float f) {
        _Float16 h = (_Float16)f;  // v_cvt_f16_f32: round to nearest even
        uint16_t bits;
        __builtin_memcpy(&bits, &h, 2);
        return bits;
    }
    static __device__ __forceinline__ uint32_t pack2(float a, float b) {
        return (uint32_t)from_float(a) | ((uint32_t)from_float(b) << 16);
    }
};

// ---------------------------------------------------------------------------------- weight packing
// Wp[kappa][cin chunk][cout slice][mtile 0..1][kstep 0..1][lane 0..63][8]: the 16-byte A-operand
// fragment of each lane for one (offset, 32 input channels, 64 output channels).  A-row m of
// m-tile t holds output channel 32*((m>>2)&1) + 16*t + 4*(m>>3) + (m&3) of the slice: with the
// 32x32 accumulator layout (lane half h, register v -> row 8*(v/4) + 4*h + v%4) a lane's
// accumulators are then the 32 consecutive channels 32*h .. 32*h+31 (m-tile t = channels
// 32*h + 16*t + v).
__global__ void k_pack_weights(const uint16_t* __restrict__ w, uint16_t* __restrict__ wp, int K3, int C_in, int C_out) {
    const int64_t total = (int64_t)K3 * C_in * C_out;
    const int nchunk = C_in / kCinChunk, nslice = C_out / kCoutSlice;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        int64_t r = e;
        const int el = (int)(r & 7); r >>= 3;
        const int lane = (int)(r & 63); r >>= 6;
        const int ks = (int)(r & 1); r >>= 1;
        const int mt = (int)(r & 1); r >>= 1;
        const int s = (int)(r % nslice); r /= nslice;
        const int c = (int)(r % nchunk); r /= nchunk;
        const int kappa = (int)r;
        const int m = lane & 31, kq = lane >> 5;
        const int cin = c * kCinChunk + ks * 16 + kq * 8 + el;
        const int cout = s * kCoutSlice + 32 * ((m >> 2) & 1) + 16 * mt + 4 * (m >> 3) + (m & 3);
        wp[e] = w[((int64_t)kappa * C_in + cin) * C_out + cout];
    }
}

#ifdef FX_CONV_TIMING
// development aid: per-workgroup phase timestamps (thread 0), read back with fx_debug_conv_timing
__device__ unsigned long long g_conv_timing[4096 * 8];
#define FX_STAMP(slot) do { if (tid == 0 && tile < 4096) g_conv_timing[tile * 8 + (slot)] = __builtin_readcyclecounter(); } while (0)
#else
#define FX_STAMP(slot) do { } while (0)
#endif

// ---------------------------------------------------------------------------------- MFMA kernel
struct ConvLds {
    unsigned char rows[(kRowCap + 1) * kRowBytes];  // 64-byte rows; 16-byte chunk q stored at q ^ ((row >> 2) & 3)
    uint16_t blocks[kMaxIdBlocks * kIdBlockElems];  // id blocks [block][voxel n][group slot]
    uint16_t perm[kTileT];
};

__device__ __forceinline__ int lds_row_offset(int row, int q) { return (int)(lds_row_code((uint32_t)row) ^ (uint32_t)(q << 4)); }

// Loop over the stencil offsets a wave needs for one 32-channel chunk.  Per offset: the ids of
// the lane's voxel column in the wave's 4 column blocks arrive with one 8-byte LDS read (fetched
// one offset ahead), the B fragments of the present column blocks are read (2 x 16 bytes per
// lane), then 4 MFMAs (2 m-tiles x 2 k-steps) per present block.  GENERAL adds the fallback for
// rows that are not staged in LDS.
template <typename T, bool GENERAL>
__device__ __forceinline__ void offsets_loop(const ConvLds& L, f32x16 (&acc)[kGroupsPerWave][2],
                                             const uint32_t (&gmask)[kGroupsPerWave], uint32_t wave_mask,
                                             int wave_block0, const typename Elem<T>::vec8* __restrict__ wbase,
                                             int64_t w_kappa_stride, int n, int h, int n_staged, int win_lo, int win_n,
                                             const int32_t* __restrict__ my_rows, const uint16_t* __restrict__ feat,
                                             int C_in, int c) {
    typedef typename Elem<T>::vec8 vec8;
    constexpr int NG = kGroupsPerWave;
    // The wave's offsets in ascending order.  Weights run two offsets ahead of the multiply in a
    // ring of three register sets (the loop is unrolled by three so that no set is ever copied);
    // ids run one offset ahead.  Steps past the last offset use offset 31, which no group has.
    const int n_off = __popc(wave_mask);
    const int k_last = 31 - __clz(wave_mask);
    const u32x2* idp = reinterpret_cast<const u32x2*>(L.blocks) + (size_t)wave_block0 * kGroup + n;
    uint32_t rest = wave_mask;            // offsets not yet fetched
    auto pop_kappa = [&]() {
        if (!rest) return 31;
        const int k = __ffs(rest) - 1;
        rest &= rest - 1;
        return k;
    };
    auto fetch_w = [&](vec8 (&w)[4], int k) {   // [mtile*2 + kstep]
        const vec8* ws = wbase + (int64_t)min(k, k_last) * w_kappa_stride;
#pragma unroll
        for (int f = 0; f < 4; ++f) w[f] = ws[f * 64];
    };
    vec8 w0[4], w1[4], w2[4];
    u32x2 idv = idp[0], idn;
    int ka = pop_kappa(), kb = pop_kappa(), it = 0;
    fetch_w(w0, ka);
    fetch_w(w1, kb);
    // one step: fetch the weights of the offset two ahead into `wfill`, multiply offset `kappa` with `wcur`
    auto step = [&](const vec8 (&wcur)[4], vec8 (&wfill)[4], int kappa, int k_fill) {
        fetch_w(wfill, k_fill);
        idn = idp[min(it + 1, n_off - 1) * kGroup];
        vec8 bf[NG][2];
#pragma unroll
        for (int gi = 0; gi < NG; ++gi) {
            if (!((gmask[gi] >> kappa) & 1u)) continue;
            const uint32_t id = (idv[gi >> 1] >> (16 * (gi & 1))) & 0xFFFFu;
            if (GENERAL) {
                const bool staged = id < (uint32_t)n_staged;
                const int row = staged ? (int)id : kRowCap;
                bf[gi][0] = *reinterpret_cast<const vec8*>(L.rows + lds_row_offset(row, h));
                bf[gi][1] = *reinterpret_cast<const vec8*>(L.rows + lds_row_offset(row, h + 2));
                const bool from_global = !staged && id != kNoRow;
                if (__any(from_global)) {
                    if (from_global) {
                        const int64_t gr = id < (uint32_t)win_n ? (int64_t)win_lo + id : (int64_t)my_rows[id - win_n];
                        const uint16_t* src = feat + gr * C_in + c * kCinChunk + h * 8;
                        bf[gi][0] = *reinterpret_cast<const vec8*>(src);
                        bf[gi][1] = *reinterpret_cast<const vec8*>(src + 16);
                    }
                }
            } else {   // id = lds_row_code(row): 16-byte piece p of the row sits at id ^ (p << 4)
                bf[gi][0] = *reinterpret_cast<const vec8*>(L.rows + (id ^ (uint32_t)(h << 4)));
                bf[gi][1] = *reinterpret_cast<const vec8*>(L.rows + (id ^ (uint32_t)((h + 2) << 4)));
            }
        }
#pragma unroll
        for (int gi = 0; gi < NG; ++gi) {
            if (!((gmask[gi] >> kappa) & 1u)) continue;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) acc[gi][mt] = Elem<T>::mfma(wcur[mt * 2 + ks], bf[gi][ks], acc[gi][mt]);
        }
        idv = idn;
        ++it;
    };
    while (it < n_off) {
        int kc = pop_kappa();
        step(w0, w2, ka, kc);
        ka = pop_kappa();
        step(w1, w0, kb, ka);
        kb = pop_kappa();
        step(w2, w1, kc, kb);
    }
}

// stage channels [32c, 32c+32) of the tile's input rows: 4 lanes x 16 bytes per row
__device__ __forceinline__ void stage_rows(ConvLds& L, int tid, int n_staged, int win_lo, int win_n,
                                           const int32_t* __restrict__ my_rows, const uint16_t* __restrict__ feat,
                                           int C_in, int c) {
    const int sub = tid & 3;
    for (int r0 = tid >> 2; r0 < n_staged; r0 += 64 * 4) {
        u32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int r = r0 + 64 * u;
            if (r < n_staged) {
                const int64_t gr = r < win_n ? (int64_t)win_lo + r : (int64_t)my_rows[r - win_n];
                v[u] = *reinterpret_cast<const u32x4*>(feat + gr * C_in + c * kCinChunk + sub * 8);
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int r = r0 + 64 * u;
            if (r < n_staged) *reinterpret_cast<u32x4*>(L.rows + lds_row_offset(r, sub)) = v[u];
        }
    }
}

// Everything a workgroup does once the tile header is known: stage, multiply, write back.
template <typename T, bool OUT_F32, bool GENERAL>
__device__ __forceinline__ void tile_body(ConvLds& L, const TileHeader* __restrict__ H, int64_t tile, int slice, int tid,
                                          const uint16_t* __restrict__ tile_perm, const int32_t* __restrict__ my_rows,
                                          const uint16_t* __restrict__ my_blocks, const uint16_t* __restrict__ feat,
                                          const uint16_t* __restrict__ wp, int C_in, int C_out, void* __restrict__ out) {
    typedef typename Elem<T>::vec8 vec8;
    constexpr int NG = kGroupsPerWave;
    const int lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, h = lane >> 5;
    const int nchunk = C_in / kCinChunk, nslice = C_out / kCoutSlice;
    const int win_lo = H->win_lo, win_n = H->win_n, n_list = H->n_list;
    const int n_blocks = H->n_blocks, n_valid = H->n_out;
    const int n_staged = (H->flags & kTileDirect) ? 0 : min(win_n + n_list, kRowCap);

    // tile metadata and the first chunk of rows -> LDS
    for (int e = tid; e < kTileT; e += kConvThreads) L.perm[e] = tile_perm[tile * kTileT + e];
    {
        const u32x4* src = reinterpret_cast<const u32x4*>(my_blocks);
        u32x4* dst = reinterpret_cast<u32x4*>(L.blocks);
        const int nb16 = n_blocks * (kIdBlockElems * 2 / 16);
        for (int e = tid; e < nb16; e += kConvThreads) dst[e] = src[e];
    }
    if (tid < kRowBytes / 16) reinterpret_cast<u32x4*>(L.rows + kRowCap * kRowBytes)[tid] = u32x4{0, 0, 0, 0};
    stage_rows(L, tid, n_staged, win_lo, win_n, my_rows, feat, C_in, 0);

    uint32_t gmask[NG];
#pragma unroll
    for (int gi = 0; gi < NG; ++gi) gmask[gi] = __builtin_amdgcn_readfirstlane(H->group_mask[tile_group_of(wave, gi)]);
    const uint32_t wave_mask = __builtin_amdgcn_readfirstlane(H->wave_mask[wave]);
    const int wave_block0 = __builtin_amdgcn_readfirstlane(H->wave_block0[wave]);

    f32x16 acc[NG][2];
#pragma unroll
    for (int gi = 0; gi < NG; ++gi)
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[gi][mt][v] = 0.f;
    FX_STAMP(1);

    for (int c = 0; c < nchunk; ++c) {
        if (c > 0) {
            __syncthreads();  // all waves are done reading the previous chunk
            stage_rows(L, tid, n_staged, win_lo, win_n, my_rows, feat, C_in, c);
        }
        __syncthreads();
        if (c == 0) FX_STAMP(2);
        if (c == 1) FX_STAMP(4);
        if (wave_mask) {
            const vec8* wbase = reinterpret_cast<const vec8*>(wp) + lane + (((int64_t)c * nslice + slice) * 4) * 64;
            const int64_t w_kappa_stride = (int64_t)nchunk * nslice * 4 * 64;
            offsets_loop<T, GENERAL>(L, acc, gmask, wave_mask, wave_block0, wbase, w_kappa_stride, n, h, n_staged, win_lo,
                                     win_n, my_rows, feat, C_in, c);
        }
        if (c == 0) FX_STAMP(3);
        if (c == 1) FX_STAMP(5);
    }
    FX_STAMP(6);

    // write-back: lane (n, h) holds output channels slice*64 + 32h .. +31 of output slot g*32 + n
#pragma unroll
    for (int gi = 0; gi < NG; ++gi) {
        const int local = L.perm[tile_group_of(wave, gi) * kGroup + n];
        if (local >= n_valid) continue;
        const int64_t o = tile * kTileT + local;
        const int64_t col = (int64_t)slice * kCoutSlice + 32 * h;
        if (OUT_F32) {
            float* dst = reinterpret_cast<float*>(out) + o * C_out + col;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4)
                    *reinterpret_cast<f32x4*>(dst + 16 * mt + 4 * v4) =
                        f32x4{acc[gi][mt][4 * v4], acc[gi][mt][4 * v4 + 1], acc[gi][mt][4 * v4 + 2], acc[gi][mt][4 * v4 + 3]};
        } else {
            uint16_t* dst = reinterpret_cast<uint16_t*>(out) + o * C_out + col;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int v8 = 0; v8 < 2; ++v8) {
                    u32x4 pk;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        pk[e] = Elem<T>::pack2(acc[gi][mt][8 * v8 + 2 * e], acc[gi][mt][8 * v8 + 2 * e + 1]);
                    *reinterpret_cast<u32x4*>(dst + 16 * mt + 8 * v8) = pk;
                }
        }
    }
}

// One workgroup = one tile of 512 consecutive outputs x one slice of 64 output channels.
// Wave w owns 4 of the tile's 16 column blocks (128 outputs): 4 x 2 accumulator tiles of 32x32.
template <typename T, bool OUT_F32>
__global__ void __launch_bounds__(kConvThreads, 2)
k_conv_mfma(const TileHeader* __restrict__ tile_hdr, const uint16_t* __restrict__ tile_perm,
            const int32_t* __restrict__ tile_rows, int row_stride, const uint16_t* __restrict__ tile_blocks,
            int block_stride, const uint16_t* __restrict__ feat, const uint16_t* __restrict__ wp,
            int C_in, int C_out, void* __restrict__ out) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    ConvLds& L = *reinterpret_cast<ConvLds*>(lds_raw);
    const int tid = threadIdx.x;
    const int64_t tile = blockIdx.x;
    const int slice = blockIdx.y;
    FX_STAMP(0);
    const TileHeader* H = tile_hdr + tile;
    const int32_t* my_rows = tile_rows + tile * (int64_t)row_stride;
    const uint16_t* my_blocks = tile_blocks + (size_t)tile * block_stride * kIdBlockElems;
    // a tile is "general" when some of its rows do not fit the LDS budget (or it is a direct tile):
    // its loop carries the global-memory fallback; all other tiles run a loop whose only global
    // loads are the weights
    const bool general = !(H->flags & kTileLdsOffsets);
    if (general)
        tile_body<T, OUT_F32, true>(L, H, tile, slice, tid, tile_perm, my_rows, my_blocks, feat, wp, C_in, C_out, out);
    else
        tile_body<T, OUT_F32, false>(L, H, tile, slice, tid, tile_perm, my_rows, my_blocks, feat, wp, C_in, C_out, out);
    FX_STAMP(7);
}

// ---------------------------------------------------------------------------------- scalar path
// One thread per (output voxel, output channel); fp32 FMA in offset-then-channel order.  Used
// for fp32 data (true fp32 products) and for channel counts the MFMA tiling does not cover.
template <int DT>
__device__ __forceinline__ float load_as_float(const void* p, int64_t i) {
    if (DT == FX_F32) return reinterpret_cast<const float*>(p)[i];
    if (DT == FX_F16) return Elem<_Float16>::to_float(reinterpret_cast<const uint16_t*>(p)[i]);
    return Elem<__bf16>::to_float(reinterpret_cast<const uint16_t*>(p)[i]);
}

template <int DT, bool OUT_F32>
__global__ void k_conv_scalar(const int32_t* __restrict__ nbmap, int64_t n_out, int K3, const void* __restrict__ feat,
                              const void* __restrict__ w, int C_in, int C_out, void* __restrict__ out) {
    const int64_t total = n_out * C_out;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const int64_t o = e / C_out;
        const int co = (int)(e - o * C_out);
        float acc = 0.f;
        for (int kappa = 0; kappa < K3; ++kappa) {
            const int32_t in = nbmap[o * K3 + kappa];
            if (in < 0) continue;
            const int64_t fb = (int64_t)in * C_in;
            const int64_t wb = (int64_t)kappa * C_in * C_out + co;
            for (int ci = 0; ci < C_in; ++ci)
                acc = fmaf(load_as_float<DT>(feat, fb + ci), load_as_float<DT>(w, wb + (int64_t)ci * C_out), acc);
        }
        if (OUT_F32) reinterpret_cast<float*>(out)[e] = acc;
        else if (DT == FX_F16) reinterpret_cast<uint16_t*>(out)[e] = Elem<_Float16>::from_float(acc);
        else reinterpret_cast<uint16_t*>(out)[e] = Elem<__bf16>::from_float(acc);
    }
}

template <typename T, bool OUT_F32>
static hipError_t launch_mfma(const fx_kmap* km, const void* feat, const void* wp, int C_in, int C_out, void* out,
                              hipStream_t st) {
    const size_t lds = sizeof(ConvLds);
    hipError_t e = hipFuncSetAttribute((const void*)k_conv_mfma<T, OUT_F32>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    dim3 grid((unsigned)km->n_tiles, (unsigned)(C_out / kCoutSlice));
    k_conv_mfma<T, OUT_F32><<<grid, kConvThreads, lds, st>>>(km->d_tile_hdr, km->d_tile_perm, km->d_tile_rows,
                                                             km->row_stride, km->d_tile_blocks, km->block_stride,
                                                             (const uint16_t*)feat, (const uint16_t*)wp, C_in, C_out,
                                                             out);
    return hipGetLastError();
}

}  // namespace fx

using namespace fx;

#ifdef FX_CONV_TIMING
extern "C" int fx_debug_conv_timing(unsigned long long* h_out, size_t bytes) {
    return (int)hipMemcpyFromSymbol(h_out, HIP_SYMBOL(g_conv_timing), bytes);
}
#endif

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
    hipStream_t st = (hipStream_t)stream;
    const bool out_f32 = (out_dt == FX_F32);
    const char* force = getenv("FVDB_HOTPATH_FORCE_SCALAR");
    const bool mfma = in_dt != FX_F32 && km->n_tiles > 0 && C_in % kCinChunk == 0 && C_out % kCoutSlice == 0 &&
                      !(force && force[0] == '1');
    if (mfma) {
        uint16_t* wp = nullptr;
        const size_t wbytes = sizeof(uint16_t) * (size_t)km->K3 * C_in * C_out;
        FX_TRY(dev_alloc((void**)&wp, wbytes, st));
        const int64_t total = (int64_t)km->K3 * C_in * C_out;
        {
            ProfScope ps(kProfPackWeights, st);
            k_pack_weights<<<(unsigned)std::min<int64_t>((total + 255) / 256, 4096), 256, 0, st>>>(
                (const uint16_t*)d_w, wp, km->K3, C_in, C_out);
        }
        hipError_t e = hipGetLastError();
        if (e == hipSuccess) {
            ProfScope ps(kProfConvMfma, st);
            if (in_dt == FX_BF16)
                e = out_f32 ? launch_mfma<__bf16, true>(km, d_feat, wp, C_in, C_out, d_out, st)
                            : launch_mfma<__bf16, false>(km, d_feat, wp, C_in, C_out, d_out, st);
            else
                e = out_f32 ? launch_mfma<_Float16, true>(km, d_feat, wp, C_in, C_out, d_out, st)
                            : launch_mfma<_Float16, false>(km, d_feat, wp, C_in, C_out, d_out, st);
        }
        dev_free(wp, st);
        if (e != hipSuccess) { set_error("convolution launch failed: %s", hipGetErrorString(e)); return FX_EDEVICE; }
        return FX_OK;
    }
    FX_TRY(kmap_ensure_dense(const_cast<fx_kmap*>(km), st));
    const int64_t total = km->n_out * C_out;
    const unsigned nb = (unsigned)std::min<int64_t>((total + 255) / 256, 1 << 20);
#define FX_SCALAR(DT)                                                                                            \
    do {                                                                                                         \
        if (out_f32) k_conv_scalar<DT, true><<<nb, 256, 0, st>>>(km->d_nbmap, km->n_out, km->K3, d_feat, d_w,    \
                                                                 C_in, C_out, d_out);                            \
        else k_conv_scalar<DT, false><<<nb, 256, 0, st>>>(km->d_nbmap, km->n_out, km->K3, d_feat, d_w, C_in,     \
                                                          C_out, d_out);                                         \
    } while (0)
    ProfScope ps(kProfConvScalar, st);
    if (in_dt == FX_F32) FX_SCALAR(FX_F32);
    else if (in_dt == FX_F16) FX_SCALAR(FX_F16);
    else FX_SCALAR(FX_BF16);
#undef FX_SCALAR
    FX_HIP_TRY(hipGetLastError());
    return FX_OK;
}
