// Sparse convolution forward (Sec. 3.5 scenario 3, re-designed for CDNA4).
//
// MFMA path.  A workgroup owns one tile of 256 consecutive output voxels.  The tile's distinct
// input rows are staged once in LDS (the paper's per-offset gathers become LDS reads), the
// per-offset products run on v_mfma_f32_16x16x32_{bf16,f16}, and -- unlike the paper's shared-
// memory scatter buffer -- every output voxel keeps its accumulators in registers for all
// offsets: a column block of 16 outputs is fixed for the whole tile, and an offset contributes
// a block only if one of the 16 has a neighbour there (missing neighbours read a zero row).
// Nothing is scattered; the write-back is one sequential range per tile.
//
// Operand roles: A = packed weights (16 output channels x 32 input channels per instruction),
// B = gathered features (32 input channels x 16 voxels), D = 16 channels x 16 voxels, so each
// lane ends up with 16 consecutive output channels of one voxel.
#include "kmap.h"

#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include <algorithm>

namespace fx {

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kCinChunk = 32;       // input channels staged in LDS at a time (one MFMA k-step)
constexpr int kCoutSlice = 64;      // output channels per wave
constexpr int kRowBytes = kCinChunk * 2;
constexpr int kRowCap = 832;        // LDS rows per tile; row kRowCap is the zero row
constexpr int kLdsBlocks = 640;     // blocks kept in LDS; further blocks are read from global memory
constexpr int kConvThreads = 256;
constexpr int kConvWaves = kConvThreads / 64;
constexpr int kGroupsPerWave = kGroupsPerTile / kConvWaves;   // 8 column blocks of 16 outputs

// ---------------------------------------------------------------------------------- element types
template <typename T> struct Elem;
template <> struct Elem<__bf16> {
    typedef bf16x8 vec8;
    static __device__ __forceinline__ f32x4 mfma(vec8 a, vec8 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ float to_float(uint16_t bits) { return __uint_as_float((uint32_t)bits << 16); }
    static __device__ __forceinline__ uint16_t from_float(float f) {  // round to nearest even
        uint32_t u = __float_as_uint(f);
        if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40);
        u += 0x7FFFu + ((u >> 16) & 1u);
        return (uint16_t)(u >> 16);
    }
};
template <> struct Elem<_Float16> {
    typedef f16x8 vec8;
    static __device__ __forceinline__ f32x4 mfma(vec8 a, vec8 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
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
};

// ---------------------------------------------------------------------------------- weight packing
// Wp[kappa][cin chunk][cout slice][mtile 0..3][lane 0..63][8]: the 16-byte A-operand fragment
// of each lane for one (offset, 32 input channels, 64 output channels).  Row m of m-tile t holds
// output channel 16*(m/4) + 4*t + (m%4) of the slice, so that a lane's 16 accumulators are 16
// consecutive output channels.
__global__ void k_pack_weights(const uint16_t* __restrict__ w, uint16_t* __restrict__ wp, int K3, int C_in, int C_out) {
    const int64_t total = (int64_t)K3 * C_in * C_out;
    const int nchunk = C_in / kCinChunk, nslice = C_out / kCoutSlice;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        int64_t r = e;
        const int el = (int)(r & 7); r >>= 3;
        const int lane = (int)(r & 63); r >>= 6;
        const int mt = (int)(r & 3); r >>= 2;
        const int s = (int)(r % nslice); r /= nslice;
        const int c = (int)(r % nchunk); r /= nchunk;
        const int kappa = (int)r;
        const int m = lane & 15, kq = lane >> 4;
        const int cin = c * kCinChunk + kq * 8 + el;
        const int cout = s * kCoutSlice + 16 * (m >> 2) + 4 * mt + (m & 3);
        wp[e] = w[((int64_t)kappa * C_in + cin) * C_out + cout];
    }
}

// ---------------------------------------------------------------------------------- MFMA kernel
struct ConvLds {
    unsigned char rows[(kRowCap + 1) * kRowBytes];  // 64-byte rows; 16-byte chunk q stored at q ^ ((row >> 2) & 3)
    uint16_t blocks[kLdsBlocks * kGroup];
    uint16_t perm[kTileT];
    uint32_t group_mask[kGroupsPerTile];
    uint32_t group_block0[kGroupsPerTile];
};

__device__ __forceinline__ int lds_row_offset(int row, int q) { return row * kRowBytes + ((q ^ ((row >> 2) & 3)) << 4); }

// One workgroup = one tile of 512 consecutive outputs x one slice of 64 output channels.
// Wave w owns column blocks 8w..8w+7 (128 outputs): 8 x 4 accumulator tiles of 16x16.
template <typename T, bool OUT_F32>
__global__ void __launch_bounds__(kConvThreads, 2)
k_conv_mfma(const TileHeader* __restrict__ tile_hdr, const uint16_t* __restrict__ tile_perm,
            const int32_t* __restrict__ tile_rows, int row_stride, const uint16_t* __restrict__ tile_blocks,
            int block_stride, int K3, const uint16_t* __restrict__ feat, const uint16_t* __restrict__ wp,
            int C_in, int C_out, void* __restrict__ out) {
    typedef typename Elem<T>::vec8 vec8;
    constexpr int NG = kGroupsPerWave;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    ConvLds& L = *reinterpret_cast<ConvLds*>(lds_raw);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, q = lane >> 4;
    const int64_t tile = blockIdx.x;
    const int slice = blockIdx.y;
    const int g0 = wave * NG;
    const int nchunk = C_in / kCinChunk, nslice = C_out / kCoutSlice;

    const TileHeader* H = tile_hdr + tile;
    const int win_lo = H->win_lo, win_n = H->win_n, n_list = H->n_list;
    const int n_blocks = H->n_blocks, n_valid = H->n_out;
    const int n_staged = (H->flags & kTileDirect) ? 0 : min(win_n + n_list, kRowCap);
    const int32_t* my_rows = tile_rows + tile * (int64_t)row_stride;
    const uint16_t* my_blocks = tile_blocks + (size_t)tile * block_stride * kGroup;

    // tile metadata -> LDS
    if (tid < kGroupsPerTile) { L.group_mask[tid] = H->group_mask[tid]; L.group_block0[tid] = H->group_block0[tid]; }
    for (int e = tid; e < kTileT; e += kConvThreads) L.perm[e] = tile_perm[tile * kTileT + e];
    {
        const u32x4* src = reinterpret_cast<const u32x4*>(my_blocks);
        u32x4* dst = reinterpret_cast<u32x4*>(L.blocks);
        const int nb2 = min(n_blocks, kLdsBlocks) * 2;
        for (int e = tid; e < nb2; e += kConvThreads) dst[e] = src[e];
    }
    if (tid < kRowBytes / 16) reinterpret_cast<u32x4*>(L.rows + kRowCap * kRowBytes)[tid] = u32x4{0, 0, 0, 0};

    f32x4 acc[NG][4];
#pragma unroll
    for (int gi = 0; gi < NG; ++gi)
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) acc[gi][mt] = f32x4{0.f, 0.f, 0.f, 0.f};

    __syncthreads();
    uint32_t gmask[NG], gblock0[NG];
    uint32_t wave_mask = 0;
#pragma unroll
    for (int gi = 0; gi < NG; ++gi) {
        gmask[gi] = __builtin_amdgcn_readfirstlane(L.group_mask[g0 + gi]);
        gblock0[gi] = __builtin_amdgcn_readfirstlane(L.group_block0[g0 + gi]);
        wave_mask |= gmask[gi];
    }

    for (int c = 0; c < nchunk; ++c) {
        if (c > 0) __syncthreads();  // all waves are done reading the previous chunk
        // stage the tile's input rows, channels [32c, 32c+32): 4 lanes x 16 bytes per row
        {
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
        __syncthreads();

        // offsets this wave needs, in order; the weights of the next one are fetched while the
        // current one is multiplied
        uint32_t todo = wave_mask;
        if (!todo) continue;
        const vec8* wbase = reinterpret_cast<const vec8*>(wp) + lane;
        auto w_ptr = [&](int kappa) { return wbase + ((((int64_t)kappa * nchunk + c) * nslice + slice) * 4) * 64; };
        vec8 wf[4], wn[4];
        {
            const vec8* ws = w_ptr(__ffs(todo) - 1);
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) wf[mt] = ws[mt * 64];
        }
        while (todo) {
            const int kappa = __ffs(todo) - 1;
            todo &= todo - 1;
            if (todo) {
                const vec8* ws = w_ptr(__ffs(todo) - 1);
#pragma unroll
                for (int mt = 0; mt < 4; ++mt) wn[mt] = ws[mt * 64];
            }
#pragma unroll
            for (int gi = 0; gi < NG; ++gi) {
                if (!((gmask[gi] >> kappa) & 1u)) continue;
                const int blk = (int)gblock0[gi] + __popc(gmask[gi] & ((1u << kappa) - 1u));
                const uint32_t id = blk < kLdsBlocks ? L.blocks[blk * kGroup + n] : my_blocks[blk * kGroup + n];
                vec8 bf;
                if (id < (uint32_t)n_staged || id == kNoRow) {
                    const int row = (id == kNoRow) ? kRowCap : (int)id;
                    bf = *reinterpret_cast<const vec8*>(L.rows + lds_row_offset(row, q));
                } else {  // row not staged (direct tile, or beyond the LDS budget): read it from global memory
                    const int64_t gr = id < (uint32_t)win_n ? (int64_t)win_lo + id : (int64_t)my_rows[id - win_n];
                    bf = *reinterpret_cast<const vec8*>(feat + gr * C_in + c * kCinChunk + q * 8);
                }
#pragma unroll
                for (int mt = 0; mt < 4; ++mt) acc[gi][mt] = Elem<T>::mfma(wf[mt], bf, acc[gi][mt]);
            }
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) wf[mt] = wn[mt];
        }
    }

    // write-back: lane (n, q) holds output channels slice*64 + 16q .. +15 of output slot g*16 + n
#pragma unroll
    for (int gi = 0; gi < NG; ++gi) {
        const int local = L.perm[(g0 + gi) * kGroup + n];
        if (local >= n_valid) continue;
        const int64_t o = tile * kTileT + local;
        const int64_t col = (int64_t)slice * kCoutSlice + 16 * q;
        if (OUT_F32) {
            float* dst = reinterpret_cast<float*>(out) + o * C_out + col;
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) *reinterpret_cast<f32x4*>(dst + 4 * mt) = acc[gi][mt];
        } else {
            uint16_t* dst = reinterpret_cast<uint16_t*>(out) + o * C_out + col;
            u32x4 pk[2];
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) {
                const uint32_t lo = Elem<T>::from_float(acc[gi][mt][0]) | ((uint32_t)Elem<T>::from_float(acc[gi][mt][1]) << 16);
                const uint32_t hi = Elem<T>::from_float(acc[gi][mt][2]) | ((uint32_t)Elem<T>::from_float(acc[gi][mt][3]) << 16);
                pk[mt >> 1][(mt & 1) * 2 + 0] = lo;
                pk[mt >> 1][(mt & 1) * 2 + 1] = hi;
            }
            reinterpret_cast<u32x4*>(dst)[0] = pk[0];
            reinterpret_cast<u32x4*>(dst)[1] = pk[1];
        }
    }
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
                                                             km->K3, (const uint16_t*)feat, (const uint16_t*)wp, C_in,
                                                             C_out, out);
    return hipGetLastError();
}

}  // namespace fx

using namespace fx;

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
