// Declarations shared by the forward and backward convolution kernels: element types with
// their MFMA instruction, vector typedefs, and the host-side pieces of the forward path that
// the backward pass reuses.
#pragma once
#include "kmap.h"

#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include <algorithm>

namespace fx {

typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) int32_t i32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kCoutSlice = 64;      // output channels per wave
constexpr int kProducerWaves = 4;
constexpr int kConvThreads = 64 * (kTileWaves + kProducerWaves);
constexpr int kMaxIdBlocks = kTileWaves * kMaxK3Tiled;

// ---------------------------------------------------------------------------------- element types
// vec8 is the 16-byte operand fragment of a lane (8 values of a 16-bit type, 4 of fp32); mma
// multiplies one fragment pair into a 32x32 accumulator tile (one instruction with k = 16 for the
// 16-bit types, four with k = 2 for fp32, whose products are true fp32 products).
template <typename T> struct Elem;
template <> struct Elem<__bf16> {
    typedef bf16x8 vec8;
    static constexpr int kBytes = 2;
    static __device__ __forceinline__ f32x16 mma(vec8 a, vec8 b, f32x16 c) { return mfma(a, b, c); }
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
        const bf16x2 h = __builtin_convertvector(f32x2{a, b}, bf16x2);
        uint32_t bits;
        __builtin_memcpy(&bits, &h, 4);
        return bits;
    }
};
template <> struct Elem<_Float16> {
    typedef f16x8 vec8;
    static constexpr int kBytes = 2;
    static __device__ __forceinline__ f32x16 mma(vec8 a, vec8 b, f32x16 c) { return mfma(a, b, c); }
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

template <> struct Elem<float> {
    typedef f32x4 vec8;
    static constexpr int kBytes = 4;
    static __device__ __forceinline__ f32x16 mma(vec8 a, vec8 b, f32x16 c) {
#pragma unroll
        for (int e = 0; e < 4; ++e) c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[e], b[e], c, 0, 0, 0);
        return c;
    }
    static __device__ __forceinline__ uint32_t pack2(float a, float) { return __float_as_uint(a); }   // never stored narrow
};

__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

template <int DT>
__device__ __forceinline__ float load_as_float(const void* p, int64_t i) {
    if (DT == FX_F32) return reinterpret_cast<const float*>(p)[i];
    if (DT == FX_F16) return Elem<_Float16>::to_float(reinterpret_cast<const uint16_t*>(p)[i]);
    return Elem<__bf16>::to_float(reinterpret_cast<const uint16_t*>(p)[i]);
}

// four consecutive elements starting at element i (i a multiple of 4, p suitably aligned)
template <int DT>
__device__ __forceinline__ f32x4 load4_as_float(const void* p, int64_t i) {
    if (DT == FX_F32) return *reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(p) + i);
    const u32x2 b = *reinterpret_cast<const u32x2*>(reinterpret_cast<const uint16_t*>(p) + i);
    f32x4 r;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const uint16_t h = (uint16_t)(b[e >> 1] >> (16 * (e & 1)));
        r[e] = DT == FX_F16 ? Elem<_Float16>::to_float(h) : Elem<__bf16>::to_float(h);
    }
    return r;
}

constexpr int kRowBufBytes = (kRowCap + 1) * kRowBytes;           // staged rows + the zero row
constexpr int kBlockBufBytes = kMaxIdBlocks * kIdBlockElems * 2;
__device__ __forceinline__ int lds_row_offset(int row, int p) { return (int)(lds_row_code((uint32_t)row) ^ (uint32_t)(p << 4)); }
typedef __attribute__((address_space(3))) void* lds_ptr_t;

// How the packed operand fragments are read from the caller's W[K^3][C_in][C_out] (two flags):
//   kWeightsForward        fragment (kappa, cin, cout) = W[kappa][cin][cout]
//   kWeightsTransposed     fragment (kappa, a, b)      = W[kappa][b][a]            (roles of the channel
//                          counts swapped: the multiply contracts over W's output channels)
//   kWeightsFlipped        fragment (kappa, cin, cout) = W[K^3-1-kappa][cin][cout] (offsets mirrored)
//   kWeightsMirrored       fragment (kappa, a, b)      = W[K^3-1-kappa][b][a]      (both)
enum WeightMode { kWeightsForward = 0, kWeightsTransposed = 1, kWeightsFlipped = 2, kWeightsMirrored = 3 };

// Every matrix-unit kernel takes the weights as the B operand: column m of n-tile t of a 64-channel slice holds
// produced channel 2*m + t, so lane m holds two adjacent channels of the voxel of each accumulator register and
// the 32 lanes of a half-wave store one whole row slice.

// Packs the weights (C_in = contracted channels, C_out = produced channels, in the sense of the
// mode) and zeroes the eight work-list counters behind them.
// elem_bytes 2 or 4; a row of the packed array covers 64 bytes of input channels (32 or 16 of them)
// and the produced channels are padded with zeros to a multiple of 64.  Returns the bytes packed.
size_t packed_weight_bytes(int K3, int C_in, int C_out, int elem_bytes);
void launch_pack_weights(const void* d_w, void* wp, int K3, int C_in, int C_out, int elem_bytes, int32_t* counters,
                         int mode, hipStream_t st);

// The forward multiply-accumulate over a map with the weights read in the given mode: d_out[o,:]
// = sum over kappa of d_feat[map(o,kappa),:] . Wmode[kappa], C_in channels in, C_out channels out.
fx_status conv_apply(const fx_kmap* km, const void* d_feat, fx_dtype in_dt, const void* d_w, int32_t C_in,
                     int32_t C_out, void* d_out, fx_dtype out_dt, hipStream_t st, int mode);
// Looks up (once per device) the device address of the static scratch array behind fx_sparse_conv_fwd_noalloc on the
// current device; fx_init calls it so that the entry point's first call does no set-up work.
fx_status conv_noalloc_setup(void** out_ptr);
// The 3x3x3 stride-1 convolution of `src` [N, C_contract] into `dst` [N, C_produce] straight from the grid, leaf by
// leaf, without a kernel map (Sec. 3.5 scenario 1); `mode` is kWeightsForward or kWeightsMirrored (input gradient).
// FX_EUNSUPPORTED for shapes its kernels do not serve.  leaf_shape_supported says so without setting an error.
// leaf_list / n_list (device; 16-bit types only): work on these leaves only instead of on all of them.
fx_status leaf_apply(const char* who, const fx_grid* g, const void* d_src, fx_dtype dt, const void* d_w, int32_t C_contract,
                     int32_t C_produce, void* d_dst, fx_dtype out_dt, hipStream_t st, int mode,
                     const int32_t* leaf_list = nullptr, const int32_t* n_list = nullptr);
inline bool leaf_shape_supported(fx_dtype dt, int C_contract, int C_produce) {
    if (dt == FX_F32) return C_contract % 4 == 0 && C_contract <= 16 && C_produce % 4 == 0 && C_produce <= 32;
    return C_contract % 32 == 0 && C_produce % 64 == 0;
}

template <typename T>
__device__ __forceinline__ typename Elem<T>::vec8 vec8_from_words(u32x4 w) {
    typename Elem<T>::vec8 v;
    __builtin_memcpy(&v, &w, 16);
    return v;
}

// The transposing LDS read of 16-bit elements (ds_read_b64_tr_b16): in every group of 16 lanes, lane 4q + e receives,
// as element j, element e of the 8 bytes that lane 4j + q addresses.  With lane 4j + q pointing at channels
// 4q .. 4q + 3 of voxel j's row, lane c of the group ends up with channel c of voxels 0..3: rows in, operand columns
// with the voxels along k out.  All 64 lanes must be active.
typedef short tr_v4s __attribute__((ext_vector_type(4)));
__device__ __forceinline__ u32x2 tr_read4(const unsigned char* p) {
    const tr_v4s v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) tr_v4s*)p);
    u32x2 w;
    __builtin_memcpy(&w, &v, 8);
    return w;
}

// Weight gradient of the 3x3x3 submanifold convolution from the leaf window (fp32 at low depth; f16 / bf16 at
// C_in % 32 == 0 and C_out % 64 == 0), and the ordered
// reduction of per-range partial sums part[n_ranges][total] into gw that all weight-gradient kernels end with
// (n_ranges = 0: gw = 0).
fx_status leaf_wgrad(const char* who, const fx_grid* g, const void* d_feat, const void* d_gout, fx_dtype dt, int32_t C_in,
                     int32_t C_out, void* d_gw, fx_dtype out_dt, hipStream_t st);
inline bool leaf_wgrad_shape_supported(fx_dtype dt, int C_in, int C_out) {
    if (dt != FX_F32) return C_in % 32 == 0 && C_out % 64 == 0;
    return (C_in == 4 || C_in == 8 || C_in == 12 || C_in == 16) && C_out >= 4 && C_out % 4 == 0 && C_out <= 32;
}
fx_status wgrad_reduce_ranges(const float* part, int n_ranges, int64_t total, void* gw, fx_dtype out_dt, hipStream_t st);
// The 16-bit leaf-window weight gradient as partial sums only: part[n_ranges][27][C_in][C_out] with
// n_ranges = leaf_wgrad16_ranges(...), over all leaves of g or over the first *n_list leaves of leaf_list.
int leaf_wgrad16_ranges(const fx_grid* g, int C_in, int C_out);
fx_status leaf_wgrad16_partial(const fx_grid* g, const void* d_feat, const void* d_gout, fx_dtype dt, int32_t C_in, int32_t C_out,
                               const int32_t* leaf_list, const int32_t* n_list, float* part, int n_ranges, hipStream_t st);

// The same sum through a dense table [n_rows, K3] of source rows (-1: none), one thread per output element
// (or per four): out[r,:] = sum over kappa with table[r][kappa] >= 0 of src[table[r][kappa],:] . W'[kappa], W' read
// from the caller's weights as `mode` says.  Serves maps without a tiled form and the inverse table.
fx_status conv_scalar_on_table(const int32_t* d_table, int64_t n_rows, int K3, const void* d_feat, fx_dtype in_dt,
                               const void* d_w, int32_t C_in, int32_t C_out, void* d_out, fx_dtype out_dt, hipStream_t st,
                               int mode);

// dst[map(o,kappa), :] for every pair of a K = stride map; see conv_bwd.hip
fx_status strided_pair_product(const fx_kmap* km, const void* d_src, fx_dtype dt, const void* d_w, int32_t C_contract,
                               int32_t C_produce, void* d_dst, fx_dtype out_dt, hipStream_t st, int mode);

}  // namespace fx
