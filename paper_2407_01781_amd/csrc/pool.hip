// Transposed convolution, factor-2 pooling and nearest-neighbour upsampling (Sec. 3.6.2: beside the
// convolution the framework offers average and max pooling on a grid / feature pair and an
// operator that upsamples by subdivision and nearest-neighbour sampling; Sec. 4.1.4's network goes
// back up to the fine resolution).  The paper gives no formulas; with map(o,kappa) the kernel map
// of a K = stride = 2 convolution from a fine grid (inputs i) to its coarse grid (outputs o):
//
//   pooling        out[o,c] = max, or mean, over the ACTIVE children i = map(o,kappa) of z[i,c]
//   upsampling     out[i,:] = z[o,:] for the one pair (o,kappa) with map(o,kappa) = i
//   transposed     out[i,:] = sum over pairs (o,kappa) with map(o,kappa) = i of z[o,:] . W[kappa]
//   convolution    (one pair per input when K = stride; on a submanifold map the sum runs over the
//                   mirrored offsets, which is the forward kernel with the offsets flipped)
//
// Pooling and upsampling move every feature row once: they are bandwidth-bound, one thread per
// 16 bytes of a row, rows of the coarse side visited in order (coalesced), rows of the fine side
// reached through the dense [N_out, 8] form of the map.
#include "conv_common.h"

namespace fx {

template <int DT>
__device__ __forceinline__ void load_vec(const void* p, int64_t byte_off, float (&v)[8]) {
    const u32x4 b = *reinterpret_cast<const u32x4*>(reinterpret_cast<const unsigned char*>(p) + byte_off);
    if (DT == FX_F32) {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = __uint_as_float(b[e]);
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint16_t h = (uint16_t)(b[e >> 1] >> (16 * (e & 1)));
            v[e] = DT == FX_F16 ? Elem<_Float16>::to_float(h) : Elem<__bf16>::to_float(h);
        }
    }
}

template <int DT>
__device__ __forceinline__ void store_vec(void* p, int64_t byte_off, const float (&v)[8]) {
    u32x4 b;
    if (DT == FX_F32) {
#pragma unroll
        for (int e = 0; e < 4; ++e) b[e] = __float_as_uint(v[e]);
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            b[e] = DT == FX_F16 ? Elem<_Float16>::pack2(v[2 * e], v[2 * e + 1]) : Elem<__bf16>::pack2(v[2 * e], v[2 * e + 1]);
    }
    *reinterpret_cast<u32x4*>(reinterpret_cast<unsigned char*>(p) + byte_off) = b;
}

// One thread per (coarse voxel, 16-byte piece of its row).  The children are visited in offset
// order; the mean is the fp32 sum in that order divided by the number of active children and
// rounded once (RNE) to the storage type; the maximum is exact in every type.
// SUM (with AVG): the plain sum, no division -- the gradient of upsampling.
template <int DT, bool AVG, bool SUM = false>
__global__ void __launch_bounds__(256)
k_pool2(const int32_t* __restrict__ nbmap, int64_t n_out, int vec_per_row, const void* __restrict__ z, void* __restrict__ out) {
    constexpr int NE = DT == FX_F32 ? 4 : 8;
    const int64_t total = n_out * vec_per_row;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x) {
        const int64_t o = t / vec_per_row;
        const int q = (int)(t - o * vec_per_row);
        float acc[8];
        int n = 0;
#pragma unroll
        for (int kappa = 0; kappa < 8; ++kappa) {
            const int32_t in = nbmap[o * 8 + kappa];
            if (in < 0) continue;
            float v[8];
            load_vec<DT>(z, ((int64_t)in * vec_per_row + q) * 16, v);
#pragma unroll
            for (int e = 0; e < NE; ++e) acc[e] = n == 0 ? v[e] : (AVG ? acc[e] + v[e] : (v[e] > acc[e] ? v[e] : acc[e]));
            ++n;
        }
        if (n == 0) {
#pragma unroll
            for (int e = 0; e < NE; ++e) acc[e] = 0.f;
        }
        if (AVG && !SUM && n > 1) {
            const float fn = (float)n;
#pragma unroll
            for (int e = 0; e < NE; ++e) acc[e] = acc[e] / fn;
        }
        store_vec<DT>(out, t * 16, acc);
    }
}

// One thread per (coarse voxel, 16-byte piece): reads the parent's piece once and copies it to every
// active child (one thread per (voxel, child slot, piece) re-read the parent's row eight times and ran
// at 0.45 of the HBM peak against 0.7 for this form).
__global__ void __launch_bounds__(256)
k_upsample2(const int32_t* __restrict__ nbmap, int64_t n_out, int vec_per_row, const void* __restrict__ z, void* __restrict__ out) {
    const int64_t total = n_out * vec_per_row;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x) {
        const int64_t o = t / vec_per_row;
        const int q = (int)(t - o * vec_per_row);
        int32_t child[8];
#pragma unroll
        for (int kappa = 0; kappa < 8; ++kappa) child[kappa] = nbmap[o * 8 + kappa];
        const u32x4 v = reinterpret_cast<const u32x4*>(z)[t];
#pragma unroll
        for (int kappa = 0; kappa < 8; ++kappa)
            if (child[kappa] >= 0) reinterpret_cast<u32x4*>(out)[(int64_t)child[kappa] * vec_per_row + q] = v;
    }
}

// element-wise fallbacks for rows that are not a multiple of 16 bytes
template <int DT, bool AVG, bool SUM = false>
__global__ void k_pool2_elem(const int32_t* __restrict__ nbmap, int64_t n_out, int C, const void* __restrict__ z,
                             void* __restrict__ out) {
    const int64_t total = n_out * C;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x) {
        const int64_t o = t / C;
        const int c = (int)(t - o * C);
        float acc = 0.f;
        int n = 0;
        for (int kappa = 0; kappa < 8; ++kappa) {
            const int32_t in = nbmap[o * 8 + kappa];
            if (in < 0) continue;
            const float v = load_as_float<DT>(z, (int64_t)in * C + c);
            acc = n == 0 ? v : (AVG ? acc + v : (v > acc ? v : acc));
            ++n;
        }
        if (AVG && !SUM && n > 1) acc = acc / (float)n;
        if (DT == FX_F32) reinterpret_cast<float*>(out)[t] = acc;
        else if (DT == FX_F16) reinterpret_cast<uint16_t*>(out)[t] = Elem<_Float16>::from_float(acc);
        else reinterpret_cast<uint16_t*>(out)[t] = Elem<__bf16>::from_float(acc);
    }
}

template <typename E>
__global__ void k_upsample2_elem(const int32_t* __restrict__ nbmap, int64_t n_out, int C, const E* __restrict__ z,
                                 E* __restrict__ out) {
    const int64_t total = n_out * 8 * C;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x) {
        const int64_t pair = t / C;
        const int32_t in = nbmap[pair];
        if (in < 0) continue;
        const int c = (int)(t - pair * C);
        out[(int64_t)in * C + c] = z[(pair >> 3) * C + c];
    }
}

// Gradient of pooling.  One thread per (coarse voxel, 16-byte piece): reads the parent's gradient piece
// once and, for max pooling, the children's pieces of the forward input (first child in offset order that
// attains the maximum takes the gradient: the one the forward pass keeps); writes every active child's
// piece -- the parent's gradient over the number of active children, or the gradient / zero.
template <int DT, bool AVG>
__global__ void __launch_bounds__(256)
k_pool2_bwd(const int32_t* __restrict__ nbmap, int64_t n_out, int vec_per_row, const void* __restrict__ z,
            const void* __restrict__ gout, void* __restrict__ gin) {
    constexpr int NE = DT == FX_F32 ? 4 : 8;
    const int64_t total = n_out * vec_per_row;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x) {
        const int64_t o = t / vec_per_row;
        const int q = (int)(t - o * vec_per_row);
        int32_t child[8];
        int n = 0;
#pragma unroll
        for (int kappa = 0; kappa < 8; ++kappa) {
            child[kappa] = nbmap[o * 8 + kappa];
            n += child[kappa] >= 0;
        }
        float g[8];
        load_vec<DT>(gout, t * 16, g);
        if (AVG) {
            if (n > 1) {
                const float fn = (float)n;
#pragma unroll
                for (int e = 0; e < NE; ++e) g[e] = g[e] / fn;
            }
#pragma unroll
            for (int kappa = 0; kappa < 8; ++kappa)
                if (child[kappa] >= 0) store_vec<DT>(gin, ((int64_t)child[kappa] * vec_per_row + q) * 16, g);
        } else {
            float best[8];
            int who[8];
            bool any = false;
#pragma unroll
            for (int kappa = 0; kappa < 8; ++kappa) {
                if (child[kappa] < 0) continue;
                float v[8];
                load_vec<DT>(z, ((int64_t)child[kappa] * vec_per_row + q) * 16, v);
#pragma unroll
                for (int e = 0; e < NE; ++e)
                    if (!any || v[e] > best[e]) { best[e] = v[e]; who[e] = kappa; }
                any = true;
            }
#pragma unroll
            for (int kappa = 0; kappa < 8; ++kappa) {
                if (child[kappa] < 0) continue;
                float r[8];
#pragma unroll
                for (int e = 0; e < NE; ++e) r[e] = who[e] == kappa ? g[e] : 0.f;
                store_vec<DT>(gin, ((int64_t)child[kappa] * vec_per_row + q) * 16, r);
            }
        }
    }
}

template <int DT, bool AVG>
__global__ void k_pool2_bwd_elem(const int32_t* __restrict__ nbmap, int64_t n_out, int C, const void* __restrict__ z,
                                 const void* __restrict__ gout, void* __restrict__ gin) {
    const int64_t total = n_out * C;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x) {
        const int64_t o = t / C;
        const int c = (int)(t - o * C);
        int n = 0, who = -1;
        float best = 0.f;
        for (int kappa = 0; kappa < 8; ++kappa) {
            const int32_t in = nbmap[o * 8 + kappa];
            if (in < 0) continue;
            if (!AVG) {
                const float v = load_as_float<DT>(z, (int64_t)in * C + c);
                if (n == 0 || v > best) { best = v; who = kappa; }
            }
            ++n;
        }
        const float g = load_as_float<DT>(gout, t);
        for (int kappa = 0; kappa < 8; ++kappa) {
            const int32_t in = nbmap[o * 8 + kappa];
            if (in < 0) continue;
            const float r = AVG ? (n > 1 ? g / (float)n : g) : (who == kappa ? g : 0.f);
            const int64_t at = (int64_t)in * C + c;
            if (DT == FX_F32) reinterpret_cast<float*>(gin)[at] = r;
            else if (DT == FX_F16) reinterpret_cast<uint16_t*>(gin)[at] = Elem<_Float16>::from_float(r);
            else reinterpret_cast<uint16_t*>(gin)[at] = Elem<__bf16>::from_float(r);
        }
    }
}

static unsigned blocks_for(int64_t total) { return (unsigned)std::max<int64_t>(1, std::min<int64_t>((total + 255) / 256, 1 << 20)); }

}  // namespace fx

using namespace fx;

static fx_status check_pair_map(const char* who, const fx_kmap* km) {
    if (!km) { set_error("%s: null kernel map", who); return FX_EINVAL; }
    if (km->K != 2 || km->stride != 2) { set_error("%s: needs the kernel map of a 2x2x2 stride-2 convolution", who); return FX_EUNSUPPORTED; }
    return FX_OK;
}

extern "C" fx_status fx_pool2(const fx_kmap* km, int32_t mode, const void* d_feat, fx_dtype dt, int32_t C, void* d_out,
                              void* stream) {
    FX_TRY(check_pair_map("fx_pool2", km));
    if ((mode != FX_POOL_MAX && mode != FX_POOL_AVG) || C < 1 || (dt != FX_F32 && dt != FX_F16 && dt != FX_BF16) ||
        (km->n_in > 0 && !d_feat) || (km->n_out > 0 && !d_out)) {
        set_error("fx_pool2: bad mode, dtype, channel count or null pointer");
        return FX_EINVAL;
    }
    if (km->n_out == 0) return FX_OK;
    hipStream_t st = (hipStream_t)stream;
    FX_TRY(kmap_ensure_dense(const_cast<fx_kmap*>(km), st));
    const int esize = dt == FX_F32 ? 4 : 2;
    const bool avg = mode == FX_POOL_AVG;
    ProfScope ps(kProfPool, st);
    if (((int64_t)C * esize) % 16 == 0) {
        const int vpr = C * esize / 16;
        const unsigned nb = blocks_for(km->n_out * vpr);
#define FX_POOL(DT) do { if (avg) k_pool2<DT, true><<<nb, 256, 0, st>>>(km->d_nbmap, km->n_out, vpr, d_feat, d_out); \
                         else k_pool2<DT, false><<<nb, 256, 0, st>>>(km->d_nbmap, km->n_out, vpr, d_feat, d_out); } while (0)
        if (dt == FX_F32) FX_POOL(FX_F32); else if (dt == FX_F16) FX_POOL(FX_F16); else FX_POOL(FX_BF16);
#undef FX_POOL
    } else {
        const unsigned nb = blocks_for(km->n_out * C);
#define FX_POOL(DT) do { if (avg) k_pool2_elem<DT, true><<<nb, 256, 0, st>>>(km->d_nbmap, km->n_out, C, d_feat, d_out); \
                         else k_pool2_elem<DT, false><<<nb, 256, 0, st>>>(km->d_nbmap, km->n_out, C, d_feat, d_out); } while (0)
        if (dt == FX_F32) FX_POOL(FX_F32); else if (dt == FX_F16) FX_POOL(FX_F16); else FX_POOL(FX_BF16);
#undef FX_POOL
    }
    FX_HIP_TRY(hipGetLastError());
    return FX_OK;
}

extern "C" fx_status fx_upsample2(const fx_kmap* km, const void* d_feat, fx_dtype dt, int32_t C, void* d_out, void* stream) {
    FX_TRY(check_pair_map("fx_upsample2", km));
    if (C < 1 || (dt != FX_F32 && dt != FX_F16 && dt != FX_BF16) || (km->n_out > 0 && !d_feat) || (km->n_in > 0 && !d_out)) {
        set_error("fx_upsample2: bad dtype, channel count or null pointer");
        return FX_EINVAL;
    }
    if (km->n_out == 0) return FX_OK;
    hipStream_t st = (hipStream_t)stream;
    FX_TRY(kmap_ensure_dense(const_cast<fx_kmap*>(km), st));
    const int esize = dt == FX_F32 ? 4 : 2;
    ProfScope ps(kProfUpsample, st);
    if (((int64_t)C * esize) % 16 == 0) {
        const int vpr = C * esize / 16;
        k_upsample2<<<blocks_for(km->n_out * vpr), 256, 0, st>>>(km->d_nbmap, km->n_out, vpr, d_feat, d_out);
    } else if (esize == 4) {
        k_upsample2_elem<uint32_t><<<blocks_for(km->n_out * 8 * C), 256, 0, st>>>(km->d_nbmap, km->n_out, C, (const uint32_t*)d_feat, (uint32_t*)d_out);
    } else {
        k_upsample2_elem<uint16_t><<<blocks_for(km->n_out * 8 * C), 256, 0, st>>>(km->d_nbmap, km->n_out, C, (const uint16_t*)d_feat, (uint16_t*)d_out);
    }
    FX_HIP_TRY(hipGetLastError());
    return FX_OK;
}

extern "C" fx_status fx_sparse_conv_transpose_fwd(const fx_kmap* km, const void* d_feat, fx_dtype dt, const void* d_w,
                                                  int32_t C_in, int32_t C_out, void* d_out, fx_dtype out_dt, void* stream) {
    if (!km || !d_w || C_in < 1 || C_out < 1 || (km->n_out > 0 && !d_feat) || (km->n_in > 0 && !d_out)) {
        set_error("fx_sparse_conv_transpose_fwd: null pointer or non-positive channel count");
        return FX_EINVAL;
    }
    if (dt != FX_F32 && dt != FX_F16 && dt != FX_BF16) { set_error("fx_sparse_conv_transpose_fwd: unknown dtype"); return FX_EINVAL; }
    if (out_dt != dt && out_dt != FX_F32) {
        set_error("fx_sparse_conv_transpose_fwd: output dtype must equal the input dtype or be fp32");
        return FX_EUNSUPPORTED;
    }
    if (km->n_in == 0) return FX_OK;
    hipStream_t st = (hipStream_t)stream;
    if (km->stride == 1) {  // symmetric map: the forward multiply over the mirrored offsets (between two grids: of the map back)
        const fx_kmap* back = km;
        if (km->gin != km->gout) {
            FX_TRY(kmap_ensure_inverse(const_cast<fx_kmap*>(km), st));
            back = km->inverse;
        }
        return conv_apply(back, d_feat, dt, d_w, C_in, C_out, d_out, out_dt, st, kWeightsFlipped);
    }
    if (km->K != km->stride) {
        // 3x3x3 stride 2: inputs are shared by up to 8 outputs; the forward kernels of strided maps over the
        // inverse map, weights as given
        FX_TRY(kmap_ensure_inverse(const_cast<fx_kmap*>(km), st));
        return conv_apply(km->inverse, d_feat, dt, d_w, C_in, C_out, d_out, out_dt, st, kWeightsForward);
    }
    // one pair per input voxel: the input-gradient kernel of the strided map with the weights read
    // forward (C_in contracted, C_out produced)
    return strided_pair_product(km, d_feat, dt, d_w, C_in, C_out, d_out, out_dt, st, kWeightsForward);
}

extern "C" fx_status fx_pool2_bwd(const fx_kmap* km, int32_t mode, const void* d_feat, const void* d_gout, fx_dtype dt,
                                  int32_t C, void* d_gin, void* stream) {
    FX_TRY(check_pair_map("fx_pool2_bwd", km));
    if ((mode != FX_POOL_MAX && mode != FX_POOL_AVG) || C < 1 || (dt != FX_F32 && dt != FX_F16 && dt != FX_BF16) ||
        (km->n_out > 0 && !d_gout) || (km->n_in > 0 && !d_gin) || (mode == FX_POOL_MAX && km->n_in > 0 && !d_feat)) {
        set_error("fx_pool2_bwd: bad mode, dtype, channel count or null pointer");
        return FX_EINVAL;
    }
    if (km->n_out == 0) return FX_OK;
    hipStream_t st = (hipStream_t)stream;
    FX_TRY(kmap_ensure_dense(const_cast<fx_kmap*>(km), st));
    const int esize = dt == FX_F32 ? 4 : 2;
    const bool avg = mode == FX_POOL_AVG;
    ProfScope ps(kProfPool, st);
    if (((int64_t)C * esize) % 16 == 0) {
        const int vpr = C * esize / 16;
        const unsigned nb = blocks_for(km->n_out * vpr);
#define FX_POOLB(DT) do { if (avg) k_pool2_bwd<DT, true><<<nb, 256, 0, st>>>(km->d_nbmap, km->n_out, vpr, d_feat, d_gout, d_gin); \
                          else k_pool2_bwd<DT, false><<<nb, 256, 0, st>>>(km->d_nbmap, km->n_out, vpr, d_feat, d_gout, d_gin); } while (0)
        if (dt == FX_F32) FX_POOLB(FX_F32); else if (dt == FX_F16) FX_POOLB(FX_F16); else FX_POOLB(FX_BF16);
#undef FX_POOLB
    } else {
        const unsigned nb = blocks_for(km->n_out * C);
#define FX_POOLB(DT) do { if (avg) k_pool2_bwd_elem<DT, true><<<nb, 256, 0, st>>>(km->d_nbmap, km->n_out, C, d_feat, d_gout, d_gin); \
                          else k_pool2_bwd_elem<DT, false><<<nb, 256, 0, st>>>(km->d_nbmap, km->n_out, C, d_feat, d_gout, d_gin); } while (0)
        if (dt == FX_F32) FX_POOLB(FX_F32); else if (dt == FX_F16) FX_POOLB(FX_F16); else FX_POOLB(FX_BF16);
#undef FX_POOLB
    }
    FX_HIP_TRY(hipGetLastError());
    return FX_OK;
}

extern "C" fx_status fx_upsample2_bwd(const fx_kmap* km, const void* d_gout, fx_dtype dt, int32_t C, void* d_gin, void* stream) {
    FX_TRY(check_pair_map("fx_upsample2_bwd", km));
    if (C < 1 || (dt != FX_F32 && dt != FX_F16 && dt != FX_BF16) || (km->n_in > 0 && !d_gout) || (km->n_out > 0 && !d_gin)) {
        set_error("fx_upsample2_bwd: bad dtype, channel count or null pointer");
        return FX_EINVAL;
    }
    if (km->n_out == 0) return FX_OK;
    hipStream_t st = (hipStream_t)stream;
    FX_TRY(kmap_ensure_dense(const_cast<fx_kmap*>(km), st));
    const int esize = dt == FX_F32 ? 4 : 2;
    ProfScope ps(kProfUpsample, st);
    if (((int64_t)C * esize) % 16 == 0) {
        const int vpr = C * esize / 16;
        const unsigned nb = blocks_for(km->n_out * vpr);
        if (dt == FX_F32) k_pool2<FX_F32, true, true><<<nb, 256, 0, st>>>(km->d_nbmap, km->n_out, vpr, d_gout, d_gin);
        else if (dt == FX_F16) k_pool2<FX_F16, true, true><<<nb, 256, 0, st>>>(km->d_nbmap, km->n_out, vpr, d_gout, d_gin);
        else k_pool2<FX_BF16, true, true><<<nb, 256, 0, st>>>(km->d_nbmap, km->n_out, vpr, d_gout, d_gin);
    } else {
        const unsigned nb = blocks_for(km->n_out * C);
        if (dt == FX_F32) k_pool2_elem<FX_F32, true, true><<<nb, 256, 0, st>>>(km->d_nbmap, km->n_out, C, d_gout, d_gin);
        else if (dt == FX_F16) k_pool2_elem<FX_F16, true, true><<<nb, 256, 0, st>>>(km->d_nbmap, km->n_out, C, d_gout, d_gin);
        else k_pool2_elem<FX_BF16, true, true><<<nb, 256, 0, st>>>(km->d_nbmap, km->n_out, C, d_gout, d_gin);
    }
    FX_HIP_TRY(hipGetLastError());
    return FX_OK;
}
