// Pooling kernels for gfx950 (Section 6 of "Communication-Optimal Convolutional Neural Nets": the convolution nest
// without the Filter, per-channel reading k = c).  HBM-bound: every Image word is needed by at most
// ceil(R/sigma_w)*ceil(S/sigma_h) outputs and those re-reads are served by L1/L2, every Out word is written once.
// One thread owns VEC adjacent images of one (h, w, c); threads are ordered images fastest, then c, so a wave's loads are
// contiguous in Image ([.][.][C][B]) and its stores are runs of B floats in Out ([.][.][.][B]).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "cacnn_internal.h"

namespace cacnn {

typedef float pf32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int pu32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t pdiv(uint32_t n, const FastDiv& f) { return f.mul ? __umulhi(n, f.mul) : n; }

// VEC values of one Image element group as floats
template <int DT, int VEC>
struct PoolLoad;
template <>
struct PoolLoad<0, 1> {
    static __device__ __forceinline__ void load(const void* base, int64_t idx, float (&v)[1]) {
        v[0] = ((const float*)base)[idx];
    }
};
template <>
struct PoolLoad<0, 4> {
    static __device__ __forceinline__ void load(const void* base, int64_t idx, float (&v)[4]) {
        const pf32x4 x = *(const pf32x4*)((const float*)base + idx);
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = x[i];
    }
};
template <>
struct PoolLoad<1, 1> {
    static __device__ __forceinline__ void load(const void* base, int64_t idx, float (&v)[1]) {
        v[0] = __uint_as_float((uint32_t)((const uint16_t*)base)[idx] << 16);
    }
};
template <>
struct PoolLoad<1, 8> {
    static __device__ __forceinline__ void load(const void* base, int64_t idx, float (&v)[8]) {
        const pu32x4 x = *(const pu32x4*)((const uint16_t*)base + idx);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(x[i] << 16);
            v[2 * i + 1] = __uint_as_float(x[i] & 0xffff0000u);
        }
    }
};

template <int DT, int MODE, int VEC>
__global__ void __launch_bounds__(256) pool_kernel(const PoolArgs a) {
    // consecutive workgroups go to different XCDs: give every XCD one contiguous run of the output instead, so the
    // rows its windows share stay in one L2
    int wg = blockIdx.x;
    if (a.n_xcd > 1) {
        const int l = (int)pdiv((uint32_t)wg, a.d_nxcd), x = wg - l * a.n_xcd;
        wg = x * a.xcd_q + min(x, a.xcd_rem) + l;
    }
    const int g = wg * 256 + threadIdx.x;
    if (g >= a.n_threads) return;
    // thread order: images fastest, then c, then the column within a chunk of TWC output columns, then h, then the
    // chunk.  An XCD's contiguous share of the workgroups is then a band of columns over all rows, so the Image rows
    // that vertically adjacent windows share are fetched into that XCD's L2 once.
    uint32_t t = (uint32_t)g;
    uint32_t q = pdiv(t, a.d_BV);
    const int bv = t - q * a.BV;
    t = q;
    q = pdiv(t, a.d_C);
    const int c = t - q * a.C;
    t = q;
    q = pdiv(t, a.d_TWC);
    const int wl = t - q * a.TWC;
    t = q;
    q = pdiv(t, a.d_H);
    const int h = t - q * a.H, w = (int)q * a.TWC + wl;
    if (w >= a.W) return;

    float acc[VEC];
    const int64_t cb = (int64_t)c * a.B + bv * VEC;
    for (int r = 0; r < a.R; ++r) {
        const int64_t xrow = ((int64_t)(a.sw * w + r) * a.IH + (int64_t)a.sh * h) * a.C * a.B + cb;
        for (int s = 0; s < a.S; ++s) {
            float v[VEC];
            PoolLoad<DT, VEC>::load(a.image, xrow + (int64_t)s * a.C * a.B, v);
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                if (r == 0 && s == 0) acc[i] = v[i];
                else if (MODE == 0) acc[i] += v[i];
                else acc[i] = fmaxf(acc[i], v[i]);
            }
        }
    }
    if (MODE == 0) {
        const float n = (float)(a.R * a.S);
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] = acc[i] / n;
    }
    float* dst = a.out + (((int64_t)c * a.H + h) * a.W + w) * a.B + bv * VEC;
    if constexpr (VEC >= 4) {
#pragma unroll
        for (int i = 0; i < VEC; i += 4) {
            const pf32x4 o = {acc[i], acc[i + 1], acc[i + 2], acc[i + 3]};
            __builtin_nontemporal_store(o, (pf32x4*)(dst + i));
        }
    } else {
        dst[0] = acc[0];
    }
}

template <int DT, int MODE, int VEC>
static int launch_one(const PoolArgs& a, void* stream) {
    hipLaunchKernelGGL((pool_kernel<DT, MODE, VEC>), dim3(a.n_wg), dim3(256), 0, (hipStream_t)stream, a);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int launch_pool(const PoolArgs& a, int dtype, int mode, int vec, void* stream) {
    if (dtype == 0) {
        if (vec == 4) return mode == 0 ? launch_one<0, 0, 4>(a, stream) : launch_one<0, 1, 4>(a, stream);
        return mode == 0 ? launch_one<0, 0, 1>(a, stream) : launch_one<0, 1, 1>(a, stream);
    }
    if (vec == 8) return mode == 0 ? launch_one<1, 0, 8>(a, stream) : launch_one<1, 1, 8>(a, stream);
    return mode == 0 ? launch_one<1, 0, 1>(a, stream) : launch_one<1, 1, 1>(a, stream);
}

}  // namespace cacnn
