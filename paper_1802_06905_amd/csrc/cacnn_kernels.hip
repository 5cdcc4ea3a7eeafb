// gfx950 (CDNA4) kernels for the blocked convolution schedule.
//
// One workgroup owns one Out tile (b_k output channels x a position tile of b_b images x b_w columns x b_h rows) and
// walks the contraction (c, r, s) in tiles, as in the blocked loop nest of Section 5 of the paper: the outer loops
// over (c, r', s') tiles are the kernel's main loop, the inner loops are the MFMA sweep.  Per contraction tile the
// Image halo tile (Section 5, item 3: its w-extent is sigma_w*(b_w-1)+b_r) and the Filter tile are staged from global
// memory into LDS; the Out tile stays in accumulator registers for the whole contraction, so each Out word is
// written exactly once and partial sums never travel (Theorem 1's first term is met with equality).
//
// MFMA mapping: rows (M) = output channels k, columns (N) = positions (b fastest, as in memory), contraction = (c,r,s).
//   fp32 : v_mfma_f32_32x32x2_f32,   A[i][kk] lane = i + 32*kk,          B[kk][j] lane = j + 32*kk
//   bf16 : v_mfma_f32_32x32x16_bf16, A[i][8g..8g+7] lane = i + 32*g,     B[8g..8g+7][j] lane = j + 32*g
//   D    : lane = j + 32*q holds rows 8*(v/4) + 4*q + (v%4), v = 0..15, of column j
// Every staged Image word is reused for all b_k channels and for every (r,s) shift that touches it -- the extra
// (RS/sigma_w sigma_h)^(1/2) reuse over matmul that the small-filter bound of Section 4.3 expresses.
//
// Kernel families in this file, in order: one tile per workgroup (any shape), pipelined persistent, wave-
// specialised (staging waves + multiplying waves), and fixed-geometry wave-specialised kernels for 3x3 (strides 1, bf16
// also 2) and 1x1 (any strides) filters and for the 7x7 stride-2 three-channel stem shape; the variant table at the end
// lists what is compiled.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>
#include <utility>

#include "cacnn_internal.h"

namespace cacnn {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ uint32_t fdiv(uint32_t n, const FastDiv& f) {
    return f.mul ? __umulhi(n, f.mul) : n;
}

struct TileCoord {
    int k0, b0, w0, h0;
};

// Workgroups are dealt round-robin to the XCDs (each with its own L2), so consecutive dispatch indices land on
// different L2s.  Give every XCD one contiguous run of the tile list instead.  The list is ordered k-tile fastest,
// then the b-tiles that share 128-byte lines of the Image (b_group of them), then w, then h, then the remaining
// image groups slowest: the workgroups that share an Image tile, its halo or its cache lines (and walk the Filter
// slices in step) then share an L2, and different XCDs mostly hold different images -- the Image is fetched from
// memory about once and the Filter once per XCD (the a_K / a_B a_W a_H replication of Section 7's parallel
// bound, with the XCDs as the processors).  Where the Filter is the bigger array the host divides the k-tiles into
// k_groups groups first (the list is then k_groups blocks, each ordered as above over its own k-tiles): an XCD sees
// 1 / k_groups of the Filter and the Image is fetched k_groups times.
// i -> tile is a bijection on [0, n): XCD x = i % n_xcd owns tiles [x*q + min(x,rem), ...) with n = n_xcd*q + rem.
__device__ __forceinline__ int xcd_tile(const KernelArgs& a, int i) {
    if (a.n_xcd <= 1) return i;
    const int l = (int)fdiv((uint32_t)i, a.d_nxcd), x = i - l * a.n_xcd;
    return x * a.xcd_q + min(x, a.xcd_rem) + l;
}

// tile list index -> tile origin; the divisors are fixed for the launch, so each division is one multiply-high
// (the host only enables the remapping and these reciprocals when the tile count keeps them exact)
__device__ __forceinline__ TileCoord tile_coords(const KernelArgs& a, int t, int KT, int TB, int TW, int TH) {
    // which group of output channels (at most 8: a few scalar compares), then the k-tile inside the group
    int kg = 0;
    for (int i = 1; i < a.k_groups; ++i) kg += (t >= i * a.grp) ? 1 : 0;
    t -= kg * a.grp;
    int q, tk;
    if (a.pos_fastest) {
        // the position tiles of one k-tile are neighbours in the list, the k-tile is the slowest index of the block
        q = (int)fdiv((uint32_t)t, a.d_npos);
        tk = kg * a.kpg + q;
        t -= q * a.npos;
    } else {
        q = (int)fdiv((uint32_t)t, a.d_tk);
        tk = kg * a.kpg + (t - q * a.kpg);
        t = q;
    }
    q = (int)fdiv((uint32_t)t, a.d_bg);
    const int tbl = t - q * a.b_group;
    t = q;
    q = (int)fdiv((uint32_t)t, a.d_tw);
    const int tw = t - q * a.tiles_w;
    t = q;
    q = (int)fdiv((uint32_t)t, a.d_th);
    const int th = t - q * a.tiles_h;
    const int tb = q * a.b_group + tbl;
    TileCoord tc;
    tc.k0 = tk * KT;
    tc.b0 = tb * TB;
    tc.w0 = tw * TW;
    tc.h0 = th * TH;
    return tc;
}

__device__ __forceinline__ TileCoord decode_tile(const KernelArgs& a, int KT, int TB, int TW, int TH) {
    return tile_coords(a, xcd_tile(a, blockIdx.x), KT, TB, TW, TH);
}

// ---------------------------------------------------------------------------------------------------------------
// fp32
// LDS: s_img[x*xpitch + (y*CT + c)*TB + b]  (+ a zeroed row at zero_off),  s_flt[k_l*fpitch + r*QE + s*CT + c]
// The contraction over (s,c) for a fixed r is one contiguous run of Q = bS*CT rows in both tiles.

template <int THREADS, int TB, int VI>
__device__ __forceinline__ void stage_image_f32(const KernelArgs& a, float* s_img, int tid, int x0, int y0, int c0,
                                                int b0) {
    constexpr int VPR = TB / VI;
    constexpr int U = 4;
    const int total = a.XS * a.YS * a.CT * VPR;
    const float* __restrict__ img = (const float*)a.image;
    for (int base = tid; base < total; base += THREADS * U) {
        float v[U][VI];
        int off[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int idx = base + u * THREADS;
            off[u] = -1;
#pragma unroll
            for (int e = 0; e < VI; ++e) v[u][e] = 0.f;
            if (idx < total) {
                const uint32_t row = (uint32_t)idx / VPR;
                const int bv = idx % VPR;
                const uint32_t t = fdiv(row, a.d_CT);
                const int c = row - t * a.CT;
                const uint32_t x = fdiv(t, a.d_YS);
                const int y = t - x * a.YS;
                const int gx = x0 + (int)x, gy = y0 + y, gc = c0 + c, gb = b0 + bv * VI;
                off[u] = (int)x * a.xpitch + (y * a.CT + c) * TB + bv * VI;
                if (gx < a.IW && gy < a.IH && gc < a.C && gb < a.B) {
                    const int64_t g = (((int64_t)gx * a.IH + gy) * a.C + gc) * a.B + gb;
                    if constexpr (VI == 4) {
                        const f32x4 q = *(const f32x4*)(img + g);
                        v[u][0] = q[0];
                        v[u][1] = q[1];
                        v[u][2] = q[2];
                        v[u][3] = q[3];
                    } else {
                        v[u][0] = img[g];
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (off[u] >= 0) {
                if constexpr (VI == 4) {
                    f32x4 q = {v[u][0], v[u][1], v[u][2], v[u][3]};
                    *(f32x4*)(s_img + off[u]) = q;
                } else {
                    s_img[off[u]] = v[u][0];
                }
            }
        }
    }
}

template <int THREADS, int KT, int VF>
__device__ __forceinline__ void stage_filter_f32(const KernelArgs& a, float* s_flt, int tid, int k0, int r0, int s0,
                                                 int c0) {
    constexpr int U = 4;
    const int CTV = a.CT / VF;
    const int total = KT * a.bR * a.bS * CTV;
    const float* __restrict__ flt = (const float*)a.filter;
    for (int base = tid; base < total; base += THREADS * U) {
        float v[U][VF];
        int off[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int idx = base + u * THREADS;
            off[u] = -1;
#pragma unroll
            for (int e = 0; e < VF; ++e) v[u][e] = 0.f;
            if (idx < total) {
                uint32_t t = fdiv((uint32_t)idx, a.d_C8);
                const int c = (idx - t * CTV) * VF;
                uint32_t t2 = fdiv(t, a.d_bS);
                const int s = t - t2 * a.bS;
                const uint32_t kl = fdiv(t2, a.d_bR);
                const int r = t2 - kl * a.bR;
                const int gk = k0 + (int)kl, gr = r0 + r, gs = s0 + s, gc = c0 + c;
                off[u] = (int)kl * a.fpitch + r * a.QE + s * a.CT + c;
                if (gk < a.K && gr < a.R && gs < a.S && gc < a.C) {
                    const int64_t g = (((int64_t)gk * a.R + gr) * a.S + gs) * a.C + gc;
                    if constexpr (VF == 4) {
                        const f32x4 q = *(const f32x4*)(flt + g);
                        v[u][0] = q[0];
                        v[u][1] = q[1];
                        v[u][2] = q[2];
                        v[u][3] = q[3];
                    } else {
                        v[u][0] = flt[g];
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (off[u] >= 0) {
#pragma unroll
                for (int e = 0; e < VF; ++e) s_flt[off[u] + e] = v[u][e];
            }
        }
    }
}

template <int WM, int WN, int MBLK, int NBLK, int TB, int TW, int TH>
__global__ void __launch_bounds__(WM* WN * 64) conv_f32_kernel(const KernelArgs a) {
    constexpr int THREADS = WM * WN * 64;
    constexpr int NT = TB * TW * TH;
    constexpr int KT = WM * MBLK * 32;
    extern __shared__ __align__(16) float smem_f[];
    float* s_img = smem_f;
    float* s_flt = smem_f + a.img_lds_elems;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;
    const int j = lane & 31, kk = lane >> 5;
    const TileCoord tc = decode_tile(a, KT, TB, TW, TH);

    int posoff[NBLK];
#pragma unroll
    for (int n = 0; n < NBLK; ++n) {
        int nn = (wn * NBLK + n) * 32 + j;
        if (nn >= NT) nn = 0;
        const int b_l = nn % TB, w_l = (nn / TB) % TW, h_l = nn / (TB * TW);
        posoff[n] = a.sw * w_l * a.xpitch + a.sh * h_l * a.ypitch + b_l;
    }

    f32x16 acc[MBLK][NBLK];
#pragma unroll
    for (int m = 0; m < MBLK; ++m)
#pragma unroll
        for (int n = 0; n < NBLK; ++n)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[m][n][v] = 0.f;

    // one-time zeros: the zero row read by the odd-length tail, and the pad column of each Filter row
    if (tid < 64) s_img[a.zero_off + tid] = 0.f;
    const int Q = a.bS * a.CT;
    if (Q & 1) {
        for (int idx = tid; idx < KT * a.bR; idx += THREADS) {
            const int kl = idx / a.bR, r = idx - kl * a.bR;
            s_flt[kl * a.fpitch + r * a.QE + Q] = 0.f;
        }
    }

    for (int r0 = 0; r0 < a.R; r0 += a.bR) {
        for (int s0 = 0; s0 < a.S; s0 += a.bS) {
            for (int c0 = 0; c0 < a.C; c0 += a.CT) {
                __syncthreads();
                const int x0 = a.sw * tc.w0 + r0, y0 = a.sh * tc.h0 + s0;
                if (a.vec_img) {
                    if constexpr (TB % 4 == 0) stage_image_f32<THREADS, TB, 4>(a, s_img, tid, x0, y0, c0, tc.b0);
                } else {
                    stage_image_f32<THREADS, TB, 1>(a, s_img, tid, x0, y0, c0, tc.b0);
                }
                if (a.vec_flt)
                    stage_filter_f32<THREADS, KT, 4>(a, s_flt, tid, tc.k0, r0, s0, c0);
                else
                    stage_filter_f32<THREADS, KT, 1>(a, s_flt, tid, tc.k0, r0, s0, c0);
                __syncthreads();

                const int rmax = min(a.bR, a.R - r0);
                for (int r = 0; r < rmax; ++r) {
                    const float* ap = s_flt + (wm * MBLK * 32 + j) * a.fpitch + r * a.QE + kk;
                    const float* bp = s_img + r * a.xpitch + kk * TB;
                    const int pairs = Q >> 1;
#pragma unroll 4
                    for (int q2 = 0; q2 < pairs; ++q2) {
                        float av[MBLK], bv[NBLK];
#pragma unroll
                        for (int m = 0; m < MBLK; ++m) av[m] = ap[m * 32 * a.fpitch + 2 * q2];
#pragma unroll
                        for (int n = 0; n < NBLK; ++n) bv[n] = bp[posoff[n] + 2 * q2 * TB];
#pragma unroll
                        for (int m = 0; m < MBLK; ++m)
#pragma unroll
                            for (int n = 0; n < NBLK; ++n)
                                acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[m], bv[n], acc[m][n], 0, 0, 0);
                    }
                    if (Q & 1) {
                        // last contraction index pairs with a zero: the kk = 1 half reads the pad column / zero row
                        float av[MBLK], bv[NBLK];
#pragma unroll
                        for (int m = 0; m < MBLK; ++m) av[m] = ap[m * 32 * a.fpitch + (Q - 1)];
#pragma unroll
                        for (int n = 0; n < NBLK; ++n)
                            bv[n] = kk ? s_img[a.zero_off + j] : bp[posoff[n] + (Q - 1) * TB];
#pragma unroll
                        for (int m = 0; m < MBLK; ++m)
#pragma unroll
                            for (int n = 0; n < NBLK; ++n)
                                acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[m], bv[n], acc[m][n], 0, 0, 0);
                    }
                }
            }
        }
    }

    // epilogue: every Out word of the tile is written once
#pragma unroll
    for (int n = 0; n < NBLK; ++n) {
        const int nn = (wn * NBLK + n) * 32 + j;
        const int b = tc.b0 + nn % TB, w = tc.w0 + (nn / TB) % TW, h = tc.h0 + nn / (TB * TW);
        const bool pos_ok = nn < NT && b < a.B && w < a.W && h < a.H;
#pragma unroll
        for (int m = 0; m < MBLK; ++m) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int k = tc.k0 + (wm * MBLK + m) * 32 + (v >> 2) * 8 + kk * 4 + (v & 3);
                if (pos_ok && k < a.K) a.out[(((int64_t)k * a.H + h) * a.W + w) * a.B + b] = acc[m][n][v];
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------------------
// bf16 inputs, fp32 accumulate
// LDS in 16-byte units (8 bf16 of consecutive c): s_img[x*xpitch + y*ypitch + c8*TB + b], so the MFMA B operand of a
// lane (8 consecutive contraction indices of one position) is one 16-byte read.  Global memory has b fastest, so the
// staging transposes 8x8 blocks in registers.  s_flt (bf16 elements): [k_l*fpitch + (r*bS+s)*CT + c].

__device__ __forceinline__ void transpose8x8_bf16(const uint4 (&in)[8], uint4 (&out)[8]) {
    // in[c] holds b0..b7 of row c; out[b] holds c0..c7 of column b
    uint32_t w[8][4];
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        w[c][0] = in[c].x;
        w[c][1] = in[c].y;
        w[c][2] = in[c].z;
        w[c][3] = in[c].w;
    }
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        uint32_t lo[4], hi[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t e = w[2 * q][m], o = w[2 * q + 1][m];
            lo[q] = (e & 0xffffu) | (o << 16);
            hi[q] = (e >> 16) | (o & 0xffff0000u);
        }
        out[2 * m] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
        out[2 * m + 1] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
    }
}

template <int THREADS, int TB>
__device__ __forceinline__ void stage_image_bf16_vec(const KernelArgs& a, uint4* s_img, int tid, int x0, int y0,
                                                     int c0, int b0) {
    constexpr int B8 = TB / 8;
    const int C8 = a.CT >> 3;
    const int total = a.XS * a.YS * C8 * B8;
    const uint16_t* __restrict__ img = (const uint16_t*)a.image;
    for (int idx = tid; idx < total; idx += THREADS) {
        const int b8 = idx % B8;
        const uint32_t t = (uint32_t)idx / B8;
        const uint32_t t2 = fdiv(t, a.d_C8);
        const int c8 = t - t2 * C8;
        const uint32_t x = fdiv(t2, a.d_YS);
        const int y = t2 - x * a.YS;
        const int gx = x0 + (int)x, gy = y0 + y, gb = b0 + b8 * 8;
        uint4 in[8], out[8];
        const bool ok = gx < a.IW && gy < a.IH && gb < a.B;
        const int64_t g0 = (((int64_t)gx * a.IH + gy) * a.C) * a.B + gb;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int gc = c0 + c8 * 8 + e;
            in[e] = make_uint4(0, 0, 0, 0);
            if (ok && gc < a.C) in[e] = *(const uint4*)(img + g0 + (int64_t)gc * a.B);
        }
        transpose8x8_bf16(in, out);
        uint4* dst = s_img + (int)x * a.xpitch + y * a.ypitch + c8 * TB + b8 * 8;
#pragma unroll
        for (int bb = 0; bb < 8; ++bb) dst[bb] = out[bb];
    }
}

template <int THREADS, int TB>
__device__ __forceinline__ void stage_image_bf16_scalar(const KernelArgs& a, uint4* s_img, int tid, int x0, int y0,
                                                        int c0, int b0) {
    const int total = a.XS * a.YS * a.CT * TB;
    const uint16_t* __restrict__ img = (const uint16_t*)a.image;
    uint16_t* s16 = (uint16_t*)s_img;
    for (int idx = tid; idx < total; idx += THREADS) {
        const int b = idx % TB;
        const uint32_t t = (uint32_t)idx / TB;
        const uint32_t t2 = fdiv(t, a.d_CT);
        const int c = t - t2 * a.CT;
        const uint32_t x = fdiv(t2, a.d_YS);
        const int y = t2 - x * a.YS;
        const int gx = x0 + (int)x, gy = y0 + y, gc = c0 + c, gb = b0 + b;
        uint16_t v = 0;
        if (gx < a.IW && gy < a.IH && gc < a.C && gb < a.B)
            v = img[(((int64_t)gx * a.IH + gy) * a.C + gc) * a.B + gb];
        s16[((int)x * a.xpitch + y * a.ypitch + (c >> 3) * TB + b) * 8 + (c & 7)] = v;
    }
}

template <int THREADS, int KT>
__device__ __forceinline__ void stage_filter_bf16(const KernelArgs& a, uint16_t* s_flt, int tid, int k0, int r0,
                                                  int s0, int c0) {
    const uint16_t* __restrict__ flt = (const uint16_t*)a.filter;
    const int RS = a.bR * a.bS;
    if (a.vec_flt) {
        const int C8 = a.CT >> 3;
        const int total = KT * RS * C8;
        for (int idx = tid; idx < total; idx += THREADS) {
            const uint32_t t = fdiv((uint32_t)idx, a.d_C8);
            const int c8 = idx - t * C8;
            const uint32_t kl = fdiv(t, a.d_RS);
            const int rs = t - kl * RS;
            const uint32_t r = fdiv((uint32_t)rs, a.d_bS);
            const int s = rs - r * a.bS;
            const int gk = k0 + (int)kl, gr = r0 + (int)r, gs = s0 + s, gc = c0 + c8 * 8;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (gk < a.K && gr < a.R && gs < a.S && gc < a.C)
                v = *(const uint4*)(flt + (((int64_t)gk * a.R + gr) * a.S + gs) * a.C + gc);
            *(uint4*)(s_flt + (int)kl * a.fpitch + rs * a.CT + c8 * 8) = v;
        }
    } else {
        const int total = KT * RS * a.CT;
        for (int idx = tid; idx < total; idx += THREADS) {
            const uint32_t t = fdiv((uint32_t)idx, a.d_CT);
            const int c = idx - t * a.CT;
            const uint32_t kl = fdiv(t, a.d_RS);
            const int rs = t - kl * RS;
            const uint32_t r = fdiv((uint32_t)rs, a.d_bS);
            const int s = rs - r * a.bS;
            const int gk = k0 + (int)kl, gr = r0 + (int)r, gs = s0 + s, gc = c0 + c;
            uint16_t v = 0;
            if (gk < a.K && gr < a.R && gs < a.S && gc < a.C)
                v = flt[(((int64_t)gk * a.R + gr) * a.S + gs) * a.C + gc];
            s_flt[(int)kl * a.fpitch + rs * a.CT + c] = v;
        }
    }
}

template <int WM, int WN, int MBLK, int NBLK, int TB, int TW, int TH>
__global__ void __launch_bounds__(WM* WN * 64) conv_bf16_kernel(const KernelArgs a) {
    constexpr int THREADS = WM * WN * 64;
    constexpr int NT = TB * TW * TH;
    constexpr int KT = WM * MBLK * 32;
    extern __shared__ __align__(16) uint4 smem_u[];
    uint4* s_img = smem_u;
    uint4* s_fltu = smem_u + a.img_lds_elems;
    uint16_t* s_flt = (uint16_t*)s_fltu;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;
    const int j = lane & 31, g = lane >> 5;
    const TileCoord tc = decode_tile(a, KT, TB, TW, TH);

    int posoff[NBLK];
#pragma unroll
    for (int n = 0; n < NBLK; ++n) {
        int nn = (wn * NBLK + n) * 32 + j;
        if (nn >= NT) nn = 0;
        const int b_l = nn % TB, w_l = (nn / TB) % TW, h_l = nn / (TB * TW);
        posoff[n] = a.sw * w_l * a.xpitch + a.sh * h_l * a.ypitch + b_l;
    }

    f32x16 acc[MBLK][NBLK];
#pragma unroll
    for (int m = 0; m < MBLK; ++m)
#pragma unroll
        for (int n = 0; n < NBLK; ++n)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[m][n][v] = 0.f;

    const int fp8 = a.fpitch >> 3;   // Filter row pitch in 16-byte units
    const int ct8 = a.CT >> 3;
    for (int r0 = 0; r0 < a.R; r0 += a.bR) {
        for (int s0 = 0; s0 < a.S; s0 += a.bS) {
            for (int c0 = 0; c0 < a.C; c0 += a.CT) {
                __syncthreads();
                const int x0 = a.sw * tc.w0 + r0, y0 = a.sh * tc.h0 + s0;
                if (a.vec_img) {
                    if constexpr (TB % 8 == 0) stage_image_bf16_vec<THREADS, TB>(a, s_img, tid, x0, y0, c0, tc.b0);
                } else {
                    stage_image_bf16_scalar<THREADS, TB>(a, s_img, tid, x0, y0, c0, tc.b0);
                }
                stage_filter_bf16<THREADS, KT>(a, s_flt, tid, tc.k0, r0, s0, c0);
                __syncthreads();

                const int rmax = min(a.bR, a.R - r0), smax = min(a.bS, a.S - s0);
                for (int r = 0; r < rmax; ++r) {
                    for (int s = 0; s < smax; ++s) {
                        const uint4* ap = s_fltu + (wm * MBLK * 32 + j) * fp8 + (r * a.bS + s) * ct8 + g;
                        const uint4* bp = s_img + r * a.xpitch + s * a.ypitch + g * TB;
                        const int steps = a.CT >> 4;
#pragma unroll 2
                        for (int cs = 0; cs < steps; ++cs) {
                            bf16x8 av[MBLK], bv[NBLK];
#pragma unroll
                            for (int m = 0; m < MBLK; ++m)
                                av[m] = __builtin_bit_cast(bf16x8, ap[m * 32 * fp8 + 2 * cs]);
#pragma unroll
                            for (int n = 0; n < NBLK; ++n)
                                bv[n] = __builtin_bit_cast(bf16x8, bp[posoff[n] + 2 * cs * TB]);
#pragma unroll
                            for (int m = 0; m < MBLK; ++m)
#pragma unroll
                                for (int n = 0; n < NBLK; ++n)
                                    acc[m][n] =
                                        __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[m], bv[n], acc[m][n], 0, 0, 0);
                        }
                    }
                }
            }
        }
    }

#pragma unroll
    for (int n = 0; n < NBLK; ++n) {
        const int nn = (wn * NBLK + n) * 32 + j;
        const int b = tc.b0 + nn % TB, w = tc.w0 + (nn / TB) % TW, h = tc.h0 + nn / (TB * TW);
        const bool pos_ok = nn < NT && b < a.B && w < a.W && h < a.H;
#pragma unroll
        for (int m = 0; m < MBLK; ++m) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int k = tc.k0 + (wm * MBLK + m) * 32 + (v >> 2) * 8 + g * 4 + (v & 3);
                if (pos_ok && k < a.K) a.out[(((int64_t)k * a.H + h) * a.W + w) * a.B + b] = acc[m][n][v];
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------------------
// Pipelined persistent kernels.
//
// A workgroup walks units u = (Out tile, contraction slice): tiles blockIdx.x, blockIdx.x + gridDim.x, ... and, inside a
// tile, the slices (r0, s0, c0) of the contraction.  While unit u is multiplied out of LDS buffer u&1, the 16-byte
// staging items of unit u+1 are already in flight from global memory into registers; they are written to the other
// LDS buffer after the multiply, so one barrier per unit suffices: a thread can only reach the stores of unit u+1
// after every thread has passed the barrier of unit u, i.e. has finished reading the buffer being overwritten.
// Which item a thread fetches is fixed for the whole kernel (it depends only on the slice geometry): its byte offset
// from the unit's origin in global memory and its LDS address are computed once, so fetching a unit costs one
// scalar base address and one load per item.  Units whose tile or slice overhangs an array take a slower path that
// checks every item and zero-fills.  The loops are finite and identical for all threads of a workgroup: every wave
// reaches every barrier.

struct UnitPos {
    int t;       // position in this workgroup's tile sequence (tile list index), >= n_tiles when exhausted
    int r0, s0, c0;
    TileCoord tc;
};

__device__ __forceinline__ TileCoord decode_tile_index(const KernelArgs& a, int t, int KT, int TB, int TW, int TH) {
    return tile_coords(a, xcd_tile(a, t), KT, TB, TW, TH);
}

__device__ __forceinline__ void advance_unit(const KernelArgs& a, UnitPos& p, int KT, int TB, int TW, int TH) {
    p.c0 += a.CT;
    if (p.c0 >= a.C) {
        p.c0 = 0;
        p.s0 += a.bS;
        if (p.s0 >= a.S) {
            p.s0 = 0;
            p.r0 += a.bR;
            if (p.r0 >= a.R) {
                p.r0 = 0;
                p.t += gridDim.x;
                if (p.t < a.n_tiles) p.tc = decode_tile_index(a, p.t, KT, TB, TW, TH);
            }
        }
    }
}

// What is uniform over one unit: buffer resources whose base is the origin of the unit's Image / Filter tile (so an
// item's address is a scalar descriptor plus a 32-bit offset; num_records is what is left of the array, and items that
// fall outside the arrays are never addressed: they read the origin and are replaced by zeros), and how far the
// arrays extend from those origins.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

struct UnitBase {
    __amdgpu_buffer_rsrc_t img, flt;
    int lx, ly, lc, lb, lk, lr, ls;
    bool img_inside, flt_inside;
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, int64_t bytes_left) {
    const int32_t n = (int32_t)(bytes_left > 0x7fffffffll ? 0x7fffffffll : bytes_left);
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, n, 0x00020000);
}

template <int ESZ>
__device__ __forceinline__ UnitBase unit_base(const KernelArgs& a, const UnitPos& p, int KT, int TB) {
    UnitBase u;
    const int x0 = a.sw * p.tc.w0 + p.r0, y0 = a.sh * p.tc.h0 + p.s0;
    const int64_t io = (((int64_t)x0 * a.IH + y0) * a.C + p.c0) * a.B + p.tc.b0;
    const int64_t fo = (((int64_t)p.tc.k0 * a.R + p.r0) * a.S + p.s0) * a.C + p.c0;
    const int64_t in = (int64_t)a.IW * a.IH * a.C * a.B, fn = (int64_t)a.K * a.R * a.S * a.C;
    u.img = make_rsrc((const char*)a.image + io * ESZ, (in - io) * ESZ);
    u.flt = make_rsrc((const char*)a.filter + fo * ESZ, (fn - fo) * ESZ);
    u.lx = a.IW - x0;
    u.ly = a.IH - y0;
    u.lc = a.C - p.c0;
    u.lb = a.B - p.tc.b0;
    u.lk = a.K - p.tc.k0;
    u.lr = a.R - p.r0;
    u.ls = a.S - p.s0;
    u.img_inside = u.lx >= a.XS && u.ly >= a.YS && u.lc >= a.CT && u.lb >= TB;
    u.flt_inside = u.lk >= KT && u.lr >= a.bR && u.ls >= a.bS && u.lc >= a.CT;
    return u;
}

__device__ __forceinline__ f32x4 buf_load_f32x4(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
    return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0));
}
__device__ __forceinline__ uint4 buf_load_u4(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0);
    return make_uint4(v[0], v[1], v[2], v[3]);
}

// ---- staging: which 16-byte items a staging thread moves, fixed for the whole kernel -------------------------------

// Per item a thread keeps two registers: the byte offset from the unit's origin in global memory and the LDS
// address.  Units that overhang an array decode the item's coordinates again to decide what to zero-fill.

template <int STHREADS, int TB, int MAXI, int MAXF>
struct F32Stager {
    static constexpr int VPR = TB / 4;
    uint32_t i_g[MAXI], f_g[MAXF];
    int i_lds[MAXI], f_lds[MAXF];
    int stid;

    __device__ __forceinline__ void img_coords(const KernelArgs& a, int idx, int& x, int& y, int& c, int& bv) const {
        const uint32_t row = (uint32_t)idx / VPR;
        bv = idx % VPR;
        const uint32_t t = fdiv(row, a.d_CT);
        c = row - t * a.CT;
        const uint32_t xx = fdiv(t, a.d_YS);
        y = t - xx * a.YS;
        x = (int)xx;
    }
    __device__ __forceinline__ void flt_coords(const KernelArgs& a, int idx, int& kl, int& r, int& s, int& c) const {
        const int CTV = a.CT >> 2;
        const uint32_t t = fdiv((uint32_t)idx, a.d_C8);
        c = (idx - t * CTV) * 4;
        const uint32_t t2 = fdiv(t, a.d_bS);
        s = t - t2 * a.bS;
        const uint32_t k = fdiv(t2, a.d_bR);
        r = t2 - k * a.bR;
        kl = (int)k;
    }

    __device__ __forceinline__ void init(const KernelArgs& a, int stid_) {
        stid = stid_;
#pragma unroll
        for (int i = 0; i < MAXI; ++i) {
            const int idx = stid + i * STHREADS;
            i_lds[i] = 0;
            i_g[i] = 0;
            if (idx < a.img_items) {
                int x, y, c, bv;
                img_coords(a, idx, x, y, c, bv);
                i_lds[i] = x * a.xpitch + (y * a.CT + c) * TB + bv * 4;
                i_g[i] = ((((uint32_t)x * a.IH + y) * a.C + c) * a.B + bv * 4) * 4u;
            }
        }
#pragma unroll
        for (int i = 0; i < MAXF; ++i) {
            const int idx = stid + i * STHREADS;
            f_lds[i] = 0;
            f_g[i] = 0;
            if (!a.flt_resident && idx < a.flt_items) {
                int kl, r, s, c;
                flt_coords(a, idx, kl, r, s, c);
                f_lds[i] = kl * a.fpitch + r * a.QE + s * a.CT + c;
                f_g[i] = ((((uint32_t)kl * a.R + r) * a.S + s) * a.C + c) * 4u;
            }
        }
    }

    __device__ __forceinline__ void issue(const KernelArgs& a, const UnitBase& u, f32x4 (&ireg)[MAXI],
                                          f32x4 (&freg)[MAXF]) const {
        issue_img(a, u, ireg);
        issue_flt(a, u, freg);
    }
    __device__ __forceinline__ void store(const KernelArgs& a, float* smem, int buf, const f32x4 (&ireg)[MAXI],
                                          const f32x4 (&freg)[MAXF]) const {
        store_img(a, smem, buf, ireg);
        store_flt(a, smem, buf, freg);
    }

    __device__ __forceinline__ void issue_img(const KernelArgs& a, const UnitBase& u, f32x4 (&ireg)[MAXI]) const {
        if (u.img_inside) {
#pragma unroll
            for (int i = 0; i < MAXI; ++i) ireg[i] = buf_load_f32x4(u.img, i_g[i], 0);
        } else {
#pragma unroll
            for (int i = 0; i < MAXI; ++i) {
                const int idx = stid + i * STHREADS;
                int x, y, c, bv;
                img_coords(a, idx, x, y, c, bv);
                const bool ok = idx < a.img_items && x < u.lx && y < u.ly && c < u.lc && bv * 4 < u.lb;
                const f32x4 v = buf_load_f32x4(u.img, ok ? i_g[i] : 0u, 0);
                const f32x4 z = {0.f, 0.f, 0.f, 0.f};
                ireg[i] = ok ? v : z;
            }
        }
    }
    __device__ __forceinline__ void issue_flt(const KernelArgs& a, const UnitBase& u, f32x4 (&freg)[MAXF]) const {
        if (!a.flt_resident) {
            if (u.flt_inside) {
#pragma unroll
                for (int i = 0; i < MAXF; ++i) freg[i] = buf_load_f32x4(u.flt, f_g[i], 0);
            } else {
#pragma unroll
                for (int i = 0; i < MAXF; ++i) {
                    const int idx = stid + i * STHREADS;
                    int kl, r, s, c;
                    flt_coords(a, idx, kl, r, s, c);
                    const bool ok = idx < a.flt_items && kl < u.lk && r < u.lr && s < u.ls && c < u.lc;
                    const f32x4 v = buf_load_f32x4(u.flt, ok ? f_g[i] : 0u, 0);
                    const f32x4 z = {0.f, 0.f, 0.f, 0.f};
                    freg[i] = ok ? v : z;
                }
            }
        }
    }

    __device__ __forceinline__ void store_img(const KernelArgs& a, float* smem, int buf,
                                              const f32x4 (&ireg)[MAXI]) const {
        float* s_img = smem + buf * a.img_buf;
#pragma unroll
        for (int i = 0; i < MAXI; ++i)
            if (stid + i * STHREADS < a.img_items) *(f32x4*)(s_img + i_lds[i]) = ireg[i];
    }
    __device__ __forceinline__ void store_flt(const KernelArgs& a, float* smem, int buf,
                                              const f32x4 (&freg)[MAXF]) const {
        if (!a.flt_resident) {
            float* s_flt = smem + a.flt_off + buf * a.flt_buf;
#pragma unroll
            for (int i = 0; i < MAXF; ++i)
                if (stid + i * STHREADS < a.flt_items) {
                    s_flt[f_lds[i] + 0] = freg[i][0];
                    s_flt[f_lds[i] + 1] = freg[i][1];
                    s_flt[f_lds[i] + 2] = freg[i][2];
                    s_flt[f_lds[i] + 3] = freg[i][3];
                }
        }
    }
};

// bf16: LDS holds the Image tile in 16-byte units of 8 consecutive channels of one position,
// s_img[x*xpitch + y*ypitch + c8*TB + (b ^ key)], so that the MFMA B operand of a lane is ONE 16-byte read (LDS reads
// run at full bandwidth only for 16-byte accesses).  Global memory has b fastest, so a staging item is an 8x8 block
// (8 channels x 8 images) that is transposed in registers; the XOR key (low three bits of b, a function of the item)
// spreads the eight 16-byte stores of neighbouring lanes over the banks and is undone, per lane, in the reads.
template <int TB>
__device__ __forceinline__ int store_key(int b8, int c8) {
    constexpr int B8 = TB / 8;
    return B8 == 4 ? ((b8 + 4 * (c8 & 1)) & 7) : (b8 & 7);
}

template <int STHREADS, int TB, int MAXI, int MAXF>
struct Bf16Stager {
    static constexpr int B8 = TB / 8;
    uint32_t i_g[MAXI], f_g[MAXF];
    int i_lds[MAXI], i_key[MAXI], f_lds[MAXF];
    uint32_t row_bytes;
    int stid;

    __device__ __forceinline__ void img_coords(const KernelArgs& a, int idx, int& x, int& y, int& c8, int& b8) const {
        const int C8 = a.CT >> 3;
        b8 = idx % B8;
        const uint32_t t = (uint32_t)idx / B8;
        const uint32_t t2 = fdiv(t, a.d_C8);
        c8 = t - t2 * C8;
        const uint32_t xx = fdiv(t2, a.d_YS);
        y = t2 - xx * a.YS;
        x = (int)xx;
    }
    __device__ __forceinline__ void flt_coords(const KernelArgs& a, int idx, int& kl, int& r, int& s, int& c8) const {
        const int C8 = a.CT >> 3, RS = a.bR * a.bS;
        const uint32_t t = fdiv((uint32_t)idx, a.d_C8);
        c8 = idx - t * C8;
        const uint32_t k = fdiv(t, a.d_RS);
        const int rs = t - k * RS;
        const uint32_t rr = fdiv((uint32_t)rs, a.d_bS);
        s = rs - rr * a.bS;
        r = (int)rr;
        kl = (int)k;
    }

    __device__ __forceinline__ void init(const KernelArgs& a, int stid_) {
        stid = stid_;
        row_bytes = (uint32_t)a.B * 2u;
#pragma unroll
        for (int i = 0; i < MAXI; ++i) {
            const int idx = stid + i * STHREADS;
            i_lds[i] = 0;
            i_g[i] = 0;
            i_key[i] = 0;
            if (idx < a.img_items) {
                int x, y, c8, b8;
                img_coords(a, idx, x, y, c8, b8);
                i_lds[i] = x * a.xpitch + y * a.ypitch + c8 * TB + b8 * 8;
                i_key[i] = store_key<TB>(b8, c8);
                i_g[i] = ((((uint32_t)x * a.IH + y) * a.C + c8 * 8) * a.B + b8 * 8) * 2u;
            }
        }
#pragma unroll
        for (int i = 0; i < MAXF; ++i) {
            const int idx = stid + i * STHREADS;
            f_lds[i] = 0;
            f_g[i] = 0;
            if (!a.flt_resident && idx < a.flt_items) {
                int kl, r, s, c8;
                flt_coords(a, idx, kl, r, s, c8);
                f_lds[i] = (kl * a.fpitch + (r * a.bS + s) * a.CT) / 8 + c8;
                f_g[i] = ((((uint32_t)kl * a.R + r) * a.S + s) * a.C + c8 * 8) * 2u;
            }
        }
    }

    __device__ __forceinline__ void issue(const KernelArgs& a, const UnitBase& u, uint4 (&ireg)[MAXI][8],
                                          uint4 (&freg)[MAXF]) const {
        issue_img(a, u, ireg);
        issue_flt(a, u, freg);
    }
    __device__ __forceinline__ void store(const KernelArgs& a, uint4* smem, int buf, const uint4 (&ireg)[MAXI][8],
                                          const uint4 (&freg)[MAXF]) const {
        store_img(a, smem, buf, ireg);
        store_flt(a, smem, buf, freg);
    }

    __device__ __forceinline__ void issue_img(const KernelArgs& a, const UnitBase& u, uint4 (&ireg)[MAXI][8]) const {
        if (u.img_inside) {
#pragma unroll
            for (int i = 0; i < MAXI; ++i)
#pragma unroll
                for (int e = 0; e < 8; ++e) ireg[i][e] = buf_load_u4(u.img, i_g[i], e * row_bytes);
        } else {
#pragma unroll
            for (int i = 0; i < MAXI; ++i) {
                const int idx = stid + i * STHREADS;
                int x, y, c8, b8;
                img_coords(a, idx, x, y, c8, b8);
                const bool ok = idx < a.img_items && x < u.lx && y < u.ly && b8 * 8 < u.lb;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const bool oke = ok && c8 * 8 + e < u.lc;
                    const uint4 v = buf_load_u4(u.img, oke ? i_g[i] + e * row_bytes : 0u, 0);
                    ireg[i][e] = oke ? v : make_uint4(0, 0, 0, 0);
                }
            }
        }
    }
    __device__ __forceinline__ void issue_flt(const KernelArgs& a, const UnitBase& u, uint4 (&freg)[MAXF]) const {
        if (!a.flt_resident) {
            if (u.flt_inside) {
#pragma unroll
                for (int i = 0; i < MAXF; ++i) freg[i] = buf_load_u4(u.flt, f_g[i], 0);
            } else {
#pragma unroll
                for (int i = 0; i < MAXF; ++i) {
                    const int idx = stid + i * STHREADS;
                    int kl, r, s, c8;
                    flt_coords(a, idx, kl, r, s, c8);
                    const bool ok = idx < a.flt_items && kl < u.lk && r < u.lr && s < u.ls && c8 * 8 < u.lc;
                    const uint4 v = buf_load_u4(u.flt, ok ? f_g[i] : 0u, 0);
                    freg[i] = ok ? v : make_uint4(0, 0, 0, 0);
                }
            }
        }
    }

    __device__ __forceinline__ void store_img(const KernelArgs& a, uint4* smem, int buf,
                                              const uint4 (&ireg)[MAXI][8]) const {
        uint4* s_img = smem + buf * a.img_buf;
#pragma unroll
        for (int i = 0; i < MAXI; ++i)
            if (stid + i * STHREADS < a.img_items) {
                // 8x8 transpose, two columns (b = 2m, 2m+1) at a time to keep few registers live
                uint4* dst = s_img + i_lds[i];
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    uint32_t lo[4], hi[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const uint4 re = ireg[i][2 * q], ro = ireg[i][2 * q + 1];
                        const uint32_t e = m == 0 ? re.x : m == 1 ? re.y : m == 2 ? re.z : re.w;
                        const uint32_t o = m == 0 ? ro.x : m == 1 ? ro.y : m == 2 ? ro.z : ro.w;
                        lo[q] = (e & 0xffffu) | (o << 16);
                        hi[q] = (e >> 16) | (o & 0xffff0000u);
                    }
                    dst[(2 * m) ^ i_key[i]] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
                    dst[(2 * m + 1) ^ i_key[i]] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
                }
            }
    }
    __device__ __forceinline__ void store_flt(const KernelArgs& a, uint4* smem, int buf,
                                              const uint4 (&freg)[MAXF]) const {
        if (!a.flt_resident) {
            uint4* s_flt = smem + a.flt_off + buf * a.flt_buf;
#pragma unroll
            for (int i = 0; i < MAXF; ++i)
                if (stid + i * STHREADS < a.flt_items) s_flt[f_lds[i]] = freg[i];
        }
    }
};

// Scheduling hint for a region that holds NMFMA matrix instructions and NDS LDS reads that do not depend on each
// other: ask the backend to issue them alternately (one MFMA, then its share of the reads), so that the reads of the
// next step are issued in the shadow of the matrix pipe instead of in front of it.  A wave issues in order: what is
// placed behind a run of MFMAs cannot start until the last of them has been issued.
template <int NMFMA, int NDS>
__device__ __forceinline__ void interleave_hint() {
    constexpr int PER = (NDS + NMFMA - 1) / NMFMA;
#pragma unroll
    for (int i = 0; i < NMFMA; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);     // one MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, PER, 0);   // up to PER LDS reads
    }
}

// The same with the reads packed PER to an MFMA at the front of the region, for regions that end in a wait for all of
// their reads: the last read then has the remaining MFMAs to land in.
template <int NMFMA, int NDS, int PER>
__device__ __forceinline__ void interleave_front_hint() {
#pragma unroll
    for (int i = 0; i < NMFMA; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (i * PER < NDS) __builtin_amdgcn_sched_group_barrier(0x100, PER, 0);
    }
}

// ---- compute: one unit out of LDS ---------------------------------------------------------------------------------

// fp32: one MFMA consumes two contraction indices.  Fragments are fetched U index pairs at a time into one of two
// register sets, so the LDS reads of the next U pairs are in flight while the MFMAs of the current U pairs issue.
template <int MBLK, int NBLK, int TB>
__device__ __forceinline__ void f32_compute_unit(const KernelArgs& a, const float* s_img, const float* s_flt,
                                                 const float* s_zero, const int (&posoff)[NBLK],
                                                 f32x16 (&acc)[MBLK][NBLK], int row0, int j, int kk, int r0) {
    constexpr int U = 4;
    const int Q = a.bS * a.CT;
    const int rmax = min(a.bR, a.R - r0);
    const int pairs = Q >> 1;
    const int chunks = pairs / U;
    for (int r = 0; r < rmax; ++r) {
        const float* ap = s_flt + (row0 + j) * a.fpitch + r * a.QE + kk;
        const float* bp = s_img + r * a.xpitch + kk * TB;
        auto load_chunk = [&](int q2, float(&av)[U][MBLK], float(&bv)[U][NBLK]) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int m = 0; m < MBLK; ++m) av[u][m] = ap[m * 32 * a.fpitch + 2 * (q2 + u)];
#pragma unroll
                for (int n = 0; n < NBLK; ++n) bv[u][n] = bp[posoff[n] + 2 * (q2 + u) * TB];
            }
        };
        auto mfma_chunk = [&](const float(&av)[U][MBLK], const float(&bv)[U][NBLK]) {
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int m = 0; m < MBLK; ++m)
#pragma unroll
                    for (int n = 0; n < NBLK; ++n)
                        acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u][m], bv[u][n], acc[m][n], 0, 0, 0);
        };
        float a0[U][MBLK], b0[U][NBLK], a1[U][MBLK], b1[U][NBLK];
        // branch-free body: past the end the last chunk is simply read again
        const int last = chunks > 0 ? chunks - 1 : 0;
        if (chunks > 0) load_chunk(0, a0, b0);
        int c = 0;
        for (; c + 2 <= chunks; c += 2) {
            load_chunk(min(c + 1, last) * U, a1, b1);
            mfma_chunk(a0, b0);
            interleave_hint<U * MBLK * NBLK, U*(MBLK + NBLK)>();
            load_chunk(min(c + 2, last) * U, a0, b0);
            mfma_chunk(a1, b1);
            interleave_hint<U * MBLK * NBLK, U*(MBLK + NBLK)>();
        }
        if (c < chunks) mfma_chunk(a0, b0);
        for (int q2 = chunks * U; q2 < pairs; ++q2) {
            float av[MBLK], bv[NBLK];
#pragma unroll
            for (int m = 0; m < MBLK; ++m) av[m] = ap[m * 32 * a.fpitch + 2 * q2];
#pragma unroll
            for (int n = 0; n < NBLK; ++n) bv[n] = bp[posoff[n] + 2 * q2 * TB];
#pragma unroll
            for (int m = 0; m < MBLK; ++m)
#pragma unroll
                for (int n = 0; n < NBLK; ++n)
                    acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[m], bv[n], acc[m][n], 0, 0, 0);
        }
        if (Q & 1) {
            // last contraction index pairs with a zero: the kk = 1 half reads the pad column / zero row
            float av[MBLK], bv[NBLK];
#pragma unroll
            for (int m = 0; m < MBLK; ++m) av[m] = ap[m * 32 * a.fpitch + (Q - 1)];
#pragma unroll
            for (int n = 0; n < NBLK; ++n) bv[n] = kk ? s_zero[j] : bp[posoff[n] + (Q - 1) * TB];
#pragma unroll
            for (int m = 0; m < MBLK; ++m)
#pragma unroll
                for (int n = 0; n < NBLK; ++n)
                    acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[m], bv[n], acc[m][n], 0, 0, 0);
        }
    }
}

// BR > 0 selects the filter-row reuse path (needs sigma_w = 1, b_r = BR, TB = 32 and one wave spanning the tile's
// width): for one filter row offset s and one 16-channel step, a wave reads the TW+BR-1 Image fragments of its row
// once and uses each of them for up to BR filter taps r -- the register-level form of the reuse that lets the
// small-filter bound of Section 4.3 sit below the matmul bound.  Fragments are double-buffered in registers so the
// LDS reads of step t+1 overlap the MFMAs of step t.
template <int MBLK, int NBLK, int TB, int TW, int BR>
__device__ __forceinline__ void bf16_compute_unit(const KernelArgs& a, const uint4* s_img, const uint4* s_flt,
                                                  const int (&posoff)[NBLK], f32x16 (&acc)[MBLK][NBLK], int row0,
                                                  int j, int g, int r0, int s0) {
    const int fp8 = a.fpitch >> 3, ct8 = a.CT >> 3;
    const int rmax = min(a.bR, a.R - r0), smax = min(a.bS, a.S - s0);
    const int steps = a.CT >> 4;
    if constexpr (BR > 0) {
        static_assert(TB == 32 && NBLK == TW, "row reuse: a wave owns TW consecutive columns of 32 images");
        constexpr int NX = TW + BR - 1;
        auto load_frags = [&](int s, int cs, bf16x8(&A)[MBLK][BR], bf16x8(&X)[NX]) {
            const uint4* ap = s_flt + (row0 + j) * fp8 + s * ct8 + g + 2 * cs;
#pragma unroll
            for (int m = 0; m < MBLK; ++m)
#pragma unroll
                for (int r = 0; r < BR; ++r) A[m][r] = __builtin_bit_cast(bf16x8, ap[m * 32 * fp8 + r * a.bS * ct8]);
            const uint4* bp = s_img + posoff[0] + s * a.ypitch + 2 * cs * TB;
#pragma unroll
            for (int x = 0; x < NX; ++x) X[x] = __builtin_bit_cast(bf16x8, bp[x * a.xpitch]);
        };
        auto mfmas = [&](const bf16x8(&A)[MBLK][BR], const bf16x8(&X)[NX]) {
#pragma unroll
            for (int r = 0; r < BR; ++r)
#pragma unroll
                for (int n = 0; n < TW; ++n)
#pragma unroll
                    for (int m = 0; m < MBLK; ++m)
                        acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[m][r], X[n + r], acc[m][n], 0, 0, 0);
        };
        // steps t = (s, cs) in order; the loop body has no branches, so the reads of step t+1 and the MFMAs of step t
        // sit in one scheduling region (past the end the last step is simply read again)
        const int T = smax * steps;
        int s_n = 0, cs_n = 0, t_n = 0;
        auto next_step = [&]() {
            const int adv = t_n < T - 1 ? 1 : 0;
            t_n += adv;
            cs_n += adv;
            const int wrap = cs_n == steps ? 1 : 0;
            cs_n = wrap ? 0 : cs_n;
            s_n += wrap;
        };
        bf16x8 A0[MBLK][BR], X0[NX], A1[MBLK][BR], X1[NX];
        load_frags(0, 0, A0, X0);
        int t = 0;
        for (; t + 2 <= T; t += 2) {
            next_step();
            load_frags(s_n, cs_n, A1, X1);
            mfmas(A0, X0);
            interleave_hint<BR * TW * MBLK, NX + MBLK * BR>();
            next_step();
            load_frags(s_n, cs_n, A0, X0);
            mfmas(A1, X1);
            interleave_hint<BR * TW * MBLK, NX + MBLK * BR>();
        }
        if (t < T) mfmas(A0, X0);
    } else {
        for (int r = 0; r < rmax; ++r) {
            for (int s = 0; s < smax; ++s) {
                const uint4* ap = s_flt + (row0 + j) * fp8 + (r * a.bS + s) * ct8 + g;
                const uint4* bp = s_img + r * a.xpitch + s * a.ypitch;
#pragma unroll 2
                for (int cs = 0; cs < steps; ++cs) {
                    bf16x8 av[MBLK], bv[NBLK];
#pragma unroll
                    for (int m = 0; m < MBLK; ++m) av[m] = __builtin_bit_cast(bf16x8, ap[m * 32 * fp8 + 2 * cs]);
#pragma unroll
                    for (int n = 0; n < NBLK; ++n) bv[n] = __builtin_bit_cast(bf16x8, bp[posoff[n] + 2 * cs * TB]);
#pragma unroll
                    for (int m = 0; m < MBLK; ++m)
#pragma unroll
                        for (int n = 0; n < NBLK; ++n)
                            acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[m], bv[n], acc[m][n], 0, 0, 0);
                }
            }
        }
    }
}

// The tile's contraction is complete: write every Out word of it once and reset the accumulators.
template <int MBLK, int NBLK, int TB, int TW, int TH>
__device__ __forceinline__ void write_tile(const KernelArgs& a, const TileCoord& tc, f32x16 (&acc)[MBLK][NBLK],
                                           int nblock0, int row0, int j, int q) {
    constexpr int NT = TB * TW * TH;
    // whole 128-byte lines per half-wave (tiles of 32 or more images, B a multiple of 32): stream them past the caches,
    // nobody reads them again; otherwise ordinary stores, so that the L2 puts the pieces of a line together
    const bool stream = TB >= 32 && a.B % 32 == 0;
#pragma unroll
    for (int n = 0; n < NBLK; ++n) {
        const int nn = (nblock0 + n) * 32 + j;
        const int b = tc.b0 + nn % TB, w = tc.w0 + (nn / TB) % TW, h = tc.h0 + nn / (TB * TW);
        const bool pos_ok = nn < NT && b < a.B && w < a.W && h < a.H;
#pragma unroll
        for (int m = 0; m < MBLK; ++m) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int k = tc.k0 + row0 + m * 32 + (v >> 2) * 8 + q * 4 + (v & 3);
                if (pos_ok && k < a.K) {
                    float* dst = &a.out[(((int64_t)k * a.H + h) * a.W + w) * a.B + b];
                    if (stream) __builtin_nontemporal_store(acc[m][n][v], dst);
                    else *dst = acc[m][n][v];
                }
                acc[m][n][v] = 0.f;
            }
        }
    }
}

template <int NBLK, int TB, int TW, int TH>
__device__ __forceinline__ void f32_posoff(const KernelArgs& a, int (&posoff)[NBLK], int nblock0, int j) {
    constexpr int NT = TB * TW * TH;
#pragma unroll
    for (int n = 0; n < NBLK; ++n) {
        int nn = (nblock0 + n) * 32 + j;
        if (nn >= NT) nn = 0;
        const int b_l = nn % TB, w_l = (nn / TB) % TW, h_l = nn / (TB * TW);
        posoff[n] = a.sw * w_l * a.xpitch + a.sh * h_l * a.ypitch + b_l;
    }
}

// LDS unit of a lane's B fragment for column block n at (r, s, c-step) = 0; c8 = 2*cs + g has the parity of g
template <int NBLK, int TB, int TW, int TH>
__device__ __forceinline__ void bf16_posoff(const KernelArgs& a, int (&posoff)[NBLK], int nblock0, int j, int g) {
    constexpr int NT = TB * TW * TH;
#pragma unroll
    for (int n = 0; n < NBLK; ++n) {
        int nn = (nblock0 + n) * 32 + j;
        if (nn >= NT) nn = 0;
        const int b_l = nn % TB, w_l = (nn / TB) % TW, h_l = nn / (TB * TW);
        const int b_sw = (b_l & ~7) | ((b_l & 7) ^ store_key<TB>(b_l >> 3, g));
        posoff[n] = a.sw * w_l * a.xpitch + a.sh * h_l * a.ypitch + g * TB + b_sw;
    }
}

// one-time zeros of the fp32 pipelined layouts: the zero row, and the pad column of every Filter row in every buffer
template <int STHREADS, int KT>
__device__ __forceinline__ void f32_pipe_zero_fill(const KernelArgs& a, float* smem, int stid) {
    if (stid < 64) smem[2 * a.img_buf + stid] = 0.f;
    const int Q = a.bS * a.CT;
    if (Q & 1) {
        const int nbuf = a.flt_resident ? 1 : 2;
        for (int idx = stid; idx < nbuf * KT * a.bR; idx += STHREADS) {
            const int bsel = idx / (KT * a.bR), rem = idx - bsel * KT * a.bR;
            const int kl = rem / a.bR, r = rem - kl * a.bR;
            smem[a.flt_off + bsel * a.flt_buf + kl * a.fpitch + r * a.QE + Q] = 0.f;
        }
    }
}

template <int MBLK, int NBLK>
__device__ __forceinline__ void zero_acc(f32x16 (&acc)[MBLK][NBLK]) {
#pragma unroll
    for (int m = 0; m < MBLK; ++m)
#pragma unroll
        for (int n = 0; n < NBLK; ++n)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[m][n][v] = 0.f;
}

__device__ __forceinline__ UnitPos first_unit(const KernelArgs& a, int KT, int TB, int TW, int TH) {
    UnitPos p;
    p.t = blockIdx.x;
    p.r0 = p.s0 = p.c0 = 0;
    p.tc = decode_tile_index(a, p.t < a.n_tiles ? p.t : 0, KT, TB, TW, TH);
    return p;
}

// ---- pipelined kernels: every wave stages and multiplies ----------------------------------------------------------

template <int WM, int WN, int MBLK, int NBLK, int TB, int TW, int TH, int MAXI, int MAXF>
__global__ void __launch_bounds__(WM* WN * 64) conv_f32_pipe_kernel(const KernelArgs a) {
    constexpr int THREADS = WM * WN * 64;
    constexpr int KT = WM * MBLK * 32;
    extern __shared__ __align__(16) float smem_f[];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WM, wn = wave / WM;
    const int j = lane & 31, kk = lane >> 5;

    int posoff[NBLK];
    f32_posoff<NBLK, TB, TW, TH>(a, posoff, wn * NBLK, j);
    F32Stager<THREADS, TB, MAXI, MAXF> st;
    st.init(a, tid);
    f32_pipe_zero_fill<THREADS, KT>(a, smem_f, tid);

    f32x4 ireg[MAXI], freg[MAXF];
    f32x16 acc[MBLK][NBLK];
    zero_acc(acc);

    UnitPos cur = first_unit(a, KT, TB, TW, TH);
    UnitPos nxt = cur;
    if (cur.t < a.n_tiles) {
        st.issue(a, unit_base<4>(a, cur, KT, TB), ireg, freg);
        advance_unit(a, nxt, KT, TB, TW, TH);
    }
    if (a.flt_resident) {
        // one Filter tile serves every unit of this workgroup: stage it once (any alignment, any C)
        if (a.vec_flt)
            stage_filter_f32<THREADS, KT, 4>(a, smem_f + a.flt_off, tid, 0, 0, 0, 0);
        else
            stage_filter_f32<THREADS, KT, 1>(a, smem_f + a.flt_off, tid, 0, 0, 0, 0);
    }
    int buf = 0;
    while (cur.t < a.n_tiles) {
        st.store(a, smem_f, buf, ireg, freg);
        __syncthreads();
        const bool have_next = nxt.t < a.n_tiles;
        if (have_next) st.issue(a, unit_base<4>(a, nxt, KT, TB), ireg, freg);
        f32_compute_unit<MBLK, NBLK, TB>(a, smem_f + buf * a.img_buf,
                                         smem_f + a.flt_off + (a.flt_resident ? 0 : buf) * a.flt_buf,
                                         smem_f + 2 * a.img_buf, posoff, acc, wm * MBLK * 32, j, kk, cur.r0);
        if (!have_next || nxt.t != cur.t)
            write_tile<MBLK, NBLK, TB, TW, TH>(a, cur.tc, acc, wn * NBLK, wm * MBLK * 32, j, kk);
        cur = nxt;
        if (have_next) advance_unit(a, nxt, KT, TB, TW, TH);
        buf ^= 1;
    }
}

template <int WM, int WN, int MBLK, int NBLK, int TB, int TW, int TH, int MAXI, int MAXF, int BR = 0>
__global__ void __launch_bounds__(WM* WN * 64) conv_bf16_pipe_kernel(const KernelArgs a) {
    constexpr int THREADS = WM * WN * 64;
    constexpr int KT = WM * MBLK * 32;
    extern __shared__ __align__(16) uint4 smem_u[];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WM, wn = wave / WM;
    const int j = lane & 31, g = lane >> 5;

    int posoff[NBLK];
    bf16_posoff<NBLK, TB, TW, TH>(a, posoff, wn * NBLK, j, g);
    Bf16Stager<THREADS, TB, MAXI, MAXF> st;
    st.init(a, tid);

    uint4 ireg[MAXI][8], freg[MAXF];
    f32x16 acc[MBLK][NBLK];
    zero_acc(acc);

    UnitPos cur = first_unit(a, KT, TB, TW, TH);
    UnitPos nxt = cur;
    if (cur.t < a.n_tiles) {
        st.issue(a, unit_base<2>(a, cur, KT, TB), ireg, freg);
        advance_unit(a, nxt, KT, TB, TW, TH);
    }
    if (a.flt_resident) stage_filter_bf16<THREADS, KT>(a, (uint16_t*)(smem_u + a.flt_off), tid, 0, 0, 0, 0);
    int buf = 0;
    while (cur.t < a.n_tiles) {
        st.store(a, smem_u, buf, ireg, freg);
        __syncthreads();
        const bool have_next = nxt.t < a.n_tiles;
        if (have_next) st.issue(a, unit_base<2>(a, nxt, KT, TB), ireg, freg);
        bf16_compute_unit<MBLK, NBLK, TB, TW, BR>(a, smem_u + buf * a.img_buf,
                                                   smem_u + a.flt_off + (a.flt_resident ? 0 : buf) * a.flt_buf, posoff,
                                                   acc, wm * MBLK * 32, j, g, cur.r0, cur.s0);
        if (!have_next || nxt.t != cur.t)
            write_tile<MBLK, NBLK, TB, TW, TH>(a, cur.tc, acc, wn * NBLK, wm * MBLK * 32, j, g);
        cur = nxt;
        if (have_next) advance_unit(a, nxt, KT, TB, TW, TH);
        buf ^= 1;
    }
}

// ---- wave-specialised kernels: 2*WM*WN waves, two per SIMD -------------------------------------------------------
// Waves [0, WM*WN) are consumers: they only read fragments from LDS, issue MFMAs and write finished Out tiles.
// Waves [WM*WN, 2*WM*WN) are producers: they only move Image and Filter words global -> registers -> LDS, two units
// ahead of the consumers (two register sets), so the memory latency and the staging arithmetic run in the shadow of
// the other wave's MFMAs on the same SIMD.  Synchronisation is one workgroup barrier per unit, B_u: a producer
// arrives after it has stored unit u, a consumer arrives before it multiplies unit u.  Passing B_u therefore tells
// the producers that unit u-1 has been multiplied (its buffer (u+1)&1 is free) and the consumers that unit u is in
// LDS.  Both roles walk the same unit sequence, so they execute the same number of barriers and the loops end.

template <int WM, int WN, int MBLK, int NBLK, int TB, int TW, int TH, int MAXI, int MAXF>
__global__ void __launch_bounds__(WM* WN * 128) conv_f32_ws_kernel(const KernelArgs a) {
    constexpr int CTHREADS = WM * WN * 64;
    constexpr int KT = WM * MBLK * 32;
    extern __shared__ __align__(16) float smem_f[];
    const int tid = threadIdx.x;
    const int wave_id = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: the role branch is wave-uniform

    if (wave_id >= WM * WN) {
        const int stid = tid - CTHREADS;
        F32Stager<CTHREADS, TB, MAXI, MAXF> st;
        st.init(a, stid);
        f32_pipe_zero_fill<CTHREADS, KT>(a, smem_f, stid);
        // Image words are fetched two units ahead (two register sets), Filter words one unit ahead
        f32x4 ireg0[MAXI], ireg1[MAXI], freg[MAXF];
        UnitPos su = first_unit(a, KT, TB, TW, TH);   // next unit to store
        UnitPos lu = su;                              // next unit whose Image tile is fetched
        UnitPos fu = su;                              // next unit whose Filter tile is fetched
        if (lu.t < a.n_tiles) {
            const UnitBase u = unit_base<4>(a, lu, KT, TB);
            st.issue_img(a, u, ireg0);
            st.issue_flt(a, u, freg);
            advance_unit(a, lu, KT, TB, TW, TH);
            advance_unit(a, fu, KT, TB, TW, TH);
        }
        if (lu.t < a.n_tiles) {
            st.issue_img(a, unit_base<4>(a, lu, KT, TB), ireg1);
            advance_unit(a, lu, KT, TB, TW, TH);
        }
        if (a.flt_resident) {
            if (a.vec_flt)
                stage_filter_f32<CTHREADS, KT, 4>(a, smem_f + a.flt_off, stid, 0, 0, 0, 0);
            else
                stage_filter_f32<CTHREADS, KT, 1>(a, smem_f + a.flt_off, stid, 0, 0, 0, 0);
        }
        while (su.t < a.n_tiles) {
            st.store_img(a, smem_f, 0, ireg0);
            st.store_flt(a, smem_f, 0, freg);
            if (lu.t < a.n_tiles) {
                st.issue_img(a, unit_base<4>(a, lu, KT, TB), ireg0);
                advance_unit(a, lu, KT, TB, TW, TH);
            }
            if (fu.t < a.n_tiles) {
                st.issue_flt(a, unit_base<4>(a, fu, KT, TB), freg);
                advance_unit(a, fu, KT, TB, TW, TH);
            }
            __syncthreads();
            advance_unit(a, su, KT, TB, TW, TH);
            if (su.t >= a.n_tiles) break;
            st.store_img(a, smem_f, 1, ireg1);
            st.store_flt(a, smem_f, 1, freg);
            if (lu.t < a.n_tiles) {
                st.issue_img(a, unit_base<4>(a, lu, KT, TB), ireg1);
                advance_unit(a, lu, KT, TB, TW, TH);
            }
            if (fu.t < a.n_tiles) {
                st.issue_flt(a, unit_base<4>(a, fu, KT, TB), freg);
                advance_unit(a, fu, KT, TB, TW, TH);
            }
            __syncthreads();
            advance_unit(a, su, KT, TB, TW, TH);
        }
    } else {
        const int lane = tid & 63, wave = wave_id;
        const int wm = wave % WM, wn = wave / WM;
        const int j = lane & 31, kk = lane >> 5;
        int posoff[NBLK];
        f32_posoff<NBLK, TB, TW, TH>(a, posoff, wn * NBLK, j);
        f32x16 acc[MBLK][NBLK];
        zero_acc(acc);
        UnitPos cur = first_unit(a, KT, TB, TW, TH);
        UnitPos nxt = cur;
        if (cur.t < a.n_tiles) advance_unit(a, nxt, KT, TB, TW, TH);
        int buf = 0;
        while (cur.t < a.n_tiles) {
            __syncthreads();
            f32_compute_unit<MBLK, NBLK, TB>(a, smem_f + buf * a.img_buf,
                                             smem_f + a.flt_off + (a.flt_resident ? 0 : buf) * a.flt_buf,
                                             smem_f + 2 * a.img_buf, posoff, acc, wm * MBLK * 32, j, kk, cur.r0);
            const bool have_next = nxt.t < a.n_tiles;
            if (!have_next || nxt.t != cur.t)
                write_tile<MBLK, NBLK, TB, TW, TH>(a, cur.tc, acc, wn * NBLK, wm * MBLK * 32, j, kk);
            cur = nxt;
            if (have_next) advance_unit(a, nxt, KT, TB, TW, TH);
            buf ^= 1;
        }
    }
}

template <int WM, int WN, int MBLK, int NBLK, int TB, int TW, int TH, int MAXI, int MAXF, int BR = 0>
__global__ void __launch_bounds__(WM* WN * 128) conv_bf16_ws_kernel(const KernelArgs a) {
    constexpr int CTHREADS = WM * WN * 64;
    constexpr int KT = WM * MBLK * 32;
    extern __shared__ __align__(16) uint4 smem_u[];
    const int tid = threadIdx.x;
    const int wave_id = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: the role branch is wave-uniform

    if (wave_id >= WM * WN) {
        const int stid = tid - CTHREADS;
        Bf16Stager<CTHREADS, TB, MAXI, MAXF> st;
        st.init(a, stid);
        // Memory latency under load is about two microseconds while a unit is multiplied in less than one, so the
        // producers keep several units in flight in registers: Image tiles ID units ahead, Filter tiles FD units ahead
        // (FD drops to 1 where two sets of each would not fit the register file).
        // The loop is unrolled over lcm(ID, FD) units so that every register set has a fixed name.
        constexpr int ID = 2, FD = (ID * MAXI * 32 + 2 * MAXF * 4 <= 160) ? 2 : 1, PERIOD = 2;
        uint4 ireg[ID][MAXI][8], freg[FD][MAXF];
        UnitPos su = first_unit(a, KT, TB, TW, TH);   // next unit to store
        UnitPos lu = su;                              // next unit whose Image tile is fetched
        UnitPos fu = su;                              // next unit whose Filter tile is fetched
#pragma unroll
        for (int d = 0; d < ID; ++d)
            if (lu.t < a.n_tiles) {
                st.issue_img(a, unit_base<2>(a, lu, KT, TB), ireg[d]);
                advance_unit(a, lu, KT, TB, TW, TH);
            }
#pragma unroll
        for (int d = 0; d < FD; ++d)
            if (fu.t < a.n_tiles) {
                st.issue_flt(a, unit_base<2>(a, fu, KT, TB), freg[d]);
                advance_unit(a, fu, KT, TB, TW, TH);
            }
        if (a.flt_resident) {
            stage_filter_bf16<CTHREADS, KT>(a, (uint16_t*)(smem_u + a.flt_off), stid, 0, 0, 0, 0);
        }
        bool done = su.t >= a.n_tiles;
        while (!done) {
#pragma unroll
            for (int ph = 0; ph < PERIOD; ++ph) {
                if (!done) {
                    st.store_img(a, smem_u, ph & 1, ireg[ph % ID]);
                    st.store_flt(a, smem_u, ph & 1, freg[ph % FD]);
                    if (lu.t < a.n_tiles) {
                        st.issue_img(a, unit_base<2>(a, lu, KT, TB), ireg[ph % ID]);
                        advance_unit(a, lu, KT, TB, TW, TH);
                    }
                    if (fu.t < a.n_tiles) {
                        st.issue_flt(a, unit_base<2>(a, fu, KT, TB), freg[ph % FD]);
                        advance_unit(a, fu, KT, TB, TW, TH);
                    }
                    __syncthreads();
                    advance_unit(a, su, KT, TB, TW, TH);
                    done = su.t >= a.n_tiles;
                }
            }
        }
    } else {
        const int lane = tid & 63, wave = wave_id;
        const int wm = wave % WM, wn = wave / WM;
        const int j = lane & 31, g = lane >> 5;
        int posoff[NBLK];
        bf16_posoff<NBLK, TB, TW, TH>(a, posoff, wn * NBLK, j, g);
        f32x16 acc[MBLK][NBLK];
        zero_acc(acc);
        UnitPos cur = first_unit(a, KT, TB, TW, TH);
        UnitPos nxt = cur;
        if (cur.t < a.n_tiles) advance_unit(a, nxt, KT, TB, TW, TH);
        int buf = 0;
        while (cur.t < a.n_tiles) {
            __syncthreads();
            bf16_compute_unit<MBLK, NBLK, TB, TW, BR>(a, smem_u + buf * a.img_buf,
                                                       smem_u + a.flt_off + (a.flt_resident ? 0 : buf) * a.flt_buf,
                                                       posoff, acc, wm * MBLK * 32, j, g, cur.r0, cur.s0);
            const bool have_next = nxt.t < a.n_tiles;
            if (!have_next || nxt.t != cur.t)
                write_tile<MBLK, NBLK, TB, TW, TH>(a, cur.tc, acc, wn * NBLK, wm * MBLK * 32, j, g);
            cur = nxt;
            if (have_next) advance_unit(a, nxt, KT, TB, TW, TH);
            buf ^= 1;
        }
    }
}

// ---- fp32 with 16-byte LDS fragments ("v4" layout) ---------------------------------------------------------------
// LDS instructions cost about the same pipe time whatever their width (measured: 4-, 8- and 16-byte reads issue at the
// same rate), so the fp32 path above, one 4-byte read per operand and MFMA, runs out of LDS issue slots before it
// runs out of MFMA time.  Here four consecutive contraction indices q = s*CT + c of one position sit in one 16-byte
// unit, img[x*xpitch + (q/4 rows)*TB + (b ^ key)], and the Filter row is 16-byte aligned, so one read per operand
// feeds four MFMAs.  An MFMA takes two indices, one per half-wave: in step e of group t the halves use
// q = 8t + e and 8t + 4 + e.  Staging items are 4 channels x 4 images, transposed by register renaming only.
// Needs CT % 4 == 0 (a channel count that is not a multiple of 4 is padded with zero channels inside LDS).

__device__ __forceinline__ int v4_swz(int b) { return (b & ~3) | ((b & 3) ^ ((b >> 3) & 3)); }

template <int STHREADS, int TB, int MAXI, int MAXF>
struct F32V4Stager {
    static constexpr int VPR = TB / 4;
    uint32_t i_g[MAXI], f_g[MAXF];
    int i_lds[MAXI], i_key[MAXI], f_lds[MAXF];
    uint32_t row_bytes;
    int stid;

    __device__ __forceinline__ void img_coords(const KernelArgs& a, int idx, int& x, int& y, int& c4, int& bv) const {
        bv = idx % VPR;
        const uint32_t t = (uint32_t)idx / VPR;
        const uint32_t G = fdiv(t, a.d_XS);           // x is the faster index: neighbouring lanes, different banks
        x = t - G * a.XS;
        const uint32_t yy = fdiv(G, a.d_C4);
        c4 = G - yy * (a.CT >> 2);
        y = (int)yy;
    }
    __device__ __forceinline__ void flt_coords(const KernelArgs& a, int idx, int& kl, int& r, int& s, int& c) const {
        const int CTV = a.CT >> 2;
        const uint32_t t = fdiv((uint32_t)idx, a.d_C4);
        c = (idx - t * CTV) * 4;
        const uint32_t t2 = fdiv(t, a.d_bS);
        s = t - t2 * a.bS;
        const uint32_t k = fdiv(t2, a.d_bR);
        r = t2 - k * a.bR;
        kl = (int)k;
    }

    __device__ __forceinline__ void init(const KernelArgs& a, int stid_) {
        stid = stid_;
        row_bytes = (uint32_t)a.B * 4u;
#pragma unroll
        for (int i = 0; i < MAXI; ++i) {
            const int idx = stid + i * STHREADS;
            i_lds[i] = 0;
            i_g[i] = 0;
            i_key[i] = 0;
            if (idx < a.img_items) {
                int x, y, c4, bv;
                img_coords(a, idx, x, y, c4, bv);
                i_lds[i] = x * a.xpitch + y * a.ypitch + c4 * TB + bv * 4;
                i_key[i] = (bv >> 1) & 3;
                i_g[i] = ((((uint32_t)x * a.IH + y) * a.C + c4 * 4) * a.B + bv * 4) * 4u;
            }
        }
#pragma unroll
        for (int i = 0; i < MAXF; ++i) {
            const int idx = stid + i * STHREADS;
            f_lds[i] = 0;
            f_g[i] = 0;
            if (!a.flt_resident && idx < a.flt_items) {
                int kl, r, s, c;
                flt_coords(a, idx, kl, r, s, c);
                f_lds[i] = (kl * a.fpitch + r * a.QE + s * a.CT + c) >> 2;
                f_g[i] = ((((uint32_t)kl * a.R + r) * a.S + s) * a.C + c) * 4u;
            }
        }
    }

    __device__ __forceinline__ void issue_img(const KernelArgs& a, const UnitBase& u, f32x4 (&ireg)[MAXI][4]) const {
        if (u.img_inside) {
#pragma unroll
            for (int i = 0; i < MAXI; ++i)
#pragma unroll
                for (int e = 0; e < 4; ++e) ireg[i][e] = buf_load_f32x4(u.img, i_g[i], e * row_bytes);
        } else {
#pragma unroll
            for (int i = 0; i < MAXI; ++i) {
                const int idx = stid + i * STHREADS;
                int x, y, c4, bv;
                img_coords(a, idx, x, y, c4, bv);
                const bool ok = idx < a.img_items && x < u.lx && y < u.ly && bv * 4 < u.lb;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const bool oke = ok && c4 * 4 + e < u.lc;
                    const f32x4 v = buf_load_f32x4(u.img, oke ? i_g[i] + e * row_bytes : 0u, 0);
                    const f32x4 z = {0.f, 0.f, 0.f, 0.f};
                    ireg[i][e] = oke ? v : z;
                }
            }
        }
    }
    __device__ __forceinline__ void issue_flt(const KernelArgs& a, const UnitBase& u, f32x4 (&freg)[MAXF]) const {
        if (!a.flt_resident) {
            if (u.flt_inside) {
#pragma unroll
                for (int i = 0; i < MAXF; ++i) freg[i] = buf_load_f32x4(u.flt, f_g[i], 0);
            } else {
#pragma unroll
                for (int i = 0; i < MAXF; ++i) {
                    const int idx = stid + i * STHREADS;
                    int kl, r, s, c;
                    flt_coords(a, idx, kl, r, s, c);
                    const bool ok = idx < a.flt_items && kl < u.lk && r < u.lr && s < u.ls && c < u.lc;
                    const f32x4 v = buf_load_f32x4(u.flt, ok ? f_g[i] : 0u, 0);
                    const f32x4 z = {0.f, 0.f, 0.f, 0.f};
                    freg[i] = ok ? v : z;
                }
            }
        }
    }
    __device__ __forceinline__ void store_img(const KernelArgs& a, f32x4* smem, int buf,
                                              const f32x4 (&ireg)[MAXI][4]) const {
        f32x4* s_img = smem + buf * a.img_buf;
#pragma unroll
        for (int i = 0; i < MAXI; ++i)
            if (stid + i * STHREADS < a.img_items) {
                f32x4* dst = s_img + i_lds[i];
#pragma unroll
                for (int bb = 0; bb < 4; ++bb) {
                    const f32x4 o = {ireg[i][0][bb], ireg[i][1][bb], ireg[i][2][bb], ireg[i][3][bb]};
                    dst[bb ^ i_key[i]] = o;
                }
            }
    }
    __device__ __forceinline__ void store_flt(const KernelArgs& a, f32x4* smem, int buf,
                                              const f32x4 (&freg)[MAXF]) const {
        if (!a.flt_resident) {
            f32x4* s_flt = smem + a.flt_off + buf * a.flt_buf;
#pragma unroll
            for (int i = 0; i < MAXF; ++i)
                if (stid + i * STHREADS < a.flt_items) s_flt[f_lds[i]] = freg[i];
        }
    }
};

// One unit out of LDS.  Groups (r, t) form one flat sequence; the fragments of the next group are read while the 4*MBLK*NBLK
// MFMAs of the current one issue (no branches in the loop body; past the end the last group is read again).
template <int MBLK, int NBLK, int TB>
__device__ __forceinline__ void f32v4_compute_unit(const KernelArgs& a, const f32x4* s_img, const f32x4* s_flt,
                                                   const f32x4* s_zero, const int (&posoff)[NBLK],
                                                   f32x16 (&acc)[MBLK][NBLK], int row0, int j, int kk, int r0) {
    const int Q = a.bS * a.CT;                 // multiple of 4
    const int G8 = a.QE >> 3;                  // groups of 8 indices per filter column
    const int rmax = min(a.bR, a.R - r0);
    const int total = rmax * G8;
    const int f4 = a.fpitch >> 2, q4 = a.QE >> 2;
    const bool half_tail = (Q & 7) != 0;       // the last group of a column has only its first four indices
    const f32x4* ap0 = s_flt + (row0 + j) * f4 + kk;
    int r_n = 0, t_n = 0, n_loaded = 0;
    auto load_group = [&](f32x4(&av)[MBLK], f32x4(&bv)[NBLK]) {
        const f32x4* ap = ap0 + r_n * q4 + 2 * t_n;
        const bool zero_half = half_tail && t_n == G8 - 1 && kk;
#pragma unroll
        for (int m = 0; m < MBLK; ++m) av[m] = ap[m * 32 * f4];
#pragma unroll
        for (int n = 0; n < NBLK; ++n)
            bv[n] = zero_half ? s_zero[j] : s_img[posoff[n] + r_n * a.xpitch + 2 * t_n * TB];
    };
    auto advance = [&]() {
        const int adv = n_loaded < total - 1 ? 1 : 0;
        n_loaded += adv;
        t_n += adv;
        const int wrap = t_n == G8 ? 1 : 0;
        t_n = wrap ? 0 : t_n;
        r_n += wrap;
    };
    auto mfma_group = [&](const f32x4(&av)[MBLK], const f32x4(&bv)[NBLK]) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int m = 0; m < MBLK; ++m)
#pragma unroll
                for (int n = 0; n < NBLK; ++n)
                    acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[m][e], bv[n][e], acc[m][n], 0, 0, 0);
    };
    f32x4 a0[MBLK], b0[NBLK], a1[MBLK], b1[NBLK];
    if (total > 0) load_group(a0, b0);
    int t = 0;
    for (; t + 2 <= total; t += 2) {
        advance();
        load_group(a1, b1);
        mfma_group(a0, b0);
        interleave_hint<4 * MBLK * NBLK, MBLK + NBLK>();
        advance();
        load_group(a0, b0);
        mfma_group(a1, b1);
        interleave_hint<4 * MBLK * NBLK, MBLK + NBLK>();
    }
    if (t < total) mfma_group(a0, b0);
}

template <int NBLK, int TB, int TW, int TH>
__device__ __forceinline__ void f32v4_posoff(const KernelArgs& a, int (&posoff)[NBLK], int nblock0, int j, int kk) {
    constexpr int NT = TB * TW * TH;
#pragma unroll
    for (int n = 0; n < NBLK; ++n) {
        int nn = (nblock0 + n) * 32 + j;
        if (nn >= NT) nn = 0;
        const int b_l = nn % TB, w_l = (nn / TB) % TW, h_l = nn / (TB * TW);
        posoff[n] = a.sw * w_l * a.xpitch + a.sh * h_l * a.ypitch + kk * TB + v4_swz(b_l);
    }
}

// Producer half of the 16-byte-fragment fp32 kernels: stages every unit of this workgroup's tile sequence, one barrier
// per unit (the consumers execute the matching barriers).
template <int CTHREADS, int KT, int TB, int TW, int TH, int MAXI, int MAXF>
__device__ __forceinline__ void f32v4_producer(const KernelArgs& a, f32x4* smem_v, int stid) {
    const int zero_off = 2 * a.img_buf;
    F32V4Stager<CTHREADS, TB, MAXI, MAXF> st;
    st.init(a, stid);
    // one-time zeros: the zero units, the pad columns of every Filter row in every buffer
    {
        const f32x4 z = {0.f, 0.f, 0.f, 0.f};
        if (stid < 32) smem_v[zero_off + stid] = z;
        const int q4 = a.QE >> 2, used4 = (a.bS * a.CT) >> 2, f4 = a.fpitch >> 2;
        const int nbuf = a.flt_resident ? 1 : 2;
        if (q4 > used4) {
            for (int idx = stid; idx < nbuf * KT * a.bR; idx += CTHREADS) {
                const int bsel = idx / (KT * a.bR), rem = idx - bsel * KT * a.bR;
                const int kl = rem / a.bR, r = rem - kl * a.bR;
                smem_v[a.flt_off + bsel * a.flt_buf + kl * f4 + r * q4 + used4] = z;
            }
        }
    }
    // Image words are fetched two units ahead (two register sets), Filter words one unit ahead
    f32x4 ireg0[MAXI][4], ireg1[MAXI][4], freg[MAXF];
    UnitPos su = first_unit(a, KT, TB, TW, TH);
    UnitPos lu = su, fu = su;
    if (lu.t < a.n_tiles) {
        const UnitBase u = unit_base<4>(a, lu, KT, TB);
        st.issue_img(a, u, ireg0);
        st.issue_flt(a, u, freg);
        advance_unit(a, lu, KT, TB, TW, TH);
        advance_unit(a, fu, KT, TB, TW, TH);
    }
    if (lu.t < a.n_tiles) {
        st.issue_img(a, unit_base<4>(a, lu, KT, TB), ireg1);
        advance_unit(a, lu, KT, TB, TW, TH);
    }
    if (a.flt_resident) {
        if (a.vec_flt)
            stage_filter_f32<CTHREADS, KT, 4>(a, (float*)(smem_v + a.flt_off), stid, 0, 0, 0, 0);
        else
            stage_filter_f32<CTHREADS, KT, 1>(a, (float*)(smem_v + a.flt_off), stid, 0, 0, 0, 0);
    }
    while (su.t < a.n_tiles) {
        st.store_img(a, smem_v, 0, ireg0);
        st.store_flt(a, smem_v, 0, freg);
        if (lu.t < a.n_tiles) {
            st.issue_img(a, unit_base<4>(a, lu, KT, TB), ireg0);
            advance_unit(a, lu, KT, TB, TW, TH);
        }
        if (fu.t < a.n_tiles) {
            st.issue_flt(a, unit_base<4>(a, fu, KT, TB), freg);
            advance_unit(a, fu, KT, TB, TW, TH);
        }
        __syncthreads();
        advance_unit(a, su, KT, TB, TW, TH);
        if (su.t >= a.n_tiles) break;
        st.store_img(a, smem_v, 1, ireg1);
        st.store_flt(a, smem_v, 1, freg);
        if (lu.t < a.n_tiles) {
            st.issue_img(a, unit_base<4>(a, lu, KT, TB), ireg1);
            advance_unit(a, lu, KT, TB, TW, TH);
        }
        if (fu.t < a.n_tiles) {
            st.issue_flt(a, unit_base<4>(a, fu, KT, TB), freg);
            advance_unit(a, fu, KT, TB, TW, TH);
        }
        __syncthreads();
        advance_unit(a, su, KT, TB, TW, TH);
    }
}

template <int WM, int WN, int MBLK, int NBLK, int TB, int TW, int TH, int MAXI, int MAXF>
__global__ void __launch_bounds__(WM* WN * 128) conv_f32v4_ws_kernel(const KernelArgs a) {
    constexpr int CTHREADS = WM * WN * 64;
    constexpr int KT = WM * MBLK * 32;
    extern __shared__ __align__(16) f32x4 smem_v[];
    const int tid = threadIdx.x;
    const int wave_id = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: the role branch is wave-uniform
    const int zero_off = 2 * a.img_buf;

    if (wave_id >= WM * WN) {
        f32v4_producer<CTHREADS, KT, TB, TW, TH, MAXI, MAXF>(a, smem_v, tid - CTHREADS);
    } else {
        const int lane = tid & 63, wave = wave_id;
        const int wm = wave % WM, wn = wave / WM;
        const int j = lane & 31, kk = lane >> 5;
        int posoff[NBLK];
        f32v4_posoff<NBLK, TB, TW, TH>(a, posoff, wn * NBLK, j, kk);
        f32x16 acc[MBLK][NBLK];
        zero_acc(acc);
        UnitPos cur = first_unit(a, KT, TB, TW, TH);
        UnitPos nxt = cur;
        if (cur.t < a.n_tiles) advance_unit(a, nxt, KT, TB, TW, TH);
        int buf = 0;
        while (cur.t < a.n_tiles) {
            __syncthreads();
            f32v4_compute_unit<MBLK, NBLK, TB>(a, smem_v + buf * a.img_buf,
                                               smem_v + a.flt_off + (a.flt_resident ? 0 : buf) * a.flt_buf,
                                               smem_v + zero_off, posoff, acc, wm * MBLK * 32, j, kk, cur.r0);
            const bool have_next = nxt.t < a.n_tiles;
            if (!have_next || nxt.t != cur.t)
                write_tile<MBLK, NBLK, TB, TW, TH>(a, cur.tc, acc, wn * NBLK, wm * MBLK * 32, j, kk);
            cur = nxt;
            if (have_next) advance_unit(a, nxt, KT, TB, TW, TH);
            buf ^= 1;
        }
    }
}

// ---- fixed-geometry kernels ("fx") ---------------------------------------------------------------------------------
// Measured on MI355X:
//  * LDS reads interleaved one to one with independent MFMAs in the same wave cost about one cycle each (a
//    register-only loop runs 32.2 cycles per bf16 32x32x16 MFMA, 33.0-33.4 with 12-21 reads per 21 MFMAs), provided
//    the wave never has to wait for one: everything a unit needs is a per-lane base register plus an immediate.
//  * A second wave on the SIMD gets few issue slots next to an MFMA stream (about one instruction per 11 cycles next
//    to bf16 MFMAs, next to fp32 MFMAs hardly any until the multiplying wave waits at the barrier), vector-ALU
//    instructions least of all.  Staging waves must therefore issue very little and no vector arithmetic in their
//    steady state: addresses are precomputed, the unit walk is scalar.
//  * Under an all-CU bf16 MFMA load the clock is power-managed (about 1.5-1.8 GHz on operands with the workloads'
//    value mix, 2.2-2.4 GHz on zeros): cycles saved beyond that point come back as a lower clock.
// With the contraction tile (c-slice, b_r = 3, b_s), unit strides and a shape that the tiles divide exactly, all
// addressing is known at compile time and a unit is straight-line code (reads and MFMAs only).
// The layout constants are the kernels' own; the launcher refuses a launch whose geometry differs.

// Out words of one 32x32 accumulator block of a tile that lies wholly inside Out: every address is a wave-uniform base
// (scalar arithmetic) plus the lane's constant 32-bit offset, which holds the lane's row group q*4*kstride and its
// column.  Resets the accumulators.
template <bool STREAM>
__device__ __forceinline__ void store_block_exact(float* base, int64_t kstride, uint32_t lane_off, f32x16& acc) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        float* const row = base + (int64_t)((v >> 2) * 8 + (v & 3)) * kstride;
        if constexpr (STREAM) __builtin_nontemporal_store(acc[v], row + lane_off);
        else row[lane_off] = acc[v];
        acc[v] = 0.f;
    }
}

// The same for a block at the edge of Out: only the rows below `rows` (this lane's count of valid output channels from
// its first row on) are stored.  Ordinary stores: at an edge the pieces of a cache line come from several instructions
// and waves, and a streaming store of a partial line was measured to cost up to twice the time.
__device__ __forceinline__ void store_block_rows(float* base, int64_t kstride, uint32_t lane_off, f32x16& acc, int rows) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int row = (v >> 2) * 8 + (v & 3);
        if (row < rows) base[(int64_t)row * kstride + lane_off] = acc[v];
        acc[v] = 0.f;
    }
}

__device__ __forceinline__ void lds_done_then_barrier() {
    // every LDS access issued so far has completed; then meet the other waves
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Wave-uniform walk over the units this workgroup stages, for the fixed-geometry kernels (C a multiple of the
// c-slice): tiles blockIdx.x, blockIdx.x + gridDim.x, ... of the tile list, and within a tile
// the contraction slices with c fastest, then s, then r in steps of b_r (one step where b_r = R; the kernels compiled
// for 1 x 1 filters take any filter one tap at a time this way).  Per unit it costs a handful of scalar instructions:
// the staging waves share the SIMD's issue slots with the MFMA stream and get few of them.
template <int ESZ, int KT, int TB, int TW, int TH, int CT, int BS>
struct FxWalk {
    int t, r0, s0, c0;
    int64_t img_org, flt_org;      // byte offsets of the current tile's Image / Filter origin (r0 = s0 = c0 = 0)
    int64_t img_bytes, flt_bytes;  // array sizes
    __device__ __forceinline__ void set_tile(const KernelArgs& a) {
        const TileCoord tc = decode_tile_index(a, t, KT, TB, TW, TH);
        img_org = ((((int64_t)a.sw * tc.w0 * a.IH + (int64_t)a.sh * tc.h0) * a.C) * a.B + tc.b0) * ESZ;
        flt_org = (int64_t)tc.k0 * a.R * a.S * a.C * ESZ;
    }
    __device__ __forceinline__ void init(const KernelArgs& a) {
        t = blockIdx.x;
        r0 = s0 = c0 = 0;
        img_bytes = (int64_t)a.IW * a.IH * a.C * a.B * ESZ;
        flt_bytes = (int64_t)a.K * a.R * a.S * a.C * ESZ;
        if (t < a.n_tiles) set_tile(a);
    }
    __device__ __forceinline__ bool valid(const KernelArgs& a) const { return t < a.n_tiles; }
    static __device__ __forceinline__ __amdgpu_buffer_rsrc_t rsrc(const void* base, int64_t off, int64_t total) {
        // in 32-bit pieces: a 64-bit compare is a vector instruction, and next to an MFMA stream the staging waves
        // hardly ever get the vector issue port
        const uint64_t left = (uint64_t)(total - off);
        const uint32_t lo = (uint32_t)left, hi = (uint32_t)(left >> 32);
        const int32_t n = (hi | (lo >> 31)) ? 0x7fffffff : (int32_t)lo;
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>((const char*)base + off), 0, n, 0x00020000);
    }
    // a descriptor of length zero: every load through it is out of range, touches no memory and returns zeros
    static __device__ __forceinline__ __amdgpu_buffer_rsrc_t empty(const void* base) {
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>((const char*)base), 0, 0, 0x00020000);
    }
    __device__ __forceinline__ __amdgpu_buffer_rsrc_t img(const KernelArgs& a) const {
        return rsrc(a.image, img_org + (int64_t)((uint32_t)((r0 * a.IH + s0) * a.C + c0) * (uint32_t)a.B) * ESZ, img_bytes);
    }
    __device__ __forceinline__ __amdgpu_buffer_rsrc_t flt(const KernelArgs& a) const {
        return rsrc(a.filter, flt_org + (int64_t)((r0 * a.S + s0) * a.C + c0) * ESZ, flt_bytes);
    }
    __device__ __forceinline__ void next(const KernelArgs& a) {
        c0 += CT;
        if (c0 >= a.C) {
            c0 = 0;
            s0 += BS;
            if (s0 >= a.S) {
                s0 = 0;
                r0 += a.bR;
                if (r0 >= a.R) {
                    r0 = 0;
                    t += gridDim.x;
                    if (t < a.n_tiles) set_tile(a);
                }
            }
        }
    }
};

// ---- fixed geometry, bf16, Image loaded straight into LDS ---------------------------------------------------------------
// A kernel that staged the Image through registers (8 loads, a 8x8 transpose of 16-bit words and 8 LDS stores per
// item, ~130 instructions per unit and staging wave) was measured to wait for its staging waves: next to a bf16 MFMA
// stream a staging wave gets about one instruction per 11 cycles.
// Here the Image words never pass through registers: a buffer load with the LDS as its destination puts 64 lanes x
// 16 bytes, in lane order, at a wave-uniform LDS address, so one instruction moves 8 channel rows of the tile's 64
// images (1 KiB) and a staging wave issues 8 or 9 of them per unit.  The Image keeps its global order in LDS,
// [x][y][c][b] with b fastest (128-byte rows), and the transpose is left to the LDS read: the transposing 64-bit read
// hands lane i of a 16-lane group the i-th 16-bit word of each of the four 32-byte runs that lanes 4e..4e+3 (e = 0..3)
// point at, so with the four runs in four consecutive channel rows a lane ends up with four channels of one image,
// and two such reads make one MFMA operand.  Which 16-byte piece of a row a lane loads is free, so rows with bit 1 of
// c set are stored with their upper and lower halves exchanged: the 16 pieces that one half-wave reads at once
// (4 rows x 64 bytes) then lie in 16 different groups of four banks.
// Data reaches LDS when it arrives, so there are three buffers: a unit's loads are issued two units ahead, and a
// staging wave waits on its own load counter before it announces the unit at the barrier.  The Filter tile (a
// quarter of the bytes) still goes through registers; its LDS stores are written as assembly so that the compiler's
// wait-count bookkeeping, which makes every LDS access it knows of wait for all outstanding loads into LDS, does not
// see them (their operands are still tracked: the store waits for its own Filter load).
// BRP: the filter's extent along w the kernel is compiled for (3, or 1 for 1 x 1 filters, where a unit is a plain
// matrix product of the Filter tile with the tile's positions).
// TBP: images per tile, 64 or 32.  With 64 a wave column (wn) takes one half of the images and all TW x TH positions; with
// 32 a row of the tile is 64 bytes, a column block is all 32 images of one position, the tile is two rows high and wave
// column wn takes row wn.
// SWP: the stride, in both directions, the kernel is compiled for (1; 2 for 3 x 3 filters on tiles of 2 x 2 positions: a
// tile then stages the 5 columns its two output columns read and, of the rows, the two that the unit's filter row reads).
// CTP: channels per unit, 32 (two 16-channel steps) or, for 1 x 1 filters, 64 (four steps): a 1 x 1 unit has a third of a
// 3 x 3 unit's MFMAs, too few to cover the barrier it ends with and the two units that its fetches run ahead.
template <int TW, int TH, int BRP = 3, int TBP = 64, int SWP = 1, int CTP = 32>
struct Bf16DirectFixed {
    static constexpr int TB = TBP, KT = 64, WM = 2, WN = 2, CT = CTP, BS = 1, BR = BRP, SW = SWP;
    static_assert(CTP == 32 || (CTP == 64 && BRP == 1), "direct bf16 geometry: 64-channel units with 1 x 1 filters");
    static constexpr int THW = TBP == 64 ? TH : 1;                  // tile rows one wave works on
    static constexpr int NBLK = TW * THW;                           // column blocks per wave
    static constexpr int C8 = CT / 8, STEPS = BS * (CT / 16);
    static constexpr int XS = SWP * (TW - 1) + BR, YS = TH - 1 + BS;  // staged columns; staged rows (one per tile row: BS = 1)
    static constexpr int YS_HOST = SWP * (TH - 1) + BS;             // the rows between the first and the last of them
    static_assert(SWP == 1 || (BS == 1 && BRP == 3 && TBP == 64), "direct bf16 geometry: strides with 3 x 3 filters, 64 images");
    static constexpr int ROW = TB * 2;                              // bytes of one (x, y, c) row
    static constexpr int IMG_BYTES = XS * YS * CT * ROW;
    static constexpr int F8 = (BR * BS * C8) | 1;                   // Filter row in 16-byte units, odd: conflict-free
    static constexpr int FLT_BYTES = KT * F8 * 16;
    static constexpr int BUF_BYTES = IMG_BYTES + FLT_BYTES, NBUF = 3, LDS_BYTES = NBUF * BUF_BYTES;
    static constexpr int PT = 256, PW = PT / 64;                    // staging threads, staging waves
    static constexpr int CPW = IMG_BYTES / 1024 / PW;               // 1 KiB Image chunks per unit and staging wave
    static constexpr int FLT_ITEMS = KT * BR * BS * C8, MAXF = FLT_ITEMS / PT, MAXI = 1;
    static constexpr int LOADS = CPW + MAXF;                        // loads one staging wave issues per unit
    static_assert(TBP == 64 || (TBP == 32 && TH == 2), "direct bf16 geometry: 64 images, or 32 images and two rows");
    static_assert(IMG_BYTES % (1024 * PW) == 0, "direct bf16 geometry: whole chunks per staging wave");
    static_assert(C8 % PW == 0, "direct bf16 geometry: chunk 4 i + p of a unit is staging wave p's i-th");
    static_assert(FLT_ITEMS % PT == 0, "direct bf16 geometry: whole Filter items per thread");
    static_assert(BUF_BYTES < 65536 && LDS_BYTES <= 160 * 1024, "direct bf16 geometry: LDS offsets and size");
    static_assert(STEPS % 2 == 0 && 2 * LOADS < 64, "direct bf16 geometry: an even number of steps per unit, load counter range");
    // tail8: the kernel instance whose last c-slice is not full (C a multiple of 8, not of 32) instead of the one for C = 0 mod 32
    static bool matches_host(const KernelArgs& a, bool tail8 = false) {
        if (tail8 ? (a.C % CT == 0 || a.C % 8 != 0) : a.C % CT != 0) return false;
        // (W, H, K and B need not be multiples of the tile, B only of the 8 images of a 16-byte load: what a tile stages
        // beyond the arrays or beyond a row's images is zeros or other rows of the Image, which only reach outputs that
        // are not stored)
        // (1 x 1 filters: any strides, a tile stages the TW x TH positions its outputs read and nothing between them)
        return ((BR == 1 && BS == 1) || (a.sw == SWP && a.sh == SWP)) && a.CT == CT && a.bS == BS && a.bR == BR && a.XS == XS &&
               a.YS == YS_HOST && a.R % BR == 0 && (BR == 1 || a.R == BR) && a.S % BS == 0 && a.B % 8 == 0 && a.vec_img && a.vec_flt;
    }
};

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
#define CACNN_LDS(T) __attribute__((address_space(3))) T

// 16-byte LDS stores regs[0..N) to addr + BASE + i * STEP, offsets in the instruction.  Assembly: the compiler must not
// count them among the LDS accesses that wait for outstanding loads into LDS (the operands are still tracked).
template <int OFF, class V>
__device__ __forceinline__ void lds_store16_at(uint32_t addr, const V& v) {
    static_assert(OFF >= 0 && OFF < 65536, "LDS store offset must fit the instruction's 16-bit field");
    asm volatile("ds_write_b128 %0, %1 offset:%2" ::"v"(addr), "v"(v), "n"(OFF) : "memory");
}
template <int BASE, int STEP, class V, size_t... I>
__device__ __forceinline__ void lds_store16_seq(uint32_t addr, const V* regs, std::index_sequence<I...>) {
    (lds_store16_at<BASE + (int)I * STEP>(addr, regs[I]), ...);
}

// s_waitcnt immediate that waits only for the vector-memory counter to drop to n (6 bits: [3:0] and [15:14])
constexpr int vmcnt_only(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

// `after` is the accumulator the last MFMA in front of the barrier writes: an MFMA touches no memory, so nothing else
// keeps the compiler from moving the barrier up over the MFMAs that are meant to cover the latency of the reads it
// waits for.
template <class ACC>
__device__ __forceinline__ void lds_done_then_barrier_known(ACC& after) {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" : "+v"(after)::"memory");
    __builtin_amdgcn_s_waitcnt(vmcnt_only(63) & ~(15 << 8));
}
__device__ __forceinline__ void lds_done_then_barrier_known() {
    lds_done_then_barrier();
    // true already: restated in a form the compiler's wait-count bookkeeping reads, so that it does not make the
    // first MFMAs behind the barrier wait for the LDS reads issued after it
    __builtin_amdgcn_s_waitcnt(vmcnt_only(63) & ~(15 << 8));
}

// The staging schedule of the direct kernels: unit u's loads are issued two units ahead (register set and Filter
// buffer u % 2), and a unit is announced at the barrier once its loads are in, which the load counter says when at most
// the next unit's LOADS loads are outstanding (loads complete in order).  The first unit is announced before anything
// else is fetched: at the start of a launch every compute unit fetches at once and the L2 caches' bandwidth sets the
// pace, so with two units requested up front the multiplying waves would start one unit's transfer time later.
// Every path is straight-line code or a loop whose state at the back edge equals its state on entry, so the
// compiler's own count of outstanding loads (it waits for a Filter register before the store that reads it) stays
// exact; a load issued under a condition would make it wait for everything.
template <int LOADS, class Issue, class Announce>
__device__ __forceinline__ void direct_staging_schedule(int total, Issue issue, Announce announce) {
    using NextUnit = std::integral_constant<int, LOADS>;
    using Nothing = std::integral_constant<int, 0>;
    if (total <= 0) return;
    issue(0);
    announce(0, Nothing{});
    if (total == 2) {
        issue(1);
        announce(1, Nothing{});
    } else if (total >= 3) {
        issue(1);
        issue(0);                   // unit 2: set 0 went to LDS with the announcement of unit 0
        int issued = 3;
        for (; issued + 2 <= total; issued += 2) {
            announce(1, NextUnit{});
            issue(1);               // the multiplying waves have left the buffer two units back: refill it
            announce(0, NextUnit{});
            issue(0);
        }
        if (total - issued == 1) {
            announce(1, NextUnit{});
            issue(1);
            announce(0, NextUnit{});
            announce(1, Nothing{});
        } else {
            announce(1, NextUnit{});
            announce(0, Nothing{});
        }
    }
}

// 64 lanes x 16 bytes from global memory (lane offset voff, wave-uniform offset soff) to dst, dst + 16, ... in lane order.
// dst is wave-uniform.  Not inside the kernel template: the host pass of the compiler rejects the 16-byte form there.
__device__ __forceinline__ void load_16_bytes_per_lane_to_lds(__amdgpu_buffer_rsrc_t r, CACNN_LDS(char)* dst, uint32_t voff,
                                                              uint32_t soff) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (CACNN_LDS(void)*)dst, 16, voff, soff, 0, 0);
}

// T8: C is a multiple of 8 but not of the 32-channel slice.  The staging waves then fill what lies beyond channel C in the
// last c-slice of every tap with zeros, for both operands, so the multiplying waves need not know: an 8-channel chunk
// of the Image beyond C is loaded through a descriptor of length zero (the range check returns zeros, which go to LDS
// like data), and a thread whose 8 Filter channels lie beyond C loads them from an offset no descriptor covers.  (Tiles
// of 32 images: a chunk holds 16 channels, one per four lanes, so there the lanes beyond C take such an offset too.)
template <int TW, int TH, int BRP = 3, int TBP = 64, int SWP = 1, bool T8 = false, int CTP = 32>
__global__ void __launch_bounds__(512) conv_bf16_direct_kernel(const KernelArgs a) {
    using GEO = Bf16DirectFixed<TW, TH, BRP, TBP, SWP, CTP>;
    static_assert(!T8 || CTP == 32 || TBP == 64, "direct bf16 kernel: a partly filled last slice of 64 channels with 64 images only");
    constexpr int TB = GEO::TB, KT = GEO::KT, CT = GEO::CT, BS = GEO::BS, BR = GEO::BR, WM = GEO::WM, NBLK = GEO::NBLK;
    constexpr int XS = GEO::XS, YS = GEO::YS, C8 = GEO::C8, F8 = GEO::F8, ROW = GEO::ROW, BUF = GEO::BUF_BYTES;
    constexpr int CTHREADS = GEO::WM * GEO::WN * 64;
    extern __shared__ __align__(16) uint4 smem_u[];
    CACNN_LDS(char)* const lds = (CACNN_LDS(char)*)smem_u;
    const int tid = threadIdx.x;
    const int wave_id = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: the role branch is wave-uniform
    const int lane = tid & 63;
    // units this workgroup works through: its tiles blockIdx.x, blockIdx.x + gridDim.x, ... times the slices of a tile
    const int n_c = (a.C + CT - 1) / CT;            // c-slices (the last one partly filled in the T8 kernels)
    const int upt = n_c * (a.S / BS) * (a.R / BR);      // (R > b_r only in the kernels for 1 x 1 filters: a unit per tap)
    int total = 0;
    for (int t = blockIdx.x; t < a.n_tiles; t += gridDim.x) total += upt;

    if (wave_id >= GEO::WM * GEO::WN) {
        const int pw = wave_id - GEO::WM * GEO::WN, stid = tid - CTHREADS;
        constexpr int MAXF = GEO::MAXF, CPW = GEO::CPW, PT = GEO::PT;
        // Image: lane L of a chunk load fetches channel row L / 8 of the chunk, 16-byte piece (L % 8) ^ 4 * (bit 1 of the row)
        const uint32_t row_bytes = (uint32_t)a.B * 2u;
        // (32 images: a chunk is 16 rows of 64 bytes, lane L fetches piece L % 4 of row L / 4, and chunk 4 i + p of a unit
        // is half (4 i + p) % 2 of position (4 i + p) / 2)
        const uint32_t ivoff = TB == 64 ? (uint32_t)(lane >> 3) * row_bytes + (uint32_t)(((lane & 7) ^ (((lane >> 4) & 1) << 2)) * 16)
                                        : (uint32_t)(lane >> 2) * row_bytes + (uint32_t)((lane & 3) * 16);
        uint32_t isoff[CPW];
#pragma unroll
        for (int i = 0; i < CPW; ++i) {
            // chunk 4 i + pw of the unit: in LDS order, position by position, a position's channels in chunks of 8 (16) rows
            const int c = GEO::PW * i + pw;
            if constexpr (TB == 64) {
                // (columns: the staged range is contiguous, except for 1 x 1 filters, where it is the outputs' own columns)
                const int xy = c / C8, grp = c % C8;
                isoff[i] = (uint32_t)(((xy / YS) * (BR == 1 ? a.sw : 1) * a.IH + (xy % YS) * a.sh) * a.C + grp * 8) * row_bytes;
            } else {
                const int xy = c / (CT / 16), grp = c % (CT / 16);
                isoff[i] = (uint32_t)(((xy / YS) * (BR == 1 ? a.sw : 1) * a.IH + (xy % YS) * a.sh) * a.C + 16 * grp) * row_bytes;
            }
        }
        // Filter: thread (kl = stid / C8, c8 = stid % C8) fetches the 16 bytes of channels 8*c8.. of output channel kl
        // for every tap (r, s) of the unit: one global offset and one LDS address per thread, the tap in the
        // instruction (scalar offset of the load, immediate of the store)
        // (64-channel units, 1 x 1 filters only: a second item, 32 channels further on)
        constexpr int TAPS = BR * BS, GQ = C8 / GEO::PW, FSTEP = GQ > 1 ? GEO::PW * 16 : C8 * 16;   // LDS bytes between items
        static_assert(MAXF == TAPS * GQ && PT == KT * GEO::PW && (GQ == 1 || TAPS == 1),
                      "direct bf16 geometry: one Filter item per thread, tap and 32 channels");
        const int f_c8 = stid % GEO::PW, f_kl = stid / GEO::PW;
        const uint32_t fg0 = ((uint32_t)f_kl * a.R * a.S * a.C + f_c8 * 8) * 2u;
        // (T8: in a c-slice that reaches beyond C, a thread whose channels lie beyond C loads from beyond every descriptor's
        // range, 2^31 or more with the tap's offset and less than 2^32: zeros)
        const uint32_t fg0_tail = T8 && f_c8 * 8 >= a.C % CT ? 0x80000000u : fg0;
        // (64-channel units: the thread's second item lies 32 channels further on)
        const uint32_t fg0_tail2 = T8 && f_c8 * 8 + 32 >= a.C % CT ? 0x80000000u : fg0;
        // (32 images: chunk 4 i + pw is half pw % 2 of a position, lane L has its channel 16 (pw % 2) + L / 4)
        const uint32_t ivoff_tail = T8 && TB == 32 && 16 * (pw & 1) + (lane >> 2) >= a.C % CT ? 0x80000000u : ivoff;
        const uint32_t fl0 = (uint32_t)(uintptr_t)(lds + GEO::IMG_BYTES + (f_kl * F8 + f_c8) * 16);
        const uint32_t fl2 = fl0 + 2 * BUF;
        uint32_t fsoff[MAXF];
#pragma unroll
        for (int i = 0; i < MAXF; ++i)
            fsoff[i] = GQ > 1 ? (uint32_t)i * GEO::PW * 16u : (uint32_t)((i / BS) * a.S + i % BS) * (uint32_t)a.C * 2u;
        FxWalk<2, KT, TB, TW, TH, CT, BS> lu;     // next unit to fetch
        lu.init(a);
        u32x4 freg[2][MAXF];
        int boff_issue = 0, boff_store = 0;       // the buffers the next fetch / the next announced unit use
        auto issue = [&](int set) {
            const __amdgpu_buffer_rsrc_t rf = lu.flt(a);
            __amdgpu_buffer_rsrc_t ri = lu.img(a);
            __amdgpu_buffer_rsrc_t ri2 = ri;          // 64-channel units: for the chunks of channels 8 pw + 32 ..
            uint32_t fgo = fg0, fgo2 = fg0;
            uint32_t ivo = ivoff;
            if constexpr (T8) {
                const int c_left = a.C - lu.c0;
                if constexpr (TB == 64) {
                    // every chunk of this staging wave holds channels 8 pw .. 8 pw + 7 of the slice (32-channel units,
                    // C8 == PW), or those and channels 8 pw + 32 .. in turns (64-channel units)
                    if (8 * pw >= c_left) ri = lu.empty(a.image);
                    if (8 * pw + 32 >= c_left) ri2 = lu.empty(a.image);
                } else {
                    if (c_left < CT) ivo = ivoff_tail;
                }
                if (c_left < CT) fgo = fg0_tail, fgo2 = fg0_tail2;
            }
#pragma unroll
            for (int i = 0; i < CPW; ++i)
                load_16_bytes_per_lane_to_lds(C8 > GEO::PW && (i & 1) ? ri2 : ri, lds + boff_issue + (i * GEO::PW + pw) * 1024, ivo,
                                              isoff[i]);
#pragma unroll
            for (int i = 0; i < MAXF; ++i) {
                const uint4 v = buf_load_u4(rf, GQ > 1 && i == 1 ? fgo2 : fgo, fsoff[i]);
                freg[set][i] = u32x4{v.x, v.y, v.z, v.w};
            }
            lu.next(a);
            boff_issue = boff_issue + BUF == GEO::NBUF * BUF ? 0 : boff_issue + BUF;
        };
        // announce the unit whose Filter words are in register set `set`: its loads are in once at most `later`
        // younger loads are outstanding (loads complete in order)
        auto announce = [&](int set, auto later) {
            __builtin_amdgcn_s_waitcnt(vmcnt_only(decltype(later)::value));
            // the buffer offset goes into the instruction (the third buffer is beyond the 16-bit field: second base
            // register), chosen by a scalar branch: a vector add here would wait for the vector issue port, which
            // the MFMA stream of the SIMD's other wave hardly ever leaves free
            if (boff_store == 0) lds_store16_seq<0, FSTEP>(fl0, freg[set], std::make_index_sequence<MAXF>{});
            else if (boff_store == BUF) lds_store16_seq<BUF, FSTEP>(fl0, freg[set], std::make_index_sequence<MAXF>{});
            else lds_store16_seq<0, FSTEP>(fl2, freg[set], std::make_index_sequence<MAXF>{});
            lds_done_then_barrier();
            boff_store = boff_store + BUF == GEO::NBUF * BUF ? 0 : boff_store + BUF;
        };
        direct_staging_schedule<GEO::LOADS>(total, issue, announce);
    } else {
        const int wm = wave_id % WM, wn = wave_id / WM;
        const int j = lane & 31, g = lane >> 5, i16 = lane & 15, jhalf = (lane >> 4) & 1;
        f32x16 acc[1][NBLK];
        zero_acc(acc);
        // per-lane LDS offsets inside a buffer: Filter row of output channel wm*32 + j, contraction half g;
        // Image: row 8g + i16/4 of a 16-channel step, the 8 bytes that hold images 4*(i16 % 4).. of this lane group
        const uint32_t al = (uint32_t)(GEO::IMG_BYTES + ((wm * 32 + j) * F8 + g) * 16);
        constexpr int THW = GEO::THW;
        const int q = (TB == 64 ? wn * 4 : 0) + 2 * jhalf + ((i16 & 3) >> 1);
        const uint32_t xl = TB == 64 ? (uint32_t)((8 * g + (i16 >> 2)) * ROW + ((q ^ (((i16 >> 3) & 1) << 2)) * 16) + (i16 & 1) * 8)
                                     : (uint32_t)((wn * CT + 8 * g + (i16 >> 2)) * ROW + q * 16 + (i16 & 1) * 8);
        bf16x8 A[2][BR], X[2][THW][XS];
        auto load_step = [&](uint32_t ab, uint32_t xb, int t, int set) {
            const int sl = t / (CT / 16), cs = t % (CT / 16);
#pragma unroll
            for (int r = 0; r < BR; ++r)
                A[set][r] = *(const CACNN_LDS(bf16x8)*)(lds + ab + ((r * BS + sl) * C8 + 2 * cs) * 16);
#pragma unroll
            for (int h = 0; h < THW; ++h)
#pragma unroll
                for (int x = 0; x < XS; ++x) {
                    CACNN_LDS(char)* const p = lds + xb + ((x * YS + h + sl) * CT + 16 * cs) * ROW;
                    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((CACNN_LDS(s16x4)*)p);
                    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((CACNN_LDS(s16x4)*)(p + 4 * ROW));
                    X[set][h][x] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                }
        };
        auto mfma_step = [&](int set) {
#pragma unroll
            for (int r = 0; r < BR; ++r)
#pragma unroll
                for (int h = 0; h < THW; ++h)
#pragma unroll
                    for (int w = 0; w < TW; ++w)
                        acc[0][h * TW + w] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[set][r], X[set][h][SWP * w + r],
                                                                                     acc[0][h * TW + w], 0, 0, 0);
        };
        const int64_t out_kstride = (int64_t)a.H * a.W * a.B;      // floats between output channels
        const uint32_t out_lane = (uint32_t)(g * 4) * (uint32_t)out_kstride + (uint32_t)((TB == 64 ? 32 * wn : 0) + j);
        int left = total, in_tile = upt, t = blockIdx.x;
        uint32_t boff = 0;
        // one unit; MORE: another one follows (its buffer is the next of the three)
        auto unit = [&](auto more) {
            constexpr bool MORE = decltype(more)::value;
            load_step(al + boff, xl + boff, 1, 1);
            mfma_step(0);
            interleave_front_hint<BR * NBLK, 2 * THW * XS + BR, 2>();
            // (units of more than two steps: the steps in between, each read under the MFMAs of the one before)
#pragma unroll
            for (int st = 1; st + 1 < GEO::STEPS; ++st) {
                load_step(al + boff, xl + boff, st + 1, (st + 1) & 1);
                mfma_step(st & 1);
                interleave_front_hint<BR * NBLK, 2 * THW * XS + BR, 2>();
            }
            if constexpr (MORE) {
                // hand the buffer back once the last fragments have landed, read the next unit's first fragments
                // under this step's MFMAs
                boff = boff + BUF == GEO::NBUF * BUF ? 0u : boff + BUF;
                lds_done_then_barrier_known(acc[0][NBLK - 1]);
                load_step(al + boff, xl + boff, 0, 0);
            }
            mfma_step(1);
            if constexpr (MORE) interleave_front_hint<BR * NBLK, 2 * THW * XS + BR, 2>();
            // keep the reads above where they are: left alone, the compiler sinks them to the top of the next
            // unit, in front of the MFMAs that need them
            asm volatile("" ::: "memory");
            --left;
            if (__builtin_expect(--in_tile == 0, 0)) {
                const TileCoord tc = decode_tile_index(a, t, KT, TB, TW, TH);
                // (B not a multiple of 32: the rows of Out are not whole cache lines, and every tile takes the path with
                // ordinary stores)
                if (tc.k0 + KT <= a.K && tc.w0 + TW <= a.W && tc.h0 + TH <= a.H && tc.b0 + TB <= a.B && a.B % 32 == 0) {
#pragma unroll
                    for (int n = 0; n < NBLK; ++n) {
                        const int hrow = TB == 64 ? n / TW : wn;
                        float* const blk = a.out + ((((int64_t)(tc.k0 + wm * 32) * a.H + tc.h0 + hrow) * a.W + tc.w0 + n % TW) * a.B + tc.b0);
                        store_block_exact<true>(blk, out_kstride, out_lane, acc[0][n]);
                    }
                } else {
                    // a tile that overhangs Out: the blocks of positions inside, this lane's image if it is inside, the
                    // rows of output channels inside.  (Where all the tile's output channels are inside, which is every
                    // tile but the last along k, a block is stored whole or not at all: with fewer images than a tile
                    // holds every tile comes here, and a test per row made such layers half as fast again.)
                    const bool lane_in = tc.b0 + (TB == 64 ? 32 * wn : 0) + j < a.B;
                    const bool k_whole = tc.k0 + KT <= a.K;
                    const int rows = lane_in ? a.K - (tc.k0 + wm * 32 + g * 4) : 0;
#pragma unroll
                    for (int n = 0; n < NBLK; ++n) {
                        const int hrow = TB == 64 ? n / TW : wn;
                        const int w = tc.w0 + n % TW, h = tc.h0 + hrow;
                        float* const blk = a.out + ((((int64_t)(tc.k0 + wm * 32) * a.H + h) * a.W + w) * a.B + tc.b0);
                        const bool blk_in = w < a.W && h < a.H;
                        if (k_whole) {
                            if (blk_in && lane_in) {
                                // (ordinary stores where the rows of Out are not whole cache lines: the L2 has to put the
                                // pieces of a line together before it is written back; streamed, such layers took up to
                                // twice as long)
                                if (a.B % 32 == 0) store_block_exact<true>(blk, out_kstride, out_lane, acc[0][n]);
                                else store_block_exact<false>(blk, out_kstride, out_lane, acc[0][n]);
                            } else {
#pragma unroll
                                for (int v = 0; v < 16; ++v) acc[0][n][v] = 0.f;
                            }
                        } else {
                            store_block_rows(blk, out_kstride, out_lane, acc[0][n], blk_in ? rows : 0);
                        }
                    }
                }
                in_tile = upt;
                t += gridDim.x;
            }
        };
        if (left > 0) {
            lds_done_then_barrier_known();      // unit 0 is staged
            load_step(al, xl, 0, 0);
            while (left > 1) unit(std::true_type{});
            unit(std::false_type{});
        }
    }
}

// ---- fixed geometry, bf16, staged through registers with a deep prefetch ----------------------------------------------
// The kernel above can have two units of fetches in flight, the two LDS buffers that are not being read.  This one was
// built to find out whether that depth is what limits it: it is not.  With fetches up to four units ahead this kernel
// takes the same time to within a few per cent on both benchmark shapes it accepts, and so does the kernel above when
// the rows of a unit are pulled into the L2 four to six units early.  (What the machine does with one unit's MFMAs
// and bytes when nothing synchronises them is measured by the probe kernels; the kernel above runs at 84 to 88 % of it.)
// It stays as a selectable variant because it halves the LDS the Image needs and makes room for an Image unit that
// serves all three filter rows.
// Here the words in flight wait in the staging waves' registers instead, of which those waves have plenty (a staging
// wave needs a dozen for its addresses): Filter words are requested three or four sub-units ahead and Image words
// two to four Image units ahead, and a set of registers is written to LDS (16-byte stores, the same layouts as above:
// the Image keeps its global order, the transposing LDS read does the rest) one sub-unit before it is multiplied.  Two
// LDS buffers of each operand then suffice, which leaves room for the other half of the paper's small-filter reuse
// (Section 4.3) inside LDS: with BSI = 3 an Image unit holds the TH + 2 rows that all three filter rows s of a c-slice
// read, staged once, and only the Filter taps change from one sub-unit (one s) to the next.
//   sub-unit  = (tile, c-slice of 32 channels, filter row s): 2 steps x 3 taps r x NBLK MFMAs per multiplying wave
//   Image unit = BSI consecutive sub-units of one c-slice (rows h0 + s0 .. h0 + s0 + TH - 2 + BSI of the tile)
// Barrier number v (one per sub-unit, executed by all eight waves) says "sub-unit v is in LDS" and, for the multiplying
// waves, "every read of sub-unit v - 1 has landed", so the staging waves may overwrite that sub-unit's buffers.
template <int TW, int TH, int BSI>
struct Bf16StagedFixed {
    static constexpr int TB = 64, KT = 64, WM = 2, WN = 2, CT = 32, BR = 3, NBLK = TW * TH;
    static constexpr int C8 = CT / 8;
    static constexpr int XS = TW + BR - 1, YSI = TH - 1 + BSI;
    static constexpr int ROW = TB * 2;                              // bytes of one (x, y, c) row
    static constexpr int IMG_BYTES = XS * YSI * CT * ROW;
    static constexpr int F8 = (BR * C8) | 1;                        // Filter row in 16-byte units, odd: conflict-free
    static constexpr int FLT_BYTES = KT * F8 * 16;
    static constexpr int FLT_OFF = 2 * IMG_BYTES, LDS_BYTES = 2 * IMG_BYTES + 2 * FLT_BYTES;
    static constexpr int PT = 256, PW = PT / 64;                    // staging threads, staging waves
    static constexpr int CPW = XS * YSI;                            // 1 KiB Image chunks per Image unit and staging wave
    static constexpr int MAXF = BR, MAXI = 1;                       // Filter items per thread and sub-unit
    static constexpr int GF = BSI == 1 ? 4 : 3;                     // Filter register sets: sub-units a Filter load runs ahead
    static constexpr int GI = BSI == 1 ? 4 : 2;                     // Image register sets: Image units an Image load runs ahead
    static constexpr int PERIOD = BSI == 1 ? 4 : 6;                 // sub-units after which every buffer and set index repeats
    static_assert(BSI == 1 || BSI == 3, "staged bf16 geometry: an Image unit serves one filter row or three");
    static_assert(C8 == PW && PT == KT * C8, "staged bf16 geometry: staging wave p moves channels 8p..8p+7; one Filter item per thread and tap");
    static_assert(PERIOD % GF == 0 && PERIOD % 2 == 0 && PERIOD % (BSI * GI) == 0, "staged bf16 geometry: static buffer rotation");
    static_assert((CPW - 1) * C8 * 1024 < 65536 && FLT_BYTES + BR * C8 * 16 < 65536, "staged bf16 geometry: LDS store offsets");
    static_assert(LDS_BYTES <= 160 * 1024, "staged bf16 geometry: LDS size");
    static_assert((GI * CPW + GF * MAXF) * 4 <= 200, "staged bf16 geometry: registers of a staging wave");
    static bool matches_host(const KernelArgs& a) {
        return a.sw == 1 && a.sh == 1 && a.CT == CT && a.bS == BSI && a.bR == BR && a.XS == XS && a.YS == YSI &&
               a.R == BR && a.S % BSI == 0 && a.C % CT == 0 && a.B % TB == 0 && a.W % TW == 0 && a.H % TH == 0 &&
               a.K % KT == 0 && a.vec_img && a.vec_flt;
    }
};

// f(integral_constant<int, 0>), f(integral_constant<int, 1>), ...: a loop whose index is a compile-time constant in every
// iteration (register sets and LDS buffers are chosen by it)
template <class F, size_t... I>
__device__ __forceinline__ void static_for(F&& f, std::index_sequence<I...>) {
    (f(std::integral_constant<int, (int)I>{}), ...);
}

// Where a staging wave is in its walk over the sub-units (or Image units) it fetches: this workgroup's tiles blockIdx.x,
// blockIdx.x + gridDim.x, ..., within a tile the c-slices, within a c-slice the filter rows s.  All scalar.
template <int KT, int TB, int TW, int TH, int CT>
struct StagedWalk {
    int t, c0, s0;
    int64_t img_org, flt_org;      // byte offsets of the current tile's Image / Filter origin (c0 = s0 = 0)
    __device__ __forceinline__ void set_tile(const KernelArgs& a) {
        const TileCoord tc = decode_tile_index(a, t, KT, TB, TW, TH);
        img_org = ((((int64_t)tc.w0 * a.IH + (int64_t)tc.h0) * a.C) * a.B + tc.b0) * 2;
        flt_org = (int64_t)tc.k0 * a.R * a.S * a.C * 2;
    }
    __device__ __forceinline__ void init(const KernelArgs& a) {
        t = blockIdx.x;
        c0 = s0 = 0;
        img_org = flt_org = 0;
        if (t < a.n_tiles) set_tile(a);
    }
    // a descriptor of the array from `off` on; of length zero once the walk has left the last tile, so that loads
    // requested past the end touch no memory and return zeros
    __device__ __forceinline__ __amdgpu_buffer_rsrc_t rsrc(const KernelArgs& a, const void* base, int64_t off, int64_t total) const {
        const bool live = t < a.n_tiles;
        const uint64_t left = (uint64_t)(total - off);
        const uint32_t lo = (uint32_t)left, hi = (uint32_t)(left >> 32);
        const int32_t n = !live ? 0 : ((hi | (lo >> 31)) ? 0x7fffffff : (int32_t)lo);
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>((const char*)base + (live ? off : 0)), 0, n, 0x00020000);
    }
    __device__ __forceinline__ __amdgpu_buffer_rsrc_t img(const KernelArgs& a, int64_t img_bytes) const {
        return rsrc(a, a.image, img_org + (int64_t)((uint32_t)(s0 * a.C + c0) * (uint32_t)a.B) * 2, img_bytes);
    }
    __device__ __forceinline__ __amdgpu_buffer_rsrc_t flt(const KernelArgs& a, int64_t flt_bytes) const {
        return rsrc(a, a.filter, flt_org + (int64_t)(s0 * a.C + c0) * 2, flt_bytes);
    }
    __device__ __forceinline__ void next(const KernelArgs& a, int ds) {
        s0 += ds;
        if (s0 >= a.S) {
            s0 = 0;
            c0 += CT;
            if (c0 >= a.C) {
                c0 = 0;
                if (t < a.n_tiles) t += gridDim.x;
                if (t < a.n_tiles) set_tile(a);
            }
        }
    }
};

template <int TW, int TH, int BSI>
__global__ void __launch_bounds__(512) conv_bf16_staged_kernel(const KernelArgs a) {
    using GEO = Bf16StagedFixed<TW, TH, BSI>;
    constexpr int TB = GEO::TB, KT = GEO::KT, CT = GEO::CT, BR = GEO::BR, WM = GEO::WM, NBLK = GEO::NBLK;
    constexpr int XS = GEO::XS, YSI = GEO::YSI, C8 = GEO::C8, F8 = GEO::F8, ROW = GEO::ROW;
    constexpr int IBUF = GEO::IMG_BYTES, FBUF = GEO::FLT_BYTES;
    constexpr int CTHREADS = GEO::WM * GEO::WN * 64;
    extern __shared__ __align__(16) uint4 smem_u[];
    CACNN_LDS(char)* const lds = (CACNN_LDS(char)*)smem_u;
    const int tid = threadIdx.x;
    const int wave_id = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: the role branch is wave-uniform
    const int lane = tid & 63;
    // sub-units this workgroup works through: its tiles blockIdx.x, blockIdx.x + gridDim.x, ... times the sub-units of a tile
    const int spt = (a.C / CT) * a.S;
    int total = 0;
    for (int t = blockIdx.x; t < a.n_tiles; t += gridDim.x) total += spt;

    if (wave_id >= GEO::WM * GEO::WN) {
        const int pw = wave_id - GEO::WM * GEO::WN, stid = tid - CTHREADS;
        constexpr int MAXF = GEO::MAXF, CPW = GEO::CPW, GF = GEO::GF, GI = GEO::GI, PERIOD = GEO::PERIOD;
        const int64_t img_bytes = (int64_t)a.IW * a.IH * a.C * a.B * 2, flt_bytes = (int64_t)a.K * a.R * a.S * a.C * 2;
        // Image: lane L of chunk i fetches channel row L / 8 of position i, 16-byte piece (L % 8) ^ 4 * (bit 1 of the row),
        // and stores it at byte 16 L of the chunk: rows with bit 1 of c set keep their halves exchanged in LDS
        const uint32_t row_bytes = (uint32_t)a.B * 2u;
        const uint32_t ivoff = (uint32_t)(lane >> 3) * row_bytes + (uint32_t)(((lane & 7) ^ (((lane >> 4) & 1) << 2)) * 16);
        uint32_t isoff[CPW];
#pragma unroll
        for (int i = 0; i < CPW; ++i)
            isoff[i] = (uint32_t)(((i / YSI) * a.IH + (i % YSI)) * a.C + pw * 8) * row_bytes;
        const uint32_t il0 = (uint32_t)(uintptr_t)(lds + pw * 1024 + lane * 16), il1 = il0 + IBUF;
        // Filter: thread (kl = stid / C8, c8 = stid % C8) fetches the 16 bytes of channels 8*c8.. of output channel kl for
        // each of the three taps r of the sub-unit's filter row
        const int f_c8 = stid % C8, f_kl = stid / C8;
        const uint32_t fg0 = ((uint32_t)f_kl * a.R * a.S * a.C + f_c8 * 8) * 2u;
        const uint32_t fl0 = (uint32_t)(uintptr_t)(lds + GEO::FLT_OFF + (f_kl * F8 + f_c8) * 16);
        uint32_t fsoff[MAXF];
#pragma unroll
        for (int i = 0; i < MAXF; ++i) fsoff[i] = (uint32_t)(i * a.S) * (uint32_t)a.C * 2u;
        StagedWalk<KT, TB, TW, TH, CT> wf, wi;    // next sub-unit whose Filter taps / next Image unit to request
        wf.init(a);
        wi.init(a);
        u32x4 freg[GF][MAXF], ireg[GI][CPW];
        auto issue_flt = [&](auto setc) {
            constexpr int set = decltype(setc)::value;
            const __amdgpu_buffer_rsrc_t rf = wf.flt(a, flt_bytes);
#pragma unroll
            for (int i = 0; i < MAXF; ++i) {
                const uint4 v = buf_load_u4(rf, fg0, fsoff[i]);
                freg[set][i] = u32x4{v.x, v.y, v.z, v.w};
            }
            wf.next(a, 1);
        };
        auto issue_img = [&](auto setc) {
            constexpr int set = decltype(setc)::value;
            const __amdgpu_buffer_rsrc_t ri = wi.img(a, img_bytes);
#pragma unroll
            for (int i = 0; i < CPW; ++i) {
                const uint4 v = buf_load_u4(ri, ivoff, isoff[i]);
                ireg[set][i] = u32x4{v.x, v.y, v.z, v.w};
            }
            wi.next(a, BSI);
        };
        // sub-unit v = J (mod PERIOD): write its registers to LDS, announce it, refill the registers it leaves
        auto step = [&](auto jc, int v) {
            constexpr int J = decltype(jc)::value;
            constexpr int fs = J % GF, fb = J % 2, is = (J / BSI) % GI, ib = (J / BSI) % 2;
            constexpr bool img_step = J % BSI == 0;
            if (v + J < total) {
                lds_store16_seq<fb * FBUF, C8 * 16>(fl0, freg[fs], std::make_index_sequence<MAXF>{});
                if constexpr (img_step)
                    lds_store16_seq<0, C8 * 1024>(ib ? il1 : il0, ireg[is], std::make_index_sequence<CPW>{});
                lds_done_then_barrier();
            }
            issue_flt(std::integral_constant<int, fs>{});
            if constexpr (img_step) issue_img(std::integral_constant<int, is>{});
        };
        static_for(issue_flt, std::make_index_sequence<GF>{});
        static_for(issue_img, std::make_index_sequence<GI>{});
        for (int v = 0; v < total; v += PERIOD)
            static_for([&](auto jc) { step(jc, v); }, std::make_index_sequence<PERIOD>{});
    } else {
        const int wm = wave_id % WM, wn = wave_id / WM;
        const int j = lane & 31, g = lane >> 5, i16 = lane & 15, jhalf = (lane >> 4) & 1;
        f32x16 acc[1][NBLK];
        zero_acc(acc);
        // per-lane LDS offsets inside a buffer: Filter row of output channel wm*32 + j, contraction half g;
        // Image: row 8g + i16/4 of a 16-channel step, the 8 bytes that hold images 4*(i16 % 4).. of this lane group
        const uint32_t al = (uint32_t)(GEO::FLT_OFF + ((wm * 32 + j) * F8 + g) * 16);
        const int q = wn * 4 + 2 * jhalf + ((i16 & 3) >> 1);
        const uint32_t xl = (uint32_t)((8 * g + (i16 >> 2)) * ROW + ((q ^ (((i16 >> 3) & 1) << 2)) * 16) + (i16 & 1) * 8);
        bf16x8 A[2][BR], X[2][TH][XS];
        // one 16-channel step cs of a sub-unit: the three taps r of its filter row, the TH x XS Image positions they read
        auto load_step = [&](uint32_t ab, uint32_t xb, int cs, int set) {
#pragma unroll
            for (int r = 0; r < BR; ++r)
                A[set][r] = *(const CACNN_LDS(bf16x8)*)(lds + ab + (r * C8 + 2 * cs) * 16);
#pragma unroll
            for (int h = 0; h < TH; ++h)
#pragma unroll
                for (int x = 0; x < XS; ++x) {
                    CACNN_LDS(char)* const p = lds + xb + ((x * YSI + h) * CT + 16 * cs) * ROW;
                    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((CACNN_LDS(s16x4)*)p);
                    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((CACNN_LDS(s16x4)*)(p + 4 * ROW));
                    X[set][h][x] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                }
        };
        auto mfma_step = [&](int set) {
#pragma unroll
            for (int r = 0; r < BR; ++r)
#pragma unroll
                for (int h = 0; h < TH; ++h)
#pragma unroll
                    for (int w = 0; w < TW; ++w)
                        acc[0][h * TW + w] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[set][r], X[set][h][w + r],
                                                                                     acc[0][h * TW + w], 0, 0, 0);
        };
        const int64_t out_kstride = (int64_t)a.H * a.W * a.B;      // floats between output channels
        const uint32_t out_lane = (uint32_t)(g * 4) * (uint32_t)out_kstride + (uint32_t)(32 * wn + j);
        int left = total, in_tile = spt, t = blockIdx.x;
        uint32_t foff = 0, ioff = 0;      // the buffers of the sub-unit being multiplied
        int sl = 0;                       // its filter row within the Image unit: the Image rows it reads start at sl
        // one sub-unit; MORE: another one follows (the other Filter buffer; the other Image buffer when an Image unit ends)
        auto unit = [&](auto more) {
            constexpr bool MORE = decltype(more)::value;
            load_step(al + foff, xl + ioff + (uint32_t)(sl * CT * ROW), 1, 1);
            mfma_step(0);
            interleave_front_hint<BR * NBLK, 2 * TH * XS + BR, 2>();
            if constexpr (MORE) {
                // hand the buffers back once the last fragments have landed, read the next sub-unit's first fragments
                // under this step's MFMAs
                foff = FBUF - foff;
                if (++sl == BSI) {
                    sl = 0;
                    ioff = IBUF - ioff;
                }
                lds_done_then_barrier_known(acc[0][NBLK - 1]);
                load_step(al + foff, xl + ioff + (uint32_t)(sl * CT * ROW), 0, 0);
            }
            mfma_step(1);
            if constexpr (MORE) interleave_front_hint<BR * NBLK, 2 * TH * XS + BR, 2>();
            // keep the reads above where they are: left alone, the compiler sinks them to the top of the next
            // sub-unit, in front of the MFMAs that need them
            asm volatile("" ::: "memory");
            --left;
            if (__builtin_expect(--in_tile == 0, 0)) {
                const TileCoord tc = decode_tile_index(a, t, KT, TB, TW, TH);
#pragma unroll
                for (int n = 0; n < NBLK; ++n) {
                    float* const blk = a.out + ((((int64_t)(tc.k0 + wm * 32) * a.H + tc.h0 + n / TW) * a.W + tc.w0 + n % TW) * a.B + tc.b0);
                    store_block_exact<true>(blk, out_kstride, out_lane, acc[0][n]);
                }
                in_tile = spt;
                t += gridDim.x;
            }
        };
        if (left > 0) {
            lds_done_then_barrier_known();      // sub-unit 0 is staged
            load_step(al, xl, 0, 0);
            while (left > 1) unit(std::true_type{});
            unit(std::false_type{});
        }
    }
}

// ---- fixed geometry, fp32, Image loaded straight into LDS -------------------------------------------------------------
// The same staging for fp32 tiles of 8 images x 4 x 4 output positions.  Next to an fp32 MFMA stream a staging wave
// gets even fewer issue slots than next to a bf16 one, and a register-staged kernel was measured with its staging
// waves arriving at the barrier as late as the multiplying ones.  An fp32 MFMA takes one word per lane and
// operand, so nothing has to be transposed: the Image keeps its global order in LDS, [x][y][c][b] with the tile's 8
// images fastest (32-byte rows, 512 bytes per position, one x plane = 6 positions + 32 bytes of padding so that the four
// output columns of an MFMA column block fall into different banks), and lane (column j, contraction half g) reads
// its word of channel c0 + 4g + t for the t-th MFMA of a group of four.  The Filter tile keeps [k][r][s][c] order (rows
// padded to 592 bytes: conflict-free 16-byte reads); a lane's 16-byte fragment holds channels c0 + 4g .. c0 + 4g + 3.
// Three Image buffers (loads into LDS two units ahead), two Filter buffers (staged through registers and stored just
// before the unit is announced).
template <int TW, int TH>
struct F32DirectFixed {
    static constexpr int TB = 8, KT = 64, WM = 2, WN = 2, CT = 16, BS = 3, BR = 3, NBLK = TH / WN, TW_ = TW, TH_ = TH;
    static constexpr int XS = TW + BR - 1, YS = TH - 1 + BS, YSL = YS, CWAVES = WM * WN;
    static constexpr int POS = CT * TB * 4;                         // bytes of one (x, y) position
    static constexpr int XP = YS * POS + 32;                        // bytes of one x plane
    static constexpr int IMG_BYTES = XS * XP, NBUF_I = 3;
    static constexpr int FP = BR * BS * CT * 4 + 16;                // bytes of one Filter row
    static constexpr int FLT_BYTES = KT * FP, NBUF_F = 2;
    static constexpr int FLT_OFF = NBUF_I * IMG_BYTES;
    static constexpr int LDS_BYTES = FLT_OFF + NBUF_F * FLT_BYTES;
    static constexpr int PT = 256, PW = PT / 64;
    static constexpr int CHUNKS = XS * YS / 2, CPW = (CHUNKS + PW - 1) / PW;   // 1 KiB chunks: two positions (y, y + 1)
    static constexpr int FLT_ITEMS = KT * BR * BS * (CT / 4), MAXF = FLT_ITEMS / PT, MAXI = 1;
    static constexpr int LOADS = CPW + MAXF;
    static constexpr int GROUPS = BR * BS * (CT / 8);               // groups of four MFMAs per column block and unit
    static_assert(TB * TW == 32 && TH % WN == 0, "direct fp32 geometry: a column block is one tile row");
    static_assert(YS % 2 == 0 && POS == 512, "direct fp32 geometry: two positions of one x plane per chunk");
    static_assert(FLT_ITEMS % PT == 0 && GROUPS % 2 == 0, "direct fp32 geometry: whole Filter items, even group count");
    static_assert(IMG_BYTES < 65536 && LDS_BYTES <= 160 * 1024 && 2 * LOADS < 64, "direct fp32 geometry: LDS offsets, size, load counter");
    static bool matches_host(const KernelArgs& a) {
        return a.sw == 1 && a.sh == 1 && a.CT == CT && a.bS == BS && a.bR == BR && a.XS == XS && a.YS == YS &&
               a.R == BR && a.S % BS == 0 && a.C % CT == 0 && a.B % TB == 0 && a.W % TW == 0 && a.H % TH == 0 &&
               a.K % KT == 0 && a.vec_img && a.vec_flt;
    }
};

// The staging waves of the fp32 direct kernels (GEO: F32DirectFixed or F32Direct16): Image chunks straight into LDS,
// Filter items through registers.
template <class GEO>
__device__ __forceinline__ void f32_direct_stage(const KernelArgs& a, CACNN_LDS(char)* const lds, int tid, int wave_id,
                                                 int lane, int total) {
    constexpr int TB = GEO::TB, KT = GEO::KT, CT = GEO::CT, BS = GEO::BS, BR = GEO::BR, TW = GEO::TW_, TH = GEO::TH_;
    constexpr int YS = GEO::YSL, XP = GEO::XP, POS = GEO::POS, FP = GEO::FP;   // YS: the rows a plane holds in LDS
    constexpr int IBUF = GEO::IMG_BYTES, FBUF = GEO::FLT_BYTES, CTHREADS = GEO::CWAVES * 64;
    const int pw = wave_id - GEO::CWAVES, stid = tid - CTHREADS;
    constexpr int MAXF = GEO::MAXF, CPW = GEO::CPW, PT = GEO::PT;
    // Image: lane L of a chunk load fetches 16-byte piece L % 32 (channel (L % 32) / 2, images 4 * (L % 2)..) of
    // position y + L / 32
    const uint32_t row_bytes = (uint32_t)a.B * 4u;
    // (strides other than 1 only reach here with 1 x 1 filters: the positions a tile stages are then sigma apart)
    const uint32_t ivoff = (uint32_t)(lane >> 5) * (uint32_t)a.sh * (uint32_t)a.C * row_bytes +
                           (uint32_t)((lane & 31) >> 1) * row_bytes + (uint32_t)(lane & 1) * 16u;
    uint32_t isoff[CPW], ildst[CPW];
#pragma unroll
    for (int i = 0; i < CPW; ++i) {
        // the waves that would run out of chunks fetch the last one again (same words to the same place)
        const int ch = min(pw + GEO::PW * i, GEO::CHUNKS - 1);
        const int x = ch / (YS / 2), yy = ch % (YS / 2);
        isoff[i] = (uint32_t)((x * a.sw * a.IH + 2 * yy * a.sh) * a.C) * row_bytes;
        ildst[i] = (uint32_t)(x * XP + yy * 2 * POS);
    }
    // Filter: thread (kl = stid / 4, c4 = stid % 4) fetches the 16 bytes of channels 4*c4.. of output channel kl for
    // every tap (r, s) of the unit: one global offset and one LDS address per thread, the tap in the instruction
    static_assert(MAXF == BR * BS && PT == KT * (CT / 4), "direct fp32 geometry: one Filter item per thread and tap");
    const int f_c4 = stid % (CT / 4), f_kl = stid / (CT / 4);
    const uint32_t fg0 = ((uint32_t)f_kl * a.R * a.S * a.C + f_c4 * 4) * 4u;
    // C not a multiple of the c-slice (the 16 x 16-block kernels, C a multiple of 4): in the last c-slice of a tap the lanes
    // whose channel lies beyond C fetch from beyond every descriptor's range (2^31 or more with the chunk's or the tap's
    // offset, less than 2^32), so the range check puts zeros into LDS for both operands and the multiplying waves run
    // the slice like any other
    const int c_tail = a.C % CT;
    const uint32_t ivoff_tail = c_tail && (int)((lane & 31) >> 1) >= c_tail ? 0x80000000u : ivoff;
    const uint32_t fg0_tail = c_tail && f_c4 * 4 >= c_tail ? 0x80000000u : fg0;
    const uint32_t fl0 = (uint32_t)(uintptr_t)(lds + GEO::FLT_OFF + f_kl * FP + f_c4 * 16);
    uint32_t fsoff[MAXF];
#pragma unroll
    for (int i = 0; i < MAXF; ++i) fsoff[i] = (uint32_t)((i / BS) * a.S + i % BS) * (uint32_t)a.C * 4u;
    FxWalk<4, KT, TB, TW, TH, CT, BS> lu;     // next unit to fetch
    lu.init(a);
    f32x4 freg[2][MAXF];
    int ioff_issue = 0;                       // Image buffer the next fetch goes to
    auto issue = [&](int set) {
        const __amdgpu_buffer_rsrc_t ri = lu.img(a), rf = lu.flt(a);
        const bool last = lu.c0 + CT > a.C;
        const uint32_t ivo = last ? ivoff_tail : ivoff, fgo = last ? fg0_tail : fg0;
#pragma unroll
        for (int i = 0; i < CPW; ++i) load_16_bytes_per_lane_to_lds(ri, lds + ioff_issue + ildst[i], ivo, isoff[i]);
#pragma unroll
        for (int i = 0; i < MAXF; ++i) freg[set][i] = buf_load_f32x4(rf, fgo, fsoff[i]);
        lu.next(a);
        ioff_issue = ioff_issue + IBUF == GEO::NBUF_I * IBUF ? 0 : ioff_issue + IBUF;
    };
    // announce the unit whose Filter words are in register set `set` (also its Filter buffer): its loads are in
    // once at most `later` younger loads are outstanding (loads complete in order).  No vector-ALU instruction
    // on this path: next to an fp32 MFMA stream a staging wave practically never gets that issue port.
    auto announce = [&](int set, auto later) {
        __builtin_amdgcn_s_waitcnt(vmcnt_only(decltype(later)::value));
        if (set == 0) lds_store16_seq<0, CT * 4>(fl0, freg[0], std::make_index_sequence<MAXF>{});
        else lds_store16_seq<FBUF, CT * 4>(fl0, freg[1], std::make_index_sequence<MAXF>{});
        lds_done_then_barrier();
    };
    direct_staging_schedule<GEO::LOADS>(total, issue, announce);
}

template <int TW, int TH>
__global__ void __launch_bounds__(512) conv_f32_direct_kernel(const KernelArgs a) {
    using GEO = F32DirectFixed<TW, TH>;
    constexpr int TB = GEO::TB, KT = GEO::KT, CT = GEO::CT, BS = GEO::BS, WM = GEO::WM, NBLK = GEO::NBLK;
    constexpr int XP = GEO::XP, POS = GEO::POS, FP = GEO::FP;
    constexpr int IBUF = GEO::IMG_BYTES, FBUF = GEO::FLT_BYTES;
    extern __shared__ __align__(16) f32x4 smem_v[];
    CACNN_LDS(char)* const lds = (CACNN_LDS(char)*)smem_v;
    const int tid = threadIdx.x;
    const int wave_id = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: the role branch is wave-uniform
    const int lane = tid & 63;
    // units this workgroup works through: its tiles blockIdx.x, blockIdx.x + gridDim.x, ... times the slices of a tile
    const int upt = (a.C / CT) * (a.S / BS);
    int total = 0;
    for (int t = blockIdx.x; t < a.n_tiles; t += gridDim.x) total += upt;

    if (wave_id >= GEO::CWAVES) {
        f32_direct_stage<GEO>(a, lds, tid, wave_id, lane, total);
    } else {
        const int wm = wave_id % WM, wn = wave_id / WM;
        const int j = lane & 31, g = lane >> 5;
        f32x16 acc[1][NBLK];
        zero_acc(acc);
        // per-lane LDS offsets: Filter row of output channel wm*32 + j, channels 4g..4g+3 of a group of 8;
        // Image: output column j / 8 of the tile row, image j % 8, channel 4g of a group of 8, tile row wn * NBLK
        const uint32_t al = (uint32_t)(GEO::FLT_OFF + (wm * 32 + j) * FP + g * 16);
        const uint32_t xl = (uint32_t)((j >> 3) * XP + wn * NBLK * POS + g * 4 * TB * 4 + (j & 7) * 4);
        f32x4 A[2];
        float X[2][NBLK][4];
        auto load_group = [&](uint32_t ab, uint32_t xb, int grp, int set) {
            const int c8 = grp % (CT / 8), rs = grp / (CT / 8);
            const int r = rs / BS, sl = rs % BS;
            A[set] = *(const CACNN_LDS(f32x4)*)(lds + ab + (rs * CT + c8 * 8) * 4);
#pragma unroll
            for (int n = 0; n < NBLK; ++n)
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    X[set][n][t] = *(const CACNN_LDS(float)*)(lds + xb + r * XP + (n + sl) * POS + (c8 * 8 + t) * TB * 4);
        };
        auto mfma_group = [&](int set) {
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int n = 0; n < NBLK; ++n)
                    acc[0][n] = __builtin_amdgcn_mfma_f32_32x32x2f32(A[set][t], X[set][n][t], acc[0][n], 0, 0, 0);
        };
        const int64_t out_kstride = (int64_t)a.H * a.W * a.B;      // floats between output channels
        const uint32_t out_lane = (uint32_t)(g * 4) * (uint32_t)out_kstride + (uint32_t)((j / TB) * a.B + j % TB);
        int left = total, in_tile = upt, t = blockIdx.x;
        uint32_t ioff = 0, foff = 0;
        // one unit; MORE: another one follows (in the next Image buffer of the three, the other Filter buffer)
        auto unit = [&](auto more) {
            constexpr bool MORE = decltype(more)::value;
#pragma unroll
            for (int grp = 0; grp < GEO::GROUPS; ++grp) {
                if (grp + 1 < GEO::GROUPS) {
                    load_group(al + foff, xl + ioff, grp + 1, (grp + 1) & 1);
                } else if constexpr (MORE) {
                    // hand the buffers back once the last fragments have landed, read the next unit's first
                    // fragments under this group's MFMAs
                    ioff = ioff + IBUF == GEO::NBUF_I * IBUF ? 0u : ioff + IBUF;
                    foff = FBUF - foff;
                    lds_done_then_barrier_known(acc[0][NBLK - 1]);
                    load_group(al + foff, xl + ioff, 0, 0);
                }
                mfma_group(grp & 1);
                if (grp + 1 < GEO::GROUPS || MORE) interleave_hint<4 * NBLK, 1 + 4 * NBLK>();
            }
            // keep the reads above where they are (the compiler would sink them to the top of the next unit)
            asm volatile("" ::: "memory");
            --left;
            if (__builtin_expect(--in_tile == 0, 0)) {
                const TileCoord tc = decode_tile_index(a, t, KT, TB, TW, TH);
#pragma unroll
                for (int n = 0; n < NBLK; ++n) {
                    float* const blk = a.out + ((((int64_t)(tc.k0 + wm * 32) * a.H + tc.h0 + wn * NBLK + n) * a.W + tc.w0) * a.B + tc.b0);
                    store_block_exact<false>(blk, out_kstride, out_lane, acc[0][n]);
                }
                in_tile = upt;
                t += gridDim.x;
            }
        };
        if (left > 0) {
            lds_done_then_barrier_known();      // unit 0 is staged
            load_group(al, xl, 0, 0);
            while (left > 1) unit(std::true_type{});
            unit(std::false_type{});
        }
    }
}

// ---- fixed geometry, fp32, 16x16 MFMA blocks -------------------------------------------------------------------------
// The same staging and LDS layouts with the tile cut into 16x16 blocks (the 16x16x4 MFMA has the 32x32x2 one's rate):
// a tile of 8 images x 2 x 7 positions is 7 column blocks of 16 (one output row each: 2 columns x 8 images), and each
// of the four multiplying waves owns 16 of the 64 output channels and all 7 blocks.  112 columns per tile instead of
// 128 is what a layer with 56 x 56 positions and 8 images wants: 224 tiles, one per compute unit, where tiles of 128
// columns leave 60 of the 256 compute units idle.
// An MFMA takes four contraction indices, one per quarter-wave q: channels 2q + e + 8h for the MFMA (h, e) of a
// 16-channel slice, so a lane's Filter words for e = 0, 1 are one 8-byte read and the Image rows of the four
// quarters are 64 bytes apart: with the two output columns of a block 32 bytes (mod 256) apart, the 64 lanes of an
// Image read fall into 64 different banks.  For fixed (r, channel) the 9 Image rows y = 0..8 serve all 7 blocks and 3 taps s
// (block j with tap s reads row j + s): 18 Image reads and 3 Filter reads per 42 MFMAs.  A plane holds 10 rows in LDS
// (whole 1 KiB chunks of two rows; the tenth is fetched and never read).
// BRS: the filter's extent in both directions (3, or 1 for 1 x 1 filters).
template <int TW, int TH, int BRS = 3>
struct F32Direct16 {
    static constexpr int TB = 8, KT = 64, CWAVES = 4, CT = 16, BS = BRS, BR = BRS, NBLK = TH, TW_ = TW, TH_ = TH;
    static constexpr int XS = TW + BR - 1, YS = TH - 1 + BS, YSL = YS + (YS & 1);
    static constexpr int POS = CT * TB * 4;                         // bytes of one (x, y) position
    static constexpr int XP = YSL * POS + 32;                       // bytes of one x plane
    static constexpr int IMG_BYTES = XS * XP, NBUF_I = 3;
    static constexpr int FP = BR * BS * CT * 4 + 16;                // bytes of one Filter row
    static constexpr int FLT_BYTES = KT * FP, NBUF_F = 2;
    static constexpr int FLT_OFF = NBUF_I * IMG_BYTES;
    static constexpr int LDS_BYTES = FLT_OFF + NBUF_F * FLT_BYTES;
    static constexpr int PT = 256, PW = PT / 64;
    static constexpr int CHUNKS = XS * YSL / 2, CPW = (CHUNKS + PW - 1) / PW;
    static constexpr int FLT_ITEMS = KT * BR * BS * (CT / 4), MAXF = FLT_ITEMS / PT, MAXI = 1;
    static constexpr int LOADS = CPW + MAXF;
    static constexpr int GROUPS = BR * (CT / 8);                    // groups of 2 * BS * NBLK MFMAs per unit
    static_assert(TB * TW == 16 && KT == CWAVES * 16, "direct fp32 16x16 geometry: a column block is one tile row, a wave 16 channels");
    static_assert(POS == 512 && (YSL * POS) % 256 == 0, "direct fp32 16x16 geometry: chunks, bank spread of the two columns");
    static_assert(FLT_ITEMS % PT == 0 && GROUPS % 2 == 0, "direct fp32 16x16 geometry: whole Filter items, even group count");
    static_assert(IMG_BYTES < 65536 && LDS_BYTES <= 160 * 1024 && 2 * LOADS < 64, "direct fp32 16x16 geometry: LDS offsets, size, load counter");
    static bool matches_host(const KernelArgs& a) {
        // (W, H and K need not be multiples of the tile: what a tile stages beyond the arrays is zeros or other rows of
        // the Image, which only reach outputs that are not stored)
        // (1 x 1 filters: any strides, a tile stages the TW x TH positions its outputs read and nothing between them)
        return (BRS == 1 || (a.sw == 1 && a.sh == 1)) && a.CT == CT && a.bS == BS && a.bR == BR && a.XS == XS && a.YS == YS &&
               a.R % BR == 0 && (BRS == 1 || a.R == BR) && a.S % BS == 0 && a.C % 4 == 0 && a.B % TB == 0 && a.vec_img && a.vec_flt;
    }
};

template <int TW, int TH, int BRS = 3>
__global__ void __launch_bounds__(512) conv_f32_direct16_kernel(const KernelArgs a) {
    using GEO = F32Direct16<TW, TH, BRS>;
    constexpr int TB = GEO::TB, KT = GEO::KT, CT = GEO::CT, BS = GEO::BS, NBLK = GEO::NBLK;
    constexpr int YS = GEO::YS, XP = GEO::XP, POS = GEO::POS, FP = GEO::FP;
    constexpr int IBUF = GEO::IMG_BYTES, FBUF = GEO::FLT_BYTES;
    extern __shared__ __align__(16) f32x4 smem_v[];
    CACNN_LDS(char)* const lds = (CACNN_LDS(char)*)smem_v;
    const int tid = threadIdx.x;
    const int wave_id = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: the role branch is wave-uniform
    const int lane = tid & 63;
    // (R > b_r only in the kernel for 1 x 1 filters: a unit per tap; the last c-slice may be partly filled)
    const int upt = ((a.C + CT - 1) / CT) * (a.S / BS) * (a.R / GEO::BR);
    int total = 0;
    for (int t = blockIdx.x; t < a.n_tiles; t += gridDim.x) total += upt;

    if (wave_id >= GEO::CWAVES) {
        f32_direct_stage<GEO>(a, lds, tid, wave_id, lane, total);
    } else {
        const int n = lane & 15, q = lane >> 4;
        f32x4 acc[NBLK];
#pragma unroll
        for (int j = 0; j < NBLK; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
        // per-lane LDS offsets: Filter row of output channel 16 * wave + n, channels 2q, 2q + 1 of a group of 8;
        // Image: output column n / 8 of the tile row, image n % 8, channel 2q of a group of 8
        const uint32_t al = (uint32_t)(GEO::FLT_OFF + (wave_id * 16 + n) * FP + q * 8);
        const uint32_t xl = (uint32_t)((n >> 3) * XP + q * 2 * TB * 4 + (n & 7) * 4);
        f32x2 A[2][BS];
        float X[2][YS][2];
        // Every read is one base register plus an offset in the instruction: a base per filter column r and channel
        // parity e for the Image (the compiler must not fold them into one, the offsets would then outgrow the
        // instruction's field and every read would need an address addition, which costs the MFMA stream an issue
        // slot), one for the Filter.  They change once per unit.
        uint32_t xr[GEO::BR][2], ar;
        auto set_bases = [&](uint32_t ioff, uint32_t foff) {
#pragma unroll
            for (int r = 0; r < GEO::BR; ++r)
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    xr[r][e] = xl + ioff + r * XP + e * TB * 4;
                    asm("" : "+v"(xr[r][e]));
                }
            ar = al + foff;
            asm("" : "+v"(ar));
        };
        auto load_group = [&](int grp, int set) {
            const int r = grp / (CT / 8), c8 = grp % (CT / 8);
#pragma unroll
            for (int s = 0; s < BS; ++s) A[set][s] = *(const CACNN_LDS(f32x2)*)(lds + ar + ((r * BS + s) * CT + c8 * 8) * 4);
#pragma unroll
            for (int y = 0; y < YS; ++y)
#pragma unroll
                for (int e = 0; e < 2; ++e)
                    X[set][y][e] = *(const CACNN_LDS(float)*)(lds + xr[r][e] + y * POS + c8 * 8 * TB * 4);
        };
        auto mfma_group = [&](int set) {
#pragma unroll
            for (int e = 0; e < 2; ++e)
#pragma unroll
                for (int s = 0; s < BS; ++s)
#pragma unroll
                    for (int j = 0; j < NBLK; ++j)
                        acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(A[set][s][e], X[set][j + s][e], acc[j], 0, 0, 0);
        };
        const int64_t out_kstride = (int64_t)a.H * a.W * a.B;      // floats between output channels
        const uint32_t out_lane = (uint32_t)(q * 4) * (uint32_t)out_kstride + (uint32_t)((n / TB) * a.B + n % TB);
        int left = total, in_tile = upt, t = blockIdx.x;
        uint32_t ioff = 0, foff = 0;
        // one unit; MORE: another one follows (in the next Image buffer of the three, the other Filter buffer)
        auto unit = [&](auto more) {
            constexpr bool MORE = decltype(more)::value;
#pragma unroll
            for (int grp = 0; grp < GEO::GROUPS; ++grp) {
                if (grp + 1 < GEO::GROUPS) {
                    load_group(grp + 1, (grp + 1) & 1);
                } else if constexpr (MORE) {
                    ioff = ioff + IBUF == GEO::NBUF_I * IBUF ? 0u : ioff + IBUF;
                    foff = FBUF - foff;
                    lds_done_then_barrier_known(acc[NBLK - 1]);
                    set_bases(ioff, foff);
                    load_group(0, 0);
                }
                mfma_group(grp & 1);
                if (grp + 1 < GEO::GROUPS || MORE) interleave_hint<2 * BS * NBLK, BS + 2 * YS>();
            }
            // keep the reads above where they are (the compiler would sink them to the top of the next unit)
            asm volatile("" ::: "memory");
            --left;
            if (__builtin_expect(--in_tile == 0, 0)) {
                const TileCoord tc = decode_tile_index(a, t, KT, TB, TW, TH);
                if (tc.k0 + KT <= a.K && tc.w0 + TW <= a.W && tc.h0 + TH <= a.H) {
#pragma unroll
                    for (int j = 0; j < NBLK; ++j) {
                        float* const blk = a.out + ((((int64_t)(tc.k0 + wave_id * 16) * a.H + tc.h0 + j) * a.W + tc.w0) * a.B + tc.b0);
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            (blk + (int64_t)v * out_kstride)[out_lane] = acc[j][v];
                            acc[j][v] = 0.f;
                        }
                    }
                } else {
                    // a tile that overhangs Out: the tile rows inside, this lane's column if it is inside, and of its four
                    // output channels those inside
                    const int rows = (tc.w0 + n / TB < a.W) ? a.K - (tc.k0 + wave_id * 16 + q * 4) : 0;
#pragma unroll
                    for (int j = 0; j < NBLK; ++j) {
                        float* const blk = a.out + ((((int64_t)(tc.k0 + wave_id * 16) * a.H + tc.h0 + j) * a.W + tc.w0) * a.B + tc.b0);
                        const int rows_j = tc.h0 + j < a.H ? rows : 0;
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            if (v < rows_j) (blk + (int64_t)v * out_kstride)[out_lane] = acc[j][v];
                            acc[j][v] = 0.f;
                        }
                    }
                }
                in_tile = upt;
                t += gridDim.x;
            }
        };
        if (left > 0) {
            lds_done_then_barrier_known();      // unit 0 is staged
            set_bases(0, 0);
            load_group(0, 0);
            while (left > 1) unit(std::true_type{});
            unit(std::false_type{});
        }
    }
}

// ---- fixed geometry, large strided filter, few channels (the stem-layer shape), Image loaded straight into LDS ------
// 7x7 taps, strides 2, three channels, 32 images per tile.  (With C = 3 the 16-byte channel fragments of the generic
// kernels would be mostly padding.)  The Image keeps its global order in LDS: one x plane is the
// run of (y, c) rows of the tile's 32 images (128 bytes each, 27 rows for a tile two output rows high), so the
// contraction over (s, c) for a fixed r is a walk down consecutive rows: row 6*h_l + q, q = 3 s + c = 0..20.  An fp32
// MFMA takes two contraction indices, one per half-wave: the halves take q and q + 11 (a constant 11 rows apart, so it
// sits in the lane's base register), 11 MFMAs per filter column r and 77 per 32x32 block where the unpadded
// contraction needs 73.5 (q = 21 does not exist: the Filter holds 0 there and the lanes that would pair it with the
// row below the window supply 0 as well, so no 0 * NaN can occur).  Planes are 4 KiB apart: a plane is 216 16-byte
// pieces, moved by four loads of 64 lanes, and the lanes beyond the last piece fetch it again into the padding.
// Filter in LDS: [k][r][22] words, rows of 155 words (odd: the 32 rows of an operand hit 32 banks).  It is staged
// once per workgroup and k-tile.  Three Image buffers, loads two tiles ahead; a tile is one unit.
template <int TW, int TH>
struct F32StemDirect {
    static constexpr int R = 7, S = 7, SW = 2, SH = 2, C = 3, TB = 32, KT = 64, WM = 2, WN = 2, NBLK = TW * TH / WN;
    static constexpr int XS = SW * (TW - 1) + R, YS = SH * (TH - 1) + S;
    static constexpr int ROWB = TB * 4;                           // bytes of one (y, c) row
    static constexpr int PIECES = YS * C * ROWB / 16;             // 16-byte pieces of one x plane
    static constexpr int XPB = 4096, PARTS = XPB / 1024;          // plane pitch; 1 KiB loads per plane
    static constexpr int Q = S * C, QH = (Q + 1) / 2, QP = 2 * QH; // 21 contraction indices per r, 11 per half-wave, 22 slots
    static constexpr int IMG_BYTES = XS * XPB, NBUF = 3;
    static constexpr int FPW = (R * QP) | 1, FLT_BYTES = KT * FPW * 4;
    static constexpr int FLT_OFF = NBUF * IMG_BYTES, LDS_BYTES = FLT_OFF + FLT_BYTES;
    static constexpr int PT = 256, PW = PT / 64, CPW = XS;        // staging wave p moves part p of every plane
    static constexpr int MAXI = 1, MAXF = 1;
    static constexpr int G0 = (QH + 1) / 2, G1 = QH - G0;         // MFMAs per column block in the two groups of one r
    static_assert(PARTS == PW && PIECES <= PARTS * 64 && PIECES > (PARTS - 1) * 64, "stem geometry: four loads per plane");
    static_assert((SH * (TH - 1) * C + QP) * ROWB <= XPB, "stem geometry: the row below the window lies inside the plane's pitch");
    static_assert((TW * TH) % WN == 0 && 2 * CPW < 64, "stem geometry: column blocks per wave, load counter range");
    static_assert(IMG_BYTES < 65536 && LDS_BYTES <= 160 * 1024, "stem geometry: LDS offsets and size");
    static bool matches_host(const KernelArgs& a) {
        // (W, H, K and B need not be multiples of the tile, B only of the 4 images of a 16-byte load: what a tile stages
        // beyond the arrays or beyond a row's images is zeros or other rows of the Image, which only reach outputs that
        // are not stored; Filter rows beyond K are staged as zeros)
        return a.sw == SW && a.sh == SH && a.R == R && a.S == S && a.C == C && a.bR == R && a.bS == S && a.CT == C &&
               a.B % 4 == 0 && a.vec_img;
    }
};

// RAGGED: the instance for shapes whose tiles overhang Out (the other one stores every tile whole: the test at the end of a
// tile and the second store path beside the first cost it 2.5 % on the benchmark shape)
template <int TW, int TH, bool RAGGED>
__global__ void __launch_bounds__(512) conv_f32_stem_direct_kernel(const KernelArgs a) {
    using GEO = F32StemDirect<TW, TH>;
    constexpr int R = GEO::R, S = GEO::S, C = GEO::C, SW = GEO::SW, SH = GEO::SH;
    constexpr int TB = GEO::TB, KT = GEO::KT, WM = GEO::WM, NBLK = GEO::NBLK, XPB = GEO::XPB, ROWB = GEO::ROWB;
    constexpr int QH = GEO::QH, QP = GEO::QP, FPW = GEO::FPW, IBUF = GEO::IMG_BYTES;
    constexpr int CTHREADS = GEO::WM * GEO::WN * 64;
    extern __shared__ __align__(16) float smem_f[];
    CACNN_LDS(char)* const lds = (CACNN_LDS(char)*)smem_f;
    const int tid = threadIdx.x;
    const int wave_id = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: the role branch is wave-uniform
    const int lane = tid & 63;
    int total = 0;                                                  // tiles of this workgroup
    for (int t = blockIdx.x; t < a.n_tiles; t += gridDim.x) ++total;

    if (wave_id >= GEO::WM * GEO::WN) {
        const int pw = wave_id - GEO::WM * GEO::WN, stid = tid - CTHREADS;
        // Image: lane L of staging wave p fetches piece 64 p + L of a plane: row piece / 8 (rows are B words apart in
        // global memory), 16 bytes (piece % 8) of its 128; lanes beyond the last piece fetch the last one again
        const int piece = min(pw * 64 + lane, GEO::PIECES - 1);
        const uint32_t ivoff = (uint32_t)(piece >> 3) * (uint32_t)a.B * 4u + (uint32_t)(piece & 7) * 16u;
        const uint32_t plane_bytes = (uint32_t)a.IH * a.C * a.B * 4u;
        FxWalk<4, KT, TB, TW, TH, C, S> lu;     // next tile to fetch
        lu.init(a);
        int ioff_issue = 0;
        auto issue = [&]() {
            const __amdgpu_buffer_rsrc_t ri = lu.img(a);
#pragma unroll
            for (int x = 0; x < GEO::XS; ++x)
                load_16_bytes_per_lane_to_lds(ri, lds + ioff_issue + x * XPB + pw * 1024, ivoff, (uint32_t)x * plane_bytes);
            lu.next(a);
            ioff_issue = ioff_issue + IBUF == GEO::NBUF * IBUF ? 0 : ioff_issue + IBUF;
        };
        auto stage_filter = [&](int k0) {
            // Filter [K][R][S][C] -> LDS [k][r][22], slot 21 zero.  The KT rows of the tile are one contiguous run in
            // global memory: read it in order (coalesced, all loads of a batch in flight together), scatter into LDS.
            float* const s_flt = smem_f + GEO::FLT_OFF / 4;
            constexpr int ROW = R * S * C, TOTAL = KT * ROW, BATCH = 8;
            const float* src = (const float*)a.filter + (int64_t)k0 * ROW;
            const int have = RAGGED ? min(KT, a.K - k0) * ROW : TOTAL;      // (a k-tile that overhangs K: the rows beyond it are zeros)
            for (int e0 = 0; e0 < TOTAL; e0 += BATCH * GEO::PT) {
                float v[BATCH];
#pragma unroll
                for (int u = 0; u < BATCH; ++u) {
                    const int e = e0 + u * GEO::PT + stid;
                    v[u] = e < have ? src[e] : 0.f;
                }
#pragma unroll
                for (int u = 0; u < BATCH; ++u) {
                    const int e = e0 + u * GEO::PT + stid;
                    if (e < TOTAL) {
                        const int kl = e / ROW, q = e % ROW;
                        s_flt[kl * FPW + (q / (S * C)) * QP + q % (S * C)] = v[u];
                    }
                }
            }
            for (int e = stid; e < KT * R; e += GEO::PT) s_flt[(e / R) * FPW + (e % R) * QP + QP - 1] = 0.f;
        };
        int flt_k0 = -1;
        int st = blockIdx.x;                    // tile about to be announced
        if (total > 0) issue();
        if (total > 1) issue();
        for (int u = 0; u < total; ++u) {
            const TileCoord tc = decode_tile_index(a, st, KT, TB, TW, TH);
            if (tc.k0 != flt_k0) {
                // the Filter tile is single-buffered: wait until the multiplying waves have finished the old one
                if (flt_k0 >= 0) lds_done_then_barrier();
                flt_k0 = tc.k0;
                stage_filter(flt_k0);
            }
            // loads complete in order: this tile is in once at most the next tile's loads are outstanding
            if (u + 1 < total) __builtin_amdgcn_s_waitcnt(vmcnt_only(GEO::CPW));
            else __builtin_amdgcn_s_waitcnt(vmcnt_only(0));
            lds_done_then_barrier();
            if (u + 2 < total) issue();         // the buffer the multiplying waves left two tiles back
            st += gridDim.x;
        }
    } else {
        const int wm = wave_id % WM, wn = wave_id / WM;
        const int j = lane & 31, g = lane >> 5;
        f32x16 acc[1][NBLK];
        zero_acc(acc);
        // per-lane LDS offsets: Filter row of output channel wm*32 + j, slots 11 g ..; Image: image j, rows 11 g ..
        const uint32_t al = (uint32_t)(GEO::FLT_OFF + ((wm * 32 + j) * FPW + g * QH) * 4);
        static_assert(NBLK == TW, "stem geometry: a wave owns one tile row");
        const uint32_t xl = (uint32_t)(j * 4 + g * QH * ROWB + wn * SH * C * ROWB);
        float A[2][GEO::G0], X[2][NBLK][GEO::G0];
        // group gi = 2 r + half: slots q0 .. q0 + n - 1 of filter column r
        auto load_group = [&](uint32_t xb, int gi, int set) {
            const int r = gi >> 1, q0 = (gi & 1) ? GEO::G0 : 0, n = (gi & 1) ? GEO::G1 : GEO::G0;
#pragma unroll
            for (int t = 0; t < n; ++t) A[set][t] = *(const CACNN_LDS(float)*)(lds + al + (r * QP + q0 + t) * 4);
#pragma unroll
            for (int nb = 0; nb < NBLK; ++nb)       // column block nb of this wave: output column nb of tile row wn
#pragma unroll
                for (int t = 0; t < n; ++t)
                    X[set][nb][t] = *(const CACNN_LDS(float)*)(lds + xb + (r + nb * SW) * XPB + (q0 + t) * ROWB);
        };
        auto mfma_group = [&](int gi, int set) {
            const int n = (gi & 1) ? GEO::G1 : GEO::G0;
#pragma unroll
            for (int t = 0; t < n; ++t)
#pragma unroll
                for (int nb = 0; nb < NBLK; ++nb) {
                    float x = X[set][nb][t];
                    // slot 21 (q = 10 in the upper half-wave) does not exist
                    if ((gi & 1) && t == n - 1) x = g ? 0.f : x;
                    acc[0][nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(A[set][t], x, acc[0][nb], 0, 0, 0);
                }
        };
        const int64_t out_kstride = (int64_t)a.H * a.W * a.B;                    // floats between output channels
        const uint32_t out_lane = (uint32_t)(g * 4) * (uint32_t)out_kstride + j;  // < 2^31: checked by the host
        int left = total, t = blockIdx.x;
        uint32_t ioff = 0;
        TileCoord tc = decode_tile_index(a, t, KT, TB, TW, TH);
        int flt_k0 = tc.k0;
        auto unit = [&](auto more) {
            constexpr bool MORE = decltype(more)::value;
            TileCoord ntc = tc;
            if constexpr (MORE) ntc = decode_tile_index(a, t + gridDim.x, KT, TB, TW, TH);
#pragma unroll
            for (int gi = 0; gi < 2 * R; ++gi) {
                if (gi + 1 < 2 * R) {
                    load_group(xl + ioff, gi + 1, (gi + 1) & 1);
                } else if constexpr (MORE) {
                    // every fragment of this tile has been requested: once they have landed the buffer goes back to
                    // the staging waves, and the first fragments of the next tile are read under this group's MFMAs
                    if (ntc.k0 != flt_k0) {
                        lds_done_then_barrier();      // done with the old Filter tile
                        flt_k0 = ntc.k0;
                    }
                    ioff = ioff + IBUF == GEO::NBUF * IBUF ? 0u : ioff + IBUF;
                    lds_done_then_barrier_known(acc[0][NBLK - 1]);
                    load_group(xl + ioff, 0, 0);
                }
                mfma_group(gi, gi & 1);
                if (gi + 1 < 2 * R || MORE) interleave_hint<GEO::G0 * NBLK, GEO::G0 * (NBLK + 1)>();
            }
            asm volatile("" ::: "memory");       // keep the reads above where they are
            // Out tile: block n is output column w_l, row h_l; a lane owns image j
            if (!RAGGED || (tc.k0 + KT <= a.K && tc.w0 + TW <= a.W && tc.h0 + TH <= a.H && tc.b0 + TB <= a.B && a.B % 32 == 0)) {
#pragma unroll
                for (int nb = 0; nb < NBLK; ++nb) {
                    float* const blk = a.out + ((((int64_t)(tc.k0 + wm * 32) * a.H + tc.h0 + wn) * a.W + tc.w0 + nb) * a.B + tc.b0);
                    store_block_exact<true>(blk, out_kstride, out_lane, acc[0][nb]);
                }
            } else {
                // a tile that overhangs Out: the blocks of positions inside, this lane's image if it is inside, the rows
                // of output channels inside
                const int rows = (tc.b0 + j < a.B && tc.h0 + wn < a.H) ? a.K - (tc.k0 + wm * 32 + g * 4) : 0;
#pragma unroll
                for (int nb = 0; nb < NBLK; ++nb) {
                    float* const blk = a.out + ((((int64_t)(tc.k0 + wm * 32) * a.H + tc.h0 + wn) * a.W + tc.w0 + nb) * a.B + tc.b0);
                    store_block_rows(blk, out_kstride, out_lane, acc[0][nb], tc.w0 + nb < a.W ? rows : 0);
                }
            }
            --left;
            t += gridDim.x;
            tc = ntc;
        };
        if (left > 0) {
            lds_done_then_barrier_known();      // tile 0 and the Filter tile are staged
            load_group(xl, 0, 0);
            while (left > 1) unit(std::true_type{});
            unit(std::false_type{});
        }
    }
}

// ---------------------------------------------------------------------------------------------------------------
// launch table

template <typename KernelT>
static int launch_kernel(KernelT kernel, bool& attr_done, int threads, const KernelArgs& a, int grid, size_t lds_bytes,
                         void* stream) {
    if (!attr_done) {
        // raise the dynamic-LDS ceiling of this kernel to the CU's full 160 KiB once
        if (hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) !=
            hipSuccess) {
            (void)hipGetLastError();
            return 1;
        }
        attr_done = true;
    }
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(threads), lds_bytes, (hipStream_t)stream, a);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

#define CACNN_VARIANT(DT, KERNEL, NAME, WM, WN, MBLK, NBLK, TB, TW, TH) \
    CACNN_VARIANT_TUNED(DT, KERNEL, NAME, 1.0f, WM, WN, MBLK, NBLK, TB, TW, TH)
#define CACNN_VARIANT_TUNED(DT, KERNEL, NAME, TUNE, WM, WN, MBLK, NBLK, TB, TW, TH)                      \
    {                                                                                                    \
        {NAME, DT, WM, WN, MBLK, NBLK, TB, TW, TH, 0, 0, 0, 2, 0, TUNE},                                             \
            [](const KernelArgs& a, int grid, size_t lds, void* stream) -> int {                         \
                static bool attr_done = false;                                                           \
                return launch_kernel(KERNEL<WM, WN, MBLK, NBLK, TB, TW, TH>, attr_done, WM * WN * 64, a, \
                                     grid, lds, stream);                                                 \
            }                                                                                            \
    }

#define CACNN_PIPE_VARIANT(DT, KERNEL, NAME, WM, WN, MBLK, NBLK, TB, TW, TH, MAXI, MAXF, OCC)                   \
    {                                                                                                          \
        {NAME, DT, WM, WN, MBLK, NBLK, TB, TW, TH, 1, MAXI, MAXF, OCC, 0, 1.0f},                               \
            [](const KernelArgs& a, int grid, size_t lds, void* stream) -> int {                               \
                static bool attr_done = false;                                                                 \
                return launch_kernel(KERNEL<WM, WN, MBLK, NBLK, TB, TW, TH, MAXI, MAXF>, attr_done,            \
                                     WM * WN * 64, a, grid, lds, stream);                                      \
            }                                                                                                  \
    }

#define CACNN_REUSE_VARIANT(NAME, WM, WN, MBLK, NBLK, TB, TW, TH, MAXI, MAXF, OCC, BR)                          \
    {                                                                                                          \
        {NAME, 1, WM, WN, MBLK, NBLK, TB, TW, TH, 1, MAXI, MAXF, OCC, BR, 1.0f},                               \
            [](const KernelArgs& a, int grid, size_t lds, void* stream) -> int {                               \
                static bool attr_done = false;                                                                 \
                return launch_kernel(conv_bf16_pipe_kernel<WM, WN, MBLK, NBLK, TB, TW, TH, MAXI, MAXF, BR>,    \
                                     attr_done, WM * WN * 64, a, grid, lds, stream);                           \
            }                                                                                                  \
    }

#define CACNN_WS_VARIANT(DT, NAME, TUNE, WM, WN, MBLK, NBLK, TB, TW, TH, MAXI, MAXF, BR, ...)                   \
    {                                                                                                          \
        {NAME, DT, WM, WN, MBLK, NBLK, TB, TW, TH, 2, MAXI, MAXF, 1, BR, TUNE},                                \
            [](const KernelArgs& a, int grid, size_t lds, void* stream) -> int {                               \
                static bool attr_done = false;                                                                 \
                return launch_kernel(__VA_ARGS__, attr_done, WM * WN * 128, a, grid, lds, stream);             \
            }                                                                                                  \
    }

// bf16 with the Image loaded straight into LDS: 64 images, 64 output channels, 32-channel slices of one filter row
#define CACNN_DIRECT_VARIANT(NAME, UNIT_US, FIXED_US, CALIB, TW, TH)                                                 \
    {                                                                                                          \
        {NAME, 1, 2, 2, 1, Bf16DirectFixed<TW, TH>::NBLK, 64, TW, TH, 2, 1, Bf16DirectFixed<TW, TH>::MAXF, 1, 3, 1.0f, 32, 3,  \
         1, Bf16DirectFixed<TW, TH>::YS, 1, 1, Bf16DirectFixed<TW, TH>::LDS_BYTES, UNIT_US, FIXED_US, 0, 2, CALIB},       \
            [](const KernelArgs& a, int grid, size_t lds, void* stream) -> int {                               \
                static bool attr_done = false;                                                                 \
                if (!Bf16DirectFixed<TW, TH>::matches_host(a) || lds != (size_t)Bf16DirectFixed<TW, TH>::LDS_BYTES) return 1; \
                return launch_kernel(conv_bf16_direct_kernel<TW, TH>, attr_done, 512, a, grid, lds, stream);    \
            }                                                                                                  \
    }

// 1 x 1 filters with 64-channel units
#define CACNN_DIRECT_1X1_C64_VARIANT(NAME, UNIT_US, FIXED_US, TW, TH)                                           \
    {                                                                                                          \
        {NAME, 1, 2, 2, 1, Bf16DirectFixed<TW, TH, 1, 64, 1, 64>::NBLK, 64, TW, TH, 2, 1, Bf16DirectFixed<TW, TH, 1, 64, 1, 64>::MAXF, 1, 1, 1.0f, 64, 1,  \
         1, Bf16DirectFixed<TW, TH, 1, 64, 1, 64>::YS, 1, 1, Bf16DirectFixed<TW, TH, 1, 64, 1, 64>::LDS_BYTES, UNIT_US, FIXED_US, 0, 2, 256, 1},  \
            [](const KernelArgs& a, int grid, size_t lds, void* stream) -> int {                               \
                static bool attr_done = false;                                                                 \
                if (!Bf16DirectFixed<TW, TH, 1, 64, 1, 64>::matches_host(a) || lds != (size_t)Bf16DirectFixed<TW, TH, 1, 64, 1, 64>::LDS_BYTES) return 1; \
                return launch_kernel(conv_bf16_direct_kernel<TW, TH, 1, 64, 1, false, 64>, attr_done, 512, a, grid, lds, stream); \
            }                                                                                                  \
    }

// ... and for C a multiple of 8 but not of 64
#define CACNN_DIRECT_1X1_C64_T8_VARIANT(NAME, UNIT_US, FIXED_US, TW, TH)                                        \
    {                                                                                                          \
        {NAME, 1, 2, 2, 1, Bf16DirectFixed<TW, TH, 1, 64, 1, 64>::NBLK, 64, TW, TH, 2, 1, Bf16DirectFixed<TW, TH, 1, 64, 1, 64>::MAXF, 1, 1, 1.0f, 64, 1,  \
         1, Bf16DirectFixed<TW, TH, 1, 64, 1, 64>::YS, 1, 1, Bf16DirectFixed<TW, TH, 1, 64, 1, 64>::LDS_BYTES, UNIT_US, FIXED_US, 0, 2, 256, 1, 1},  \
            [](const KernelArgs& a, int grid, size_t lds, void* stream) -> int {                               \
                static bool attr_done = false;                                                                 \
                if (!Bf16DirectFixed<TW, TH, 1, 64, 1, 64>::matches_host(a, true) || lds != (size_t)Bf16DirectFixed<TW, TH, 1, 64, 1, 64>::LDS_BYTES) return 1; \
                return launch_kernel(conv_bf16_direct_kernel<TW, TH, 1, 64, 1, true, 64>, attr_done, 512, a, grid, lds, stream); \
            }                                                                                                  \
    }

// the same for C a multiple of 8 but not of 32 (BR = 3 or 1): the staging waves zero-fill the last c-slice
#define CACNN_DIRECT_T8_VARIANT(NAME, UNIT_US, FIXED_US, CALIB, TW, TH, BR)                                    \
    {                                                                                                          \
        {NAME, 1, 2, 2, 1, Bf16DirectFixed<TW, TH, BR>::NBLK, 64, TW, TH, 2, 1, Bf16DirectFixed<TW, TH, BR>::MAXF, 1, BR, 1.0f, 32, BR,  \
         1, Bf16DirectFixed<TW, TH, BR>::YS, 1, 1, Bf16DirectFixed<TW, TH, BR>::LDS_BYTES, UNIT_US, FIXED_US, 0, 2, CALIB, BR == 1, 1},  \
            [](const KernelArgs& a, int grid, size_t lds, void* stream) -> int {                               \
                static bool attr_done = false;                                                                 \
                if (!Bf16DirectFixed<TW, TH, BR>::matches_host(a, true) || lds != (size_t)Bf16DirectFixed<TW, TH, BR>::LDS_BYTES) return 1; \
                return launch_kernel(conv_bf16_direct_kernel<TW, TH, BR, 64, 1, true>, attr_done, 512, a, grid, lds, stream); \
            }                                                                                                  \
    }

// the same for strides 2
#define CACNN_DIRECT_S2_VARIANT(NAME, UNIT_US, FIXED_US, CALIB, TW, TH)                                         \
    {                                                                                                          \
        {NAME, 1, 2, 2, 1, Bf16DirectFixed<TW, TH, 3, 64, 2>::NBLK, 64, TW, TH, 2, 1, Bf16DirectFixed<TW, TH, 3, 64, 2>::MAXF, 1, 3, 1.0f, 32, 3,  \
         1, Bf16DirectFixed<TW, TH, 3, 64, 2>::YS_HOST, 2, 2, Bf16DirectFixed<TW, TH, 3, 64, 2>::LDS_BYTES, UNIT_US, FIXED_US, 0, 2, CALIB},  \
            [](const KernelArgs& a, int grid, size_t lds, void* stream) -> int {                               \
                static bool attr_done = false;                                                                 \
                if (!Bf16DirectFixed<TW, TH, 3, 64, 2>::matches_host(a) || lds != (size_t)Bf16DirectFixed<TW, TH, 3, 64, 2>::LDS_BYTES) return 1; \
                return launch_kernel(conv_bf16_direct_kernel<TW, TH, 3, 64, 2>, attr_done, 512, a, grid, lds, stream); \
            }                                                                                                  \
    }

// the same with 32 images per tile (two rows of TW positions), for 3 x 3 (BR = 3) or 1 x 1 (BR = 1) filters
#define CACNN_DIRECT_B32_VARIANT(NAME, UNIT_US, FIXED_US, TW, BR)                                               \
    {                                                                                                          \
        {NAME, 1, 2, 2, 1, Bf16DirectFixed<TW, 2, BR, 32>::NBLK, 32, TW, 2, 2, 1, Bf16DirectFixed<TW, 2, BR, 32>::MAXF, 1, BR, 1.0f, 32, BR,  \
         1, Bf16DirectFixed<TW, 2, BR, 32>::YS, 1, 1, Bf16DirectFixed<TW, 2, BR, 32>::LDS_BYTES, UNIT_US, FIXED_US, 0, 2, 256, BR == 1},  \
            [](const KernelArgs& a, int grid, size_t lds, void* stream) -> int {                               \
                static bool attr_done = false;                                                                 \
                if (!Bf16DirectFixed<TW, 2, BR, 32>::matches_host(a) || lds != (size_t)Bf16DirectFixed<TW, 2, BR, 32>::LDS_BYTES) return 1; \
                return launch_kernel(conv_bf16_direct_kernel<TW, 2, BR, 32>, attr_done, 512, a, grid, lds, stream); \
            }                                                                                                  \
    }

// the same for C a multiple of 8 but not of 32
#define CACNN_DIRECT_B32_T8_VARIANT(NAME, UNIT_US, FIXED_US, TW, BR)                                            \
    {                                                                                                          \
        {NAME, 1, 2, 2, 1, Bf16DirectFixed<TW, 2, BR, 32>::NBLK, 32, TW, 2, 2, 1, Bf16DirectFixed<TW, 2, BR, 32>::MAXF, 1, BR, 1.0f, 32, BR,  \
         1, Bf16DirectFixed<TW, 2, BR, 32>::YS, 1, 1, Bf16DirectFixed<TW, 2, BR, 32>::LDS_BYTES, UNIT_US, FIXED_US, 0, 2, 256, BR == 1, 1},  \
            [](const KernelArgs& a, int grid, size_t lds, void* stream) -> int {                               \
                static bool attr_done = false;                                                                 \
                if (!Bf16DirectFixed<TW, 2, BR, 32>::matches_host(a, true) || lds != (size_t)Bf16DirectFixed<TW, 2, BR, 32>::LDS_BYTES) return 1; \
                return launch_kernel(conv_bf16_direct_kernel<TW, 2, BR, 32, 1, true>, attr_done, 512, a, grid, lds, stream); \
            }                                                                                                  \
    }

// the same for 1 x 1 filters
#define CACNN_DIRECT_1X1_VARIANT(NAME, UNIT_US, FIXED_US, TW, TH)                                               \
    {                                                                                                          \
        {NAME, 1, 2, 2, 1, Bf16DirectFixed<TW, TH, 1>::NBLK, 64, TW, TH, 2, 1, Bf16DirectFixed<TW, TH, 1>::MAXF, 1, 1, 1.0f, 32, 1,  \
         1, Bf16DirectFixed<TW, TH, 1>::YS, 1, 1, Bf16DirectFixed<TW, TH, 1>::LDS_BYTES, UNIT_US, FIXED_US, 0, 2, 256, 1}, \
            [](const KernelArgs& a, int grid, size_t lds, void* stream) -> int {                               \
                static bool attr_done = false;                                                                 \
                if (!Bf16DirectFixed<TW, TH, 1>::matches_host(a) || lds != (size_t)Bf16DirectFixed<TW, TH, 1>::LDS_BYTES) return 1; \
                return launch_kernel(conv_bf16_direct_kernel<TW, TH, 1>, attr_done, 512, a, grid, lds, stream); \
            }                                                                                                  \
    }

// bf16 staged through registers with a deep prefetch: 64 images, 64 output channels, 32-channel slices, Image units of BSI filter rows
#define CACNN_STAGED_VARIANT(NAME, UNIT_US, FIXED_US, CALIB, TW, TH, BSI)                                            \
    {                                                                                                          \
        {NAME, 1, 2, 2, 1, Bf16StagedFixed<TW, TH, BSI>::NBLK, 64, TW, TH, 2, 1, Bf16StagedFixed<TW, TH, BSI>::MAXF, 1, 3, 1.0f, 32, 3,  \
         BSI, Bf16StagedFixed<TW, TH, BSI>::YSI, 1, 1, Bf16StagedFixed<TW, TH, BSI>::LDS_BYTES, UNIT_US, FIXED_US, 0, 0, CALIB},  \
            [](const KernelArgs& a, int grid, size_t lds, void* stream) -> int {                               \
                static bool attr_done = false;                                                                 \
                if (!Bf16StagedFixed<TW, TH, BSI>::matches_host(a) || lds != (size_t)Bf16StagedFixed<TW, TH, BSI>::LDS_BYTES) return 1; \
                return launch_kernel(conv_bf16_staged_kernel<TW, TH, BSI>, attr_done, 512, a, grid, lds, stream); \
            }                                                                                                  \
    }

// fp32 with the Image loaded straight into LDS: 8 images x 4 x 4 positions, 64 output channels, 16-channel slices of three filter rows
#define CACNN_F32_DIRECT_VARIANT(NAME, UNIT_US, FIXED_US, TW, TH)                                               \
    {                                                                                                          \
        {NAME, 0, 2, 2, 1, F32DirectFixed<TW, TH>::NBLK, 8, TW, TH, 2, 1, F32DirectFixed<TW, TH>::MAXF, 1, -4, 1.0f, 16, 3,    \
         3, F32DirectFixed<TW, TH>::YS, 1, 1, F32DirectFixed<TW, TH>::LDS_BYTES, UNIT_US, FIXED_US, 0},         \
            [](const KernelArgs& a, int grid, size_t lds, void* stream) -> int {                               \
                static bool attr_done = false;                                                                 \
                if (!F32DirectFixed<TW, TH>::matches_host(a) || lds != (size_t)F32DirectFixed<TW, TH>::LDS_BYTES) return 1; \
                return launch_kernel(conv_f32_direct_kernel<TW, TH>, attr_done, 512, a, grid, lds, stream);     \
            }                                                                                                  \
    }

// the same with 16x16 MFMA blocks: 8 images x 2 x 7 positions
#define CACNN_F32_DIRECT16_VARIANT(NAME, UNIT_US, FIXED_US, TW, TH)                                             \
    {                                                                                                          \
        {NAME, 0, 2, 2, 1, F32Direct16<TW, TH>::NBLK, 8, TW, TH, 2, 1, F32Direct16<TW, TH>::MAXF, 1, -4, 1.0f, 16, 3,    \
         3, F32Direct16<TW, TH>::YS, 1, 1, F32Direct16<TW, TH>::LDS_BYTES, UNIT_US, FIXED_US, 0, 1, 0, 0, 2},               \
            [](const KernelArgs& a, int grid, size_t lds, void* stream) -> int {                               \
                static bool attr_done = false;                                                                 \
                if (!F32Direct16<TW, TH>::matches_host(a) || lds != (size_t)F32Direct16<TW, TH>::LDS_BYTES) return 1; \
                return launch_kernel(conv_f32_direct16_kernel<TW, TH>, attr_done, 512, a, grid, lds, stream);   \
            }                                                                                                  \
    }

// the same for 1 x 1 filters
#define CACNN_F32_DIRECT16_1X1_VARIANT(NAME, UNIT_US, FIXED_US, TW, TH)                                         \
    {                                                                                                          \
        {NAME, 0, 2, 2, 1, F32Direct16<TW, TH, 1>::NBLK, 8, TW, TH, 2, 1, F32Direct16<TW, TH, 1>::MAXF, 1, -4, 1.0f, 16, 1,    \
         1, F32Direct16<TW, TH, 1>::YS, 1, 1, F32Direct16<TW, TH, 1>::LDS_BYTES, UNIT_US, FIXED_US, 0, 1, 0, 1, 2},         \
            [](const KernelArgs& a, int grid, size_t lds, void* stream) -> int {                               \
                static bool attr_done = false;                                                                 \
                if (!F32Direct16<TW, TH, 1>::matches_host(a) || lds != (size_t)F32Direct16<TW, TH, 1>::LDS_BYTES) return 1; \
                return launch_kernel(conv_f32_direct16_kernel<TW, TH, 1>, attr_done, 512, a, grid, lds, stream); \
            }                                                                                                  \
    }

static const Variant g_variants[] = {
    // fp32
    CACNN_VARIANT(0, conv_f32_kernel, "f32 k32 b1w16h16 w1x4 m1n2", 1, 4, 1, 2, 1, 16, 16),
    CACNN_VARIANT(0, conv_f32_kernel, "f32 k64 b8w4h4 w2x2 m1n2", 2, 2, 1, 2, 8, 4, 4),
    CACNN_VARIANT(0, conv_f32_kernel, "f32 k64 b32w4h2 w2x2 m1n4", 2, 2, 1, 4, 32, 4, 2),
    CACNN_VARIANT(0, conv_f32_kernel, "f32 k64 b32w2h2 w2x2 m1n2", 2, 2, 1, 2, 32, 2, 2),
    CACNN_VARIANT(0, conv_f32_kernel, "f32 k64 b4w8h4 w2x2 m1n2", 2, 2, 1, 2, 4, 8, 4),
    // one position per tile: the staged Image range is b_r x b_s whatever the strides are (the fallback for strides so
    // large that a tile of several positions would span more than the LDS holds)
    // (priced at four times the model's figure: it is the last resort, not a competitor of the tiles above)
    CACNN_VARIANT_TUNED(0, conv_f32_kernel, "f32 k64 b32w1h1 w2x1 m1n1", 4.0f, 2, 1, 1, 1, 32, 1, 1),
    // bf16
    CACNN_VARIANT(1, conv_bf16_kernel, "bf16 k128 b32w2h2 w2x2 m2n2", 2, 2, 2, 2, 32, 2, 2),
    CACNN_VARIANT(1, conv_bf16_kernel, "bf16 k128 b32w7h1 w4x1 m1n7", 4, 1, 1, 7, 32, 7, 1),
    CACNN_VARIANT(1, conv_bf16_kernel, "bf16 k64 b8w4h4 w2x2 m1n2", 2, 2, 1, 2, 8, 4, 4),
    CACNN_VARIANT(1, conv_bf16_kernel, "bf16 k32 b1w16h16 w1x4 m1n2", 1, 4, 1, 2, 1, 16, 16),
    CACNN_VARIANT(1, conv_bf16_kernel, "bf16 k64 b64w2h1 w2x2 m1n2", 2, 2, 1, 2, 64, 2, 1),
    CACNN_VARIANT_TUNED(1, conv_bf16_kernel, "bf16 k64 b32w1h1 w2x1 m1n1", 4.0f, 2, 1, 1, 1, 32, 1, 1),
    // pipelined, fp32
    CACNN_PIPE_VARIANT(0, conv_f32_pipe_kernel, "f32 pipe k64 b8w4h4 w2x2 m1n2", 2, 2, 1, 2, 8, 4, 4, 6, 10, 1),
    CACNN_PIPE_VARIANT(0, conv_f32_pipe_kernel, "f32 pipe k64 b8w8h4 w2x2 m1n4", 2, 2, 1, 4, 8, 8, 4, 10, 10, 1),
    CACNN_PIPE_VARIANT(0, conv_f32_pipe_kernel, "f32 pipe k64 b32w4h2 w2x2 m1n4", 2, 2, 1, 4, 32, 4, 2, 12, 10, 1),
    CACNN_PIPE_VARIANT(0, conv_f32_pipe_kernel, "f32 pipe k64 b32w2h2 w2x2 m1n2", 2, 2, 1, 2, 32, 2, 2, 8, 10, 1),
    // pipelined, bf16 (MAXI counts 8x8 staging blocks, MAXF 16-byte Filter chunks)
    CACNN_PIPE_VARIANT(1, conv_bf16_pipe_kernel, "bf16 pipe k128 b32w2h2 w2x2 m2n2", 2, 2, 2, 2, 32, 2, 2, 1, 10, 1),
    CACNN_PIPE_VARIANT(1, conv_bf16_pipe_kernel, "bf16 pipe k128 b32w7h1 w4x1 m1n7", 4, 1, 1, 7, 32, 7, 1, 1, 10, 1),
    CACNN_PIPE_VARIANT(1, conv_bf16_pipe_kernel, "bf16 pipe k64 b64w2h1 w2x2 m1n2", 2, 2, 1, 2, 64, 2, 1, 1, 6, 2),
    CACNN_PIPE_VARIANT(1, conv_bf16_pipe_kernel, "bf16 pipe k128 b64w2h2 w2x2 m2n4", 2, 2, 2, 4, 64, 2, 2, 1, 10, 1),
    CACNN_PIPE_VARIANT(1, conv_bf16_pipe_kernel, "bf16 pipe k64 b16w4h2 w2x2 m1n2", 2, 2, 1, 2, 16, 4, 2, 1, 6, 2),
    CACNN_PIPE_VARIANT(1, conv_bf16_pipe_kernel, "bf16 pipe k64 b8w4h4 w2x2 m1n2", 2, 2, 1, 2, 8, 4, 4, 1, 6, 2),
    // pipelined bf16 with filter-row reuse (3 taps)
    CACNN_REUSE_VARIANT("bf16 pipe3 k128 b32w2h2 w2x2 m2n2", 2, 2, 2, 2, 32, 2, 2, 1, 10, 1, 3),
    CACNN_REUSE_VARIANT("bf16 pipe3 k128 b32w7h1 w4x1 m1n7", 4, 1, 1, 7, 32, 7, 1, 1, 10, 1, 3),
    CACNN_REUSE_VARIANT("bf16 pipe3 k64 b32w7h2 w2x2 m1n7", 2, 2, 1, 7, 32, 7, 2, 2, 6, 1, 3),
    CACNN_REUSE_VARIANT("bf16 pipe3 k128 b32w4h1 w4x1 m1n4", 4, 1, 1, 4, 32, 4, 1, 1, 10, 1, 3),
    // wave-specialised (producer waves + consumer waves), fp32
    CACNN_WS_VARIANT(0, "f32 ws k64 b8w4h4 w2x2 m1n2", 1.0f, 2, 2, 1, 2, 8, 4, 4, 6, 10, 0,
                     conv_f32_ws_kernel<2, 2, 1, 2, 8, 4, 4, 6, 10>),
    CACNN_WS_VARIANT(0, "f32 ws k64 b8w8h4 w2x2 m1n4", 1.0f, 2, 2, 1, 4, 8, 8, 4, 10, 10, 0,
                     conv_f32_ws_kernel<2, 2, 1, 4, 8, 8, 4, 10, 10>),
    CACNN_WS_VARIANT(0, "f32 ws k64 b32w4h2 w2x2 m1n4", 1.0f, 2, 2, 1, 4, 32, 4, 2, 12, 10, 0,
                     conv_f32_ws_kernel<2, 2, 1, 4, 32, 4, 2, 12, 10>),
    CACNN_WS_VARIANT(0, "f32 ws k64 b32w2h2 w2x2 m1n2", 1.0f, 2, 2, 1, 2, 32, 2, 2, 8, 10, 0,
                     conv_f32_ws_kernel<2, 2, 1, 2, 32, 2, 2, 8, 10>),
    // wave-specialised fp32 with 16-byte LDS fragments
    CACNN_WS_VARIANT(0, "f32 ws4 k64 b8w4h4 w2x2 m1n2", 1.0f, 2, 2, 1, 2, 8, 4, 4, 2, 10, -4,
                     conv_f32v4_ws_kernel<2, 2, 1, 2, 8, 4, 4, 2, 10>),
    CACNN_WS_VARIANT(0, "f32 ws4 k64 b8w8h4 w2x2 m1n4", 1.0f, 2, 2, 1, 4, 8, 8, 4, 3, 10, -4,
                     conv_f32v4_ws_kernel<2, 2, 1, 4, 8, 8, 4, 3, 10>),
    CACNN_WS_VARIANT(0, "f32 ws4 k64 b32w4h2 w2x2 m1n4", 1.0f, 2, 2, 1, 4, 32, 4, 2, 4, 10, -4,
                     conv_f32v4_ws_kernel<2, 2, 1, 4, 32, 4, 2, 4, 10>),
    CACNN_WS_VARIANT(0, "f32 ws4 k64 b32w2h2 w2x2 m1n2", 1.0f, 2, 2, 1, 2, 32, 2, 2, 3, 10, -4,
                     conv_f32v4_ws_kernel<2, 2, 1, 2, 32, 2, 2, 3, 10>),
    CACNN_WS_VARIANT(0, "f32 ws4 k64 b16w4h2 w2x2 m1n2", 1.0f, 2, 2, 1, 2, 16, 4, 2, 3, 10, -4,
                     conv_f32v4_ws_kernel<2, 2, 1, 2, 16, 4, 2, 3, 10>),
    // fixed-geometry kernels (3x3 and 1x1 taps; the first needs shapes its tiles divide exactly, the others mask their Out stores)
    CACNN_F32_DIRECT_VARIANT("f32 fxd k64 b8w4h4 w2x2 m1n2 c16r3s3", 4.4f, 3.0f, 4, 4),
    CACNN_F32_DIRECT16_VARIANT("f32 fxd16 k64 b8w2h7 w4x1 m1n7 c16r3s3", 4.1f, 2.6f, 2, 7),
    CACNN_F32_DIRECT16_1X1_VARIANT("f32 fxd16 k64 b8w2h7 w4x1 m1n7 c16r1s1", 0.50f, 2.6f, 2, 7),
    CACNN_DIRECT_VARIANT("bf16 fxd k64 b64w7h1 w2x2 m1n7 c32r3s1", 1.0f, 4.5f, 224, 7, 1),
    CACNN_DIRECT_VARIANT("bf16 fxd k64 b64w2h2 w2x2 m1n4 c32r3s1", 0.62f, 4.2f, 196, 2, 2),
    CACNN_DIRECT_S2_VARIANT("bf16 fxd k64 b64w2h2 w2x2 m1n4 c32r3s1 s2", 0.85f, 4.2f, 224, 2, 2),
    CACNN_DIRECT_T8_VARIANT("bf16 fxd k64 b64w7h1 w2x2 m1n7 c32r3s1 t8", 1.0f, 4.5f, 224, 7, 1, 3),
    CACNN_DIRECT_T8_VARIANT("bf16 fxd k64 b64w2h2 w2x2 m1n4 c32r3s1 t8", 0.62f, 4.2f, 196, 2, 2, 3),
    CACNN_DIRECT_T8_VARIANT("bf16 fxd k64 b64w7h1 w2x2 m1n7 c32r1s1 t8", 0.57f, 4.5f, 256, 7, 1, 1),
    CACNN_DIRECT_T8_VARIANT("bf16 fxd k64 b64w2h2 w2x2 m1n4 c32r1s1 t8", 0.35f, 4.2f, 256, 2, 2, 1),
    CACNN_DIRECT_1X1_VARIANT("bf16 fxd k64 b64w7h1 w2x2 m1n7 c32r1s1", 0.57f, 4.5f, 7, 1),
    CACNN_DIRECT_1X1_VARIANT("bf16 fxd k64 b64w2h2 w2x2 m1n4 c32r1s1", 0.35f, 4.2f, 2, 2),
    CACNN_DIRECT_1X1_C64_VARIANT("bf16 fxd k64 b64w2h2 w2x2 m1n4 c64r1s1", 0.61f, 4.2f, 2, 2),
    CACNN_DIRECT_1X1_C64_T8_VARIANT("bf16 fxd k64 b64w2h2 w2x2 m1n4 c64r1s1 t8", 0.61f, 4.2f, 2, 2),
    CACNN_DIRECT_B32_VARIANT("bf16 fxd k64 b32w7h2 w2x2 m1n7 c32r3s1", 1.1f, 4.5f, 7, 3),
    CACNN_DIRECT_B32_VARIANT("bf16 fxd k64 b32w7h2 w2x2 m1n7 c32r1s1", 0.64f, 4.5f, 7, 1),
    CACNN_DIRECT_B32_T8_VARIANT("bf16 fxd k64 b32w7h2 w2x2 m1n7 c32r3s1 t8", 1.1f, 4.5f, 7, 3),
    CACNN_DIRECT_B32_T8_VARIANT("bf16 fxd k64 b32w7h2 w2x2 m1n7 c32r1s1 t8", 0.64f, 4.5f, 7, 1),
    CACNN_STAGED_VARIANT("bf16 fxr k64 b64w7h1 w2x2 m1n7 c32r3s1", 1.1f, 4.5f, 224, 7, 1, 1),
    CACNN_STAGED_VARIANT("bf16 fxr k64 b64w2h2 w2x2 m1n4 c32r3s3", 2.0f, 4.2f, 196, 2, 2, 3),
    // fixed geometry for the stem-layer shape: 7x7 taps, strides 2, three channels
    {{"f32 fxsd k64 b32w2h2 w2x2 m1n2 c3r7s7 s2", 0, 2, 2, 1, F32StemDirect<2, 2>::NBLK, 32, 2, 2, 2, 1, 1, 1, 0, 1.0f, 3, 7, 7,
      F32StemDirect<2, 2>::YS, 2, 2, F32StemDirect<2, 2>::LDS_BYTES, 5.15f, 4.5f, 1, 2},
     [](const KernelArgs& a, int grid, size_t lds, void* stream) -> int {
         static bool attr_done = false;
         if (!F32StemDirect<2, 2>::matches_host(a) || lds != (size_t)F32StemDirect<2, 2>::LDS_BYTES) return 1;
         static bool attr_done_ragged = false;
         if (a.B % 32 == 0 && a.W % 2 == 0 && a.H % 2 == 0 && a.K % 64 == 0)
             return launch_kernel(conv_f32_stem_direct_kernel<2, 2, false>, attr_done, 512, a, grid, lds, stream);
         return launch_kernel(conv_f32_stem_direct_kernel<2, 2, true>, attr_done_ragged, 512, a, grid, lds, stream);
     }},
    // wave-specialised, bf16
    CACNN_WS_VARIANT(1, "bf16 ws k128 b32w2h2 w2x2 m2n2", 1.05f, 2, 2, 2, 2, 32, 2, 2, 1, 9, 0,
                     conv_bf16_ws_kernel<2, 2, 2, 2, 32, 2, 2, 1, 9, 0>),
    CACNN_WS_VARIANT(1, "bf16 ws3 k128 b32w2h2 w2x2 m2n2", 1.0f, 2, 2, 2, 2, 32, 2, 2, 1, 9, 3,
                     conv_bf16_ws_kernel<2, 2, 2, 2, 32, 2, 2, 1, 9, 3>),
    CACNN_WS_VARIANT(1, "bf16 ws3 k128 b32w7h1 w4x1 m1n7", 1.0f, 4, 1, 1, 7, 32, 7, 1, 1, 9, 3,
                     conv_bf16_ws_kernel<4, 1, 1, 7, 32, 7, 1, 1, 9, 3>),
    CACNN_WS_VARIANT(1, "bf16 ws3 k64 b32w7h2 w2x2 m1n7", 1.9f, 2, 2, 1, 7, 32, 7, 2, 2, 6, 3,
                     conv_bf16_ws_kernel<2, 2, 1, 7, 32, 7, 2, 2, 6, 3>),
    CACNN_WS_VARIANT(1, "bf16 ws3 k128 b32w4h1 w4x1 m1n4", 1.5f, 4, 1, 1, 4, 32, 4, 1, 1, 9, 3,
                     conv_bf16_ws_kernel<4, 1, 1, 4, 32, 4, 1, 1, 9, 3>),
    CACNN_WS_VARIANT(1, "bf16 ws k64 b8w4h4 w2x2 m1n2", 3.0f, 2, 2, 1, 2, 8, 4, 4, 1, 6, 0,
                     conv_bf16_ws_kernel<2, 2, 1, 2, 8, 4, 4, 1, 6, 0>),
};

int num_variants() { return (int)(sizeof(g_variants) / sizeof(g_variants[0])); }
const Variant& variant(int i) { return g_variants[i]; }

}  // namespace cacnn
