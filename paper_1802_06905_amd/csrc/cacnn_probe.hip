// Measurement support for gfx950: what this machine sustains, to read the convolution's rates against.
//   mfma_rate_kernel  a register-only MFMA loop on every compute unit (one wavefront per SIMD, the same instruction
//                     mix as the convolution kernels' inner step: 21 MFMAs on 7 accumulators, 3 + 9 operand fragments)
//   copy_kernel       a streaming copy through HBM
//   lds_fill_kernel   every compute unit filling its LDS from a window of global memory with the loads the convolution's
//                     staging waves use: with a window that fits an L2 this is the rate at which the L2s feed the LDS
// The published peaks assume the peak clock; under an all-CU matrix load the clock is power-managed and depends on
// how much the operand bits toggle, so the sustained MFMA rate is a property of the box and of the data.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "cacnn_internal.h"

namespace cacnn {

typedef float pr_f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 pr_bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int pr_u32x4 __attribute__((ext_vector_type(4)));

// operands: 4096 32-bit words.  DT 0: fp32 32x32x2 MFMAs, DT 1: bf16 32x32x16 MFMAs.  One launch issues
// gridDim.x * 4 * iters * 42 MFMAs.  The accumulators go to sink so that nothing is optimised away.
template <int DT>
__global__ void __launch_bounds__(256) mfma_rate_kernel(const uint32_t* operands, float* sink, int iters) {
    const int tid = threadIdx.x, lane = tid & 63;
    pr_f32x16 acc[7];
#pragma unroll
    for (int n = 0; n < 7; ++n)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[n][v] = 0.f;
    if constexpr (DT == 0) {
        float A[3], X[9];
#pragma unroll
        for (int r = 0; r < 3; ++r) A[r] = __uint_as_float(operands[(lane + 64 * r) & 4095]);
#pragma unroll
        for (int x = 0; x < 9; ++x) X[x] = __uint_as_float(operands[(lane + 64 * (3 + x)) & 4095]);
        for (int it = 0; it < 2 * iters; ++it) {
#pragma unroll
            for (int r = 0; r < 3; ++r)
#pragma unroll
                for (int w = 0; w < 7; ++w) acc[w] = __builtin_amdgcn_mfma_f32_32x32x2f32(A[r], X[w + r], acc[w], 0, 0, 0);
        }
    } else {
        pr_bf16x8 A[3], X[9];
        const pr_u32x4* const op = (const pr_u32x4*)operands;      // 1024 16-byte fragments
#pragma unroll
        for (int r = 0; r < 3; ++r) A[r] = __builtin_bit_cast(pr_bf16x8, op[(lane + 64 * r) & 1023]);
#pragma unroll
        for (int x = 0; x < 9; ++x) X[x] = __builtin_bit_cast(pr_bf16x8, op[(lane + 64 * (3 + x)) & 1023]);
        for (int it = 0; it < 2 * iters; ++it) {
#pragma unroll
            for (int r = 0; r < 3; ++r)
#pragma unroll
                for (int w = 0; w < 7; ++w)
                    acc[w] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[r], X[w + r], acc[w], 0, 0, 0);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int n = 0; n < 7; ++n)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[n][v];
    sink[blockIdx.x * 256 + tid] = s;
}

// dst[i] = src[i] for n 16-byte words; every wave reads and writes whole 1 KiB runs, streaming hints on both sides
__global__ void __launch_bounds__(256) copy_kernel(const pr_u32x4* src, pr_u32x4* dst, size_t n) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride)
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// Each of the four waves of a workgroup moves, `iters` times, twelve 1 KiB chunks (64 lanes x 16 bytes, LDS destination)
// from the window [src, src + window) into its own 12 KiB of LDS, with the twelve loads of the previous round still in
// flight.  A window below 64 MiB is shared: chunk numbers advance so that the workgroups of an XCD read different chunks at
// any one time and every chunk is read by many of them (what an L2 serves).  A larger window is divided among the
// workgroups, each streaming round and round through its own part, so that nothing a workgroup reads has been read by
// another one (what comes from behind the L2s).  window is a power of two, at least 64 KiB.
__global__ void __launch_bounds__(256) lds_fill_kernel(const char* src, uint32_t window, int iters, float* sink) {
    __shared__ __align__(16) char lds[4 * 12 * 1024];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(src), 0, (int)window, 0x00020000);
    const uint32_t chunks = window >> 10;
    const bool shared = window < (64u << 20);
    const uint32_t part = shared ? chunks : chunks / gridDim.x;       // chunks this workgroup walks through
    const uint32_t base = shared ? 0u : blockIdx.x * part;
    uint32_t chunk = shared ? (blockIdx.x * 53u + wave * 12u) & (chunks - 1) : (wave * 12u) % part;
    __attribute__((address_space(3))) char* const mine = (__attribute__((address_space(3))) char*)lds + wave * 12 * 1024;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 12; ++i) {
            uint32_t c = chunk + i;                 // chunk < part and part >= 64: one conditional step wraps it
            c = c >= part ? c - part : c;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (__attribute__((address_space(3))) void*)(mine + i * 1024), 16,
                                                     (uint32_t)lane * 16u, (base + c) << 10, 0, 0);
        }
        chunk = (chunk + (shared ? 48u * 5u + 12u : 48u)) % part;
        __builtin_amdgcn_s_waitcnt((12 & 15) | ((12 >> 4) << 14) | (7 << 4) | (15 << 8));   // all but the last twelve loads are in
    }
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    sink[blockIdx.x * 256 + threadIdx.x] = (float)(unsigned char)lds[threadIdx.x * 16];
}

// Both at once, in the proportions of a bf16 convolution kernel's unit: waves 0-3 of a workgroup of eight run the bf16
// MFMA loop of that kernel's multiplying waves (per step 3 taps x TW x THW MFMAs on TW x THW accumulators, two steps per
// iteration), waves 4-7 the LDS fill from a shared window (12 KiB per iteration and wave).  Either count may be zero.
// What the two cost each other when nothing synchronises them.
// <TW, THW> = <7, 1>: the tile of 64 images x 7 x 1 positions (42 MFMAs per iteration and wave); <2, 2>: 64 images x 2 x 2
// positions (24 MFMAs per iteration and wave).
// lds_reads = 0: the MFMA loop is register-only.  1: before every step a wave reads its 3 + THW x (TW + 2) operand
// fragments from the LDS the other waves are filling, with the instructions, the addresses and the bank pattern of the
// convolution kernel's multiplying waves (16-byte reads of a Filter row, pairs of transposing 8-byte reads of Image rows,
// laid out as one buffer of that kernel: (TW + 2) x THW x 32 Image rows of 128 bytes, then 64 Filter rows of 13 x 16
// bytes); still no dependence between the two kinds of waves.
// barrier = 1 (the host passes it only with mfma_iters == fill_iters, so that all eight waves execute the same number
// of barriers): once per iteration all eight waves meet at a workgroup barrier, as the kernel's waves do once per unit.
typedef short pr_s16x4 __attribute__((ext_vector_type(4)));
#define CACNN_PROBE_LDS(T) __attribute__((address_space(3))) T
template <int TW, int THW>
__global__ void __launch_bounds__(512) mfma_and_fill_kernel(const uint32_t* operands, const char* src, uint32_t window,
                                                            int mfma_iters, int fill_iters, int lds_reads, int barrier,
                                                            float* sink) {
    constexpr int NBLK = TW * THW, XS = TW + 2, NX = THW * XS, IMG_BYTES = XS * THW * 32 * 128;
    static_assert(IMG_BYTES + 64 * 13 * 16 <= 50 * 1024 && 3 + NX <= 1024 / 64, "probe geometry: LDS size, operand fragments");
    __shared__ __align__(16) char lds[50 * 1024];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    float result = 0.f;
    if (lds_reads) {
        // what is read before the first fill arrives (or all the time, without a fill), and the end of the Filter rows,
        // which no fill reaches: the operand words, over and over
        for (int i = threadIdx.x; i < (int)sizeof(lds) / 16; i += 512) ((pr_u32x4*)lds)[i] = ((const pr_u32x4*)operands)[i & 1023];
        __syncthreads();
    }
    if (wave < 4) {
        pr_f32x16 acc[NBLK];
#pragma unroll
        for (int n = 0; n < NBLK; ++n)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[n][v] = 0.f;
        pr_bf16x8 A[3], X[NX];
        const pr_u32x4* const op = (const pr_u32x4*)operands;
#pragma unroll
        for (int r = 0; r < 3; ++r) A[r] = __builtin_bit_cast(pr_bf16x8, op[(lane + 64 * r) & 1023]);
#pragma unroll
        for (int x = 0; x < NX; ++x) X[x] = __builtin_bit_cast(pr_bf16x8, op[(lane + 64 * (3 + x)) & 1023]);
        auto mfma_step = [&]() {
#pragma unroll
            for (int r = 0; r < 3; ++r)
#pragma unroll
                for (int h = 0; h < THW; ++h)
#pragma unroll
                    for (int w = 0; w < TW; ++w)
                        acc[h * TW + w] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[r], X[h * XS + w + r], acc[h * TW + w], 0, 0, 0);
        };
        if (!lds_reads) {
            for (int it = 0; it < 2 * mfma_iters; ++it) {
                mfma_step();
                if (barrier && (it & 1)) __builtin_amdgcn_s_barrier();
            }
        } else {
            // the multiplying waves' lane offsets (wave = wm + 2 wn; rows of 128 bytes, halves of rows with bit 1 of the
            // channel set exchanged; Filter rows of 13 x 16 bytes behind the Image rows)
            const int wm = wave & 1, wn = wave >> 1;
            const int j = lane & 31, g = lane >> 5, i16 = lane & 15, jhalf = (lane >> 4) & 1;
            const int q = wn * 4 + 2 * jhalf + ((i16 & 3) >> 1);
            const uint32_t al = (uint32_t)(IMG_BYTES + ((wm * 32 + j) * 13 + g) * 16);
            const uint32_t xl = (uint32_t)((8 * g + (i16 >> 2)) * 128 + ((q ^ (((i16 >> 3) & 1) << 2)) * 16) + (i16 & 1) * 8);
            CACNN_PROBE_LDS(char)* const l3 = (CACNN_PROBE_LDS(char)*)lds;
            for (int it = 0; it < 2 * mfma_iters; ++it) {
                const int cs = it & 1;
                pr_bf16x8 An[3], Xn[NX];
#pragma unroll
                for (int r = 0; r < 3; ++r) An[r] = *(const CACNN_PROBE_LDS(pr_bf16x8)*)(l3 + al + (r * 4 + 2 * cs) * 16);
#pragma unroll
                for (int h = 0; h < THW; ++h)
#pragma unroll
                    for (int x = 0; x < XS; ++x) {
                        CACNN_PROBE_LDS(char)* const p = l3 + xl + ((x * THW + h) * 32 + 16 * cs) * 128;
                        const pr_s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((CACNN_PROBE_LDS(pr_s16x4)*)p);
                        const pr_s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((CACNN_PROBE_LDS(pr_s16x4)*)(p + 4 * 128));
                        Xn[h * XS + x] = __builtin_bit_cast(pr_bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                    }
                // this step's MFMAs run on the fragments read during the last step, under these reads
                mfma_step();
#pragma unroll
                for (int r = 0; r < 3; ++r) A[r] = An[r];
#pragma unroll
                for (int x = 0; x < NX; ++x) X[x] = Xn[x];
                asm volatile("" ::: "memory");      // the LDS changes under the reads: every step reads again
                // as in the kernel: once per unit, when this step's reads have landed, meet the other waves
                if (barrier && (it & 1)) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            }
        }
#pragma unroll
        for (int n = 0; n < NBLK; ++n)
#pragma unroll
            for (int v = 0; v < 16; ++v) result += acc[n][v];
    } else {
        const int fw = wave - 4;
        const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(src), 0, (int)window, 0x00020000);
        const uint32_t chunks = window >> 10;
        uint32_t chunk = (blockIdx.x * 53u + fw * 12u) & (chunks - 1);
        __attribute__((address_space(3))) char* const mine = (__attribute__((address_space(3))) char*)lds + fw * 12 * 1024;
        for (int it = 0; it < fill_iters; ++it) {
#pragma unroll
            for (int i = 0; i < 12; ++i)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (__attribute__((address_space(3))) void*)(mine + i * 1024), 16,
                                                         (uint32_t)lane * 16u, ((chunk + i) & (chunks - 1)) << 10, 0, 0);
            chunk = (chunk + 48u * 5u + 12u) & (chunks - 1);
            __builtin_amdgcn_s_waitcnt((12 & 15) | ((12 >> 4) << 14) | (7 << 4) | (15 << 8));
            // (the loads of the iteration before have landed: the kernel's staging waves announce a unit here)
            if (barrier) __builtin_amdgcn_s_barrier();
        }
        __builtin_amdgcn_s_waitcnt(0);
    }
    if (wave < 4) sink[blockIdx.x * 256 + threadIdx.x] = result;
}

template <int TW, int THW>
static int launch_mfma_and_fill(const void* operands, const void* src, uint32_t window, int mfma_iters, int fill_iters, int lds_reads,
                                int barrier, float* sink, int grid, void* stream) {
    // 46 KiB of unused dynamic LDS on top of the kernel's own 50 KiB: no second workgroup fits the compute unit, so a
    // grid below the CU count leaves exactly that many compute units idle
    static bool attr_done = false;
    if (!attr_done) {
        if (hipFuncSetAttribute((const void*)mfma_and_fill_kernel<TW, THW>, hipFuncAttributeMaxDynamicSharedMemorySize, 46 * 1024) !=
            hipSuccess) {
            (void)hipGetLastError();
            return 1;
        }
        attr_done = true;
    }
    hipLaunchKernelGGL((mfma_and_fill_kernel<TW, THW>), dim3(grid), dim3(512), 46 * 1024, (hipStream_t)stream,
                       (const uint32_t*)operands, (const char*)src, window, mfma_iters, fill_iters, lds_reads, barrier, sink);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

// tile: 0 = 64 images x 7 x 1 positions, 1 = 64 images x 2 x 2 positions
int launch_mfma_and_fill_probe(int tile, const void* operands, const void* src, uint32_t window, int mfma_iters, int fill_iters,
                               int lds_reads, int barrier, float* sink, int grid, void* stream) {
    if (barrier && mfma_iters != fill_iters) return 1;      // the waves would not meet
    return tile == 0 ? launch_mfma_and_fill<7, 1>(operands, src, window, mfma_iters, fill_iters, lds_reads, barrier, sink, grid, stream)
                     : launch_mfma_and_fill<2, 2>(operands, src, window, mfma_iters, fill_iters, lds_reads, barrier, sink, grid, stream);
}

int launch_lds_fill_probe(const void* src, uint32_t window, int iters, float* sink, int grid, void* stream) {
    hipLaunchKernelGGL(lds_fill_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const char*)src, window, iters, sink);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int launch_mfma_probe(int dtype, const void* operands, float* sink, int iters, int grid, void* stream) {
    if (dtype == 0)
        hipLaunchKernelGGL(mfma_rate_kernel<0>, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const uint32_t*)operands,
                           sink, iters);
    else
        hipLaunchKernelGGL(mfma_rate_kernel<1>, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const uint32_t*)operands,
                           sink, iters);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int launch_copy_probe(const void* src, void* dst, size_t bytes, int grid, void* stream) {
    hipLaunchKernelGGL(copy_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const pr_u32x4*)src, (pr_u32x4*)dst,
                       bytes / 16);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

}  // namespace cacnn
