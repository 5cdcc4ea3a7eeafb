// Internal interface between the host planner/dispatcher (cacnn_host.cpp) and the gfx950 kernels
// (cacnn_kernels.hip).  Not part of the public ABI.
#ifndef CACNN_INTERNAL_H
#define CACNN_INTERNAL_H

#include <stddef.h>
#include <stdint.h>

namespace cacnn {

// Division of small unsigned numbers by a run-time constant with one multiply-high.
// Exact for n * d < 2^32 (the staged-tile indices it is used on are bounded by the LDS size).
struct FastDiv {
    uint32_t mul;  // floor(2^32 / d) + 1, or 0 when d == 1
    uint32_t d;
};

inline FastDiv make_fastdiv(uint32_t d) {
    FastDiv f;
    f.d = d;
    f.mul = (d <= 1) ? 0u : (uint32_t)((0x100000000ull / d) + 1ull);
    return f;
}

// Geometry of one compiled kernel variant: the workgroup's Out tile is KT output channels by a position tile of
// TB images x TW output columns x TH output rows, flattened as n = (h_l*TW + w_l)*TB + b_l and cut into MFMA
// column blocks of 32.  WM x WN wavefronts; each owns MBLK x NBLK MFMA tiles of 32x32.
struct VariantInfo {
    const char* name;
    int dtype;  // cacnn_dtype
    int WM, WN, MBLK, NBLK, TB, TW, TH;
    // 0: one workgroup per Out tile, staging and MFMA alternate (works for every shape and alignment).
    // 1: persistent workgroups walk a list of (tile, contraction slice) units; the next unit's Image and Filter
    //    words are fetched into registers while the current one is multiplied, LDS is double-buffered.
    //    Needs 16-byte-legal operands and a slice that fits MAXI/MAXF staging items per thread.
    // 2: as 1, with twice the waves: half of them only stage (two units ahead), the other half only multiply.
    int pipelined;
    int MAXI, MAXF;
    int occ;    // workgroups of this kernel one compute unit can hold at once, as far as registers go
    int reuse_r;  // > 0: filter-row reuse path compiled for exactly this many taps per contraction tile (sigma_w = 1);
                  // -4: fp32 kernel with the 16-byte-fragment LDS layout (c-slices in multiples of 4 channels)
    float tune;   // measured time of this variant relative to what the planner's cost model predicts (1 = as modelled)
    // fixed-geometry kernels: the only contraction tile (c-slice, b_r, b_s) the kernel was compiled for (0 = any)
    // and the staged Image rows sigma_h*(TH-1)+b_s it assumes
    int fx_ct = 0, fx_br = 0, fx_bs = 0, fx_ys = 0;
    int fx_sw = 1, fx_sh = 1;   // the strides it assumes
    int fx_lds = 0;             // the fixed-geometry kernels' own LDS layout, bytes (they all have one)
    // measured on MI355X with every CU busy: microseconds per unit (tile and contraction slice) of one workgroup, and the
    // fixed part of a launch (first loads, last Out tile, dispatch); the planner prices these kernels with them
    float fx_unit_us = 0.f, fx_fixed_us = 0.f;
    int fx_whole = 0;           // 1: with its own LDS layout, the kernel takes a tile's whole contraction as one unit (C == fx_ct, S == fx_bs)
    int fx_ragged = 0;          // 1: W, H and K need not be multiples of the tile (the kernel masks its Out stores); 2: nor B
    int fx_calib_cus = 0;       // > 0 (bf16): the busy compute units fx_unit_us was measured with.  The chip's bf16 MFMA rate is
                                // power-limited, so a unit takes longer the more compute units work at once
    int fx_any_stride = 0;      // 1 (1 x 1 filters): any strides; a tile stages exactly the TW x TH positions its outputs read
    int fx_tail8 = 0;           // 0: C = 0 mod fx_ct; 1: the instance for C a multiple of 8 but not of fx_ct (the last c-slice partly
                                // filled); 2 (fp32): any C that is a multiple of 4
    int KT() const { return WM * MBLK * 32; }
    int NT() const { return TB * TW * TH; }
    int threads() const { return WM * WN * (pipelined == 2 ? 128 : 64); }
    int staging_threads() const { return WM * WN * 64; }
    bool f32v4() const { return reuse_r == -4; }
    int cgran() const { return dtype == 0 ? (f32v4() ? 4 : 1) : 16; }  // contraction granularity of the c-slice
};

// Everything a kernel needs, passed by value.
struct KernelArgs {
    const void* image;
    const void* filter;
    float* out;
    int32_t B, C, K, W, H, R, S, sw, sh, IW, IH;
    int32_t bR, bS, CT;       // contraction tile: r-range, s-range, c-slice (CT multiple of cgran)
    int32_t XS, YS;           // staged Image extents: sw*(TW-1)+bR, sh*(TH-1)+bS
    int32_t xpitch, ypitch;   // LDS pitches of the staged Image tile (fp32: floats; bf16: 16-byte units)
    int32_t fpitch;           // LDS pitch of one Filter row (one k), in elements
    int32_t QE;               // fp32: per-r contraction length bS*CT rounded up to even
    int32_t img_lds_elems;    // fp32: floats before the Filter tile; bf16: 16-byte units before it
    int32_t zero_off;         // fp32: offset (floats) of a zeroed row of 64 floats inside the Image region
    int32_t tiles_k, tiles_b, tiles_w, tiles_h;
    int32_t vec_img, vec_flt; // 1 = 16-byte global loads are legal for this operand
    FastDiv d_CT, d_YS, d_bS, d_bR, d_C8, d_RS, d_XS, d_C4;
    // pipelined kernels only
    int32_t n_tiles;          // Out tiles in the whole problem (all kernels)
    int32_t n_xcd;            // XCDs the dispatcher deals workgroups to (8 on MI355X); 1 = no remapping
    int32_t b_group;          // consecutive b-tiles whose Image rows share 128-byte lines (divides tiles_b)
    int32_t xcd_q, xcd_rem;   // n_tiles = n_xcd * xcd_q + xcd_rem
    // the tile list is k_groups blocks of grp tiles; inside a block the kpg k-tiles of the group are the fastest index
    // (k_groups = 1: the whole list is one block with all tiles_k k-tiles fastest); d_tk divides by kpg
    int32_t k_groups, kpg, grp;
    int32_t pos_fastest;      // 1: inside a block the position tiles of a k-tile are the fastest index, the k-tile the slowest
    int32_t npos;             // position tiles per block, grp / kpg
    FastDiv d_npos;           // its reciprocal
    FastDiv d_nxcd, d_tk, d_bg, d_tw, d_th;   // reciprocals of n_xcd, tiles_k, b_group, tiles_w, tiles_h
    int32_t img_items, flt_items;   // 16-byte staging items per slice
    int32_t img_buf, flt_buf; // size of one LDS buffer of each operand (fp32: floats; bf16: 16-byte units)
    int32_t flt_off;          // where the Filter buffers start (same unit)
    int32_t flt_resident;     // 1 = the Filter tile is the same for every unit of a workgroup: staged once
};

typedef int (*LaunchFn)(const KernelArgs& a, int grid, size_t lds_bytes, void* stream);

struct Variant {
    VariantInfo info;
    LaunchFn launch;
};

// Pooling (cacnn_pool.hip): everything the kernel needs, by value.
struct PoolArgs {
    const void* image;
    float* out;
    int32_t B, C, W, H, R, S, sw, sh, IH;
    int32_t BV;               // groups of VEC adjacent images per (x, y, c): B / VEC
    int32_t TWC;              // output columns per chunk (the last chunk may overhang W)
    int32_t n_threads;        // chunks * H * TWC * C * BV
    int32_t n_wg, n_xcd, xcd_q, xcd_rem;   // workgroups, and the XCD remapping of their order
    FastDiv d_BV, d_C, d_TWC, d_H, d_nxcd;
};
// dtype: cacnn_dtype; mode: cacnn_pool_mode; vec: images per thread (1, or 4 for fp32 / 8 for bf16). 0 = launched.
int launch_pool(const PoolArgs& a, int dtype, int mode, int vec, void* stream);

// Measurement kernels (cacnn_probe.hip).  0 = launched.
int launch_mfma_probe(int dtype, const void* operands, float* sink, int iters, int grid, void* stream);
int launch_copy_probe(const void* src, void* dst, size_t bytes, int grid, void* stream);
int launch_lds_fill_probe(const void* src, uint32_t window, int iters, float* sink, int grid, void* stream);
int launch_mfma_and_fill_probe(int tile, const void* operands, const void* src, uint32_t window, int mfma_iters, int fill_iters,
                               int lds_reads, int barrier, float* sink, int grid, void* stream);

// Defined in cacnn_kernels.hip.
int num_variants();
const Variant& variant(int i);

}  // namespace cacnn
#endif
