/*
 * cacnn -- communication-avoiding convolution for AMD MI355X (gfx950), C ABI.
 *
 * The library computes the seven-nested-loop convolution analysed in "Communication-Optimal Convolutional
 * Neural Nets" (Demmel, Dinh; arXiv 1802.06905), evaluates the paper's lower bound on words moved, and plans
 * the tiling it launches.  HBM plays the paper's slow memory; one compute unit's LDS (plus its register file)
 * plays the cache of M words.
 *
 * Conventions shared by every entry point
 *   - Problem parameters follow the paper's problem statement (Section 2): B images, C input channels,
 *     K output channels, W x H OUTPUT extents, R x S filter extents (R pairs with w, S with h), strides
 *     sigma_w, sigma_h.  F = B*C*K*W*H*R*S multiply-adds.
 *   - Arrays are dense, row-major in the paper's index order, last index fastest:
 *         Image  [IW][IH][C][B]   IW = sigma_w*(W-1)+R,  IH = sigma_h*(H-1)+S   (the touched extent; no padding)
 *         Filter [K][R][S][C]
 *         Out    [K][H][W][B]     always fp32
 *     Note the transposition the paper itself has: Image's first axis pairs with (r, w), its second with
 *     (s, h), while Out is indexed (k, h, w, b).
 *   - Every function returns a cacnn_status (0 = success).  Nothing throws, aborts or prints.
 *   - "words" are elements, as in the paper (it has a single word size).
 */
#ifndef CACNN_H
#define CACNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CACNN_OK = 0,
    CACNN_ERR_NULL = 1,         /* a required pointer is NULL */
    CACNN_ERR_INVALID_ARG = 2,  /* a dimension or stride < 1, M <= 1, a size that overflows the kernel's indexing */
    CACNN_ERR_UNSUPPORTED = 3,  /* unknown dtype, unknown variant, plan that does not fit the machine */
    CACNN_ERR_LAUNCH = 4,       /* the HIP runtime refused the launch */
    CACNN_ERR_NO_DEVICE = 5     /* no usable GPU */
} cacnn_status;

/* Section 2 of the paper: the nine integers that define one convolution.  W and H are OUTPUT extents. */
typedef struct {
    int64_t B, C, K, W, H, R, S, sigma_w, sigma_h;
} cacnn_problem;

typedef enum {
    CACNN_F32 = 0,         /* fp32 Image and Filter, fp32 multiply-accumulate (fp32 MFMA, no reduced-precision mode) */
    CACNN_BF16_F32ACC = 1  /* bf16 Image and Filter (raw 16-bit patterns), fp32 accumulate (bf16 MFMA) */
} cacnn_dtype;

/* Theorem 1 (Section 4): the five terms, their maximum and which term it is (0-based, first of equals). */
typedef struct {
    double term[5];  /* BKWH, sw*sh*BCWH, CKRS, BCKWHRS/M, BCKWH*sqrt(RS*sw*sh/M) */
    double bound;
    int32_t argmax;
} cacnn_bound;

/* The fast memory a tile has to fit.  Passing NULL where one is accepted means the MI355X defaults
 * (160 KiB LDS per compute unit, 512 KiB vector registers per compute unit, 256 compute units). */
typedef struct {
    int64_t lds_bytes;
    int64_t vgpr_bytes_per_cu;
    int64_t num_cu;
} cacnn_machine;

/* Result of planning.  The first block is the paper's own linear program (Section 5, the program over the
 * logs of the nine tile sizes) solved at M = lds_bytes / input element size: it is prior art for an abstract
 * machine and is reported for comparison.  The second block is the tiling the GPU kernel is launched with;
 * it is re-derived for LDS capacity, the accumulator registers and MFMA fragment shapes. */
typedef struct {
    /* --- paper LP at M = LDS words; order b,c,k,w,h,r',r'',s',s'' (r = sigma_w*r' + r'', s likewise) --- */
    double lp_tile[9];
    double lp_volume;        /* G*: product of lp_tile */
    double lp_cost_words;    /* F*M/G*  (Section 5.2) */
    double bound_words;      /* Theorem 1 at the same M */
    int32_t paper_case;      /* Appendix A leaf for strides 1, its number without the dots: 11 .. 19, 110 = Cases 1.1 .. 1.9,
                                1.10; 21, 221, 2221, 2222 = Cases 2.1 .. 2.2.2.2; 0 = strides are not both 1 */
    /* --- tiling launched on the GPU --- */
    int32_t variant;         /* index into the compiled kernel table, see cacnn_variant_name */
    int32_t b_b, b_c, b_k, b_w, b_h;       /* tile of (b,c,k,w,h) held by one workgroup per contraction step */
    int32_t b_r1, b_r2, b_s1, b_s2;        /* lifted filter tile: the kernel stages b_r = contiguous r range;
                                              b_r2 = min(sigma_w, b_r), b_r1 = ceil(b_r / sigma_w) */
    int32_t b_r, b_s;
    int32_t grid[3];
    int32_t block;           /* threads per workgroup */
    int64_t lds_bytes_used;
    double tile_volume;      /* b_b*b_c*b_k*b_w*b_h*b_r*b_s */
    double predicted_words;  /* words this schedule moves between HBM/L2 and the compute units:
                                staged Image halo tiles + staged Filter tiles + Out written once.  Every workgroup
                                stages what its tile needs (nothing is shared between workgroups), the staged Image
                                tile is the contiguous range sigma*(b-1)+b_r by sigma*(b-1)+b_s clipped to the array
                                (so it includes untouched rows when a stride exceeds the tile's filter extent, and a
                                full b_r, b_s range where the last contraction tile is ragged) */
    int32_t xcd_split_k;     /* Section 7 with the eight XCDs (each has its own L2) as the processors: the XCDs are
                                divided into this many groups of output channels (a_K; 1, 2, 4 or 8, a divisor of the
                                k-tile count) and 8 / a_K ranges of positions.  Chosen together with xcd_walk by the
                                per-XCD cache model of cacnn_two_level_plan (the layout whose modelled fetches from
                                behind the L2s are fewest).  cacnn_conv_forward_with_plan: 0 = choose. */
    int32_t xcd_walk;        /* order of an XCD's run of tiles: 0 = the k-tiles of a position tile are neighbours (the
                                Image tile is fetched once, the Filter rows of the k-group stream past once per round of
                                workgroups), 1 = the position tiles of a k-tile are neighbours (the other way round).
                                Chosen with xcd_split_k by cacnn_two_level_plan's model; with_plan: used as given. */
} cacnn_plan;

/*
 * Theorem 1 (Section 4; also Section 1): lower bound on words moved between a slow memory and a cache of
 * M_words words, for any execution order of the loop nest.  Host only; needs no GPU.
 *   problem  in   host pointer
 *   M_words  in   cache size in words, must be > 0
 *   out      out  host pointer, caller-owned
 * The constant hidden in the paper's Omega is taken as 1 and nothing is floored.  If a stride exceeds its
 * filter extent (outside the paper's assumption sigma <= R) it is clamped to the extent in terms 2 and 5,
 * since only touched Image elements count.
 * Errors: CACNN_ERR_NULL; CACNN_ERR_INVALID_ARG for any parameter < 1 or M_words <= 0 (out untouched).
 */
int cacnn_lower_bound(const cacnn_problem* problem, double M_words, cacnn_bound* out);

/*
 * Section 5 (optimal tiling as a linear program) and Appendix A (case analysis), then the re-derivation for
 * gfx950: chooses the kernel variant, the workgroup tile and the contraction tile that minimise a cost model
 * of staged words and machine fill, subject to LDS bytes and accumulator registers.  Host only; needs no GPU.
 *   problem  in   host pointer
 *   dtype    in   cacnn_dtype
 *   machine  in   host pointer or NULL for MI355X defaults
 *   out      out  host pointer, caller-owned
 * Several tilings reach the same optimal volume (Appendix A says so); only lp_volume / lp_cost_words are
 * unique, lp_tile is one optimiser.
 * Errors: CACNN_ERR_NULL, CACNN_ERR_INVALID_ARG (bad dimensions; machine->lds_bytes too small for any tile),
 * CACNN_ERR_UNSUPPORTED (dtype).
 */
int cacnn_tile_plan(const cacnn_problem* problem, int dtype, const cacnn_machine* machine, cacnn_plan* out);

/*
 * Eq. (1) of the paper (Section 2): Out(k,h,w,b) = sum over c,r,s of
 *     Image(r + sigma_w*w, s + sigma_h*h, c, b) * Filter(k,r,s,c),
 * executed as the blocked schedule of Section 5 on the GPU: each workgroup owns one Out tile, walks the
 * contraction (c, r, s) in tiles, stages the Image halo tile and the Filter tile in LDS and multiplies on MFMA.
 *   problem  in   host pointer
 *   dtype    in   cacnn_dtype
 *   image    in   DEVICE pointer, IW*IH*C*B elements (fp32, or bf16 bit patterns), read-only
 *   filter   in   DEVICE pointer, K*R*S*C elements, same element type as image, read-only
 *   out      out  DEVICE pointer, K*H*W*B fp32; OVERWRITTEN with the full sum (the paper's += from zero);
 *                 must not alias the inputs
 *   hip_stream    hipStream_t cast to void*; NULL is the default stream
 * The call enqueues work on the stream and returns; it never synchronises, allocates no device memory and
 * keeps no reference to the buffers.  The caller owns all three buffers.  Pointers must be aligned to their
 * element size; 16-byte alignment enables the vector paths.
 * Parameters outside the paper's assumptions (sigma > R, R > sigma_w*W) are computed correctly.
 * Errors: CACNN_ERR_NULL, CACNN_ERR_INVALID_ARG (dimension < 1, element counts beyond 2^31-1 per array, or so many
 * tiles along one dimension that tiles * tiles-per-dimension reaches 2^32),
 * CACNN_ERR_UNSUPPORTED (dtype), CACNN_ERR_NO_DEVICE, CACNN_ERR_LAUNCH.  On error nothing is enqueued.
 */
int cacnn_conv_forward(const cacnn_problem* problem, int dtype, const void* image, const void* filter,
                       void* out, void* hip_stream);

/*
 * Same computation as cacnn_conv_forward, launched with a caller-supplied plan instead of the planner's
 * choice (Section 5: any admissible tiling computes the same sums; Appendix A: several are optimal).
 * Only plan->variant, b_c, b_r, b_s are read; the workgroup tile is a property of the variant.  b_c is rounded
 * up to the variant's contraction granularity.  Used by tests (every variant must agree with the oracle on
 * every shape) and for tuning.
 * Extra errors: CACNN_ERR_UNSUPPORTED if the variant does not exist, is for the other dtype, or the tile does
 * not fit in LDS.
 */
int cacnn_conv_forward_with_plan(const cacnn_problem* problem, int dtype, const cacnn_plan* plan,
                                 const void* image, const void* filter, void* out, void* hip_stream);

/*
 * The plan cacnn_tile_plan would make if `variant_index` were the only compiled kernel: that variant with the
 * contraction tile the planner's cost model likes best for it, and the model's estimate of the launch time in
 * microseconds (model_us, may be NULL) with its terms in compute-unit cycles (model_terms, 5 doubles, may be NULL: Out
 * tiles per compute unit, MFMA time of a tile, staging time of a tile, contraction slices per tile, Out drain).  What
 * cacnn_tune times per variant; exposed so that the cost model can be compared with measurements and fitted to them
 * (bench.py --planner-sweep, --planner-compare).  Host only.
 * Errors: NULL -> CACNN_ERR_NULL; bad dims -> CACNN_ERR_INVALID_ARG; a variant of the other dtype, out of range, or one
 * that does not accept the problem -> CACNN_ERR_UNSUPPORTED.
 */
int cacnn_plan_variant(const cacnn_problem* problem, int dtype, int variant_index, cacnn_plan* out, double* model_us,
                       double* model_terms);

/*
 * Measured plan selection for problems the cost model was not calibrated on: runs every kernel variant that accepts
 * the problem (each with the contraction tile the model prefers for it) a few times on the caller's buffers, keeps
 * the fastest, and remembers it for later cacnn_conv_forward calls with the same problem, dtype and operand alignment.
 * Unlike the other entry points it SYNCHRONISES with hip_stream (it reads event timings) and creates and destroys two
 * HIP events; it allocates no device memory.  `out` is overwritten by every candidate and ends up holding a valid
 * result.  Arguments as for cacnn_conv_forward; out_plan (host, may be NULL) receives the chosen plan.
 * Errors: as cacnn_conv_forward; CACNN_ERR_UNSUPPORTED if no variant accepts the problem.
 */
int cacnn_tune(const cacnn_problem* problem, int dtype, const void* image, const void* filter, void* out,
               void* hip_stream, cacnn_plan* out_plan);

/*
 * Section 7 ("Parallel Algorithm"): p processors share one memory, each gets one block B/a_B x K/a_K x W/a_W x H/a_H of
 * the output and runs the sequential algorithm on it.  Total traffic is bounded below by
 *     max(BKWH, a_K*sw*sh*BCWH, a_B*a_W*a_H*CKRS, BCKWHRS/M, BCKWH*sqrt(RS*sw*sh/M)):
 * the Image term is replicated over the a_K groups of output channels, the Filter term over the a_B*a_W*a_H groups
 * of positions.  Host only.
 * cacnn_parallel_bound: the five terms for a given division (strides clamped as in cacnn_lower_bound).
 * cacnn_work_division: the division to use for p processors.  Readings the paper leaves open: an a may be anything
 * from 1 to the size of its dimension; the work is divided over as many processors as the dimensions allow (the
 * largest product a_B*a_K*a_W*a_H <= p); among those the maximum above is minimised, ties go to the least replicated
 * traffic a_K*term2 + a_B*a_W*a_H*term3, then to the lexicographically smallest (a_B, a_K, a_W, a_H).
 * Errors: CACNN_ERR_NULL; CACNN_ERR_INVALID_ARG for any parameter < 1, M_words <= 0, an a above its dimension,
 * p > 4096 (outputs untouched).
 */
typedef struct {
    int32_t a_b, a_k, a_w, a_h;
} cacnn_division;
int cacnn_parallel_bound(const cacnn_problem* problem, double M_words, const cacnn_division* a, cacnn_bound* out);

int cacnn_work_division(const cacnn_problem* problem, double M_words, int32_t p, cacnn_division* out_a,
                        cacnn_bound* out_bound);

/*
 * Pooling (Section 6 of the paper, "Application to Pooling"): the convolution's loop nest without the Filter,
 *     Out(k,h,w,b) (+)= Image(r + sigma_w*w, s + sigma_h*h, c, b),
 * where (+) adds the element divided by R*S (average) or keeps the maximum.  The printed nest runs over k and c
 * independently although no array carries both; it is executed as per-channel pooling, k = c, so problem->K must equal
 * problem->C.  Arrays and layouts as for cacnn_conv_forward (Image [IW][IH][C][B] fp32 or bf16, Out [K][H][W][B] fp32).
 */
typedef enum {
    CACNN_POOL_AVG = 0,  /* Out = (1/(R*S)) * sum over the window, summed in fp32 in the order r, then s */
    CACNN_POOL_MAX = 1   /* Out = maximum over the window (exact; a NaN in the window is ignored unless all are NaN) */
} cacnn_pool_mode;

/* Section 6: the three terms BKWH, sw*sh*BCWH, BCKWHRS/M, their maximum and which one it is (first of equals). */
typedef struct {
    double term[3];
    double bound;
    int32_t argmax;
} cacnn_pool_bound;

/*
 * Section 6: lower bound on words moved by the pooling nest as printed (all seven loops; for the per-channel reading
 * the multiply-free work is F/K, and the array-size terms are what binds).  Host only.  Strides above the window
 * extent are clamped in the Image term as in cacnn_lower_bound.
 * Errors: CACNN_ERR_NULL; CACNN_ERR_INVALID_ARG for any parameter < 1 or M_words <= 0 (out untouched).
 */
int cacnn_pool_lower_bound(const cacnn_problem* problem, double M_words, cacnn_pool_bound* out);

/*
 * Section 6, executed on the GPU: one thread per (h, w, c, group of adjacent images) reads its R*S window elements
 * with coalesced vector loads (c and b are contiguous in Image) and writes its Out words once.  HBM-bound.
 *   problem  in   host pointer; problem->K must equal problem->C
 *   dtype    in   cacnn_dtype of the Image (Out is fp32)
 *   mode     in   cacnn_pool_mode
 *   image    in   DEVICE pointer, IW*IH*C*B elements, read-only
 *   out      out  DEVICE pointer, K*H*W*B fp32, overwritten; must not alias image
 *   hip_stream    hipStream_t cast to void*; NULL is the default stream
 * Enqueues and returns; never synchronises, allocates nothing, keeps no reference.
 * Errors: CACNN_ERR_NULL, CACNN_ERR_INVALID_ARG (dimension < 1, K != C, element counts beyond 2^31-1 per array,
 * misaligned pointers), CACNN_ERR_UNSUPPORTED (dtype, mode), CACNN_ERR_NO_DEVICE, CACNN_ERR_LAUNCH.
 */
int cacnn_pool_forward(const cacnn_problem* problem, int dtype, int mode, const void* image, void* out,
                       void* hip_stream);

/*
 * Measurement support: what this machine sustains, for reading the convolution's rates against (the published peaks
 * assume the peak clock; under an all-CU matrix load the clock is power-managed and depends on the operand bits).
 *
 * cacnn_probe_mfma: a register-only MFMA loop, one workgroup of four wavefronts on each of the 256 compute units, with
 * the instruction mix of the convolution kernels' inner step (21 MFMAs on 7 accumulators, 3 + 9 operand fragments).
 *   dtype        in   CACNN_F32 (32x32x2 fp32 MFMAs, 4096 flops each) or CACNN_BF16_F32ACC (32x32x16 bf16, 32768 flops)
 *   operands     in   DEVICE pointer, 16-byte aligned, 16 KiB: the operand fragments are taken from here (fp32 words or
 *                     packed bf16 pairs); all zeros gives the rate with nothing toggling
 *   sink         out  DEVICE pointer, 65536 fp32, overwritten with sums of the accumulators (so the work is kept)
 *   iters        in   1 .. 2^24; the launch issues 256 * 4 * iters * 42 MFMAs, returned in *mfma_issued (host)
 * cacnn_probe_copy: dst[0..bytes) = src[0..bytes) with streaming loads and stores: bytes read and bytes written.
 *   src, dst     DEVICE pointers, 16-byte aligned, not overlapping; bytes a positive multiple of 16
 * cacnn_probe_lds_fill: every compute unit fills its LDS from the window [src, src + window_bytes) with the loads the
 * convolution's staging waves use (64 lanes x 16 bytes to a wave-uniform LDS address, 24 KiB in flight per wave): with a
 * window that fits one L2 (say 2 MiB) the rate at which the L2s feed the LDS of all compute units at once; with a
 * window far beyond the L2s, the rate from behind them.
 *   src          in   DEVICE pointer, 16-byte aligned, at least window_bytes long
 *   window_bytes in   a power of two, 64 KiB .. 1 GiB
 *   sink         out  DEVICE pointer, 65536 fp32 (overwritten)
 *   iters        in   1 .. 2^20; the launch moves 256 * 48 KiB * iters bytes, returned in *bytes_moved (host)
 * cacnn_probe_mfma_and_fill: both at once in the proportions of the bf16 convolution's unit, with nothing that
 * synchronises them: on every compute unit four wavefronts run the bf16 MFMA loop (mfma_iters x 42 MFMAs each) while four
 * others fill the LDS from a shared window (fill_iters x 12 KiB each); either count may be 0 (not both).
 *   operands     as for cacnn_probe_mfma; src, window_bytes (64 KiB .. 32 MiB), sink as for cacnn_probe_lds_fill
 * cacnn_probe_mfma_and_fill_on: the same on `compute_units` compute units only (1 .. 256; one workgroup each, the others
 * idle): what a compute unit's rate is when fewer of them work, i.e. how much of the rate is the whole chip's (its
 * power-managed clock) and how much the compute unit's own.
 *   tile         0: the MFMA loop of the kernel with tiles of 64 images x 7 x 1 positions (mfma_iters x 42 MFMAs per
 *                wavefront, as cacnn_probe_mfma_and_fill); 1: of the kernel with tiles of 64 images x 2 x 2 positions
 *                (mfma_iters x 24 MFMAs per wavefront on 4 accumulators)
 *   mode         bit 0: the MFMA wavefronts read their operand fragments from the LDS that the others are filling, before
 *                every half iteration, with the instructions and the addresses of that kernel's multiplying wavefronts (3
 *                16-byte reads and 18 or 16 transposing 8-byte reads); the LDS starts out as copies of the operand words
 *                (clear: register-only MFMA loop).  bit 1: all eight wavefronts meet at a workgroup barrier once per
 *                iteration, as that kernel's do once per unit; needs mfma_iters == fill_iters
 * All of them enqueue on hip_stream and return; they never synchronise and allocate nothing.  The caller times them.
 * Errors: CACNN_ERR_NULL, CACNN_ERR_INVALID_ARG (alignment, sizes, iters), CACNN_ERR_UNSUPPORTED (dtype),
 * CACNN_ERR_NO_DEVICE, CACNN_ERR_LAUNCH.
 */
int cacnn_probe_mfma(int dtype, const void* operands, float* sink, int32_t iters, int64_t* mfma_issued, void* hip_stream);
int cacnn_probe_copy(const void* src, void* dst, size_t bytes, void* hip_stream);
int cacnn_probe_lds_fill(const void* src, size_t window_bytes, float* sink, int32_t iters, void* hip_stream, int64_t* bytes_moved);
int cacnn_probe_mfma_and_fill(const void* operands, const void* src, size_t window_bytes, float* sink, int32_t mfma_iters,
                              int32_t fill_iters, void* hip_stream);
int cacnn_probe_mfma_and_fill_on(int32_t compute_units, int32_t tile, int32_t mode, const void* operands, const void* src,
                                 size_t window_bytes, float* sink, int32_t mfma_iters, int32_t fill_iters, void* hip_stream);

/* Number of compiled kernel variants, and a static, NUL-terminated description of one
 * ("f32 k64 b8w4h4 ..."); NULL if the index is out of range.  Host only. */
int cacnn_variant_count(void);
const char* cacnn_variant_name(int variant);

/* Static, NUL-terminated text for a status code (never NULL). */
const char* cacnn_status_string(int status);

/*
 * Two memory levels (Section 4.1: any level of a hierarchy can play the fast memory; Section 7 with the eight XCDs, each
 * with its own L2, as the processors): the workgroup's LDS tile of cacnn_tile_plan inside an L2-level tile.  Host only.
 *   - the Section 5 linear program and Theorem 1 at M = one L2 in input words (lp_*, bound_words), and that LP's tile
 *     rounded to whole LDS tiles (l2_tile_*, in elements: what the paper's schedule would keep in one L2);
 *   - for every admissible way of laying an XCD's run of tiles out -- a_K groups of k-tiles (1, 2, 4, 8, a divisor of the
 *     k-tile count) times the walk order inside a group (cacnn_plan.xcd_walk) -- the words the eight L2s fetch according
 *     to a model of the launch: a workgroup's n-th tile belongs to round n, an XCD's round reads the Filter rows of its
 *     k-tiles and the Image footprints (halo included) of its position tiles, each L2 keeps what it read in LRU order
 *     up to its size, and Out is written once.  Position tiles whose halos overlap each fetch the overlap: that is
 *     what the counters show on MI355X (a line has left the L2 before the neighbouring tile asks for it);
 *   - a_k / walk: candidates are taken in the order a_K = 1, 2, 4, 8, walk 0 before 1, and a later one replaces the
 *     choice only if it saves 3 % of the chosen one's words; cacnn_tile_plan puts them into xcd_split_k / xcd_walk.
 * machine_l2 NULL = MI355X (4 MiB, 8 XCDs, 32 compute units each).  Problems with more than a hundred thousand tiles are not
 * simulated: n_candidates = 0 and a_k is the closed-form choice that minimises a_K*|Image| + (8/a_K)*|Filter|.
 * Errors: as cacnn_tile_plan.
 */
typedef struct {
    int64_t l2_bytes;
    int32_t n_xcd, cu_per_xcd;
} cacnn_machine_l2;

typedef struct {
    double lp_tile[9];       /* Section 5 LP at M = L2 words, order b,c,k,w,h,r',r'',s',s'' */
    double lp_volume, lp_cost_words, bound_words;
    int32_t l2_tile_b, l2_tile_k, l2_tile_w, l2_tile_h;   /* lp_tile rounded to whole LDS tiles, clipped to the problem */
    int32_t a_k, walk;       /* the chosen layout of an XCD's run */
    int32_t n_candidates;
    int32_t cand_a_k[8], cand_walk[8];
    double cand_words[8];    /* modelled words fetched by the L2s plus Out once, per candidate */
    double chosen_words;     /* the chosen candidate's (0 when nothing was simulated) */
    double parallel_bound_words;   /* Section 7's expression at M = L2 words for the chosen a_K and the positions divided
                                      over the remaining 8 / a_K (images first, then rows, then columns) */
} cacnn_l2_plan;

int cacnn_two_level_plan(const cacnn_problem* problem, int dtype, const cacnn_machine* machine,
                         const cacnn_machine_l2* machine_l2, cacnn_l2_plan* out);

/*
 * Closed-form tiling (Section 5.1, "Determining the optimal tiling", and the partition algorithm of its figure).
 * The parameter space theta = log_M (B, C, K, W, H, R, S, sigma_w, sigma_h) is cut into convex regions, in each of
 * which the optimiser of the Section 5 LP is one affine function of theta; the table compiled into the library was
 * produced offline by paper_1802_06905_amd/closed_form.py (exact rational arithmetic; a tie-break in the objective
 * makes the optimiser unique, so there is one region per affine map).  This call evaluates it: no LP is solved.
 *   M        fast-memory size in words, > 1.
 *   region   index of the region that holds theta (borders belong to both neighbours; the optimum agrees there);
 *   theta    the nine logs after clamping into the tabulated box (a loop bound above M acts like M, and a stride
 *            above its filter extent like that extent: neither changes the LP's feasible set);
 *   l, tile  the tile logs (base M) and sizes M^l, order b,c,k,w,h,r',r'',s',s'';
 *   log_volume, volume, cost_words = F*M/volume (Section 5.2), bound_words = Theorem 1 at M;
 *   worst_violation  the largest amount by which l breaks a row of the LP (rounding only: <= 1e-9).
 * Errors: NULL pointer -> CACNN_ERR_NULL; non-positive dimension or M <= 1 -> CACNN_ERR_INVALID_ARG.  Host-only.
 */
typedef struct {
    int32_t region, n_regions;
    double theta[9];
    double l[9];
    double tile[9];
    double log_volume, volume, cost_words, bound_words;
    double worst_violation;
} cacnn_closed_form;

int cacnn_closed_form_tiling(const cacnn_problem* problem, double M, cacnn_closed_form* out);

#ifdef __cplusplus
}
#endif
#endif /* CACNN_H */
