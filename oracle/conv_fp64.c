/*
 * Oracle: the seven-nested-loop convolution of the paper, written out as its definition.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, obviously-correct CPU reference that the
 * GPU library is checked against.  It shares no code with the GPU path; only tests, the smoke check
 * and the benchmark's cpu_baseline leg may build or call it.
 *
 * What it computes (paper, Section 2 "CNN Model", Eq. (1), the loop nest labelled eqn_CNN):
 *
 *     for b, c, k, w, h, r, s:
 *         Out(k,h,w,b) += Image(r + sigma_w*w, s + sigma_h*h, c, b) * Filter(k,r,s,c)
 *
 * starting from Out = 0.  All arithmetic is fp64; fp32 (or bf16-valued fp32) inputs are widened exactly.
 *
 * Readings of the paper taken here (the paper does not fix them):
 *   - storage: dense row-major in the printed index order, last index fastest:
 *       Image [IW][IH][C][B],  Filter [K][R][S][C],  Out [K][H][W][B];
 *   - Image extent is the touched one, IW = sigma_w*(W-1)+R, IH = sigma_h*(H-1)+S (Section 2 prints the
 *     asymptotic over-estimate sigma_w*W+R);
 *   - the first Image axis pairs with (r, w, sigma_w), the second with (s, h, sigma_h), while Out is
 *     indexed (k,h,w,b): taken literally;
 *   - no padding.
 *
 * Loop order: (k,h,w) outside, (c,r,s) inside, b innermost so that the unit-stride index is the inner
 * loop.  The paper allows any order ("the same arithmetic operations in an arbitrary order", Section 1);
 * in fp64 the order only affects rounding at the 1e-16 level.
 *
 * Also returns Abs(k,h,w,b) = sum |Image * Filter| over the same (c,r,s): the denominator of the parity
 * tolerance.
 */
#include <stdint.h>
#include <stdlib.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int64_t B, C, K, W, H, R, S, sigma_w, sigma_h;
} oracle_problem;

static inline int64_t img_index(const oracle_problem *p, int64_t x, int64_t y, int64_t c, int64_t b) {
    const int64_t IH = p->sigma_h * (p->H - 1) + p->S;
    return ((x * IH + y) * p->C + c) * p->B + b;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Full convolution.  image/filter are fp32 values (bf16 configs pass bf16-rounded values stored as fp32).
 * out and abs_out (may be NULL) are fp64 arrays of K*H*W*B elements.  Returns 0, or -1 on bad arguments. */
int oracle_conv_fp64(const oracle_problem *p, const float *image, const float *filter,
                     double *out, double *abs_out, int threads) {
    if (!p || !image || !filter || !out) return -1;
    if (p->B < 1 || p->C < 1 || p->K < 1 || p->W < 1 || p->H < 1 || p->R < 1 || p->S < 1 ||
        p->sigma_w < 1 || p->sigma_h < 1) return -1;
    const int64_t B = p->B, C = p->C, K = p->K, W = p->W, H = p->H, R = p->R, S = p->S;
    const int64_t sw = p->sigma_w, sh = p->sigma_h;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#else
    (void)threads;
#endif
    #pragma omp parallel
    {
        double *acc = (double *)malloc(sizeof(double) * (size_t)B);
        double *aab = (double *)malloc(sizeof(double) * (size_t)B);
        #pragma omp for collapse(2) schedule(static)
        for (int64_t k = 0; k < K; ++k) {
            for (int64_t h = 0; h < H; ++h) {
                for (int64_t w = 0; w < W; ++w) {
                    for (int64_t b = 0; b < B; ++b) { acc[b] = 0.0; aab[b] = 0.0; }
                    for (int64_t c = 0; c < C; ++c) {
                        for (int64_t r = 0; r < R; ++r) {
                            for (int64_t s = 0; s < S; ++s) {
                                const double f = (double)filter[((k * R + r) * S + s) * C + c];
                                const float *im = image + img_index(p, r + sw * w, s + sh * h, c, 0);
                                for (int64_t b = 0; b < B; ++b) {
                                    const double prod = (double)im[b] * f;
                                    acc[b] += prod;
                                    aab[b] += fabs(prod);
                                }
                            }
                        }
                    }
                    double *o = out + ((k * H + h) * W + w) * B;
                    for (int64_t b = 0; b < B; ++b) o[b] = acc[b];
                    if (abs_out) {
                        double *a = abs_out + ((k * H + h) * W + w) * B;
                        for (int64_t b = 0; b < B; ++b) a[b] = aab[b];
                    }
                }
            }
        }
        free(acc);
        free(aab);
    }
    return 0;
}

/* The same sum for a list of n output coordinates (k,h,w,b), one at a time: used where the full array is
 * too slow to compute on the CPU.  coords is n x 4 int64, row = (k,h,w,b). */
int oracle_conv_fp64_at(const oracle_problem *p, const float *image, const float *filter,
                        const int64_t *coords, int64_t n, double *out, double *abs_out) {
    if (!p || !image || !filter || !coords || !out) return -1;
    const int64_t C = p->C, R = p->R, S = p->S;
    const int64_t sw = p->sigma_w, sh = p->sigma_h;
    for (int64_t i = 0; i < n; ++i) {
        const int64_t k = coords[4 * i + 0], h = coords[4 * i + 1], w = coords[4 * i + 2], b = coords[4 * i + 3];
        if (k < 0 || k >= p->K || h < 0 || h >= p->H || w < 0 || w >= p->W || b < 0 || b >= p->B) return -1;
    }
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        const int64_t k = coords[4 * i + 0], h = coords[4 * i + 1], w = coords[4 * i + 2], b = coords[4 * i + 3];
        double acc = 0.0, aab = 0.0;
        for (int64_t c = 0; c < C; ++c)
            for (int64_t r = 0; r < R; ++r)
                for (int64_t s = 0; s < S; ++s) {
                    const double prod = (double)image[img_index(p, r + sw * w, s + sh * h, c, b)] *
                                        (double)filter[((k * R + r) * S + s) * C + c];
                    acc += prod;
                    aab += fabs(prod);
                }
        out[i] = acc;
        if (abs_out) abs_out[i] = aab;
    }
    return 0;
}
