// Host side of the cacnn C ABI: Theorem 1's bound, the tiling linear program of Section 5, the Appendix A case
// analysis, the gfx950 tile planner, argument validation and the launch dispatcher.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <limits>
#include <list>
#include <mutex>
#include <unordered_map>
#include <vector>

#include "../../include/cacnn.h"
#include "cacnn_internal.h"

using namespace cacnn;

namespace {

#include "cacnn_closed_form_table.inc"

const cacnn_machine kDefaultMachine = {160 * 1024, 512 * 1024, 256};

bool valid_problem(const cacnn_problem* p) {
    const int64_t v[9] = {p->B, p->C, p->K, p->W, p->H, p->R, p->S, p->sigma_w, p->sigma_h};
    for (int64_t x : v)
        if (x < 1) return false;
    return true;
}

// product with overflow detection; returns false on overflow past lim
bool mul_check(int64_t a, int64_t b, int64_t lim, int64_t* out) {
    if (a != 0 && b > lim / a) return false;
    *out = a * b;
    return true;
}

// ------------------------------------------------------------------------------------------------------------
// Section 5: the linear program over l_x = log_M(tile size of x), x in (b,c,k,w,h,r',r'',s',s'').
// maximise sum l_x  s.t.  l >= 0, each tile within its loop bound, Out / Filter / Image footprints <= M, the Image
// footprint (b_w + b_r')(b_h + b_s') being bounded term by term.  All right-hand sides are >= 0, so the slack basis
// is feasible and a plain primal simplex (Bland's rule) suffices.
struct LpSolution {
    double l[9];
    double log_volume;
};

// M_out, M_flt, M_img: the words the Out, Filter and Image tiles may occupy (the paper's LP has one M for all three; the
// gfx950 budget has accumulator registers for Out and LDS for the other two).  l[] and log_volume are logarithms to base
// `base`.
LpSolution solve_tiling_lp(const cacnn_problem& p, double M_out, double M_flt, double M_img, double base) {
    const int n = 9;
    enum { b_, c_, k_, w_, h_, r1_, r2_, s1_, s2_ };
    const double lnM = std::log(base);
    auto lg = [&](double x) { return std::log(x) / lnM; };
    const double sw = (double)std::min(p.sigma_w, p.R), sh = (double)std::min(p.sigma_h, p.S);

    std::vector<std::vector<double>> A;
    std::vector<double> rhs;
    auto row = [&](std::initializer_list<int> vars, double r) {
        std::vector<double> a(n, 0.0);
        for (int v : vars) a[v] += 1.0;
        A.push_back(a);
        rhs.push_back(std::max(r, 0.0));
    };
    row({b_}, lg((double)p.B));
    row({c_}, lg((double)p.C));
    row({k_}, lg((double)p.K));
    row({w_}, lg((double)p.W));
    row({h_}, lg((double)p.H));
    row({r2_}, lg(sw));
    row({s2_}, lg(sh));
    row({r1_}, lg((double)p.R) - lg(sw));
    row({s1_}, lg((double)p.S) - lg(sh));
    row({b_, k_, w_, h_}, lg(M_out));                    // Out tile
    row({c_, k_, r1_, r2_, s1_, s2_}, lg(M_flt));        // Filter tile
    row({b_, c_, w_, h_, r2_, s2_}, lg(M_img));          // Image tile, four products
    row({b_, c_, w_, s1_, r2_, s2_}, lg(M_img));
    row({b_, c_, r1_, h_, r2_, s2_}, lg(M_img));
    row({b_, c_, r1_, s1_, r2_, s2_}, lg(M_img));

    const int m = (int)A.size();
    // tableau: m rows x (n + m + 1) columns, objective row last; maximise sum x  <=>  reduced costs start at -1
    const int cols = n + m + 1;
    std::vector<std::vector<double>> T(m + 1, std::vector<double>(cols, 0.0));
    std::vector<int> basis(m);
    for (int i = 0; i < m; ++i) {
        for (int jx = 0; jx < n; ++jx) T[i][jx] = A[i][jx];
        T[i][n + i] = 1.0;
        T[i][cols - 1] = rhs[i];
        basis[i] = n + i;
    }
    for (int jx = 0; jx < n; ++jx) T[m][jx] = -1.0;
    const double eps = 1e-12;
    for (int iter = 0; iter < 10000; ++iter) {
        int enter = -1;
        for (int jx = 0; jx < n + m; ++jx)
            if (T[m][jx] < -1e-10) {
                enter = jx;  // Bland: lowest index
                break;
            }
        if (enter < 0) break;
        int leave = -1;
        double best = 0.0;
        for (int i = 0; i < m; ++i) {
            if (T[i][enter] > eps) {
                const double ratio = T[i][cols - 1] / T[i][enter];
                if (leave < 0 || ratio < best - 1e-14 || (std::fabs(ratio - best) <= 1e-14 && basis[i] < basis[leave])) {
                    leave = i;
                    best = ratio;
                }
            }
        }
        if (leave < 0) break;  // unbounded: cannot happen, every variable is capped
        const double piv = T[leave][enter];
        for (int jx = 0; jx < cols; ++jx) T[leave][jx] /= piv;
        for (int i = 0; i <= m; ++i) {
            if (i == leave) continue;
            const double f = T[i][enter];
            if (f != 0.0)
                for (int jx = 0; jx < cols; ++jx) T[i][jx] -= f * T[leave][jx];
        }
        basis[leave] = enter;
    }
    LpSolution s;
    for (int jx = 0; jx < n; ++jx) s.l[jx] = 0.0;
    for (int i = 0; i < m; ++i)
        if (basis[i] < n) s.l[basis[i]] = std::max(0.0, T[i][cols - 1]);
    s.log_volume = 0.0;
    for (int jx = 0; jx < n; ++jx) s.log_volume += s.l[jx];
    return s;
}

LpSolution solve_tiling_lp(const cacnn_problem& p, double M) { return solve_tiling_lp(p, M, M, M, M); }

// Appendix A, Theorem 2 (strides 1): which leaf of the decision tree the shape falls in.
int appendix_a_case(const cacnn_problem& p, double M) {
    if (p.sigma_w != 1 || p.sigma_h != 1) return 0;
    const double img = (double)p.C * p.H * p.W * p.B, flt = (double)p.K * p.C * p.R * p.S,
                 out = (double)p.K * p.H * p.W * p.B;
    if (std::min(img, std::min(flt, out)) <= M) {
        // Case 1, by which arrays exceed M (the sub-cases of the proof of the Case 1 lemma)
        const bool bi = img > M, bf = flt > M, bo = out > M;
        const double hwb = (double)p.H * p.W * p.B;
        if (!bi && !bf && !bo) return 11;
        if (bi && !bf && !bo) return 12;
        if (bo && !bf && !bi) return 13;
        if (bf && !bi && !bo) return (double)p.K * p.C <= M ? 14 : 15;
        if (bi && bo) return 16;
        if (bi && bf) return (double)p.K >= hwb ? 17 : 18;
        return (double)p.C >= hwb ? 19 : 110;
    }
    const double RS = (double)p.R * p.S, BHW = (double)p.B * p.H * p.W;
    if (RS >= M) return 21;
    if (M * RS >= BHW * BHW) return 221;
    if ((double)std::min(p.C, p.K) >= std::sqrt(M / RS)) return 2221;
    return 2222;
}

void bound_terms(const cacnn_problem& p, double M, cacnn_bound* out) {
    const double sw = (double)std::min(p.sigma_w, p.R), sh = (double)std::min(p.sigma_h, p.S);
    const double B = (double)p.B, C = (double)p.C, K = (double)p.K, W = (double)p.W, H = (double)p.H, R = (double)p.R,
                 S = (double)p.S;
    out->term[0] = B * K * W * H;
    out->term[1] = sw * sh * B * C * W * H;
    out->term[2] = C * K * R * S;
    out->term[3] = B * C * K * W * H * R * S / M;
    out->term[4] = B * C * K * W * H * std::sqrt(R * S * sw * sh / M);
    out->argmax = 0;
    for (int i = 1; i < 5; ++i)
        if (out->term[i] > out->term[out->argmax]) out->argmax = i;
    out->bound = out->term[out->argmax];
}

// Section 7: Theorem 1's terms with the Image replicated over the a_K groups of output channels and the Filter over
// the a_B a_W a_H groups of positions.
void parallel_terms(const cacnn_problem& p, double M, int64_t ab, int64_t ak, int64_t aw, int64_t ah, cacnn_bound* out) {
    bound_terms(p, M, out);
    out->term[1] *= (double)ak;
    out->term[2] *= (double)ab * (double)aw * (double)ah;
    out->argmax = 0;
    for (int i = 1; i < 5; ++i)
        if (out->term[i] > out->term[out->argmax]) out->argmax = i;
    out->bound = out->term[out->argmax];
}

// ------------------------------------------------------------------------------------------------------------
// gfx950 tile geometry for one (variant, contraction tile)

int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
int64_t round_up(int64_t a, int64_t b) { return ceil_div(a, b) * b; }

struct Geometry {
    int CT, bR, bS, XS, YS, xpitch, ypitch, fpitch, QE, img_lds_elems, zero_off;
    int64_t lds_bytes;
    // pipelined variants
    int img_items, flt_items, img_buf, flt_buf, flt_off, flt_resident;
    int64_t n_slices;
    bool legal;   // the variant can run this geometry (staging items fit, packed fields fit)
};

Geometry make_geometry(const VariantInfo& v, const cacnn_problem& p, int CT, int bR, int bS, bool vec_img) {
    Geometry g;
    std::memset(&g, 0, sizeof(g));
    g.legal = true;
    g.CT = CT;
    g.bR = bR;
    g.bS = bS;
    {
        // Extents first, in 64 bits: a stride can be anything up to 2^31, and everything below is 32-bit arithmetic on
        // products of these.  A tile whose staged Image range or Filter tile cannot fit twice the largest LDS is refused
        // here; past this check every factor and every product of them stays below 2^20.
        // (a 1 x 1 kernel that takes any strides stages the positions its outputs read, not the range between them)
        const int64_t XS = v.fx_any_stride ? v.TW : p.sigma_w * (int64_t)(v.TW - 1) + bR,
                      YS = v.fx_any_stride ? v.TH : p.sigma_h * (int64_t)(v.TH - 1) + bS;
        const double esz0 = v.dtype == CACNN_F32 ? 4.0 : 2.0, cap = 2.0 * 160.0 * 1024.0;
        if (XS < 1 || YS < 1 || (double)XS * (double)YS * (double)CT * (double)v.TB * esz0 > cap ||
            (double)v.KT() * (double)bR * (double)bS * (double)CT * esz0 > cap) {
            g.legal = false;
            g.lds_bytes = INT64_MAX;
            return g;
        }
        g.XS = (int)XS;
        g.YS = (int)YS;
    }
    const int64_t Cpad = round_up(p.C, v.cgran());
    g.n_slices = ceil_div(p.R, bR) * ceil_div(p.S, bS) * ceil_div(Cpad, CT);
    g.flt_resident = (g.n_slices == 1 && ceil_div(p.K, v.KT()) == 1 && v.fx_ct == 0) ? 1 : 0;
    const int nbuf_f = g.flt_resident ? 1 : 2;
    if (v.fx_lds > 0) {
        // a fixed-geometry kernel: its own LDS layout, contraction tile and strides, a shape the tiles divide exactly
        g.lds_bytes = v.fx_lds;
        g.img_items = g.flt_items = 1;
        g.legal = CT == v.fx_ct && bR == v.fx_br && bS == v.fx_bs && g.YS == v.fx_ys &&
                  (v.fx_any_stride || (p.sigma_w == v.fx_sw && p.sigma_h == v.fx_sh)) &&
                  // (the kernels compiled for 1 x 1 filters take any filter one tap at a time)
                  (p.R == bR || (v.fx_any_stride && bR == 1)) && p.S % bS == 0 &&
                  (v.fx_tail8 == 2 ? p.C % 4 == 0 : v.fx_tail8 ? (p.C % CT != 0 && p.C % 8 == 0) : p.C % CT == 0) && vec_img &&
                  (v.fx_ragged == 2 || p.B % v.TB == 0) &&
                  (v.fx_ragged || (p.W % v.TW == 0 && p.H % v.TH == 0 && p.K % v.KT() == 0));
        if (v.fx_whole && (p.S != bS || p.C != CT)) g.legal = false;
        // staged words are addressed by 32-bit byte offsets from the unit's origin
        const double esz = v.dtype == CACNN_F32 ? 4.0 : 2.0;
        const double IHd = (double)(p.sigma_h * (p.H - 1) + p.S);
        const double reach = v.fx_any_stride ? (double)p.sigma_w * v.TW + (double)p.R : (double)(g.XS + 1);
        if (reach * IHd * (double)p.C * (double)p.B * esz >= 2147483648.0) g.legal = false;
        if ((double)(v.KT() + 1) * (double)p.R * (double)p.S * (double)p.C * esz >= 2147483648.0) g.legal = false;
        return g;
    }
    if (v.dtype == CACNN_F32 && v.f32v4()) {
        // 16-byte units: four consecutive contraction indices of one position
        const int G = CT / 4;
        g.ypitch = G * v.TB;
        const int base = g.YS * g.ypitch;
        int pad = 0;
        if (v.TB < 32) {
            // eight neighbouring staging lanes (b-quads fastest, then x) must land in eight different 16-byte slots
            const int want = v.TB >= 16 ? 2 : 1;
            while (((base + pad) & 7) != want) ++pad;
        }
        g.xpitch = base + pad;
        g.QE = (int)round_up((int64_t)bS * CT, 8);
        int f4 = bR * g.QE / 4;
        if ((f4 & 1) == 0) f4 += 1;     // odd count of 16-byte units: conflict-free A fragments
        g.fpitch = 4 * f4;
        g.img_buf = g.XS * g.xpitch;
        g.zero_off = 2 * g.img_buf;
        g.flt_off = g.zero_off + 32;
        g.flt_buf = v.KT() * f4;
        g.lds_bytes = 16ll * (g.flt_off + (int64_t)nbuf_f * g.flt_buf);
        g.img_items = g.XS * g.YS * G * (v.TB / 4);
        g.flt_items = v.KT() * bR * bS * G;
        g.legal = vec_img && v.TB % 4 == 0 && CT % 4 == 0 && (g.flt_resident || p.C % 4 == 0);
    } else if (v.dtype == CACNN_F32) {
        g.ypitch = CT * v.TB;
        int base = g.YS * g.ypitch;
        int pad = 0;
        if (v.TB < 32) {
            // spread the position groups of one MFMA column block over the 32 LDS banks: sigma_w * xpitch = TB (mod 32)
            int best = -1;
            for (int t = 0; t < 64; ++t) {
                if (vec_img && ((base + t) % 4) != 0) continue;
                if (best < 0) best = t;
                if (((int64_t)p.sigma_w * (base + t)) % 32 == v.TB % 32) {
                    best = t;
                    break;
                }
            }
            pad = best < 0 ? 0 : best;
        }
        g.xpitch = base + pad;
        g.QE = bS * CT + ((bS * CT) & 1);
        g.fpitch = bR * g.QE;
        if ((g.fpitch & 1) == 0) g.fpitch += 1;  // odd pitch: the 32 rows of an A fragment hit 32 different banks
        if (!v.pipelined) {
            g.zero_off = g.XS * g.xpitch;
            g.img_lds_elems = (int)round_up(g.zero_off + 64, 4);
            g.lds_bytes = 4ll * (g.img_lds_elems + (int64_t)v.KT() * g.fpitch);
        } else {
            g.img_buf = (int)round_up((int64_t)g.XS * g.xpitch, 4);
            g.zero_off = 2 * g.img_buf;
            g.flt_off = g.zero_off + 64;
            g.flt_buf = (int)round_up((int64_t)v.KT() * g.fpitch, 4);
            g.lds_bytes = 4ll * (g.flt_off + (int64_t)nbuf_f * g.flt_buf);
            g.img_items = g.XS * g.YS * CT * (v.TB / 4);
            g.flt_items = v.KT() * bR * bS * (CT / 4);
            g.legal = vec_img && v.TB % 4 == 0 && (g.flt_resident || (CT % 4 == 0 && p.C % 4 == 0));
        }
    } else {
        const int C8 = CT / 8;
        int f8 = bR * bS * C8;          // Filter row in 16-byte units; odd count keeps 16-byte reads conflict-free
        if ((f8 & 1) == 0) f8 += 1;
        g.fpitch = f8 * 8;
        g.ypitch = C8 * v.TB;           // 16-byte units, [c/8][b][8 c]
        g.xpitch = g.YS * g.ypitch;
        if (!v.pipelined) {
            g.img_lds_elems = g.XS * g.xpitch;
            g.lds_bytes = 16ll * g.img_lds_elems + 2ll * v.KT() * g.fpitch;
        } else {
            g.img_buf = g.XS * g.xpitch;
            g.flt_off = 2 * g.img_buf;
            g.flt_buf = v.KT() * f8;
            g.lds_bytes = 16ll * (g.flt_off + (int64_t)nbuf_f * g.flt_buf);
            g.img_items = g.XS * g.YS * C8 * (v.TB / 8);    // 8 channels x 8 images each
            g.flt_items = v.KT() * bR * bS * C8;
            g.legal = vec_img && v.TB % 8 == 0 && (g.flt_resident || p.C % 8 == 0);
        }
    }
    if (v.reuse_r > 0 && (bR != v.reuse_r || p.sigma_w != 1)) g.legal = false;
    if (v.pipelined) {
        const int64_t thr = v.staging_threads();
        if (g.img_items > v.MAXI * thr || (!g.flt_resident && g.flt_items > v.MAXF * thr)) g.legal = false;
        if (g.XS > 1023 || g.YS > 1023 || CT > 1023 || bR > 127 || bS > 127 || v.KT() > 256) g.legal = false;
        // staging items are addressed by 32-bit byte offsets from the unit's origin
        const double esz = v.dtype == CACNN_F32 ? 4.0 : 2.0;
        const double IHd = (double)(p.sigma_h * (p.H - 1) + p.S);
        const double reach = v.fx_any_stride ? (double)p.sigma_w * v.TW + 1.0 : (double)(g.XS + 1);
        if (reach * IHd * (double)p.C * (double)p.B * esz >= 2147483648.0) g.legal = false;
        if ((double)(v.KT() + 1) * (double)p.R * (double)p.S * (double)p.C * esz >= 2147483648.0) g.legal = false;
    }
    return g;
}

struct Choice {
    int variant = -1;
    Geometry g{};
    double cost = 0.0;
    int64_t n_wg = 0;
    double words = 0.0;       // words staged from global memory by the whole grid
    double img_words = 0.0;   // the Image part of them
    // the cost model's terms for the chosen geometry, in CU cycles: tiles per CU, MFMA time, staging time and
    // contraction slices per tile, Out drain
    double terms[5] = {0.0, 0.0, 0.0, 0.0, 0.0};
};

// words staged from global memory by the whole grid for one variant/geometry, clipped to the arrays
double staged_words(const VariantInfo& v, const cacnn_problem& p, const Geometry& g, double* image_words) {
    const int64_t tiles_k = ceil_div(p.K, v.KT()), tiles_b = ceil_div(p.B, v.TB), tiles_w = ceil_div(p.W, v.TW),
                  tiles_h = ceil_div(p.H, v.TH);
    const int64_t IW = p.sigma_w * (p.W - 1) + p.R, IH = p.sigma_h * (p.H - 1) + p.S;
    double sum_x = 0.0, sum_y = 0.0;
    for (int64_t r0 = 0; r0 < p.R; r0 += g.bR)
        for (int64_t tw = 0; tw < tiles_w; ++tw) {
            const int64_t lo = p.sigma_w * tw * v.TW + r0;
            sum_x += (double)std::max<int64_t>(0, std::min<int64_t>(IW, lo + g.XS) - lo);
        }
    for (int64_t s0 = 0; s0 < p.S; s0 += g.bS)
        for (int64_t th = 0; th < tiles_h; ++th) {
            const int64_t lo = p.sigma_h * th * v.TH + s0;
            sum_y += (double)std::max<int64_t>(0, std::min<int64_t>(IH, lo + g.YS) - lo);
        }
    const double image = (double)tiles_k * sum_x * sum_y * (double)p.C * (double)p.B;
    const double filter = (double)tiles_b * tiles_w * tiles_h * (double)p.K * p.R * p.S * p.C;
    if (image_words) *image_words = image;
    return image + filter;
}

bool vec_img_ok(const VariantInfo& v, const cacnn_problem& p) {
    const int vi = v.dtype == CACNN_F32 ? 4 : 8;
    return v.TB % vi == 0 && p.B % vi == 0;
}

// Cost model in CU cycles: MFMA issue time of one wavefront plus the staging time of the workgroup, times the
// number of workgroups a compute unit has to run.  Staging overlaps MFMA only when two workgroups share a CU.
// Coefficients of the generic kernels' cost model (see evaluate): cycles per MFMA-pipe cycle, per staging cycle, per
// contraction slice, per Out-drain cycle, and the constant part of a launch.
struct ModelCoef {
    double mfma, stage, slice, drain, fixed;
};

const ModelCoef& model_coef(const VariantInfo& v) {
    static const ModelCoef one_tile_bf16 = {4.926, 1.741, 7.1, 0.02466, 17060.0};
    static const ModelCoef one_tile_f32 = {2.459, 2.334, 8696.0, 0.1144, 1322.0};
    static const ModelCoef pipe_bf16 = {2.696, 0.0, 5385.0, 0.0928, 15510.0};
    static const ModelCoef pipe3_bf16 = {1.525, 0.0, 4127.0, 0.0, 27740.0};
    static const ModelCoef pipe_f32 = {1.667, 0.0, 6584.0, 0.1336, 4643.0};
    static const ModelCoef ws_bf16 = {2.236, 0.0, 2918.0, 0.0, 24020.0};
    static const ModelCoef ws3_bf16 = {1.358, 0.0, 1926.0, 0.0, 34050.0};
    static const ModelCoef ws_f32 = {1.514, 0.0, 2807.0, 0.2543, 11870.0};
    static const ModelCoef ws4_f32 = {1.284, 0.0, 5212.0, 0.2865, 7469.0};
    const bool f32 = v.dtype == CACNN_F32;
    if (v.pipelined == 0) return f32 ? one_tile_f32 : one_tile_bf16;
    if (v.pipelined == 1) return f32 ? pipe_f32 : (v.reuse_r > 0 ? pipe3_bf16 : pipe_bf16);
    return f32 ? (v.f32v4() ? ws4_f32 : ws_f32) : (v.reuse_r > 0 ? ws3_bf16 : ws_bf16);
}

bool evaluate(int vi, const cacnn_problem& p, const cacnn_machine& mach, Choice* best) {
    const VariantInfo& v = variant(vi).info;
    // fp32 slices in multiples of 4 channels keep the 16-byte Filter loads legal
    const int gran = (v.dtype == CACNN_F32 && p.C % 4 == 0) ? 4 : v.cgran();   // v.cgran() is 4 for the v4 layout
    const int Cpad = (int)std::min<int64_t>(round_up(p.C, gran), 1 << 20);
    // candidate contraction tiles: every even split of the (padded) channel range, and halvings of the s and r ranges
    std::vector<int> cts;
    for (int d = 1; d <= 64; ++d) {
        const int ct = (int)round_up(ceil_div(Cpad, d), gran);
        if (cts.empty() || cts.back() != ct) cts.push_back(ct);
        if (ct == gran) break;
    }
    if (v.fx_ct > 0) cts.assign(1, v.fx_ct);      // a fixed-geometry kernel has one c-slice (it may exceed a small C)
    const bool vimg = vec_img_ok(v, p);
    bool found = false;
    const int64_t tiles_k = ceil_div(p.K, v.KT()), tiles_b = ceil_div(p.B, v.TB), tiles_w = ceil_div(p.W, v.TW),
                  tiles_h = ceil_div(p.H, v.TH);
    int64_t n_wg = 0, t = 0;
    if (!mul_check(tiles_k, tiles_b, INT32_MAX, &t) || !mul_check(t, tiles_w, INT32_MAX, &t) ||
        !mul_check(t, tiles_h, INT32_MAX, &n_wg))
        return false;
    const double ebytes = v.dtype == CACNN_F32 ? 4.0 : 2.0;
    // global runs shorter than 32 bytes along b waste the rest of each 32-byte sector
    const double run_bytes = (double)std::min<int64_t>(v.TB, p.B) * ebytes;
    const double waste = std::max(1.0, 32.0 / run_bytes);
    for (int bR = (int)std::min<int64_t>(p.R, 1 << 12); bR >= 1; bR = (bR + 1) / 2 == bR ? 0 : (bR + 1) / 2) {
        for (int bS = (int)std::min<int64_t>(p.S, 1 << 12); bS >= 1; bS = (bS + 1) / 2 == bS ? 0 : (bS + 1) / 2) {
            for (int ct : cts) {
                const Geometry g = make_geometry(v, p, ct, bR, bS, vimg);
                if (!g.legal || g.lds_bytes > mach.lds_bytes) continue;
                double img_words = 0.0;
                const double words = staged_words(v, p, g, &img_words);
                // Cost model, in compute-unit cycles, for the generic kernels.  Four quantities of the launch:
                //   t_mfma   MFMA pipe time of one wavefront for one Out tile (64 cycles per fp32 32x32x2, 32 per bf16
                //            32x32x16);
                //   t_stage  staged bytes of the tile at 16 B/clk (runs shorter than 32 bytes along b waste the rest of
                //            each sector);
                //   n_ctiles contraction slices per tile (each costs a barrier and exposed latency);
                //   t_out    the Out tile draining to HBM at ~1 TB/s for the whole chip;
                // and per_cu, the Out tiles a compute unit runs one after the other.  The launch time is a non-negative
                // linear combination of them plus a constant, with one set of coefficients per kernel family, fitted
                // (least squares on the relative error) to the measured launch times of every generic variant on 28
                // calibration layers (bench.py --planner-sweep calibration).
                // (a kernel that reuses Image fragments over three taps r runs a last r-slice of fewer taps at the cost of a
                // whole one)
                const double r_run = v.reuse_r > 0 ? (double)round_up(p.R, v.reuse_r) : (double)p.R;
                const double ksteps = v.dtype != CACNN_F32 ? r_run * p.S * (Cpad / 16)
                                      : v.f32v4()          ? (double)p.R * (double)round_up((int64_t)p.S * Cpad, 8) / 2.0
                                                           : (double)p.R * ceil_div((int64_t)p.S * Cpad, 2);
                const double t_mfma = (v.dtype == CACNN_F32 ? 64.0 : 32.0) * v.MBLK * v.NBLK * ksteps;
                const double t_stage = (img_words * waste + (words - img_words)) * ebytes / (double)n_wg / 16.0;
                const double n_ctiles = (double)g.n_slices;
                const double t_out = (double)v.KT() * v.NT() * 4.0 * waste * (double)mach.num_cu / 1.0e12 * 2.4e9;
                const ModelCoef& mc = model_coef(v);
                const double per_cu = (double)ceil_div(n_wg, mach.num_cu);
                double cost = per_cu * (mc.mfma * t_mfma + mc.stage * t_stage + mc.slice * n_ctiles) +
                              mc.drain * t_out / std::max(1.0, std::min(per_cu, 4.0)) + mc.fixed;
                // the fixed-geometry kernels run one schedule: priced by what a unit was measured to take
                if (v.fx_unit_us > 0.f) {
                    double rounds = per_cu;
                    if (v.fx_calib_cus > 0) {
                        // the bf16 MFMA rate is the chip's (its power-managed clock), not the compute unit's: measured, a unit
                        // takes 1.13 to 1.2 times as long on 256 busy compute units as on 224 or 196, and 0.72 to 0.8 times
                        // on 128; (n / n_calibration)^0.8, not below 0.75, is within a few per cent of those.  Full rounds of
                        // tiles run on all compute units, the last round on what is left.
                        auto scale = [&](double busy) { return std::max(0.75, std::pow(busy / (double)v.fx_calib_cus, 0.8)); };
                        const int64_t full = n_wg / mach.num_cu, rest = n_wg % mach.num_cu;
                        rounds = (double)full * scale((double)mach.num_cu) + (rest ? scale((double)rest) : 0.0);
                    }
                    // a compute unit that runs several tiles one after the other pays, for each one after the first, the
                    // empty pipeline at the tile's start and the stores at its end (about 2 us, measured on 1 x 1 layers
                    // of 1 to 4 units per tile); the first tile's share is in the variant's fixed time
                    const double tile_us = v.fx_calib_cus > 0 ? 2.0 * (per_cu - 1.0) : 0.0;
                    // (a bf16 kernel compiled for 1 x 1 filters that walks the taps of a larger filter: its units were
                    // measured to take 1.1 to 1.17 times a 1 x 1 layer's on 3 x 3 layers with strides 2)
                    const double taps = v.fx_calib_cus > 0 && v.fx_any_stride && (p.R > 1 || p.S > 1) ? 1.12 : 1.0;
                    cost = (rounds * n_ctiles * (double)v.fx_unit_us * taps + tile_us + (double)v.fx_fixed_us) * 2400.0;
                }
                if (best->variant < 0 || cost < best->cost) {
                    best->variant = vi;
                    best->g = g;
                    best->cost = cost;
                    best->n_wg = n_wg;
                    best->words = words;
                    best->img_words = img_words;
                    best->terms[0] = per_cu;
                    best->terms[1] = t_mfma;
                    best->terms[2] = t_stage;
                    best->terms[3] = n_ctiles;
                    best->terms[4] = t_out;
                }
                found = true;
            }
        }
    }
    return found;
}

// ------------------------------------------------------------------------------------------------------------
// The generic kernels' tile, sized from the Section 5 linear program at the gfx950 budget.  The paper bounds three
// tiles by one M; here the Out tile lives in accumulator registers (at most 7 MFMA blocks of 32 x 32 per multiplying
// wave, four such waves: 28672 words) and the Image and Filter tiles share the LDS, double-buffered, so each may take a
// quarter of it (the paper's own slack: per-array bounds instead of a bound on the sum).  The LP's optimum gives the
// Out tile's two extents k* and P* = b*w*h and says how much of the filter a contraction tile should cover; the compiled
// variant nearest to (k*, P*) in log distance is launched, where padding (tile extents beyond the problem's), an uneven
// or short tile count over the compute units (Section 7: divide the output over all processors) and the kernel family
// (measured ratios between the one-tile, pipelined and wave-specialised kernels on the same tile) add to the distance.
// The contraction tile is the one of largest volume b_c b_r b_s the LDS really holds, whole filter extents first as in
// the LP's optimum for R S << M (Appendix A, Case 2.2.2.1: b_R = R, b_S = S).
struct GpuLpTile {
    double k, P, c, r, s;
};

GpuLpTile solve_gpu_lp(const cacnn_problem& p, int dtype, const cacnn_machine& mach) {
    const double esz = dtype == CACNN_F32 ? 4.0 : 2.0;
    const double M_acc = 28672.0, M_lds = std::max(2.0, (double)mach.lds_bytes / (4.0 * esz));
    const LpSolution s = solve_tiling_lp(p, M_acc, M_lds, M_lds, std::exp(1.0));
    GpuLpTile t;
    t.k = std::exp(s.l[2]);
    t.P = std::exp(s.l[0] + s.l[3] + s.l[4]);
    t.c = std::exp(s.l[1]);
    t.r = std::exp(s.l[5] + s.l[6]);
    t.s = std::exp(s.l[7] + s.l[8]);
    return t;
}

bool evaluate_lp(int vi, const cacnn_problem& p, const cacnn_machine& mach, const GpuLpTile& lp, Choice* best) {
    const VariantInfo& v = variant(vi).info;
    const int gran = (v.dtype == CACNN_F32 && p.C % 4 == 0) ? 4 : v.cgran();
    const int Cpad = (int)std::min<int64_t>(round_up(p.C, gran), 1 << 20);
    const bool vimg = vec_img_ok(v, p);
    const int64_t tiles_k = ceil_div(p.K, v.KT()), tiles_b = ceil_div(p.B, v.TB), tiles_w = ceil_div(p.W, v.TW),
                  tiles_h = ceil_div(p.H, v.TH);
    int64_t n_wg = 0, t = 0;
    if (!mul_check(tiles_k, tiles_b, INT32_MAX, &t) || !mul_check(t, tiles_w, INT32_MAX, &t) ||
        !mul_check(t, tiles_h, INT32_MAX, &n_wg))
        return false;
    // the contraction tile of largest volume that is legal and fits: whole filter extents first, then the c-slice
    Geometry g_best{};
    double vol_best = -1.0;
    for (int bR = (int)std::min<int64_t>(p.R, 1 << 12); bR >= 1; bR = (bR + 1) / 2 == bR ? 0 : (bR + 1) / 2)
        for (int bS = (int)std::min<int64_t>(p.S, 1 << 12); bS >= 1; bS = (bS + 1) / 2 == bS ? 0 : (bS + 1) / 2)
            for (int d = 1; d <= 64; ++d) {
                const int ct = (int)round_up(ceil_div(Cpad, d), gran);
                const Geometry g = make_geometry(v, p, ct, bR, bS, vimg);
                if (g.legal && g.lds_bytes <= mach.lds_bytes) {
                    // volume, with a premium on covering the filter extents (the halo re-staging the LP's optimum avoids)
                    const double vol = (double)std::min<int64_t>(ct, p.C) * bR * bS * ((int64_t)bR * bS == p.R * p.S ? 4.0 : 1.0);
                    if (vol > vol_best) {
                        vol_best = vol;
                        g_best = g;
                    }
                    break;      // smaller c-slices of the same (b_r, b_s) only lose volume
                }
                if (ct == gran) break;
            }
    if (vol_best < 0.0) return false;
    const double ku = (double)std::min<int64_t>(v.KT(), p.K);
    const double Pu = (double)std::min<int64_t>(v.TB, p.B) * (double)std::min<int64_t>(v.TW, p.W) * (double)std::min<int64_t>(v.TH, p.H);
    double dist = std::fabs(std::log(ku / lp.k)) + std::fabs(std::log(Pu / lp.P));
    dist += std::log((double)v.KT() * v.NT() / (ku * Pu));                          // padded MFMA rows and columns
    // global runs along b shorter than a 64-byte half line use a fraction of every line they touch
    dist += std::log(std::max(1.0, 64.0 / ((double)std::min<int64_t>(v.TB, p.B) * (v.dtype == CACNN_F32 ? 4.0 : 2.0))));
    const int64_t resident = std::max<int64_t>(1, std::min<int64_t>(v.occ, mach.lds_bytes / std::max<int64_t>(1, g_best.lds_bytes)));
    const double slots = (double)mach.num_cu * (v.pipelined ? 1.0 : (double)resident);
    dist += std::log((double)ceil_div(n_wg, (int64_t)slots) * slots / (double)n_wg);    // idle or unevenly loaded compute units
    dist += v.pipelined == 2 ? 0.0 : (v.pipelined == 1 ? std::log(1.3) : std::log(2.5));  // kernel family
    dist += std::log((double)v.tune);
    if (best->variant < 0 || dist < best->cost) {
        best->variant = vi;
        best->g = g_best;
        best->cost = dist;
        best->n_wg = n_wg;
        best->words = staged_words(v, p, g_best, &best->img_words);
    }
    return true;
}

// Measured against the fastest of all variants (cacnn_tune) on sixteen mid-size and ragged layers, the LP-sized choice is
// 1.38x slower in the geometric mean (worst 2.1x) and the calibrated cycle model 1.34x (worst 2.5x): on problems this
// small what separates the variants is how well each kernel family keeps its pipeline full, which neither the LP nor
// the model prices well.  The cycle model stays the default; CACNN_PLANNER=lp selects the LP-sized choice.
bool planner_uses_lp() {
    static const bool lp = [] {
        const char* e = std::getenv("CACNN_PLANNER");
        return e && std::strcmp(e, "lp") == 0;
    }();
    return lp;
}

// workgroups launched: one per Out tile, or for the persistent kernels as many as the machine holds at once
int64_t launch_grid(const VariantInfo& v, const Geometry& g, int64_t n_tiles, const cacnn_machine& mach) {
    if (!v.pipelined) return n_tiles;
    const int64_t resident =
        std::max<int64_t>(1, std::min<int64_t>(v.occ, mach.lds_bytes / std::max<int64_t>(1, g.lds_bytes)));
    return std::min<int64_t>(n_tiles, mach.num_cu * resident);
}

// XCD count used for the tile remapping; CACNN_XCDS=1 switches the remapping off (debugging aid)
int xcd_count() {
    static int n = [] {
        const char* e = std::getenv("CACNN_XCDS");
        const int v = e ? std::atoi(e) : 8;
        return v >= 1 && v <= 64 ? v : 8;
    }();
    return n;
}

// Section 7 with the XCDs as the processors and the arrays' real sizes: divide the XCDs into a_K groups of output
// channels and n_xcd / a_K ranges of positions; an XCD then fetches 1 / a_K of the Filter and the Image is fetched a_K
// times over all XCDs.  a_K must divide both the XCD count and the k-tile count (whole k-tiles per group).
int choose_xcd_split_k(const cacnn_problem& p, int dtype, int64_t tiles_k, int n_xcd) {
    const double esz = dtype == CACNN_F32 ? 4.0 : 2.0;
    const double img = (double)(p.sigma_w * (p.W - 1) + p.R) * (double)(p.sigma_h * (p.H - 1) + p.S) * (double)p.C *
                       (double)p.B * esz;
    const double flt = (double)p.K * p.R * p.S * p.C * esz;
    int best = 1;
    double best_bytes = img + (double)n_xcd * flt;
    for (int ak = 2; ak <= n_xcd; ak *= 2) {
        if (n_xcd % ak || tiles_k % ak) continue;
        const double bytes = (double)ak * img + (double)(n_xcd / ak) * flt;
        if (bytes < best_bytes) {
            best = ak;
            best_bytes = bytes;
        }
    }
    return best;
}

// ------------------------------------------------------------------------------------------------------------
// Two levels: the words the XCDs' L2s fetch for one way of laying out an XCD's run of tiles (a_K groups of k-tiles, walk
// order inside a group).  A model of the launch: workgroup i belongs to XCD i % n_xcd and takes the tiles at places
// i / n_xcd, i / n_xcd + grid / n_xcd, ... of its XCD's contiguous run of the tile list; an XCD's round n is every
// workgroup's n-th tile; a tile reads the Filter rows of its k-tile (one atom) and the Image columns of its position
// tile (one atom per input pixel and image group: all channels); an L2 keeps atoms in LRU order up to its size.
struct L2Machine {
    double words;      // one L2, in input words
    int n_xcd, cu_per_xcd;
};
constexpr L2Machine kDefaultL2Bytes = {4.0 * 1024.0 * 1024.0, 8, 32};

struct TileGeom {
    int KT, TB, TW, TH, b_group;
    int64_t grid;
};

int b_group_of(const VariantInfo& v, int dtype, int64_t tiles_b) {
    // b-tiles that read different pieces of the same 128-byte Image lines stay adjacent in the tile order
    const int64_t esz = dtype == CACNN_F32 ? 4 : 2;
    const int64_t want = std::max<int64_t>(1, 128 / (int64_t)(v.TB * esz));
    int g_b = 1;
    for (int d = 1; d <= tiles_b && d <= want; ++d)
        if (tiles_b % d == 0) g_b = d;
    return g_b;
}

// -1: not simulated (too large)
double l2_model_words(const cacnn_problem& p, const TileGeom& tg, int a_k, int walk, const L2Machine& m2) {
    const int64_t tk = ceil_div(p.K, tg.KT), tb = ceil_div(p.B, tg.TB), tw = ceil_div(p.W, tg.TW), th = ceil_div(p.H, tg.TH);
    const int64_t npos = tb * tw * th, n_tiles = tk * npos, kpg = tk / a_k;
    const int64_t IW = p.sigma_w * (p.W - 1) + p.R, IH = p.sigma_h * (p.H - 1) + p.S;
    const int64_t XS = p.sigma_w * (tg.TW - 1) + p.R, YS = p.sigma_h * (tg.TH - 1) + p.S;
    if ((double)n_tiles > 1.0e5) return -1.0;     // the walk costs about half a microsecond per tile and candidate
    const int64_t q = n_tiles / m2.n_xcd, rem = n_tiles % m2.n_xcd;
    const int64_t per_xcd = std::max<int64_t>(1, tg.grid / m2.n_xcd);
    double total = 0.0;
    std::vector<int64_t> atoms;
    for (int x = 0; x < m2.n_xcd; ++x) {
        const int64_t lo = x * q + std::min<int64_t>(x, rem), hi = lo + q + (x < rem ? 1 : 0);
        // LRU over atom ids: id < tk is the Filter atom of a k-tile, tk + position tile the Image footprint of that tile.
        // Position tiles that overlap in their halo are separate atoms: measured, an XCD's L2 serves a line to the
        // workgroups of one position tile (they fetch it in the same microsecond) but has turned it over before a
        // neighbouring position tile asks for it.
        std::list<std::pair<int64_t, double>> lru;
        std::unordered_map<int64_t, std::list<std::pair<int64_t, double>>::iterator> where;
        double used = 0.0;
        for (int64_t n0 = lo; n0 < hi; n0 += per_xcd) {
            atoms.clear();
            for (int64_t t = n0; t < std::min(hi, n0 + per_xcd); ++t) {
                const int64_t kg = t / (kpg * npos), tl = t - kg * kpg * npos;
                int64_t k_l, pos;
                if (walk == 0) {
                    k_l = tl % kpg;
                    pos = tl / kpg;
                } else {
                    pos = tl % npos;
                    k_l = tl / npos;
                }
                const int64_t b_lo = pos % tg.b_group, w_i = (pos / tg.b_group) % tw, h_i = (pos / (tg.b_group * tw)) % th,
                              b_i = (pos / (tg.b_group * tw * th)) * tg.b_group + b_lo;
                atoms.push_back(kg * kpg + k_l);
                atoms.push_back(tk + (b_i * tw + w_i) * th + h_i);
            }
            std::sort(atoms.begin(), atoms.end());
            atoms.erase(std::unique(atoms.begin(), atoms.end()), atoms.end());
            for (int64_t id : atoms) {
                auto it = where.find(id);
                if (it != where.end()) {
                    lru.splice(lru.end(), lru, it->second);
                    continue;
                }
                double sz;
                if (id < tk) {
                    sz = (double)std::min<int64_t>(tg.KT, p.K - id * tg.KT) * (double)p.R * p.S * p.C;
                } else {
                    const int64_t pt = id - tk, h_i = pt % th, w_i = (pt / th) % tw, b_i = pt / (th * tw);
                    const int64_t xs = std::min(IW, p.sigma_w * w_i * tg.TW + XS) - p.sigma_w * w_i * tg.TW,
                                  ys = std::min(IH, p.sigma_h * h_i * tg.TH + YS) - p.sigma_h * h_i * tg.TH;
                    sz = (double)std::min<int64_t>(tg.TB, p.B - b_i * tg.TB) * (double)p.C * (double)(xs * ys);
                }
                total += sz;
                lru.emplace_back(id, sz);
                where[id] = std::prev(lru.end());
                used += sz;
                while (used > m2.words && lru.size() > 1) {
                    used -= lru.front().second;
                    where.erase(lru.front().first);
                    lru.pop_front();
                }
            }
        }
    }
    return total + (double)p.K * p.H * p.W * p.B;
}

struct L2Choice {
    int a_k = 1, walk = 0, n = 0;
    int cand_a_k[8] = {0}, cand_walk[8] = {0};
    double cand_words[8] = {0.0};
    double words = 0.0;
};

L2Choice choose_l2_layout(const cacnn_problem& p, int dtype, const VariantInfo& v, int64_t grid, const L2Machine& m2) {
    L2Choice c;
    const int64_t tk = ceil_div(p.K, v.KT());
    TileGeom tg{v.KT(), v.TB, v.TW, v.TH, b_group_of(v, dtype, ceil_div(p.B, v.TB)), grid};
    const int64_t n_tiles = tk * ceil_div(p.B, v.TB) * ceil_div(p.W, v.TW) * ceil_div(p.H, v.TH);
    for (int ak = 1; ak <= m2.n_xcd && ak <= 8; ak *= 2) {
        if (m2.n_xcd % ak || tk % ak) continue;
        for (int walk = 0; walk < 2; ++walk) {
            // the walk order only differs when a group has several k-tiles; its decoding needs n_tiles * npos < 2^32
            if (walk == 1 && (tk / ak < 2 || (double)n_tiles * (double)(n_tiles / tk) >= 4294967296.0)) continue;
            const double w = l2_model_words(p, tg, ak, walk, m2);
            if (w < 0.0) {
                c = L2Choice();
                c.a_k = choose_xcd_split_k(p, dtype, tk, m2.n_xcd);
                return c;
            }
            c.cand_a_k[c.n] = ak;
            c.cand_walk[c.n] = walk;
            c.cand_words[c.n] = w;
            // a later layout must save more than the few per cent the model is off by on the measured layouts
            if (c.n == 0 || w < 0.97 * c.words) {
                c.words = w;
                c.a_k = ak;
                c.walk = walk;
            }
            ++c.n;
        }
    }
    return c;
}

int fill_plan(const cacnn_problem& p, int dtype, const cacnn_machine& mach, const Choice& ch, cacnn_plan* out) {
    const VariantInfo& v = variant(ch.variant).info;
    const double esz = dtype == CACNN_F32 ? 4.0 : 2.0;
    const double M = (double)mach.lds_bytes / esz;
    std::memset(out, 0, sizeof(*out));
    if (M > 1.0) {
        const LpSolution s = solve_tiling_lp(p, M);
        for (int i = 0; i < 9; ++i) out->lp_tile[i] = std::pow(M, s.l[i]);
        out->lp_volume = std::pow(M, s.log_volume);
        const double F = (double)p.B * p.C * p.K * p.W * p.H * p.R * p.S;
        out->lp_cost_words = F * M / out->lp_volume;
        cacnn_bound b;
        bound_terms(p, M, &b);
        out->bound_words = b.bound;
        out->paper_case = appendix_a_case(p, M);
    }
    out->variant = ch.variant;
    out->b_b = v.TB;
    out->b_c = ch.g.CT;
    out->b_k = v.KT();
    out->b_w = v.TW;
    out->b_h = v.TH;
    out->b_r = ch.g.bR;
    out->b_s = ch.g.bS;
    out->b_r2 = (int32_t)std::min<int64_t>(p.sigma_w, ch.g.bR);
    out->b_r1 = (int32_t)ceil_div(ch.g.bR, std::max<int64_t>(1, std::min<int64_t>(p.sigma_w, p.R)));
    out->b_s2 = (int32_t)std::min<int64_t>(p.sigma_h, ch.g.bS);
    out->b_s1 = (int32_t)ceil_div(ch.g.bS, std::max<int64_t>(1, std::min<int64_t>(p.sigma_h, p.S)));
    out->grid[0] = (int32_t)launch_grid(v, ch.g, ch.n_wg, mach);
    out->grid[1] = 1;
    out->grid[2] = 1;
    out->block = v.threads();
    out->lds_bytes_used = ch.g.lds_bytes;
    out->tile_volume = (double)v.TB * ch.g.CT * v.KT() * v.TW * v.TH * ch.g.bR * ch.g.bS;
    double staged = ch.words;
    // a kernel that takes a tile's whole contraction as one unit keeps its Filter tile while the output channels stay
    // the same: with one k-tile it is staged once per workgroup, not once per Out tile
    if (v.fx_whole && ceil_div(p.K, v.KT()) == 1)
        staged = ch.img_words + (double)out->grid[0] * (double)p.K * p.R * p.S * p.C;
    out->predicted_words = staged + (double)p.K * p.H * p.W * p.B;
    {
        L2Machine m2 = kDefaultL2Bytes;
        m2.words /= esz;
        m2.n_xcd = xcd_count();
        const L2Choice l2 = choose_l2_layout(p, dtype, v, out->grid[0], m2);
        out->xcd_split_k = l2.a_k;
        out->xcd_walk = l2.walk;
    }
    return CACNN_OK;
}

// per-array element counts must fit the kernels' 31-bit tile arithmetic
int validate_dims(const cacnn_problem& pr) {
    const cacnn_problem* p = &pr;
    const int64_t IW = p->sigma_w * (p->W - 1) + p->R, IH = p->sigma_h * (p->H - 1) + p->S;
    int64_t t;
    const int64_t lim = INT32_MAX;
    if (p->sigma_w > lim || p->sigma_h > lim || p->W > lim || p->H > lim || p->R > lim || p->S > lim ||
        IW > lim || IH > lim || IW < 1 || IH < 1)
        return CACNN_ERR_INVALID_ARG;
    if (!mul_check(IW, IH, lim, &t) || !mul_check(t, p->C, lim, &t) || !mul_check(t, p->B, lim, &t))
        return CACNN_ERR_INVALID_ARG;
    if (!mul_check(p->K, p->R, lim, &t) || !mul_check(t, p->S, lim, &t) || !mul_check(t, p->C, lim, &t))
        return CACNN_ERR_INVALID_ARG;
    if (!mul_check(p->K, p->H, lim, &t) || !mul_check(t, p->W, lim, &t) || !mul_check(t, p->B, lim, &t))
        return CACNN_ERR_INVALID_ARG;
    return CACNN_OK;
}

int plan_impl(const cacnn_problem* p, int dtype, const cacnn_machine* machine, cacnn_plan* out,
              bool allow_pipelined = true) {
    if (!p || !out) return CACNN_ERR_NULL;
    if (!valid_problem(p)) return CACNN_ERR_INVALID_ARG;
    if (dtype != CACNN_F32 && dtype != CACNN_BF16_F32ACC) return CACNN_ERR_UNSUPPORTED;
    cacnn_machine mach = machine ? *machine : kDefaultMachine;
    if (mach.lds_bytes < 1024 || mach.num_cu < 1) return CACNN_ERR_INVALID_ARG;
    mach.lds_bytes = std::min<int64_t>(mach.lds_bytes, 160 * 1024);  // the kernels cannot address more
    {
        const int vrc = validate_dims(*p);
        if (vrc != CACNN_OK) return vrc;
    }
    Choice best;
    // Where a fixed-geometry kernel fits the problem and gives at least an eighth of the machine a tile, it has beaten
    // every generic kernel measured (by 2-3x on mid-size layers), and its cost above is a measurement while the
    // generic kernels' is a model: choose among those first.
    for (int vi = 0; vi < num_variants() && allow_pipelined; ++vi)
        if (variant(vi).info.dtype == dtype && variant(vi).info.fx_ct > 0) evaluate(vi, *p, mach, &best);
    // ... unless half or more of its tiles' outputs lie outside Out (fewer images than a tile holds, mostly): then the generic
    // kernels, which have tiles of 8 and 16 images, compete with it on the estimated time
    bool mostly_padding = false;
    if (best.variant >= 0) {
        const VariantInfo& bv = variant(best.variant).info;
        const double padded = (double)best.n_wg * bv.KT() * bv.NT();
        // (fp32: also where exactly half lie outside; the generic fp32 kernels' estimates are within 10 %, the bf16 ones' are
        // up to a third too low, and a half-empty bf16 tile was still the fastest on seven of seven such layers)
        const double useful = (double)p->B * p->K * p->W * p->H;
        mostly_padding = dtype == CACNN_F32 ? useful <= 0.5 * padded : useful < 0.5 * padded;
    }
    // ... or it is the fp32 kernel for 1 x 1 filters walking the taps of a larger filter, which re-stages the Image once
    // per tap: there the generic fp32 kernels, whose model is within 10 % of their measured times, win on some layers
    const bool f32_taps = best.variant >= 0 && dtype == CACNN_F32 && variant(best.variant).info.fx_any_stride && (p->R > 1 || p->S > 1);
    if (best.variant < 0 || best.n_wg * 8 < mach.num_cu || mostly_padding || f32_taps) {
        const bool use_lp = planner_uses_lp() && !((mostly_padding || f32_taps) && best.n_wg * 8 >= mach.num_cu);
        if (use_lp) best = Choice();
        // a bf16 fixed-geometry kernel that competes is given a head start of a quarter of its time: on such layers its
        // price was up to a quarter too high and the generic bf16 kernels' up to a quarter too low, and where the pick was
        // wrong the generic kernel lost up to 1.5 x, the fixed-geometry one 1.15 x
        const int fx_variant = best.variant;
        const double fx_cost = best.cost;
        if (fx_variant >= 0 && dtype != CACNN_F32) best.cost *= 0.75;
        const GpuLpTile lp = solve_gpu_lp(*p, dtype, mach);
        for (int vi = 0; vi < num_variants(); ++vi) {
            if (variant(vi).info.dtype != dtype) continue;
            if (variant(vi).info.pipelined && !allow_pipelined) continue;
            if (variant(vi).info.fx_ct > 0) continue;      // already in
            if (use_lp) evaluate_lp(vi, *p, mach, lp, &best);
            else evaluate(vi, *p, mach, &best);
        }
        if (best.variant == fx_variant && fx_variant >= 0) best.cost = fx_cost;
    }
    if (best.variant < 0) return CACNN_ERR_INVALID_ARG;  // nothing fits the given LDS size
    return fill_plan(*p, dtype, mach, best, out);
}

bool g_device_checked = false;
bool g_device_ok = false;
std::mutex g_mutex;

bool have_device() {
    std::lock_guard<std::mutex> lock(g_mutex);
    if (!g_device_checked) {
        int n = 0;
        const hipError_t e = hipGetDeviceCount(&n);
        if (e != hipSuccess) (void)hipGetLastError();
        g_device_ok = (e == hipSuccess && n > 0);
        g_device_checked = true;
    }
    return g_device_ok;
}

// layouts chosen by the two-level model for launches that name none, keyed by (problem, dtype, variant, grid): the model
// walks every tile of every candidate, which is host time a launch loop should pay once
struct LayoutEntry {
    cacnn_problem p;
    int dtype, vi;
    int64_t grid;
    int a_k, walk;
};
std::vector<LayoutEntry> g_layouts;

void cached_l2_layout(const cacnn_problem& p, int dtype, int vi, int64_t grid, const L2Machine& m2, int* a_k, int* walk) {
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        for (const LayoutEntry& e : g_layouts)
            if (e.dtype == dtype && e.vi == vi && e.grid == grid && std::memcmp(&e.p, &p, sizeof(cacnn_problem)) == 0) {
                *a_k = e.a_k;
                *walk = e.walk;
                return;
            }
    }
    const L2Choice l2 = choose_l2_layout(p, dtype, variant(vi).info, grid, m2);
    *a_k = l2.a_k;
    *walk = l2.walk;
    std::lock_guard<std::mutex> lock(g_mutex);
    if (g_layouts.size() >= 64) g_layouts.erase(g_layouts.begin());
    g_layouts.push_back(LayoutEntry{p, dtype, vi, grid, l2.a_k, l2.walk});
}

int launch_with(const cacnn_problem& p, int dtype, int vi, int CT, int bR, int bS, int split_k, int walk, const void* image,
                const void* filter, void* out, void* stream) {
    const Variant& var = variant(vi);
    const VariantInfo& v = var.info;
    const bool aligned_img = (reinterpret_cast<uintptr_t>(image) % 16) == 0;
    const bool aligned_flt = (reinterpret_cast<uintptr_t>(filter) % 16) == 0;
    const size_t esz = dtype == CACNN_F32 ? 4 : 2;
    if (reinterpret_cast<uintptr_t>(image) % esz || reinterpret_cast<uintptr_t>(filter) % esz ||
        reinterpret_cast<uintptr_t>(out) % 4)
        return CACNN_ERR_INVALID_ARG;
    const bool vimg = vec_img_ok(v, p) && aligned_img;
    const Geometry g = make_geometry(v, p, CT, bR, bS, vimg);
    if (!g.legal || g.lds_bytes > 160 * 1024 || g.lds_bytes < 1) return CACNN_ERR_UNSUPPORTED;
    if (v.pipelined && !aligned_flt && !g.flt_resident) return CACNN_ERR_UNSUPPORTED;

    KernelArgs a;
    std::memset(&a, 0, sizeof(a));
    a.image = image;
    a.filter = filter;
    a.out = (float*)out;
    a.B = (int32_t)p.B;
    a.C = (int32_t)p.C;
    a.K = (int32_t)p.K;
    a.W = (int32_t)p.W;
    a.H = (int32_t)p.H;
    a.R = (int32_t)p.R;
    a.S = (int32_t)p.S;
    a.sw = (int32_t)p.sigma_w;
    a.sh = (int32_t)p.sigma_h;
    a.IW = (int32_t)(p.sigma_w * (p.W - 1) + p.R);
    a.IH = (int32_t)(p.sigma_h * (p.H - 1) + p.S);
    a.bR = g.bR;
    a.bS = g.bS;
    a.CT = g.CT;
    a.XS = g.XS;
    a.YS = g.YS;
    a.xpitch = g.xpitch;
    a.ypitch = g.ypitch;
    a.fpitch = g.fpitch;
    a.QE = g.QE;
    a.img_lds_elems = g.img_lds_elems;
    a.zero_off = g.zero_off;
    a.tiles_k = (int32_t)ceil_div(p.K, v.KT());
    a.tiles_b = (int32_t)ceil_div(p.B, v.TB);
    a.tiles_w = (int32_t)ceil_div(p.W, v.TW);
    a.tiles_h = (int32_t)ceil_div(p.H, v.TH);
    a.vec_img = vimg ? 1 : 0;
    if (dtype == CACNN_F32)
        a.vec_flt = (aligned_flt && p.C % 4 == 0 && g.CT % 4 == 0) ? 1 : 0;
    else
        a.vec_flt = (aligned_flt && p.C % 8 == 0) ? 1 : 0;
    a.d_CT = make_fastdiv((uint32_t)g.CT);
    a.d_YS = make_fastdiv((uint32_t)g.YS);
    a.d_bS = make_fastdiv((uint32_t)g.bS);
    a.d_bR = make_fastdiv((uint32_t)g.bR);
    a.d_RS = make_fastdiv((uint32_t)(g.bR * g.bS));
    a.d_XS = make_fastdiv((uint32_t)g.XS);
    a.d_C4 = make_fastdiv((uint32_t)std::max(1, g.CT / 4));
    if (dtype == CACNN_F32)
        a.d_C8 = make_fastdiv((uint32_t)(a.vec_flt ? g.CT / 4 : g.CT));
    else
        a.d_C8 = make_fastdiv((uint32_t)(g.CT / 8));
    int64_t grid = 0, t = 0;
    if (!mul_check(a.tiles_k, a.tiles_b, INT32_MAX, &t) || !mul_check(t, a.tiles_w, INT32_MAX, &t) ||
        !mul_check(t, a.tiles_h, INT32_MAX, &grid))
        return CACNN_ERR_INVALID_ARG;
    a.n_tiles = (int32_t)grid;
    a.n_xcd = xcd_count();
    {
        // b-tiles that read different pieces of the same 128-byte Image lines stay adjacent in the tile order
        const int64_t want = std::max<int64_t>(1, 128 / (int64_t)(v.TB * esz));
        int g_b = 1;
        for (int d = 1; d <= a.tiles_b && d <= want; ++d)
            if (a.tiles_b % d == 0) g_b = d;
        a.b_group = g_b;
    }
    // tile-list decoding divides by launch constants with one multiply-high each, exact while dividend * divisor < 2^32
    if ((int64_t)a.n_tiles * std::max<int64_t>(std::max(a.tiles_k, a.tiles_w), std::max(a.tiles_h, 64)) >= (1ll << 32))
        return CACNN_ERR_INVALID_ARG;
    a.xcd_q = a.n_tiles / a.n_xcd;
    a.xcd_rem = a.n_tiles % a.n_xcd;
    a.d_nxcd = make_fastdiv((uint32_t)a.n_xcd);
    if (split_k == 0) {
        // no layout given: the two-level model's choice for this variant and grid
        L2Machine m2 = kDefaultL2Bytes;
        m2.words /= (double)esz;
        m2.n_xcd = a.n_xcd;
        cached_l2_layout(p, dtype, vi, launch_grid(v, g, grid, kDefaultMachine), m2, &split_k, &walk);
    }
    if (split_k < 1 || split_k > 8 || (split_k & (split_k - 1)) || a.tiles_k % split_k) return CACNN_ERR_INVALID_ARG;
    if (walk != 0 && walk != 1) return CACNN_ERR_INVALID_ARG;
    a.k_groups = split_k;
    a.kpg = a.tiles_k / split_k;
    a.grp = a.n_tiles / split_k;
    a.npos = a.grp / a.kpg;
    // positions fastest needs a division by the position tiles of a block: exact while n_tiles * npos < 2^32
    if (walk == 1 && (double)a.n_tiles * (double)a.npos >= 4294967296.0) return CACNN_ERR_INVALID_ARG;
    a.pos_fastest = walk;
    a.d_npos = make_fastdiv((uint32_t)a.npos);
    a.d_tk = make_fastdiv((uint32_t)a.kpg);
    a.d_bg = make_fastdiv((uint32_t)a.b_group);
    a.d_tw = make_fastdiv((uint32_t)a.tiles_w);
    a.d_th = make_fastdiv((uint32_t)a.tiles_h);
    a.img_items = g.img_items;
    a.flt_items = g.flt_items;
    a.img_buf = g.img_buf;
    a.flt_buf = g.flt_buf;
    a.flt_off = g.flt_off;
    a.flt_resident = g.flt_resident;
    grid = launch_grid(v, g, grid, kDefaultMachine);
    if (!have_device()) return CACNN_ERR_NO_DEVICE;
    return var.launch(a, (int)grid, (size_t)g.lds_bytes, stream) == 0 ? CACNN_OK : CACNN_ERR_LAUNCH;
}

// plan cache of cacnn_conv_forward, keyed by (problem, dtype | misaligned << 8)
struct PlanEntry {
    cacnn_problem p;
    int key;
    cacnn_plan plan;
};
std::vector<PlanEntry> g_plans;

bool lookup_plan(const cacnn_problem& p, int key, cacnn_plan* out) {
    std::lock_guard<std::mutex> lock(g_mutex);
    for (const PlanEntry& e : g_plans)
        if (e.key == key && std::memcmp(&e.p, &p, sizeof(cacnn_problem)) == 0) {
            *out = e.plan;
            return true;
        }
    return false;
}

void store_plan(const cacnn_problem& p, int key, const cacnn_plan& plan) {
    std::lock_guard<std::mutex> lock(g_mutex);
    for (PlanEntry& e : g_plans)
        if (e.key == key && std::memcmp(&e.p, &p, sizeof(cacnn_problem)) == 0) {
            e.plan = plan;
            return;
        }
    if (g_plans.size() >= 64) g_plans.erase(g_plans.begin());
    g_plans.push_back(PlanEntry{p, key, plan});
}

}  // namespace

extern "C" {

int cacnn_lower_bound(const cacnn_problem* problem, double M_words, cacnn_bound* out) {
    if (!problem || !out) return CACNN_ERR_NULL;
    if (!valid_problem(problem) || !(M_words > 0.0) || !std::isfinite(M_words)) return CACNN_ERR_INVALID_ARG;
    bound_terms(*problem, M_words, out);
    return CACNN_OK;
}

int cacnn_tile_plan(const cacnn_problem* problem, int dtype, const cacnn_machine* machine, cacnn_plan* out) {
    return plan_impl(problem, dtype, machine, out);
}

int cacnn_conv_forward(const cacnn_problem* problem, int dtype, const void* image, const void* filter, void* out,
                       void* hip_stream) {
    if (!problem || !image || !filter || !out) return CACNN_ERR_NULL;
    if (dtype != CACNN_F32 && dtype != CACNN_BF16_F32ACC) return CACNN_ERR_UNSUPPORTED;
    // plans are cached per (problem, dtype): planning costs tens of microseconds, a launch a few.
    // The pipelined kernels need 16-byte aligned operands; a misaligned call is planned without them.
    const bool aligned = reinterpret_cast<uintptr_t>(image) % 16 == 0 && reinterpret_cast<uintptr_t>(filter) % 16 == 0;
    const int key = dtype | (aligned ? 0 : 0x100);
    cacnn_plan plan;
    if (!lookup_plan(*problem, key, &plan)) {
        const int rc = plan_impl(problem, dtype, nullptr, &plan, aligned);
        if (rc != CACNN_OK) return rc;
        store_plan(*problem, key, plan);
    }
    return launch_with(*problem, dtype, plan.variant, plan.b_c, plan.b_r, plan.b_s, plan.xcd_split_k, plan.xcd_walk, image, filter, out,
                       hip_stream);
}

int cacnn_conv_forward_with_plan(const cacnn_problem* problem, int dtype, const cacnn_plan* plan, const void* image,
                                 const void* filter, void* out, void* hip_stream) {
    if (!problem || !plan || !image || !filter || !out) return CACNN_ERR_NULL;
    if (dtype != CACNN_F32 && dtype != CACNN_BF16_F32ACC) return CACNN_ERR_UNSUPPORTED;
    if (!valid_problem(problem)) return CACNN_ERR_INVALID_ARG;
    const int rc = validate_dims(*problem);
    if (rc != CACNN_OK) return rc;
    if (plan->variant < 0 || plan->variant >= num_variants()) return CACNN_ERR_UNSUPPORTED;
    const VariantInfo& v = variant(plan->variant).info;
    if (v.dtype != dtype) return CACNN_ERR_UNSUPPORTED;
    if (plan->b_c < 1 || plan->b_r < 1 || plan->b_s < 1) return CACNN_ERR_INVALID_ARG;
    const int64_t Cpad = round_up(problem->C, v.cgran());
    // (a fixed-geometry kernel's c-slice is its own, also where it exceeds a small C)
    const int CT = v.fx_ct > 0 && plan->b_c == v.fx_ct ? v.fx_ct : (int)std::min<int64_t>(round_up(plan->b_c, v.cgran()), Cpad);
    const int bR = (int)std::min<int64_t>(plan->b_r, problem->R);
    const int bS = (int)std::min<int64_t>(plan->b_s, problem->S);
    if (plan->xcd_split_k < 0) return CACNN_ERR_INVALID_ARG;
    return launch_with(*problem, dtype, plan->variant, CT, bR, bS, plan->xcd_split_k, plan->xcd_walk, image, filter, out, hip_stream);
}

int cacnn_parallel_bound(const cacnn_problem* problem, double M_words, const cacnn_division* a, cacnn_bound* out) {
    if (!problem || !a || !out) return CACNN_ERR_NULL;
    if (!valid_problem(problem) || !(M_words > 0.0) || !std::isfinite(M_words)) return CACNN_ERR_INVALID_ARG;
    const cacnn_problem& p = *problem;
    if (a->a_b < 1 || a->a_k < 1 || a->a_w < 1 || a->a_h < 1 || a->a_b > p.B || a->a_k > p.K || a->a_w > p.W ||
        a->a_h > p.H)
        return CACNN_ERR_INVALID_ARG;
    parallel_terms(p, M_words, a->a_b, a->a_k, a->a_w, a->a_h, out);
    return CACNN_OK;
}

int cacnn_work_division(const cacnn_problem* problem, double M_words, int32_t p_count, cacnn_division* out_a,
                        cacnn_bound* out_bound) {
    if (!problem || !out_a || !out_bound) return CACNN_ERR_NULL;
    if (!valid_problem(problem) || !(M_words > 0.0) || !std::isfinite(M_words) || p_count < 1 || p_count > 4096)
        return CACNN_ERR_INVALID_ARG;
    const cacnn_problem& p = *problem;
    bool have = false;
    int64_t best_prod = 0;
    double best_rep = 0.0;
    cacnn_division best_a = {1, 1, 1, 1};
    cacnn_bound best_b;
    std::memset(&best_b, 0, sizeof(best_b));
    // every admissible division, in lexicographic order (so the first of equals is the lexicographically smallest)
    for (int64_t ab = 1; ab <= std::min<int64_t>(p.B, p_count); ++ab)
        for (int64_t ak = 1; ak <= std::min<int64_t>(p.K, p_count / ab); ++ak)
            for (int64_t aw = 1; aw <= std::min<int64_t>(p.W, p_count / (ab * ak)); ++aw)
                for (int64_t ah = 1; ah <= std::min<int64_t>(p.H, p_count / (ab * ak * aw)); ++ah) {
                    cacnn_bound b;
                    parallel_terms(p, M_words, ab, ak, aw, ah, &b);
                    const int64_t prod = ab * ak * aw * ah;
                    const double rep = b.term[1] + b.term[2];
                    const bool better = !have || prod > best_prod ||
                                        (prod == best_prod && (b.bound < best_b.bound ||
                                                               (b.bound == best_b.bound && rep < best_rep)));
                    if (better) {
                        have = true;
                        best_prod = prod;
                        best_rep = rep;
                        best_b = b;
                        best_a = cacnn_division{(int32_t)ab, (int32_t)ak, (int32_t)aw, (int32_t)ah};
                    }
                }
    *out_a = best_a;
    *out_bound = best_b;
    return CACNN_OK;
}

int cacnn_tune(const cacnn_problem* problem, int dtype, const void* image, const void* filter, void* out, void* hip_stream,
               cacnn_plan* out_plan) {
    if (!problem || !image || !filter || !out) return CACNN_ERR_NULL;
    if (dtype != CACNN_F32 && dtype != CACNN_BF16_F32ACC) return CACNN_ERR_UNSUPPORTED;
    if (!valid_problem(problem)) return CACNN_ERR_INVALID_ARG;
    {
        const int vrc = validate_dims(*problem);
        if (vrc != CACNN_OK) return vrc;
    }
    if (!have_device()) return CACNN_ERR_NO_DEVICE;
    const bool aligned = reinterpret_cast<uintptr_t>(image) % 16 == 0 && reinterpret_cast<uintptr_t>(filter) % 16 == 0;
    const int key = dtype | (aligned ? 0 : 0x100);
    hipStream_t stream = (hipStream_t)hip_stream;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return CACNN_ERR_LAUNCH;
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        return CACNN_ERR_LAUNCH;
    }
    // every kernel variant that accepts the problem, each with the contraction tile the cost model likes best for it
    Choice best;
    float best_ms = 0.f;
    int status = CACNN_ERR_UNSUPPORTED;
    for (int vi = 0; vi < num_variants(); ++vi) {
        const VariantInfo& v = variant(vi).info;
        if (v.dtype != dtype || (v.pipelined && !aligned)) continue;
        Choice c;
        if (!evaluate(vi, *problem, kDefaultMachine, &c)) continue;
        constexpr int WARM = 2, TIMED = 5;
        bool ok = true;
        for (int i = 0; i < WARM + TIMED && ok; ++i) {
            if (i == WARM) ok = hipEventRecord(e0, stream) == hipSuccess;
            ok = ok && launch_with(*problem, dtype, vi, c.g.CT, c.g.bR, c.g.bS, 0, 0, image, filter, out, hip_stream) == CACNN_OK;
        }
        if (!ok) continue;
        float ms = 0.f;
        if (hipEventRecord(e1, stream) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
            hipEventElapsedTime(&ms, e0, e1) != hipSuccess) {
            status = CACNN_ERR_LAUNCH;
            continue;
        }
        if (best.variant < 0 || ms < best_ms) {
            best = c;
            best_ms = ms;
        }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (best.variant < 0) return status;
    cacnn_plan plan;
    const int rc = fill_plan(*problem, dtype, kDefaultMachine, best, &plan);
    if (rc != CACNN_OK) return rc;
    store_plan(*problem, key, plan);
    if (out_plan) *out_plan = plan;
    return CACNN_OK;
}

int cacnn_plan_variant(const cacnn_problem* problem, int dtype, int variant_index, cacnn_plan* out, double* model_us,
                       double* model_terms) {
    if (!problem || !out) return CACNN_ERR_NULL;
    if (!valid_problem(problem)) return CACNN_ERR_INVALID_ARG;
    if (dtype != CACNN_F32 && dtype != CACNN_BF16_F32ACC) return CACNN_ERR_UNSUPPORTED;
    if (variant_index < 0 || variant_index >= num_variants() || variant(variant_index).info.dtype != dtype)
        return CACNN_ERR_UNSUPPORTED;
    {
        const int vrc = validate_dims(*problem);
        if (vrc != CACNN_OK) return vrc;
    }
    Choice c;
    if (!evaluate(variant_index, *problem, kDefaultMachine, &c)) return CACNN_ERR_UNSUPPORTED;
    if (model_us) *model_us = c.cost / 2400.0;
    if (model_terms)
        for (int i = 0; i < 5; ++i) model_terms[i] = c.terms[i];
    return fill_plan(*problem, dtype, kDefaultMachine, c, out);
}

int cacnn_two_level_plan(const cacnn_problem* problem, int dtype, const cacnn_machine* machine,
                         const cacnn_machine_l2* machine_l2, cacnn_l2_plan* out) {
    if (!problem || !out) return CACNN_ERR_NULL;
    cacnn_plan plan;
    const int rc = plan_impl(problem, dtype, machine, &plan);
    if (rc != CACNN_OK) return rc;
    const cacnn_problem& p = *problem;
    const double esz = dtype == CACNN_F32 ? 4.0 : 2.0;
    L2Machine m2 = kDefaultL2Bytes;
    if (machine_l2) {
        if (machine_l2->l2_bytes < 1024 || machine_l2->n_xcd < 1 || machine_l2->n_xcd > 8 ||
            (machine_l2->n_xcd & (machine_l2->n_xcd - 1)) || machine_l2->cu_per_xcd < 1)
            return CACNN_ERR_INVALID_ARG;
        m2.words = (double)machine_l2->l2_bytes;
        m2.n_xcd = machine_l2->n_xcd;
        m2.cu_per_xcd = machine_l2->cu_per_xcd;
    }
    m2.words /= esz;
    std::memset(out, 0, sizeof(*out));
    const double M = m2.words;
    const LpSolution s = solve_tiling_lp(p, M);
    for (int i = 0; i < 9; ++i) out->lp_tile[i] = std::pow(M, s.l[i]);
    out->lp_volume = std::pow(M, s.log_volume);
    out->lp_cost_words = (double)p.B * p.C * p.K * p.W * p.H * p.R * p.S * M / out->lp_volume;
    cacnn_bound b;
    bound_terms(p, M, &b);
    out->bound_words = b.bound;
    // the LP's tile rounded to whole LDS tiles
    auto whole = [](double lp, int tile, int64_t extent) {
        const int64_t n = std::max<int64_t>(1, (int64_t)std::floor(lp / tile + 0.5));
        return (int32_t)std::min<int64_t>(n * tile, round_up(extent, tile));
    };
    out->l2_tile_b = whole(out->lp_tile[0], plan.b_b, p.B);
    out->l2_tile_k = whole(out->lp_tile[2], plan.b_k, p.K);
    out->l2_tile_w = whole(out->lp_tile[3], plan.b_w, p.W);
    out->l2_tile_h = whole(out->lp_tile[4], plan.b_h, p.H);
    const VariantInfo& v = variant(plan.variant).info;
    const int64_t grid = machine_l2 ? std::min<int64_t>(plan.grid[0], (int64_t)m2.n_xcd * m2.cu_per_xcd) : plan.grid[0];
    const L2Choice l2 = choose_l2_layout(p, dtype, v, grid, m2);
    out->a_k = l2.a_k;
    out->walk = l2.walk;
    out->n_candidates = l2.n;
    for (int i = 0; i < l2.n; ++i) {
        out->cand_a_k[i] = l2.cand_a_k[i];
        out->cand_walk[i] = l2.cand_walk[i];
        out->cand_words[i] = l2.cand_words[i];
    }
    out->chosen_words = l2.words;
    {
        // Section 7 for the chosen a_K, the positions divided over the remaining processors: images, then rows, then columns
        int64_t rest = m2.n_xcd / l2.a_k, ab = 1, ah = 1, aw = 1;
        for (int64_t* a : {&ab, &ah, &aw}) {
            const int64_t extent = a == &ab ? p.B : (a == &ah ? p.H : p.W);
            while (*a * 2 <= std::min<int64_t>(rest, extent)) *a *= 2;
            rest /= *a;
        }
        cacnn_bound pb;
        parallel_terms(p, M, ab, l2.a_k, aw, ah, &pb);
        out->parallel_bound_words = pb.bound;
    }
    return CACNN_OK;
}

int cacnn_pool_lower_bound(const cacnn_problem* problem, double M_words, cacnn_pool_bound* out) {
    if (!problem || !out) return CACNN_ERR_NULL;
    if (!valid_problem(problem) || !(M_words > 0.0) || !std::isfinite(M_words)) return CACNN_ERR_INVALID_ARG;
    const cacnn_problem& p = *problem;
    const double sw = (double)std::min(p.sigma_w, p.R), sh = (double)std::min(p.sigma_h, p.S);
    const double bkwh = (double)p.B * p.K * p.W * p.H, bcwh = (double)p.B * p.C * p.W * p.H;
    out->term[0] = bkwh;
    out->term[1] = sw * sh * bcwh;
    out->term[2] = bkwh * (double)p.C * p.R * p.S / M_words;
    out->argmax = 0;
    for (int i = 1; i < 3; ++i)
        if (out->term[i] > out->term[out->argmax]) out->argmax = i;
    out->bound = out->term[out->argmax];
    return CACNN_OK;
}

int cacnn_pool_forward(const cacnn_problem* problem, int dtype, int mode, const void* image, void* out,
                       void* hip_stream) {
    if (!problem || !image || !out) return CACNN_ERR_NULL;
    if (dtype != CACNN_F32 && dtype != CACNN_BF16_F32ACC) return CACNN_ERR_UNSUPPORTED;
    if (mode != CACNN_POOL_AVG && mode != CACNN_POOL_MAX) return CACNN_ERR_UNSUPPORTED;
    if (!valid_problem(problem) || problem->K != problem->C) return CACNN_ERR_INVALID_ARG;
    const cacnn_problem& p = *problem;
    {
        // element counts of Image and Out within the kernel's 32-bit indexing
        const int64_t lim = INT32_MAX;
        if (p.sigma_w > lim || p.sigma_h > lim || p.W > lim || p.H > lim || p.R > lim || p.S > lim) return CACNN_ERR_INVALID_ARG;
        const int64_t IW = p.sigma_w * (p.W - 1) + p.R, IH = p.sigma_h * (p.H - 1) + p.S;
        int64_t t;
        if (IW > lim || IH > lim || !mul_check(IW, IH, lim, &t) || !mul_check(t, p.C, lim, &t) || !mul_check(t, p.B, lim, &t))
            return CACNN_ERR_INVALID_ARG;
        if (!mul_check(p.K, p.H, lim, &t) || !mul_check(t, p.W, lim, &t) || !mul_check(t, p.B, lim, &t))
            return CACNN_ERR_INVALID_ARG;
    }
    const size_t esz = dtype == CACNN_F32 ? 4 : 2;
    if (reinterpret_cast<uintptr_t>(image) % esz || reinterpret_cast<uintptr_t>(out) % 4) return CACNN_ERR_INVALID_ARG;
    const int full = dtype == CACNN_F32 ? 4 : 8;
    const bool wide = p.B % full == 0 && reinterpret_cast<uintptr_t>(image) % 16 == 0 &&
                      reinterpret_cast<uintptr_t>(out) % 16 == 0;
    const int vec = wide ? full : 1;
    PoolArgs a;
    std::memset(&a, 0, sizeof(a));
    a.image = image;
    a.out = (float*)out;
    a.B = (int32_t)p.B;
    a.C = (int32_t)p.C;
    a.W = (int32_t)p.W;
    a.H = (int32_t)p.H;
    a.R = (int32_t)p.R;
    a.S = (int32_t)p.S;
    a.sw = (int32_t)p.sigma_w;
    a.sh = (int32_t)p.sigma_h;
    a.IH = (int32_t)(p.sigma_h * (p.H - 1) + p.S);
    a.BV = (int32_t)(p.B / vec);
    a.n_xcd = xcd_count();
    a.TWC = (int32_t)ceil_div(p.W, a.n_xcd);              // one band of output columns per XCD
    const int64_t chunks = ceil_div(p.W, a.TWC);
    int64_t n = 0;
    if (!mul_check(p.H, chunks * a.TWC, INT32_MAX, &n) || !mul_check(n, p.C, INT32_MAX, &n) ||
        !mul_check(n, a.BV, INT32_MAX, &n))
        return CACNN_ERR_INVALID_ARG;
    a.n_threads = (int32_t)n;
    a.n_wg = (int32_t)ceil_div(n, 256);
    // the reciprocal divisions in the kernel are exact while dividend * divisor < 2^32
    if ((double)n * (double)std::max<int64_t>(std::max<int64_t>(a.BV, p.C), std::max<int64_t>(p.H, 64)) >= 4294967296.0)
        return CACNN_ERR_INVALID_ARG;
    a.xcd_q = a.n_wg / a.n_xcd;
    a.xcd_rem = a.n_wg % a.n_xcd;
    a.d_BV = make_fastdiv((uint32_t)a.BV);
    a.d_C = make_fastdiv((uint32_t)a.C);
    a.d_TWC = make_fastdiv((uint32_t)a.TWC);
    a.d_H = make_fastdiv((uint32_t)a.H);
    a.d_nxcd = make_fastdiv((uint32_t)a.n_xcd);
    if (!have_device()) return CACNN_ERR_NO_DEVICE;
    return launch_pool(a, dtype, mode, vec, hip_stream) == 0 ? CACNN_OK : CACNN_ERR_LAUNCH;
}

int cacnn_probe_mfma(int dtype, const void* operands, float* sink, int32_t iters, int64_t* mfma_issued, void* hip_stream) {
    if (!operands || !sink || !mfma_issued) return CACNN_ERR_NULL;
    if (dtype != CACNN_F32 && dtype != CACNN_BF16_F32ACC) return CACNN_ERR_UNSUPPORTED;
    if (iters < 1 || iters > (1 << 24) || reinterpret_cast<uintptr_t>(operands) % 16 || reinterpret_cast<uintptr_t>(sink) % 4)
        return CACNN_ERR_INVALID_ARG;
    if (!have_device()) return CACNN_ERR_NO_DEVICE;
    const int grid = kDefaultMachine.num_cu;
    *mfma_issued = (int64_t)grid * 4 * iters * 42;
    return launch_mfma_probe(dtype, operands, sink, iters, grid, hip_stream) == 0 ? CACNN_OK : CACNN_ERR_LAUNCH;
}

int cacnn_probe_lds_fill(const void* src, size_t window_bytes, float* sink, int32_t iters, void* hip_stream, int64_t* bytes_moved) {
    if (!src || !sink || !bytes_moved) return CACNN_ERR_NULL;
    if (window_bytes < 65536 || window_bytes > (1ull << 30) || (window_bytes & (window_bytes - 1)) || iters < 1 ||
        iters > (1 << 20) || reinterpret_cast<uintptr_t>(src) % 16)
        return CACNN_ERR_INVALID_ARG;
    if (!have_device()) return CACNN_ERR_NO_DEVICE;
    const int grid = kDefaultMachine.num_cu;
    *bytes_moved = (int64_t)grid * 4 * 12 * 1024 * iters;
    return launch_lds_fill_probe(src, (uint32_t)window_bytes, iters, sink, grid, hip_stream) == 0 ? CACNN_OK : CACNN_ERR_LAUNCH;
}

int cacnn_probe_mfma_and_fill(const void* operands, const void* src, size_t window_bytes, float* sink, int32_t mfma_iters,
                              int32_t fill_iters, void* hip_stream) {
    return cacnn_probe_mfma_and_fill_on((int32_t)kDefaultMachine.num_cu, 0, 0, operands, src, window_bytes, sink, mfma_iters,
                                        fill_iters, hip_stream);
}

int cacnn_probe_mfma_and_fill_on(int32_t compute_units, int32_t tile, int32_t mode, const void* operands, const void* src,
                                 size_t window_bytes, float* sink, int32_t mfma_iters, int32_t fill_iters, void* hip_stream) {
    if (!operands || !src || !sink) return CACNN_ERR_NULL;
    // mode: bit 0 = operands read from LDS, bit 1 = a workgroup barrier per iteration (equal iteration counts only)
    if (compute_units < 1 || compute_units > kDefaultMachine.num_cu || mode < 0 || mode > 3 || (tile != 0 && tile != 1))
        return CACNN_ERR_INVALID_ARG;
    if ((mode & 2) && mfma_iters != fill_iters) return CACNN_ERR_INVALID_ARG;
    if (window_bytes < 65536 || window_bytes > (32u << 20) || (window_bytes & (window_bytes - 1)) || mfma_iters < 0 ||
        fill_iters < 0 || mfma_iters > (1 << 20) || fill_iters > (1 << 20) || (mfma_iters == 0 && fill_iters == 0) ||
        reinterpret_cast<uintptr_t>(src) % 16 || reinterpret_cast<uintptr_t>(operands) % 16)
        return CACNN_ERR_INVALID_ARG;
    if (!have_device()) return CACNN_ERR_NO_DEVICE;
    return launch_mfma_and_fill_probe(tile, operands, src, (uint32_t)window_bytes, mfma_iters, fill_iters, mode & 1, (mode >> 1) & 1, sink, compute_units,
                                      hip_stream) == 0
               ? CACNN_OK
               : CACNN_ERR_LAUNCH;
}

int cacnn_probe_copy(const void* src, void* dst, size_t bytes, void* hip_stream) {
    if (!src || !dst) return CACNN_ERR_NULL;
    if (bytes == 0 || bytes % 16 || reinterpret_cast<uintptr_t>(src) % 16 || reinterpret_cast<uintptr_t>(dst) % 16)
        return CACNN_ERR_INVALID_ARG;
    if (!have_device()) return CACNN_ERR_NO_DEVICE;
    return launch_copy_probe(src, dst, bytes, kDefaultMachine.num_cu * 8, hip_stream) == 0 ? CACNN_OK : CACNN_ERR_LAUNCH;
}

// Section 5.1: the tabulated closed form.  theta is clamped into the tabulated box first; a region is a set of faces
// a.theta <= b with integer coefficients, its form nine integer rows over a common denominator.
int cacnn_closed_form_tiling(const cacnn_problem* p, double M, cacnn_closed_form* out) {
    if (!p || !out) return CACNN_ERR_NULL;
    if (!valid_problem(p) || !(M > 1.0)) return CACNN_ERR_INVALID_ARG;
    std::memset(out, 0, sizeof(*out));
    const double lnM = std::log(M);
    auto lg = [&](int64_t v) { return std::log((double)v) / lnM; };
    double th[9] = {lg(p->B), lg(p->C), lg(p->K), lg(p->W), lg(p->H), lg(p->R), lg(p->S), lg(p->sigma_w), lg(p->sigma_h)};
    for (int i = 0; i < 5; ++i) th[i] = std::min(th[i], 1.0);
    for (int i = 0; i < 2; ++i) {       // (R, sigma_w), (S, sigma_h): the LP sees min(sigma, extent) and extent / sigma
        double sg = std::min(th[7 + i], th[5 + i]);
        const double rest = std::min(th[5 + i] - sg, 1.0);
        sg = std::min(sg, 1.0);
        th[7 + i] = sg;
        th[5 + i] = sg + rest;
    }
    int best = 0;
    double best_v = std::numeric_limits<double>::infinity();
    for (int r = 0; r < kClosedFormRegions; ++r) {
        double worst = -std::numeric_limits<double>::infinity();
        for (int f = kClosedFormRegion[r][0]; f < kClosedFormRegion[r][0] + kClosedFormRegion[r][1]; ++f) {
            double v = -(double)kClosedFormFace[f][9];
            for (int j = 0; j < 9; ++j) v += (double)kClosedFormFace[f][j] * th[j];
            worst = std::max(worst, v);
        }
        if (worst < best_v) {
            best_v = worst;
            best = r;
        }
        if (worst <= 1e-12) break;
    }
    const int form = kClosedFormRegion[best][2];
    out->region = best;
    out->n_regions = kClosedFormRegions;
    double sum = 0.0;
    for (int i = 0; i < 9; ++i) {
        double v = (double)kClosedFormNum[form][i][9];
        for (int j = 0; j < 9; ++j) v += (double)kClosedFormNum[form][i][j] * th[j];
        v /= (double)kClosedFormDen[form];
        out->theta[i] = th[i];
        out->l[i] = std::max(v, 0.0);
        out->tile[i] = std::pow(M, out->l[i]);
        sum += out->l[i];
    }
    // how far l is from satisfying the LP's rows (the same rows solve_tiling_lp builds)
    {
        const double* l = out->l;
        const double rows[15] = {l[0] - th[0], l[1] - th[1], l[2] - th[2], l[3] - th[3], l[4] - th[4], l[6] - th[7], l[8] - th[8],
                                 l[5] - (th[5] - th[7]), l[7] - (th[6] - th[8]),
                                 l[0] + l[2] + l[3] + l[4] - 1.0, l[1] + l[2] + l[5] + l[6] + l[7] + l[8] - 1.0,
                                 l[0] + l[1] + l[3] + l[4] + l[6] + l[8] - 1.0, l[0] + l[1] + l[3] + l[7] + l[6] + l[8] - 1.0,
                                 l[0] + l[1] + l[5] + l[4] + l[6] + l[8] - 1.0, l[0] + l[1] + l[5] + l[7] + l[6] + l[8] - 1.0};
        double worst = 0.0;
        for (double v : rows) worst = std::max(worst, v);
        out->worst_violation = worst;
    }
    out->log_volume = sum;
    out->volume = std::pow(M, sum);
    const double F = (double)p->B * p->C * p->K * p->W * p->H * p->R * p->S;
    out->cost_words = F * M / out->volume;
    cacnn_bound b;
    bound_terms(*p, M, &b);
    out->bound_words = b.bound;
    return CACNN_OK;
}

int cacnn_variant_count(void) { return num_variants(); }

const char* cacnn_variant_name(int i) {
    if (i < 0 || i >= num_variants()) return nullptr;
    return variant(i).info.name;
}

const char* cacnn_status_string(int status) {
    switch (status) {
        case CACNN_OK: return "ok";
        case CACNN_ERR_NULL: return "null pointer argument";
        case CACNN_ERR_INVALID_ARG: return "invalid argument";
        case CACNN_ERR_UNSUPPORTED: return "unsupported dtype, variant or plan";
        case CACNN_ERR_LAUNCH: return "kernel launch failed";
        case CACNN_ERR_NO_DEVICE: return "no usable GPU";
        default: return "unknown status";
    }
}

}  // extern "C"
