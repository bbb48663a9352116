/*
 * CPU oracle for sensitivity-guided, row-parallel, Hessian-compensated layer
 * quantization.  TEST INFRASTRUCTURE ONLY: plain, slow, fp64, written from the
 * paper's equations.  It shares no code with the GPU library and must never be
 * reached from the product path; only the tests, the smoke check and the
 * "cpu_baseline" leg of the benchmark call it.
 *
 * Notation follows the paper: W is d_row x d_col (row-major, fp32 input),
 * X is d_col x N (row-major, fp32 input), Hinv is the inverse of the damped
 * Hessian, "quant" is rounding onto a fixed uniform grid.
 *
 * What each routine follows:
 *   oracle_hessian        Section 3, Eq. 2: the layer objective |WX - W^X|^2 is
 *                         quadratic in each row of W with Hessian 2 X X^T; the
 *                         build divides by the number of calibration columns N.
 *   oracle_damp           Section 6.1 (implementation details): a damping value
 *                         is added to the diagonal of H.
 *   oracle_spd_inverse    Section 5, item 1: Cholesky factor, then the inverse
 *                         from the factor.
 *   oracle_grid           Section 3 (OBQ paragraph): "a fixed grid of width
 *                         Delta"; here the asymmetric min-max grid per row or
 *                         per (row, column group), frozen from the original W.
 *   oracle_sensitivity    Section 3, Eq. 10 and Section 4.2 steps 1-2:
 *                         L = (quant(w) - w)^2 / (2 [Hinv]_jj), S_j = sum_i L_ij.
 *   oracle_order          Section 4.2 step 3: columns by S_j, descending.
 *   oracle_column_key,    Section 4.1 and Table 3: the other sort keys of the ablation
 *   oracle_order_dir      ("err" = summed squared quantization error, "w" = summed squared
 *                         weight, "sensi" = S_j) and both directions ("des", "asc").
 *   oracle_column_loop    Section 4.2 steps 4-5 with Eq. 9 (row form of Eq. 11)
 *                         and Eq. 12: quantize a whole column, push the error
 *                         into the columns not yet quantized, eliminate the
 *                         column from the one shared Hinv.
 *   oracle_loss_eval      Section 3, Eq. 4: 1/2 dw^T H dw summed over rows.
 *
 * Everything is fp64 and in the order the paper states; the only parallelism
 * is OpenMP over independent rows / matrix entries (and "omp simd" on the long
 * dot products, whose summation order the definitions do not fix).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_EINVAL -1
#define ORACLE_ENOMEM -2
#define ORACLE_ENOTPD -4

/* Number of OpenMP threads the parallel loops below will use. */
int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* H = (2/N) X X^T, X given as fp32 d x N with row stride ld.  Full d x d. */
int oracle_hessian(const float *X, int64_t d, int64_t N, int64_t ld, double *H)
{
    if (!X || !H || d <= 0 || N <= 0 || ld < N) return ORACLE_EINVAL;
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t a = 0; a < d; ++a) {
        const float *xa = X + a * ld;
        for (int64_t b = 0; b <= a; ++b) {
            const float *xb = X + b * ld;
            double s = 0.0;
#pragma omp simd reduction(+ : s)
            for (int64_t n = 0; n < N; ++n) s += (double)xa[n] * (double)xb[n];
            s = 2.0 * s / (double)N;
            H[a * d + b] = s;
            H[b * d + a] = s;
        }
    }
    return ORACLE_OK;
}

/* H += (damp * mean(diag H) + damp_abs) I.  Returns the addend via *lambda. */
int oracle_damp(double *H, int64_t d, double damp, double damp_abs, double *lambda)
{
    if (!H || d <= 0) return ORACLE_EINVAL;
    double tr = 0.0;
    for (int64_t a = 0; a < d; ++a) tr += H[a * d + a];
    double lam = damp * (tr / (double)d) + damp_abs;
    for (int64_t a = 0; a < d; ++a) H[a * d + a] += lam;
    if (lambda) *lambda = lam;
    return ORACLE_OK;
}

/* Hinv = H^-1 for symmetric positive definite H: H = L L^T, then L^-1 by
 * forward substitution, then Hinv = L^-T L^-1. */
int oracle_spd_inverse(const double *H, int64_t d, double *Hinv)
{
    if (!H || !Hinv || d <= 0) return ORACLE_EINVAL;
    double *L = (double *)calloc((size_t)d * d, sizeof(double));
    double *Li = (double *)calloc((size_t)d * d, sizeof(double));
    if (!L || !Li) { free(L); free(Li); return ORACLE_ENOMEM; }
    int status = ORACLE_OK;
    /* Cholesky, column by column: the diagonal entry, then the column below it. */
    for (int64_t b = 0; b < d && status == ORACLE_OK; ++b) {
        double s = H[b * d + b];
        for (int64_t k = 0; k < b; ++k) s -= L[b * d + k] * L[b * d + k];
        if (!(s > 0.0)) { status = ORACLE_ENOTPD; break; }
        const double lbb = sqrt(s);
        L[b * d + b] = lbb;
#pragma omp parallel for schedule(static)
        for (int64_t a = b + 1; a < d; ++a) {
            double dot = 0.0;
#pragma omp simd reduction(+ : dot)
            for (int64_t k = 0; k < b; ++k) dot += L[a * d + k] * L[b * d + k];
            L[a * d + b] = (H[a * d + b] - dot) / lbb;
        }
    }
    if (status == ORACLE_OK) {
        /* Column c of L^-1 solves L y = e_c. */
#pragma omp parallel for schedule(dynamic, 8)
        for (int64_t c = 0; c < d; ++c) {
            for (int64_t a = c; a < d; ++a) {
                double s = (a == c) ? 1.0 : 0.0;
                for (int64_t k = c; k < a; ++k) s -= L[a * d + k] * Li[k * d + c];
                Li[a * d + c] = s / L[a * d + a];
            }
        }
        /* Hinv[a][b] = sum_k Li[k][a] Li[k][b], k >= max(a, b). */
#pragma omp parallel for schedule(dynamic, 8)
        for (int64_t a = 0; a < d; ++a) {
            for (int64_t b = 0; b <= a; ++b) {
                double s = 0.0;
                for (int64_t k = a; k < d; ++k) s += Li[k * d + a] * Li[k * d + b];
                Hinv[a * d + b] = s;
                Hinv[b * d + a] = s;
            }
        }
    }
    free(L);
    free(Li);
    return status;
}

static int64_t groups_of(int64_t d, int64_t group) { return group > 0 ? d / group : 1; }

/* Asymmetric min-max grid per row (group == 0) or per (row, group of `group`
 * consecutive original columns).  Range is widened to contain 0.
 * scale, zero: d_row x G. */
int oracle_grid(const float *W, int64_t d_row, int64_t d_col, int bits, int64_t group,
                double *scale, double *zero)
{
    if (!W || !scale || !zero || d_row <= 0 || d_col <= 0 || bits < 1 || bits > 32) return ORACLE_EINVAL;
    if (group < 0 || (group > 0 && d_col % group != 0)) return ORACLE_EINVAL;
    const int64_t G = groups_of(d_col, group);
    const int64_t gs = group > 0 ? group : d_col;
    const double maxq = ldexp(1.0, bits) - 1.0;
    for (int64_t i = 0; i < d_row; ++i) {
        for (int64_t g = 0; g < G; ++g) {
            double lo = 0.0, hi = 0.0;
            for (int64_t j = g * gs; j < (g + 1) * gs; ++j) {
                double w = (double)W[i * d_col + j];
                if (w < lo) lo = w;
                if (w > hi) hi = w;
            }
            if (hi == lo) {
                scale[i * G + g] = 1.0;
                zero[i * G + g] = 0.0;
            } else {
                double s = (hi - lo) / maxq;
                scale[i * G + g] = s;
                zero[i * G + g] = rint(-lo / s);
            }
        }
    }
    return ORACLE_OK;
}

/* code = clamp(rint(w / scale) + zero, 0, maxq); rint is round-half-to-even. */
static inline double grid_code(double w, double scale, double zero, double maxq)
{
    double c = rint(w / scale) + zero;
    if (c < 0.0) c = 0.0;
    if (c > maxq) c = maxq;
    return c;
}

static inline double grid_value(double code, double scale, double zero)
{
    return scale * (code - zero);
}

/* S_j = sum_i (quant(w_ij) - w_ij)^2 / (2 Hinv_jj), initial W and initial Hinv. */
int oracle_sensitivity(const float *W, int64_t d_row, int64_t d_col, const double *Hinv_diag,
                       int bits, int64_t group, const double *scale, const double *zero, double *S)
{
    if (!W || !Hinv_diag || !scale || !zero || !S) return ORACLE_EINVAL;
    const int64_t G = groups_of(d_col, group);
    const int64_t gs = group > 0 ? group : d_col;
    const double maxq = ldexp(1.0, bits) - 1.0;
    for (int64_t j = 0; j < d_col; ++j) {
        const int64_t g = j / gs;
        double s = 0.0;
        for (int64_t i = 0; i < d_row; ++i) {
            double w = (double)W[i * d_col + j];
            double q = grid_value(grid_code(w, scale[i * G + g], zero[i * G + g], maxq),
                                  scale[i * G + g], zero[i * G + g]);
            s += (q - w) * (q - w) / (2.0 * Hinv_diag[j]);
        }
        S[j] = s;
    }
    return ORACLE_OK;
}

/* Column sort keys of the ordering ablation (Section 4.1, Table 3), aggregated per column
 * as in Section 4.2 step 2.  kind 0 "sensi": sum_i (quant(w) - w)^2 / (2 Hinv_jj);
 * kind 1 "err": sum_i (quant(w) - w)^2;  kind 2 "w": sum_i w^2. */
int oracle_column_key(const float *W, int64_t d_row, int64_t d_col, const double *Hinv_diag, int bits,
                      int64_t group, const double *scale, const double *zero, int kind, double *key)
{
    if (!W || !scale || !zero || !key || kind < 0 || kind > 2) return ORACLE_EINVAL;
    if (kind == 0) return oracle_sensitivity(W, d_row, d_col, Hinv_diag, bits, group, scale, zero, key);
    const int64_t G = groups_of(d_col, group);
    const int64_t gs = group > 0 ? group : d_col;
    const double maxq = ldexp(1.0, bits) - 1.0;
    for (int64_t j = 0; j < d_col; ++j) {
        const int64_t g = j / gs;
        double s = 0.0;
        for (int64_t i = 0; i < d_row; ++i) {
            const double w = (double)W[i * d_col + j];
            if (kind == 1) {
                const double q = grid_value(grid_code(w, scale[i * G + g], zero[i * G + g], maxq),
                                            scale[i * G + g], zero[i * G + g]);
                s += (q - w) * (q - w);
            } else {
                s += w * w;
            }
        }
        key[j] = s;
    }
    return ORACLE_OK;
}

/* perm = columns by key, descending (ascending = 0) or ascending (ascending = 1); equal keys
 * keep the smaller index first. */
int oracle_order_dir(const double *S, int64_t d, int ascending, int32_t *perm)
{
    if (!S || !perm || d <= 0) return ORACLE_EINVAL;
    for (int64_t j = 0; j < d; ++j) perm[j] = (int32_t)j;
    /* insertion sort: stable, d is a few thousand at most */
    for (int64_t a = 1; a < d; ++a) {
        int32_t v = perm[a];
        int64_t b = a - 1;
        while (b >= 0 && (ascending ? S[perm[b]] > S[v] : S[perm[b]] < S[v])) {
            perm[b + 1] = perm[b];
            --b;
        }
        perm[b + 1] = v;
    }
    return ORACLE_OK;
}

/* perm = columns by S descending; equal scores keep the smaller index first. */
int oracle_order(const double *S, int64_t d, int32_t *perm)
{
    return oracle_order_dir(S, d, 0, perm);
}

/*
 * The column loop.  Inputs: original W (fp32), Hinv (d x d, fp64, full
 * symmetric; overwritten with the running shared inverse), processing order
 * perm, the frozen grid.  Columns are addressed through perm; nothing is
 * physically permuted.
 *
 * For step t, j = perm[t], Rem = columns not yet processed (j included):
 *   q_ij   = quant(w_ij)                                   for all rows i
 *   loss  += sum_i (w_ij - q_ij)^2 / (2 Hinv_jj)
 *   e_i    = (w_ij - q_ij) / Hinv_jj
 *   w_ik  -= e_i Hinv_jk                                   k in Rem \ {j}
 *   Hinv_ab -= Hinv_aj Hinv_jb / Hinv_jj                   a, b in Rem \ {j}
 *
 * steps: number of columns to process (d_col for all).
 * Outputs (original column order): codes (int64), Q (quantized values; columns
 * not processed keep 0), Wwork (running weights; processed columns hold the
 * value they had when they were quantized), Hinv (running; rows and columns of
 * processed indices are set to 0), loss.
 */
static int column_loop_impl(const float *W, int64_t d_row, int64_t d_col, double *Hinv,
                            const int32_t *perm, int32_t *perm_dyn, int bits, int64_t group,
                            const double *scale, const double *zero, int64_t steps,
                            int64_t *codes, double *Q, double *Wwork, double *loss)
{
    if (!W || !Hinv || (!perm && !perm_dyn) || !scale || !zero || !codes || !Q || !Wwork || !loss)
        return ORACLE_EINVAL;
    if (steps < 0 || steps > d_col) return ORACLE_EINVAL;
    const int64_t d = d_col;
    const int64_t G = groups_of(d_col, group);
    const int64_t gs = group > 0 ? group : d_col;
    const double maxq = ldexp(1.0, bits) - 1.0;
    unsigned char *done = (unsigned char *)calloc((size_t)d, 1);
    double *rowj = (double *)malloc((size_t)d * sizeof(double));
    double *lossrow = (double *)calloc((size_t)d_row, sizeof(double));
    double *score = (double *)calloc((size_t)d, sizeof(double));
    if (!done || !rowj || !lossrow || !score) {
        free(done); free(rowj); free(lossrow); free(score);
        return ORACLE_ENOMEM;
    }
    for (int64_t i = 0; i < d_row * d_col; ++i) {
        Wwork[i] = (double)W[i];
        Q[i] = 0.0;
        codes[i] = 0;
    }
    int status = ORACLE_OK;
    for (int64_t t = 0; t < steps; ++t) {
        int64_t j;
        if (perm_dyn) {
            /* Dynamic order: the scores of Eq. 10 are recomputed from the current weights and the
             * current shared inverse; the column with the largest score is next (the first such
             * column in index order when several are equal). */
#pragma omp parallel for schedule(static)
            for (int64_t k = 0; k < d; ++k) {
                if (done[k]) continue;
                const int64_t gk = k / gs;
                const double hkk = Hinv[k * d + k];
                double sk = 0.0;
                for (int64_t i = 0; i < d_row; ++i) {
                    const double w = Wwork[i * d + k];
                    const double s = scale[i * G + gk], z = zero[i * G + gk];
                    const double diff = grid_value(grid_code(w, s, z, maxq), s, z) - w;
                    sk += diff * diff / (2.0 * hkk);
                }
                score[k] = sk;
            }
            j = -1;
            for (int64_t k = 0; k < d; ++k)
                if (!done[k] && (j < 0 || score[k] > score[j])) j = k;
            perm_dyn[t] = (int32_t)j;
        } else {
            j = perm[t];
        }
        if (j < 0 || j >= d || done[j]) { status = ORACLE_EINVAL; break; }
        const double hjj = Hinv[j * d + j];
        if (!(hjj > 0.0)) { status = ORACLE_ENOTPD; break; }
        const int64_t g = j / gs;
        for (int64_t k = 0; k < d; ++k) rowj[k] = Hinv[j * d + k];
        done[j] = 1;
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < d_row; ++i) {
            double *w = Wwork + i * d;
            const double s = scale[i * G + g], z = zero[i * G + g];
            const double c = grid_code(w[j], s, z, maxq);
            const double q = grid_value(c, s, z);
            codes[i * d + j] = (int64_t)c;
            Q[i * d + j] = q;
            const double diff = w[j] - q;
            lossrow[i] += diff * diff / (2.0 * hjj);
            const double e = diff / hjj;
            for (int64_t k = 0; k < d; ++k)
                if (!done[k]) w[k] -= e * rowj[k];
        }
#pragma omp parallel for schedule(static)
        for (int64_t a = 0; a < d; ++a) {
            if (done[a]) continue;
            const double haj = rowj[a]; /* Hinv is symmetric: Hinv_aj = Hinv_ja */
            double *ra = Hinv + a * d;
            const double f = haj / hjj;
            for (int64_t b = 0; b < d; ++b)
                if (!done[b]) ra[b] -= f * rowj[b];
        }
        for (int64_t k = 0; k < d; ++k) {
            Hinv[j * d + k] = 0.0;
            Hinv[k * d + j] = 0.0;
        }
    }
    double total = 0.0;
    for (int64_t i = 0; i < d_row; ++i) total += lossrow[i];
    *loss = total;
    if (perm_dyn) {
        /* columns not reached (steps < d_col) follow in index order */
        int64_t t = steps;
        for (int64_t k = 0; k < d && status == ORACLE_OK; ++k)
            if (!done[k]) perm_dyn[t++] = (int32_t)k;
    }
    free(done);
    free(rowj);
    free(lossrow);
    free(score);
    return status;
}

int oracle_column_loop(const float *W, int64_t d_row, int64_t d_col, double *Hinv,
                       const int32_t *perm, int bits, int64_t group,
                       const double *scale, const double *zero, int64_t steps,
                       int64_t *codes, double *Q, double *Wwork, double *loss)
{
    if (!perm) return ORACLE_EINVAL;
    return column_loop_impl(W, d_row, d_col, Hinv, perm, NULL, bits, group, scale, zero, steps,
                            codes, Q, Wwork, loss);
}

/*
 * The same loop with the order decided step by step (the reading of Section 5 in which the
 * sorting is repeated for every column): before each step the scores S_k of Eq. 10 are
 * recomputed for every column not yet processed, from the current (compensated) weights and
 * the diagonal of the current shared inverse, and the column with the largest score is taken.
 * perm_out[t] receives the column processed at step t.
 */
int oracle_column_loop_dynamic(const float *W, int64_t d_row, int64_t d_col, double *Hinv,
                               int32_t *perm_out, int bits, int64_t group,
                               const double *scale, const double *zero, int64_t steps,
                               int64_t *codes, double *Q, double *Wwork, double *loss)
{
    if (!perm_out) return ORACLE_EINVAL;
    return column_loop_impl(W, d_row, d_col, Hinv, NULL, perm_out, bits, group, scale, zero, steps,
                            codes, Q, Wwork, loss);
}

/*
 * The baseline the method is derived from (Section 4.2, first paragraphs): OBQ quantizes every
 * row on its own.  Each row keeps its own copy of the inverse Hessian, picks at every step the
 * not-yet-quantized weight with the SMALLEST loss term (quant(w_p) - w_p)^2 / (2 [Hinv]_pp)
 * (Eq. 10; the first such weight in index order when several are equal), quantizes it,
 * compensates the rest of the row (Eq. 9 / 11) and eliminates index p from the row's own
 * inverse (Eq. 12).  Cost O(d_row d_col^3) against O(d_col^3 + d_row d_col^2) of the shared-inverse
 * loop above.  Same frozen grid, same arithmetic per step as oracle_column_loop.
 *
 * row_begin .. row_end: the rows to process (a sample of rows is enough to measure the per-row
 * cost and loss; rows do not interact).  Outputs are full d_row x d_col arrays of which only those
 * rows are written; order (may be NULL) receives, per row, the index processed at each step;
 * lossrow (d_row) the row's accumulated loss.
 */
int oracle_obq_rows(const float *W, int64_t d_row, int64_t d_col, const double *Hinv0,
                    int bits, int64_t group, const double *scale, const double *zero,
                    int64_t row_begin, int64_t row_end,
                    int64_t *codes, double *Q, int32_t *order, double *lossrow)
{
    if (!W || !Hinv0 || !scale || !zero || !codes || !Q || !lossrow) return ORACLE_EINVAL;
    if (row_begin < 0 || row_end > d_row || row_begin > row_end) return ORACLE_EINVAL;
    const int64_t d = d_col;
    const int64_t G = groups_of(d_col, group);
    const int64_t gs = group > 0 ? group : d_col;
    const double maxq = ldexp(1.0, bits) - 1.0;
    int status = ORACLE_OK;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = row_begin; i < row_end; ++i) {
        double *Hc = (double *)malloc((size_t)d * d * sizeof(double));
        double *w = (double *)malloc((size_t)d * sizeof(double));
        double *rowj = (double *)malloc((size_t)d * sizeof(double));
        unsigned char *done = (unsigned char *)calloc((size_t)d, 1);
        if (!Hc || !w || !rowj || !done) {
#pragma omp critical
            status = ORACLE_ENOMEM;
            free(Hc); free(w); free(rowj); free(done);
            continue;
        }
        memcpy(Hc, Hinv0, (size_t)d * d * sizeof(double));
        for (int64_t k = 0; k < d; ++k) w[k] = (double)W[i * d + k];
        double loss = 0.0;
        for (int64_t t = 0; t < d; ++t) {
            int64_t j = -1;
            double best = 0.0;
            for (int64_t k = 0; k < d; ++k) {
                if (done[k]) continue;
                const double s = scale[i * G + k / gs], z = zero[i * G + k / gs];
                const double diff = grid_value(grid_code(w[k], s, z, maxq), s, z) - w[k];
                const double sk = diff * diff / (2.0 * Hc[k * d + k]);
                if (j < 0 || sk < best) { j = k; best = sk; }
            }
            const double hjj = Hc[j * d + j];
            if (!(hjj > 0.0)) {
#pragma omp critical
                status = ORACLE_ENOTPD;
                break;
            }
            for (int64_t k = 0; k < d; ++k) rowj[k] = Hc[j * d + k];
            done[j] = 1;
            if (order) order[i * d + t] = (int32_t)j;
            const double s = scale[i * G + j / gs], z = zero[i * G + j / gs];
            const double c = grid_code(w[j], s, z, maxq);
            const double q = grid_value(c, s, z);
            codes[i * d + j] = (int64_t)c;
            Q[i * d + j] = q;
            const double diff = w[j] - q;
            loss += diff * diff / (2.0 * hjj);
            const double e = diff / hjj;
            for (int64_t k = 0; k < d; ++k)
                if (!done[k]) w[k] -= e * rowj[k];
            for (int64_t a = 0; a < d; ++a) {
                if (done[a]) continue;
                const double f = rowj[a] / hjj;
                double *ra = Hc + a * d;
                for (int64_t b = 0; b < d; ++b)
                    if (!done[b]) ra[b] -= f * rowj[b];
            }
        }
        lossrow[i] = loss;
        free(Hc); free(w); free(rowj); free(done);
    }
    return status;
}

/* 1/2 tr((W - Q) H (W - Q)^T), H fp64 d x d. */
int oracle_loss_eval(const float *W, const double *Q, const double *H, int64_t d_row, int64_t d_col,
                     double *loss)
{
    if (!W || !Q || !H || !loss) return ORACLE_EINVAL;
    const int64_t d = d_col;
    double total = 0.0;
#pragma omp parallel for schedule(static) reduction(+ : total)
    for (int64_t i = 0; i < d_row; ++i) {
        double acc = 0.0;
        for (int64_t a = 0; a < d; ++a) {
            const double da = (double)W[i * d + a] - Q[i * d + a];
            double s = 0.0;
            for (int64_t b = 0; b < d; ++b) s += H[a * d + b] * ((double)W[i * d + b] - Q[i * d + b]);
            acc += da * s;
        }
        total += 0.5 * acc;
    }
    *loss = total;
    return ORACLE_OK;
}

/* (1/N) |(W - Q) X|_F^2 computed directly from X (no Hessian). */
int oracle_output_error(const float *W, const double *Q, const float *X, int64_t d_row, int64_t d_col,
                        int64_t N, int64_t ld, double *err)
{
    if (!W || !Q || !X || !err) return ORACLE_EINVAL;
    double total = 0.0;
#pragma omp parallel for schedule(static) reduction(+ : total)
    for (int64_t i = 0; i < d_row; ++i) {
        double acc = 0.0;
        for (int64_t n = 0; n < N; ++n) {
            double y = 0.0;
            for (int64_t a = 0; a < d_col; ++a)
                y += ((double)W[i * d_col + a] - Q[i * d_col + a]) * (double)X[a * ld + n];
            acc += y * y;
        }
        total += acc;
    }
    *err = total / (double)N;
    return ORACLE_OK;
}
