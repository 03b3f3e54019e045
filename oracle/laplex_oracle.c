/*
 * CPU oracle for the LAPLEX apply.  TEST INFRASTRUCTURE ONLY: the product path
 * never links, loads or calls anything in this file; it shares no code, header
 * or table with the HIP kernels.  Everything is fp64 (callers widen the fp32
 * inputs first, the protocol of App. "Numerical accuracy"), plain loops, no
 * blocking and no reordering beyond what the cited definition or theorem
 * states.
 *
 * Notation of this repository: L is k x n, a[0..k) are the OUTPUT anchors,
 * b[0..n) the INPUT anchors, L_ij = exp(-|a_i - b_j|) (Introduction, the
 * Laplace-kernel matrix).  Batched data are batch-minor: x[j*ldx + t] is batch
 * column t of input j.
 *
 * Two independent routes to the same numbers:
 *   A  brute force, the definition written out, O(n k batch);
 *   B  Theorem "Dual reduction via the b-axis" (App. B.3): inputs sorted by
 *      the caller, two recurrences along the input axis (Sec. 3 "Symmetric
 *      case"), one binary search per output and a two-term evaluation.
 *   C  the definition restricted to a window |a_i - b_j| <= W around a
 *      sampled output (truncation below exp(-W) * sum|x|).
 *
 * Pins (tests/test_oracle_pins.py): exact-rational worked examples from
 * tests/golden/, the geometric closed form on a uniform grid, the tridiagonal
 * inverse of the symmetric kernel, the CountSketch / zero-temperature limit
 * (App. A, Lemma 1 and Prop. 1), symmetry / unit diagonal of the Gram form,
 * translation and reflection invariance, central finite differences for every
 * gradient, and route A against route B against numpy's dense matmul.  No
 * function here is parity-unpinned.
 *
 * Anchor gradient at a tie (a_i == b_j, duplicated anchors, the Gram
 * diagonal): |.| has no derivative there and the paper prints no formula; the
 * reading taken is sgn(0) = 0, the central-difference limit and what automatic
 * differentiation of the dense definition yields.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double sgn(double v) { return (v > 0.0) - (v < 0.0); }

/* ------------------------------------------------------------------------ */
/* Route A: the definition.                                                  */
/* ------------------------------------------------------------------------ */

/* y[i*ldy+t] = sum_j exp(-|a_i-b_j|) x[j*ldx+t];  tol[i*ldy+t] the same sum
 * over |x| (the denominator of the acceptance bound); tol may be NULL. */
int oracle_apply_brute(const double* a, int64_t k, const double* b, int64_t n,
                       const double* x, int64_t ldx, int64_t batch,
                       double* y, double* tol, int64_t ldy)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < k; ++i) {
        for (int64_t t = 0; t < batch; ++t) {
            y[i * ldy + t] = 0.0;
            if (tol) tol[i * ldy + t] = 0.0;
        }
        for (int64_t j = 0; j < n; ++j) {
            const double w = exp(-fabs(a[i] - b[j]));
            for (int64_t t = 0; t < batch; ++t) {
                y[i * ldy + t] += w * x[j * ldx + t];
                if (tol) tol[i * ldy + t] += w * fabs(x[j * ldx + t]);
            }
        }
    }
    return 0;
}

/* Gradients of  sum_{i,t} g[i*ldg+t] * y[i*ldy+t]  by differentiating the
 * definition term by term:
 *   gx[j,t] =  sum_i L_ij g[i,t]
 *   ga[i]   = -sum_t g[i,t] sum_j sgn(a_i-b_j) L_ij x[j,t]
 *   gb[j]   = +sum_t x[j,t] sum_i sgn(a_i-b_j) L_ij g[i,t]
 * tgx/tga/tgb: the same sums over absolute values of the summands (ties
 * included).  Any output pointer may be NULL. */
int oracle_apply_backward_brute(const double* a, int64_t k, const double* b, int64_t n,
                                const double* x, int64_t ldx,
                                const double* g, int64_t ldg, int64_t batch,
                                double* gx, double* tgx, int64_t ldgx,
                                double* ga, double* tga, double* gb, double* tgb)
{
    const size_t nb = (size_t)(batch ? batch : 1);
    if (gx || gb) {
#pragma omp parallel
        {
            /* per batch column: s = sum L g, sa = sum L |g|, sd = sum sgn L g */
            double* s = (double*)malloc(3 * nb * sizeof(double));
            double* sa = s + nb;
            double* sd = sa + nb;
#pragma omp for schedule(static)
            for (int64_t j = 0; j < n; ++j) {
                for (int64_t t = 0; t < batch; ++t) s[t] = sa[t] = sd[t] = 0.0;
                for (int64_t i = 0; i < k; ++i) {
                    const double w = exp(-fabs(a[i] - b[j]));
                    const double sg = sgn(a[i] - b[j]);
                    for (int64_t t = 0; t < batch; ++t) {
                        s[t] += w * g[i * ldg + t];
                        sa[t] += w * fabs(g[i * ldg + t]);
                        sd[t] += sg * w * g[i * ldg + t];
                    }
                }
                double accb = 0.0, acct = 0.0;
                for (int64_t t = 0; t < batch; ++t) {
                    if (gx) gx[j * ldgx + t] = s[t];
                    if (tgx) tgx[j * ldgx + t] = sa[t];
                    accb += x[j * ldx + t] * sd[t];
                    acct += fabs(x[j * ldx + t]) * sa[t];
                }
                if (gb) gb[j] = accb;
                if (tgb) tgb[j] = acct;
            }
            free(s);
        }
    }
    if (ga) {
#pragma omp parallel
        {
            double* sd = (double*)malloc(2 * nb * sizeof(double));
            double* sa = sd + nb;
#pragma omp for schedule(static)
            for (int64_t i = 0; i < k; ++i) {
                for (int64_t t = 0; t < batch; ++t) sd[t] = sa[t] = 0.0;
                for (int64_t j = 0; j < n; ++j) {
                    const double w = exp(-fabs(a[i] - b[j]));
                    const double sg = sgn(a[i] - b[j]);
                    for (int64_t t = 0; t < batch; ++t) {
                        sd[t] += sg * w * x[j * ldx + t];
                        sa[t] += w * fabs(x[j * ldx + t]);
                    }
                }
                double acca = 0.0, acct = 0.0;
                for (int64_t t = 0; t < batch; ++t) {
                    acca -= g[i * ldg + t] * sd[t];
                    acct += fabs(g[i * ldg + t]) * sa[t];
                }
                ga[i] = acca;
                if (tga) tga[i] = acct;
            }
            free(sd);
        }
    }
    return 0;
}

/* Square (Gram) form K = L(a,a), K_ij = exp(-|a_i-a_j|) (Sec. 3 "Symmetric
 * case"): y = K x. */
int oracle_gram_brute(const double* a, int64_t n, const double* x, int64_t ldx,
                      int64_t batch, double* y, double* tol, int64_t ldy)
{
    return oracle_apply_brute(a, n, a, n, x, ldx, batch, y, tol, ldy);
}

/* Gradients of sum g.y for y = K x:  gx = K g (K is symmetric) and, since a_m
 * enters row m and column m of K,
 *   ga[m] = sum_t [ g[m,t] sum_j s_mj K_mj x[j,t] + x[m,t] sum_i s_mi K_im g[i,t] ],
 *   s_mj = -sgn(a_m - a_j)   (the diagonal contributes 0). */
int oracle_gram_backward_brute(const double* a, int64_t n, const double* x, int64_t ldx,
                               const double* g, int64_t ldg, int64_t batch,
                               double* gx, double* tgx, int64_t ldgx,
                               double* ga, double* tga)
{
    const size_t nb = (size_t)(batch ? batch : 1);
#pragma omp parallel
    {
        double* kg = (double*)malloc(5 * nb * sizeof(double));
        double* kga = kg + nb;   /* sum K |g| */
        double* kxa = kga + nb;  /* sum K |x| */
        double* dx = kxa + nb;   /* sum s K x */
        double* dg = dx + nb;    /* sum s K g */
#pragma omp for schedule(static)
        for (int64_t m = 0; m < n; ++m) {
            for (int64_t t = 0; t < batch; ++t) kg[t] = kga[t] = kxa[t] = dx[t] = dg[t] = 0.0;
            for (int64_t j = 0; j < n; ++j) {
                const double w = exp(-fabs(a[m] - a[j]));
                const double s = -sgn(a[m] - a[j]);
                for (int64_t t = 0; t < batch; ++t) {
                    kg[t] += w * g[j * ldg + t];
                    kga[t] += w * fabs(g[j * ldg + t]);
                    kxa[t] += w * fabs(x[j * ldx + t]);
                    dx[t] += s * w * x[j * ldx + t];
                    dg[t] += s * w * g[j * ldg + t];
                }
            }
            double acc = 0.0, acct = 0.0;
            for (int64_t t = 0; t < batch; ++t) {
                if (gx) gx[m * ldgx + t] = kg[t];
                if (tgx) tgx[m * ldgx + t] = kga[t];
                acc += g[m * ldg + t] * dx[t] + x[m * ldx + t] * dg[t];
                acct += fabs(g[m * ldg + t]) * kxa[t] + fabs(x[m * ldx + t]) * kga[t];
            }
            if (ga) ga[m] = acc;
            if (tga) tga[m] = acct;
        }
        free(kg);
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Route B: Theorem "Dual reduction via the b-axis".                         */
/* ------------------------------------------------------------------------ */

/* number of s[0..m) strictly below q / not above q (s ascending) */
static int64_t count_below(const double* s, int64_t m, double q)
{
    int64_t lo = 0, hi = m;
    while (lo < hi) { int64_t mid = lo + (hi - lo) / 2; if (s[mid] < q) lo = mid + 1; else hi = mid; }
    return lo;
}
static int64_t count_not_above(const double* s, int64_t m, double q)
{
    int64_t lo = 0, hi = m;
    while (lo < hi) { int64_t mid = lo + (hi - lo) / 2; if (s[mid] <= q) lo = mid + 1; else hi = mid; }
    return lo;
}

/*
 * Source anchors s[0..m) ASCENDING with values val[j*ldv+t] (the caller has
 * already put them in that order), query anchors q[0..nq).  With
 *   u_j = val_j + exp(s_{j-1}-s_j) u_{j-1}     (prefix recurrence)
 *   v_j = val_j + exp(s_j-s_{j+1}) v_{j+1}     (suffix recurrence)
 * and, per query, hi = #{s_j <= q}, lo = #{s_j < q}, the theorem's two terms
 * give
 *   left_incl  = sum_{s_j <= q} exp(s_j-q) val_j = exp(s_{hi-1}-q) u_{hi-1}
 *   left_strict= sum_{s_j <  q} exp(s_j-q) val_j = exp(s_{lo-1}-q) u_{lo-1}
 *   right_strict=sum_{s_j >  q} exp(q-s_j) val_j = exp(q-s_hi) v_hi
 * (a term whose index does not exist is 0).  Outputs are nq x batch with
 * leading dimension ldo; any may be NULL.  All exponents are <= 0.
 * use_abs != 0 runs on |val| (for the tolerance denominators).
 */
int oracle_dual_sums(const double* s, int64_t m, const double* val, int64_t ldv,
                     int64_t batch, const double* q, int64_t nq, int use_abs,
                     double* left_incl, double* left_strict, double* right_strict,
                     int64_t ldo)
{
    if (m == 0) {
        for (int64_t i = 0; i < nq; ++i)
            for (int64_t t = 0; t < batch; ++t) {
                if (left_incl) left_incl[i * ldo + t] = 0.0;
                if (left_strict) left_strict[i * ldo + t] = 0.0;
                if (right_strict) right_strict[i * ldo + t] = 0.0;
            }
        return 0;
    }
    int64_t* lo = (int64_t*)malloc(sizeof(int64_t) * (size_t)(nq ? nq : 1));
    int64_t* hi = (int64_t*)malloc(sizeof(int64_t) * (size_t)(nq ? nq : 1));
    if (!lo || !hi) { free(lo); free(hi); return -1; }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nq; ++i) {
        lo[i] = count_below(s, m, q[i]);
        hi[i] = count_not_above(s, m, q[i]);
    }
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t t = 0; t < batch; ++t) {
        double* u = (double*)malloc(sizeof(double) * (size_t)m);
        double* v = (double*)malloc(sizeof(double) * (size_t)m);
        if (!u || !v) {
            free(u); free(v);
#pragma omp atomic write
            fail = 1;
            continue;
        }
        for (int64_t j = 0; j < m; ++j) {
            double w = val[j * ldv + t];
            if (use_abs) w = fabs(w);
            u[j] = (j == 0) ? w : w + exp(s[j - 1] - s[j]) * u[j - 1];
        }
        for (int64_t j = m - 1; j >= 0; --j) {
            double w = val[j * ldv + t];
            if (use_abs) w = fabs(w);
            v[j] = (j == m - 1) ? w : w + exp(s[j] - s[j + 1]) * v[j + 1];
        }
        for (int64_t i = 0; i < nq; ++i) {
            if (left_incl)
                left_incl[i * ldo + t] = hi[i] >= 1 ? exp(s[hi[i] - 1] - q[i]) * u[hi[i] - 1] : 0.0;
            if (left_strict)
                left_strict[i * ldo + t] = lo[i] >= 1 ? exp(s[lo[i] - 1] - q[i]) * u[lo[i] - 1] : 0.0;
            if (right_strict)
                right_strict[i * ldo + t] = hi[i] < m ? exp(q[i] - s[hi[i]]) * v[hi[i]] : 0.0;
        }
        free(u); free(v);
    }
    free(lo); free(hi);
    return fail ? -1 : 0;
}

/* ------------------------------------------------------------------------ */
/* Route C: the definition inside a window, for sampled outputs.             */
/* ------------------------------------------------------------------------ */

/* b_sorted ascending with x_sorted in the same order (batch column 0 of a
 * batch-minor array with leading dimension ldx).  For each sampled anchor
 * q[i]: y[i] = sum over j with |q_i - b_j| <= window of exp(-|q_i-b_j|) x_j
 * and tol[i] the same over |x_j|. */
int oracle_apply_window(const double* b_sorted, int64_t n, const double* x_sorted,
                        int64_t ldx, const double* q, int64_t nq, double window,
                        double* y, double* tol)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nq; ++i) {
        const int64_t j0 = count_below(b_sorted, n, q[i] - window);
        const int64_t j1 = count_not_above(b_sorted, n, q[i] + window);
        double s = 0.0, sa = 0.0;
        for (int64_t j = j0; j < j1; ++j) {
            const double w = exp(-fabs(q[i] - b_sorted[j]));
            s += w * x_sorted[j * ldx];
            sa += w * fabs(x_sorted[j * ldx]);
        }
        y[i] = s;
        if (tol) tol[i] = sa;
    }
    return 0;
}
