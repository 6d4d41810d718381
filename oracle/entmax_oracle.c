/*
 * Float64 CPU oracle for alpha-entmax attention and its gradient.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code with the HIP path and is
 * never linked into, imported by or called from the product.
 *
 * What it computes, per (batch, head) and per query row r (AdaSplash-2 paper):
 *   s_j   = <q_r, k_j> / sqrt(d)                         (Eq. 2)
 *   x_j   = (alpha-1) s_j
 *   tau*  = unique root of  sum_j [x_j - tau]_+^{1/(alpha-1)} = 1   (Eq. 3, Eq. 4)
 *   p_j   = [x_j - tau*]_+^{1/(alpha-1)},  O_r = sum_j p_j v_j       (Eq. 2, Eq. 3)
 * tau* is found by the sort-based exact solvers for alpha = 2 and alpha = 1.5
 * (Sec. 2.4 "Sorting-based solvers", App. A) and by bisection on the bracket
 * of Eq. 5 otherwise (Sec. 2.4 "Bisection").
 * Causal masking (not written in Alg. 1-3, used by every benchmark of Sec. 4.2):
 * key j is visible to query r iff j <= r; hidden keys take no part in anything.
 *
 * Gradient (Sec. 3.3 "Backward pass", App. B part (ii), Alg. 2-3), for the
 * scalar L = sum(O * dO):
 *   g_j  = <dO_r, v_j>
 *   u_j  = p_j^{2-alpha} on the support (p_j > 0), 0 off it
 *   delta_r = sum_j u_j g_j / sum_j u_j
 *   ds_j = u_j (g_j - delta_r)
 *   dQ_r = sum_j ds_j k_j / sqrt(d);  dK_j += ds_j q_r / sqrt(d);  dV_j += p_j dO_r
 * The delta printed in the "Require" lines of Alg. 2-3 is garbled (it has no dO
 * and uses S for P); the form above is the one that follows from differentiating
 * Eq. 3 under sum_j p_j = 1 and is pinned by finite differences in the tests.
 *
 * Only entries with x_j > max_j x_j - 1 are handed to the sort / the bisection:
 * by Eq. 5 tau* >= max x - 1, so no other entry can be positive.  The tests
 * check that this restriction changes nothing.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_EBADARG -1
#define ORACLE_ENOMEM -2

static int cmp_desc(const void* a, const void* b) {
    double x = *(const double*)a, y = *(const double*)b;
    return (x < y) - (x > y);
}

/* f(tau) of Eq. 4 over the given entries. */
double oracle_f(const double* x, long n, double alpha, double tau) {
    double r = 1.0 / (alpha - 1.0), acc = 0.0;
    for (long j = 0; j < n; ++j) {
        double y = x[j] - tau;
        if (y > 0.0) acc += pow(y, r);
    }
    return acc - 1.0;
}

/* Bisection on the Eq. 5 bracket [max x - 1, max x - n^{1-alpha}] until the
 * bracket is narrower than tol; returns its midpoint. */
double oracle_tau_bisect(const double* x, long n, double alpha, double tol) {
    double mx = x[0];
    for (long j = 1; j < n; ++j) if (x[j] > mx) mx = x[j];
    double lo = mx - 1.0, hi = mx - pow((double)n, 1.0 - alpha);
    /* f(lo) >= 0 >= f(hi) */
    while (hi - lo > tol) {
        double mid = 0.5 * (lo + hi);
        if (mid <= lo || mid >= hi) break; /* bracket at floating point resolution */
        if (oracle_f(x, n, alpha, mid) >= 0.0) lo = mid; else hi = mid;
    }
    return 0.5 * (lo + hi);
}

/* Sort-based exact threshold for alpha = 2 (linear equation per top-k set) and
 * alpha = 1.5 (quadratic equation per top-k set); App. A.  `work` holds n doubles.
 * Returns NaN for any other alpha. */
double oracle_tau_sort(const double* x, long n, double alpha, double* work) {
    memcpy(work, x, (size_t)n * sizeof(double));
    qsort(work, (size_t)n, sizeof(double), cmp_desc);
    double best = NAN;
    if (alpha == 2.0) {
        double s1 = 0.0;
        for (long k = 1; k <= n; ++k) {
            s1 += work[k - 1];
            double t = (s1 - 1.0) / (double)k;          /* sum_{top k}(x - t) = 1 */
            if (work[k - 1] > t) best = t;               /* largest k whose k-th entry is active */
        }
    } else if (alpha == 1.5) {
        double s1 = 0.0, s2 = 0.0;
        for (long k = 1; k <= n; ++k) {
            s1 += work[k - 1];
            s2 += work[k - 1] * work[k - 1];
            /* sum_{top k}(x - t)^2 = 1  <=>  k t^2 - 2 s1 t + s2 - 1 = 0, smaller root */
            double mean = s1 / (double)k;
            double disc = mean * mean - (s2 - 1.0) / (double)k;
            if (disc < 0.0) disc = 0.0;
            double t = mean - sqrt(disc);
            if (work[k - 1] > t) best = t;
        }
    }
    return best;
}

/* Exact threshold of one row: x holds (alpha-1)*s for the visible keys.
 * full != 0 disables the restriction to entries above max x - 1 (used by tests). */
double oracle_tau_row(const double* x, long n, double alpha, int full, double* work /* 2n doubles */) {
    double mx = x[0];
    for (long j = 1; j < n; ++j) if (x[j] > mx) mx = x[j];
    double* cand = work;
    long m = 0;
    if (full) { memcpy(cand, x, (size_t)n * sizeof(double)); m = n; }
    else for (long j = 0; j < n; ++j) if (x[j] > mx - 1.0) cand[m++] = x[j];
    if (alpha == 2.0 || alpha == 1.5) return oracle_tau_sort(cand, m, alpha, work + n);
    /* bisection: the bracket's upper end uses the number of visible keys n, as in Eq. 5 */
    double lo = mx - 1.0, hi = mx - pow((double)n, 1.0 - alpha);
    while (hi - lo > 1e-12) {
        double mid = 0.5 * (lo + hi);
        if (mid <= lo || mid >= hi) break;
        if (oracle_f(cand, m, alpha, mid) >= 0.0) lo = mid; else hi = mid;
    }
    return 0.5 * (lo + hi);
}

/* p_j = [x_j - tau]_+^{1/(alpha-1)}  (Eq. 3) */
static inline double entmax_p(double x, double tau, double alpha) {
    double y = x - tau;
    if (y <= 0.0) return 0.0;
    if (alpha == 2.0) return y;
    if (alpha == 1.5) return y * y;
    return pow(y, 1.0 / (alpha - 1.0));
}

/*
 * Forward.  Q,K,V: [B,H,N,d] contiguous doubles.  Outputs (all caller-allocated):
 *   O      [B,H,N,d]
 *   tau    [B,H,N]      raw convention: p = [(alpha-1) s - tau]_+^{1/(alpha-1)}
 *   margin [B,H,T,T]    T = N/tile; margin[I][J] = max over rows r of query tile I and
 *                       visible keys j of key tile J of (x_rj - tau_r); -inf when no key of
 *                       the tile is visible to any row.  Block-mask bit = margin > 0.  May be NULL.
 *   P      [B,H,N,N]    the probabilities (0 for hidden keys).  May be NULL (tiny cases only).
 */
int oracle_entmax_attn_fwd(const double* Q, const double* K, const double* V,
                           int B, int H, int N, int d, double alpha, int causal, int tile,
                           double* O, double* tau, double* margin, double* P) {
    if (!Q || !K || !V || !O || !tau) return ORACLE_EBADARG;
    if (!(alpha > 1.0) || B <= 0 || H <= 0 || N <= 0 || d <= 0) return ORACLE_EBADARG;
    if (margin && (tile <= 0 || N % tile != 0)) return ORACLE_EBADARG;
    const long BH = (long)B * H;
    const int T = margin ? N / tile : 0;
    const double inv_sqrt_d = 1.0 / sqrt((double)d);
    if (margin) for (long i = 0; i < BH * T * T; ++i) margin[i] = -INFINITY;
    int err = 0;
#pragma omp parallel
    {
        double* x = (double*)malloc((size_t)N * sizeof(double));
        double* work = (double*)malloc((size_t)3 * N * sizeof(double));
        if (!x || !work) {
#pragma omp atomic write
            err = 1;
        } else {
            /* one (head, query tile) per task when margins are wanted, so that no two
             * threads write the same margin entry */
            const int RT = margin ? tile : 1;
            const long ntask = BH * (N / RT);
#pragma omp for schedule(dynamic, 1)
            for (long task = 0; task < ntask; ++task) {
                const long bh = task / (N / RT);
                const int r0 = (int)(task % (N / RT)) * RT;
                const double* q_h = Q + bh * (long)N * d;
                const double* k_h = K + bh * (long)N * d;
                const double* v_h = V + bh * (long)N * d;
                for (int r = r0; r < r0 + RT; ++r) {
                    const int nvis = causal ? r + 1 : N;
                    const double* q = q_h + (long)r * d;
                    for (int j = 0; j < nvis; ++j) {
                        const double* k = k_h + (long)j * d;
                        double s = 0.0;
                        for (int c = 0; c < d; ++c) s += q[c] * k[c];
                        x[j] = (alpha - 1.0) * (s * inv_sqrt_d);
                    }
                    const double t = oracle_tau_row(x, nvis, alpha, 0, work);
                    tau[bh * N + r] = t;
                    double* o = O + (bh * (long)N + r) * d;
                    for (int c = 0; c < d; ++c) o[c] = 0.0;
                    for (int j = 0; j < nvis; ++j) {
                        const double p = entmax_p(x[j], t, alpha);
                        if (P) P[(bh * (long)N + r) * N + j] = p;
                        if (p > 0.0) {
                            const double* v = v_h + (long)j * d;
                            for (int c = 0; c < d; ++c) o[c] += p * v[c];
                        }
                    }
                    if (P) for (int j = nvis; j < N; ++j) P[(bh * (long)N + r) * N + j] = 0.0;
                    if (margin) {
                        double* mrow = margin + (bh * T + r / tile) * (long)T;
                        for (int j = 0; j < nvis; ++j) {
                            const double mg = x[j] - t;
                            if (mg > mrow[j / tile]) mrow[j / tile] = mg;
                        }
                    }
                }
            }
        }
        free(x); free(work);
    }
    return err ? ORACLE_ENOMEM : ORACLE_OK;
}

/*
 * Backward of L = sum(O * dO).  Recomputes tau* and p itself (it takes nothing
 * from any forward result).  dQ, dK, dV: [B,H,N,d], caller-allocated, overwritten.
 * delta (may be NULL): [B,H,N].
 */
int oracle_entmax_attn_bwd(const double* Q, const double* K, const double* V, const double* dO,
                           int B, int H, int N, int d, double alpha, int causal,
                           double* dQ, double* dK, double* dV, double* delta) {
    if (!Q || !K || !V || !dO || !dQ || !dK || !dV) return ORACLE_EBADARG;
    if (!(alpha > 1.0) || B <= 0 || H <= 0 || N <= 0 || d <= 0) return ORACLE_EBADARG;
    const long BH = (long)B * H;
    const double inv_sqrt_d = 1.0 / sqrt((double)d);
    const long total = BH * (long)N * d;
    for (long i = 0; i < total; ++i) { dQ[i] = 0.0; dK[i] = 0.0; dV[i] = 0.0; }
    int err = 0;
#pragma omp parallel
    {
        double* x = (double*)malloc((size_t)N * sizeof(double));
        double* work = (double*)malloc((size_t)3 * N * sizeof(double));
        if (!x || !work) {
#pragma omp atomic write
            err = 1;
        } else {
#pragma omp for schedule(dynamic, 16)
            for (long row = 0; row < BH * N; ++row) {
                const long bh = row / N;
                const int r = (int)(row % N);
                const int nvis = causal ? r + 1 : N;
                const double* q = Q + row * d;
                const double* go = dO + row * d;
                const double* k_h = K + bh * (long)N * d;
                const double* v_h = V + bh * (long)N * d;
                for (int j = 0; j < nvis; ++j) {
                    const double* k = k_h + (long)j * d;
                    double s = 0.0;
                    for (int c = 0; c < d; ++c) s += q[c] * k[c];
                    x[j] = (alpha - 1.0) * (s * inv_sqrt_d);
                }
                const double t = oracle_tau_row(x, nvis, alpha, 0, work);
                /* delta_r = sum u g / sum u over the support */
                double num = 0.0, den = 0.0;
                for (int j = 0; j < nvis; ++j) {
                    const double p = entmax_p(x[j], t, alpha);
                    if (p > 0.0) {
                        const double u = (alpha == 2.0) ? 1.0 : pow(p, 2.0 - alpha);
                        const double* v = v_h + (long)j * d;
                        double g = 0.0;
                        for (int c = 0; c < d; ++c) g += go[c] * v[c];
                        num += u * g; den += u;
                    }
                }
                const double dl = num / den;   /* the support is never empty */
                if (delta) delta[row] = dl;
                double* dq = dQ + row * d;
                for (int j = 0; j < nvis; ++j) {
                    const double p = entmax_p(x[j], t, alpha);
                    if (p > 0.0) {
                        const double u = (alpha == 2.0) ? 1.0 : pow(p, 2.0 - alpha);
                        const double* v = v_h + (long)j * d;
                        const double* k = k_h + (long)j * d;
                        double g = 0.0;
                        for (int c = 0; c < d; ++c) g += go[c] * v[c];
                        const double ds = u * (g - dl);
                        double* dk = dK + (bh * (long)N + j) * d;
                        double* dv = dV + (bh * (long)N + j) * d;
                        for (int c = 0; c < d; ++c) {
                            dq[c] += ds * k[c] * inv_sqrt_d;
#pragma omp atomic
                            dk[c] += ds * q[c] * inv_sqrt_d;
#pragma omp atomic
                            dv[c] += p * go[c];
                        }
                    }
                }
            }
        }
        free(x); free(work);
    }
    return err ? ORACLE_ENOMEM : ORACLE_OK;
}

/* Plain entmax of one score vector s (not pre-scaled): p and tau (raw convention). */
int oracle_entmax(const double* s, long n, double alpha, int full, double* p, double* tau_out) {
    if (!s || !p || n <= 0 || !(alpha > 1.0)) return ORACLE_EBADARG;
    double* x = (double*)malloc((size_t)n * sizeof(double));
    double* work = (double*)malloc((size_t)3 * n * sizeof(double));
    if (!x || !work) { free(x); free(work); return ORACLE_ENOMEM; }
    for (long j = 0; j < n; ++j) x[j] = (alpha - 1.0) * s[j];
    const double t = oracle_tau_row(x, n, alpha, full, work);
    for (long j = 0; j < n; ++j) p[j] = entmax_p(x[j], t, alpha);
    if (tau_out) *tau_out = t;
    free(x); free(work);
    return ORACLE_OK;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
