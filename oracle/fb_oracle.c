/*
 * fb_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, double-precision CPU forward-backward over an HMM given as an
 * arc list, written out from the definitions in the paper (Algorithm section):
 *
 *   alpha recursion  Eq. 2 (scalar) / Eq. 4 (matrix) / Eq. 13 (log semifield)
 *   beta recursion   Eq. 3 / Eq. 5 / Eq. 14
 *   state posterior  Eq. 1 / Eq. 15
 *   semifield ops    Eq. 8-12: a (+) b = log(e^a + e^b), a (x) b = a + b,
 *                    a (/) b = a - b, zero = -inf, one = 0
 *   LF-MMI           Eq. 16 (objective) and Eq. 17 (its derivative)
 *
 * One sequence at a time, frame by frame, every step a scan over the whole arc
 * list.  No blocking, no fusion, no scaling tricks: doubles have the range.
 * Only tests, the smoke check and the CPU-baseline leg of the benchmark may
 * call this file; the GPU library shares nothing with it.
 *
 * Readings of the paper adopted here (the paper is silent or garbled there):
 *   - Eq. 2 sums over z_{n-1} (it prints z_n, which is the free variable).
 *   - Eq. 5 / Eq. 14 print v_n next to beta_{n+1}; the scalar Eq. 3 has
 *     p(x_{n+1} | z_{n+1}), so v_{n+1} is used.
 *   - T[i][j] is the weight of the arc i -> j (row = source), which is the only
 *     reading under which Eq. 4 multiplies alpha by T transposed.
 *   - The paper gives no initial / final condition.  alpha_0 = init (x) v_0 (the
 *     first state emits the first frame) and beta_{last} = final; the paper's
 *     case "sum over all states of alpha_N" (Eq. 1) is final == 0 everywhere.
 *   - State k emits through pdf[k]: v_n[k] = emis[n][pdf[k]]; the derivative of
 *     log Z w.r.t. emis[n][d] is the sum of the posteriors of the states tied
 *     to d (chain rule applied to Eq. 17's phi).
 *   - Variable lengths: a sequence of T frames is simply run over frames
 *     0..T-1; padded frames have posterior 0.
 *   - An empty or all-zero (+)-sum is the semiring zero, never NaN;
 *     exp(zero - finite) = 0; if log Z is zero the posteriors are all 0.
 *   - Parallel arcs stay separate arcs; their weights (+)-add.
 *
 * Every function here is pinned by tests/test_oracle_*.py (brute-force path
 * enumeration, dense probability-domain matrices, closed forms, invariants,
 * finite differences, a hand-computed example).  Nothing is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ZERO_BAR (-INFINITY)

typedef struct {
    int32_t K;
    int64_t E;
    const int32_t *src, *dst;
    const float *logw;
    const int32_t *pdf;
    const float *init, *fin;
} graph_t;

/* y[j] = (+)-sum over arcs e with head[e] == j of ( w[e] (x) x[tail[e]] ), j in [lo, hi).
 * Two scans of the arc list: the largest term of every sum, then the sum of
 * exponentials relative to it (the usual stable evaluation of Eq. 8). */
static void semiring_matvec(int64_t E, const int32_t *tail, const int32_t *head, const float *w,
                            int64_t elo, int64_t ehi, int32_t lo, int32_t hi,
                            const double *x, double *y, double *mx)
{
    (void)E;
    for (int32_t j = lo; j < hi; ++j) { mx[j] = ZERO_BAR; y[j] = 0.0; }
    for (int64_t e = elo; e < ehi; ++e) {
        double t = (double)w[e] + x[tail[e]];
        if (t > mx[head[e]]) mx[head[e]] = t;
    }
    for (int64_t e = elo; e < ehi; ++e) {
        int32_t j = head[e];
        if (mx[j] == ZERO_BAR) continue;
        double t = (double)w[e] + x[tail[e]];
        y[j] += exp(t - mx[j]);
    }
    for (int32_t j = lo; j < hi; ++j)
        y[j] = (mx[j] == ZERO_BAR) ? ZERO_BAR : mx[j] + log(y[j]);
}

static double lse_pairs(const double *a, const float *b, int32_t lo, int32_t hi)
{
    double m = ZERO_BAR;
    for (int32_t k = lo; k < hi; ++k) { double t = a[k] + (double)b[k]; if (t > m) m = t; }
    if (m == ZERO_BAR) return ZERO_BAR;
    double s = 0.0;
    for (int32_t k = lo; k < hi; ++k) s += exp(a[k] + (double)b[k] - m);
    return m + log(s);
}

/* Forward-backward of one sequence over the states [klo, khi) and the arcs
 * [elo, ehi) of g (the whole graph when it is shared; one diagonal block when
 * graphs are packed).  emis: T rows of D floats, row stride ld.  alpha, beta,
 * gamma: [T][khi-klo] doubles; rho: [T][D] doubles (gamma, rho nullable).
 * Returns log Z. */
static double fb_sequence(const graph_t *g, int32_t klo, int32_t khi, int64_t elo, int64_t ehi,
                          const float *emis, int64_t ld, int32_t D, int32_t T,
                          double *alpha, double *beta, double *gamma, double *rho)
{
    int32_t Kb = khi - klo;
    double *x = (double *)malloc(sizeof(double) * (size_t)g->K);
    double *y = (double *)malloc(sizeof(double) * (size_t)g->K);
    double *mx = (double *)malloc(sizeof(double) * (size_t)g->K);
    double logz;

    /* alpha_0 = init (x) v_0 ;  alpha_n = v_n o (T^t alpha_{n-1})   (Eq. 13) */
    for (int32_t n = 0; n < T; ++n) {
        const float *v = emis + (int64_t)n * ld;
        double *a = alpha + (int64_t)n * Kb;
        if (n == 0) {
            for (int32_t k = klo; k < khi; ++k) a[k - klo] = (double)g->init[k] + (double)v[g->pdf[k]];
        } else {
            const double *ap = alpha + (int64_t)(n - 1) * Kb;
            for (int32_t k = klo; k < khi; ++k) x[k] = ap[k - klo];
            semiring_matvec(g->E, g->src, g->dst, g->logw, elo, ehi, klo, khi, x, y, mx);
            for (int32_t k = klo; k < khi; ++k) a[k - klo] = (double)v[g->pdf[k]] + y[k];
        }
    }
    /* log Z = (+)-sum_k alpha_{T-1}[k] (x) final[k]   (denominator of Eq. 1) */
    for (int32_t k = klo; k < khi; ++k) x[k] = alpha[(int64_t)(T - 1) * Kb + (k - klo)];
    logz = lse_pairs(x, g->fin, klo, khi);

    /* beta_{T-1} = final ;  beta_n = T (beta_{n+1} o v_{n+1})   (Eq. 14) */
    for (int32_t n = T - 1; n >= 0; --n) {
        double *bn = beta + (int64_t)n * Kb;
        if (n == T - 1) {
            for (int32_t k = klo; k < khi; ++k) bn[k - klo] = (double)g->fin[k];
        } else {
            const float *v = emis + (int64_t)(n + 1) * ld;
            const double *bp = beta + (int64_t)(n + 1) * Kb;
            for (int32_t k = klo; k < khi; ++k) x[k] = bp[k - klo] + (double)v[g->pdf[k]];
            /* roles of the arc ends swapped: gather at the destination, write at the source */
            semiring_matvec(g->E, g->dst, g->src, g->logw, elo, ehi, klo, khi, x, y, mx);
            for (int32_t k = klo; k < khi; ++k) bn[k - klo] = y[k];
        }
    }
    /* gamma_n[k] = exp(alpha_n[k] (x) beta_n[k] (/) log Z)   (Eq. 15);
     * rho_n[d] = sum of gamma_n over the states tied to pdf d */
    if (gamma || rho) {
        for (int32_t n = 0; n < T; ++n) {
            if (rho) for (int32_t d = 0; d < D; ++d) rho[(int64_t)n * D + d] = 0.0;
            for (int32_t k = klo; k < khi; ++k) {
                double a = alpha[(int64_t)n * Kb + (k - klo)], b = beta[(int64_t)n * Kb + (k - klo)];
                double p = (a == ZERO_BAR || b == ZERO_BAR || logz == ZERO_BAR) ? 0.0 : exp(a + b - logz);
                if (gamma) gamma[(int64_t)n * Kb + (k - klo)] = p;
                if (rho) rho[(int64_t)n * D + g->pdf[k]] += p;
            }
        }
    }
    free(x); free(y); free(mx);
    return logz;
}

static void block_range(const graph_t *g, const int32_t *state_off, const int64_t *arc_off,
                        int32_t b, int32_t *klo, int32_t *khi, int64_t *elo, int64_t *ehi)
{
    if (state_off) { *klo = state_off[b]; *khi = state_off[b + 1]; *elo = arc_off[b]; *ehi = arc_off[b + 1]; }
    else { *klo = 0; *khi = g->K; *elo = 0; *ehi = g->E; }
}

/*
 * Forward-backward of the selected sequences sel[0..nsel) of a batch.
 *
 * Graph: K states, E arcs in any order for a shared graph (state_off == NULL);
 * for packed graphs state_off[B+1] gives each sequence's state range and the
 * arcs must be grouped by sequence with arc_off[B+1] giving each group.
 * emis: [B][N][D] floats; lengths[B].
 * Outputs for the i-th selected sequence b = sel[i], with Kb its state count
 * and ooff[i] the offset (in elements) of its block in alpha/beta/gamma:
 *   alpha/beta/gamma + ooff[i] : [lengths[b]][Kb] doubles (gamma nullable)
 *   rho + i*N*D : [N][D] doubles, rows >= lengths[b] zero (nullable)
 *   logz[i]
 * Returns 0, or -1 on a malformed argument.
 */
int fbo_forward_backward(int32_t K, int64_t E, const int32_t *src, const int32_t *dst, const float *logw,
                         const int32_t *pdf, const float *init, const float *fin,
                         const int32_t *state_off, const int64_t *arc_off,
                         const float *emis, const int32_t *lengths, int32_t B, int32_t N, int32_t D,
                         const int32_t *sel, int32_t nsel, const int64_t *ooff,
                         double *alpha, double *beta, double *gamma, double *rho, double *logz)
{
    graph_t g = { K, E, src, dst, logw, pdf, init, fin };
    if (K <= 0 || E < 0 || B <= 0 || N <= 0 || D <= 0 || nsel < 0) return -1;
    for (int32_t i = 0; i < nsel; ++i)
        if (sel[i] < 0 || sel[i] >= B || lengths[sel[i]] < 1 || lengths[sel[i]] > N) return -1;
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t i = 0; i < nsel; ++i) {
        int32_t b = sel[i], klo, khi; int64_t elo, ehi;
        block_range(&g, state_off, arc_off, b, &klo, &khi, &elo, &ehi);
        int32_t T = lengths[b];
        double *r = rho ? rho + (int64_t)i * N * D : NULL;
        if (r) memset(r, 0, sizeof(double) * (size_t)N * D);
        double z = fb_sequence(&g, klo, khi, elo, ehi, emis + (int64_t)b * N * D, D, D, T,
                               alpha + ooff[i], beta + ooff[i], gamma ? gamma + ooff[i] : NULL, r);
        logz[i] = z;
        if (z != z) bad = 1;
    }
    return bad ? -2 : 0;
}

/*
 * LF-MMI objective and derivative for the selected sequences (Eq. 16, Eq. 17):
 *   logz_num[i], logz_den[i]; grad + i*N*D : [N][D] = rho_num - rho_den (rows
 *   past the sequence's length are zero).  The objective of the selection is
 *   the sum over i of logz_num[i] - logz_den[i], left to the caller.
 * den: shared graph.  num: packed graphs (state_off / arc_off as above).
 */
int fbo_lfmmi(int32_t Kd, int64_t Ed, const int32_t *dsrc, const int32_t *ddst, const float *dlogw,
              const int32_t *dpdf, const float *dinit, const float *dfin,
              int32_t Kn, int64_t En, const int32_t *nsrc, const int32_t *ndst, const float *nlogw,
              const int32_t *npdf, const float *ninit, const float *nfin,
              const int32_t *state_off, const int64_t *arc_off,
              const float *emis, const int32_t *lengths, int32_t B, int32_t N, int32_t D,
              const int32_t *sel, int32_t nsel,
              double *logz_num, double *logz_den, double *grad)
{
    graph_t gd = { Kd, Ed, dsrc, ddst, dlogw, dpdf, dinit, dfin };
    graph_t gn = { Kn, En, nsrc, ndst, nlogw, npdf, ninit, nfin };
    if (Kd <= 0 || Kn <= 0 || B <= 0 || N <= 0 || D <= 0 || !state_off || !arc_off) return -1;
    for (int32_t i = 0; i < nsel; ++i)
        if (sel[i] < 0 || sel[i] >= B || lengths[sel[i]] < 1 || lengths[sel[i]] > N) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t i = 0; i < nsel; ++i) {
        int32_t b = sel[i], T = lengths[b];
        const float *em = emis + (int64_t)b * N * D;
        double *gr = grad + (int64_t)i * N * D;
        memset(gr, 0, sizeof(double) * (size_t)N * D);
        double *rho = (double *)malloc(sizeof(double) * (size_t)T * D);

        /* numerator: this utterance's own graph */
        int32_t klo = state_off[b], khi = state_off[b + 1], Kb = khi - klo;
        double *a = (double *)malloc(sizeof(double) * (size_t)T * Kb);
        double *bt = (double *)malloc(sizeof(double) * (size_t)T * Kb);
        logz_num[i] = fb_sequence(&gn, klo, khi, arc_off[b], arc_off[b + 1], em, D, D, T, a, bt, NULL, rho);
        for (int64_t t = 0; t < (int64_t)T * D; ++t) gr[t] += rho[t];
        free(a); free(bt);

        /* denominator: the graph shared by all utterances */
        a = (double *)malloc(sizeof(double) * (size_t)T * Kd);
        bt = (double *)malloc(sizeof(double) * (size_t)T * Kd);
        logz_den[i] = fb_sequence(&gd, 0, Kd, 0, Ed, em, D, D, T, a, bt, NULL, rho);
        for (int64_t t = 0; t < (int64_t)T * D; ++t) gr[t] -= rho[t];
        free(a); free(bt); free(rho);
    }
    return 0;
}

int fbo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void fbo_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
