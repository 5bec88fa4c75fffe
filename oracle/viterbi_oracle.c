/*
 * viterbi_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * The extension the paper's last section (conclusion and future work) names:
 * the same forward recursion with the log semiring replaced by the tropical
 * semiring, a (+) b = max(a, b), a (x) b = a + b, zero = -inf, one = 0, which
 * is the Viterbi algorithm.  Written out plainly in double precision, one
 * sequence at a time, every step a scan over the whole arc list:
 *
 *   delta_0[k] = init[k] + v_0[k]
 *   delta_n[j] = v_n[j] + max over arcs e into j of ( w_e + delta_{n-1}[src_e] )   (Eq. 13 with (+) = max)
 *   psi_n[j]   = the source state of an arc that attains that maximum (the first such arc in the list)
 *   score      = max_k ( delta_{T-1}[k] + final[k] )                               (Eq. 1's denominator with (+) = max)
 *   path       = back-pointers followed from a state that attains the score
 *
 * Same readings as the log-semiring oracle (start state emits frame 0, v_n[k] =
 * emis[n][pdf[k]], lengths give the frames that count).  Several paths may attain
 * the score; the score is unique, the path returned here is one of them.
 * Pinned by tests/test_viterbi_pins.py: exhaustive path enumeration, the limit
 * temperature * log Z(1 / temperature) -> score of the pinned log-semiring
 * oracle, and the bounds score <= log Z <= score + log(number of paths).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

/*
 * Best path of the selected sequences sel[0..nsel) of a batch.  Graph and emissions as in
 * fbo_forward_backward (packed graphs: arcs grouped by sequence, arc_off[B+1]).
 * score[i]; path + i*N: N int32, the state (global numbering) at every frame < lengths[b], -1 after,
 * all -1 when the score is -inf.  Returns 0, or -1 on a malformed argument.
 */
int vto_viterbi(int32_t K, int64_t E, const int32_t *src, const int32_t *dst, const float *logw,
                const int32_t *pdf, const float *init, const float *fin,
                const int32_t *state_off, const int64_t *arc_off,
                const float *emis, const int32_t *lengths, int32_t B, int32_t N, int32_t D,
                const int32_t *sel, int32_t nsel, double *score, int32_t *path)
{
    if (K <= 0 || E < 0 || B <= 0 || N <= 0 || D <= 0 || nsel < 0) return -1;
    for (int32_t i = 0; i < nsel; ++i)
        if (sel[i] < 0 || sel[i] >= B || lengths[sel[i]] < 1 || lengths[sel[i]] > N) return -1;
    for (int32_t i = 0; i < nsel; ++i) {
        const int32_t b = sel[i], T = lengths[b];
        const int32_t klo = state_off ? state_off[b] : 0, khi = state_off ? state_off[b + 1] : K;
        const int64_t elo = state_off ? arc_off[b] : 0, ehi = state_off ? arc_off[b + 1] : E;
        const float *em = emis + (int64_t)b * N * D;
        double *prev = (double *)malloc(sizeof(double) * (size_t)K);
        double *cur = (double *)malloc(sizeof(double) * (size_t)K);
        int32_t *psi = (int32_t *)malloc(sizeof(int32_t) * (size_t)T * (size_t)K);
        for (int32_t k = klo; k < khi; ++k) prev[k] = (double)init[k] + (double)em[pdf[k]];
        for (int32_t n = 1; n < T; ++n) {
            const float *v = em + (int64_t)n * D;
            for (int32_t k = klo; k < khi; ++k) { cur[k] = -INFINITY; psi[(int64_t)n * K + k] = -1; }
            for (int64_t e = elo; e < ehi; ++e) {
                const double t = (double)logw[e] + prev[src[e]];
                if (t > cur[dst[e]]) { cur[dst[e]] = t; psi[(int64_t)n * K + dst[e]] = src[e]; }
            }
            for (int32_t k = klo; k < khi; ++k) cur[k] += (double)v[pdf[k]];
            double *sw = prev; prev = cur; cur = sw;
        }
        double best = -INFINITY;
        int32_t at = -1;
        for (int32_t k = klo; k < khi; ++k) {
            const double t = prev[k] + (double)fin[k];
            if (t > best) { best = t; at = k; }
        }
        score[i] = best;
        for (int32_t n = 0; n < N; ++n) path[(int64_t)i * N + n] = -1;
        for (int32_t n = T - 1; n >= 0 && at >= 0; --n) {
            path[(int64_t)i * N + n] = at;
            if (n > 0) at = psi[(int64_t)n * K + at];
        }
        free(prev); free(cur); free(psi);
    }
    return 0;
}
