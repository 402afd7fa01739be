/*
 * Plain fp64 CPU oracle of the semi-Markov CRF forward-backward pass.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing on the product path may call this file:
 * it exists so that the GPU library can be checked against a slow, obviously
 * correct implementation of the textbook O(T*K*C^2) recurrence.  It shares no
 * code, tables or helpers with the HIP kernels.
 *
 * What it computes (per sequence b of true length L = lengths[b]):
 *   - the emission baseline nu[c] and the centred prefix sums S[t,c]
 *     (paper Eq. 1 and Eq. 2, masked mean over the L valid positions);
 *   - the edge potential psi(t,k,c,c') of Eq. 4,
 *         psi = S[t,c] - S[t-k,c] + dur[k-1,c] + trans[c',c] + bs[t-k,c] + be[t-1,c],
 *     where bs / be are the optional boundary projections of the "Boundary
 *     Projections" section (start score of the segment's first token, end score of
 *     its last token; zero when absent), to which the optional scalar sequence
 *     boundaries pi_start[c] / pi_end[c] are added at token 0 / token L-1
 *     (appendix on boundary handling, composition rule); optionally trans carries a
 *     duration index, trans[k-1,c',c] (the [K,C,C] transition whose gradient the
 *     gradient-workspace section allocates), and so does its gradient;
 *   - log-forward messages alpha[t,c] by the recurrence of Algorithm 1
 *     (alpha[0,:] = 0, k <= min(K,t)) but with the FULL table kept: no ring
 *     buffer, no checkpoints, no normalisation;
 *   - logZ = LSE_c alpha[L,c]  (Algorithm 1, last line, with T -> L);
 *   - log-backward messages beta[t,c'] (Algorithm 3: beta[L,:] = 0,
 *     k <= min(K, L-t)), again as a full table;
 *   - segment marginals mu(t,k,c,c') = exp(alpha[t,c'] + psi(t+k,k,c,c')
 *     + beta[t+k,c] - logZ) ("Gradient Computation" section) and from them the
 *     expected sufficient statistics of the "Gradient Formulas" section:
 *         gS[t+k,c] += mu,  gS[t,c] -= mu,
 *         gTr[c',c] += w*mu, gD[k-1,c] += w*mu       (w = upstream dL/dlogZ_b),
 *     and, since psi is linear in them, gPs[t,c] += w*mu, gPe[t+k-1,c] += w*mu for the
 *     boundary projections (gradients of the scalar boundaries: the rows of token 0 /
 *     token L-1 summed over sequences); the posterior that a segment boundary falls at
 *     position t, sum_c exp(alpha[t,c] + beta[t,c] - logZ);
 *   - the chain rule through Eq. 2 and Eq. 1 (the paper leaves this to
 *     autograd): pm[u,c] = sum_{t>u} gS[t,c] is the gradient w.r.t. the centred
 *     emission, i.e. the posterior that token u carries label c, and
 *     gE[u,c] = w*(pm[u,c] - mean_u' pm[u',c]) is the gradient w.r.t. the raw
 *     emission when centring is on (w*pm[u,c] when it is off).
 *
 * Logsumexp of an empty set is a true -inf; every LSE is max-shifted and
 * guarded so that -inf inputs never produce NaN.  No clamps are applied.
 *
 * Threading: OpenMP over sequences; when there are fewer sequences than
 * threads the destination-label loop inside a position is split as well.
 * Neither changes the arithmetic or its order for any single output element.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double lse_pair_guard(double m, double s) {
    /* m = running max, s = sum of exp(x - m); returns max + log(sum) */
    if (m == -INFINITY) return -INFINITY;
    return m + log(s);
}

/* tks = 0: trans is [C,C] as in Eq. 4; tks = C*C: trans is [K,C,C], one matrix per duration
 * (the duration-indexed transition of the gradient-workspace section). */
#define PSI(t, k, c, cp) (S[(size_t)(t) * C + (c)] - S[(size_t)((t) - (k)) * C + (c)] \
                          + dur[(size_t)((k) - 1) * C + (c)] \
                          + trans[(size_t)((k) - 1) * tks + (size_t)(cp) * C + (c)] \
                          + bs[(size_t)((t) - (k)) * C + (c)] + be[(size_t)((t) - 1) * C + (c)])

/* Eq. 1 (masked mean over the L valid positions) and Eq. 2 (S[0,c] = 0,
 * S[t,c] = sum_{u<t} (f[u,c] - nu[c])).  S must hold (L+1)*C zeros on entry. */
static void oracle_prefix_sums(const double *f, int L, int C, int center, double *nu, double *S)
{
    for (int c = 0; c < C; ++c) nu[c] = 0.0;
    if (center && L > 0) {
        for (int c = 0; c < C; ++c) {
            double acc = 0.0;
            for (int u = 0; u < L; ++u) acc += f[(size_t)u * C + c];
            nu[c] = acc / (double)L;
        }
    }
    for (int t = 1; t <= L; ++t)
        for (int c = 0; c < C; ++c)
            S[(size_t)t * C + c] = S[(size_t)(t - 1) * C + c] + (f[(size_t)(t - 1) * C + c] - nu[c]);
}

/* Algorithm 1 with the whole table kept (alpha[0,:] = 0); returns
 * logZ = LSE_c alpha[L,c]. */
static double oracle_forward(const double *S, const double *trans, size_t tks, const double *dur,
                             const double *bs, const double *be,
                             int L, int K, int C, int inner_threads, double *alpha)
{
    (void)inner_threads;
    for (int c = 0; c < C; ++c) alpha[c] = 0.0;
    for (int t = 1; t <= L; ++t) {
        int kmax = K < t ? K : t;
#pragma omp parallel for num_threads(inner_threads) if (inner_threads > 1) schedule(static)
        for (int c = 0; c < C; ++c) {
            double m = -INFINITY;
            for (int k = 1; k <= kmax; ++k)
                for (int cp = 0; cp < C; ++cp) {
                    double x = alpha[(size_t)(t - k) * C + cp] + PSI(t, k, c, cp);
                    if (x > m) m = x;
                }
            double s = 0.0;
            if (m != -INFINITY)
                for (int k = 1; k <= kmax; ++k)
                    for (int cp = 0; cp < C; ++cp)
                        s += exp(alpha[(size_t)(t - k) * C + cp] + PSI(t, k, c, cp) - m);
            alpha[(size_t)t * C + c] = lse_pair_guard(m, s);
        }
    }
    double m = -INFINITY, s = 0.0;
    for (int c = 0; c < C; ++c)
        if (alpha[(size_t)L * C + c] > m) m = alpha[(size_t)L * C + c];
    if (m != -INFINITY)
        for (int c = 0; c < C; ++c) s += exp(alpha[(size_t)L * C + c] - m);
    return lse_pair_guard(m, s);
}

/* Start / end scores per token for one sequence: the boundary projections (or zeros)
 * plus the scalar sequence boundaries at token 0 / token L-1.  Rows 0..L-1 (at least one
 * row is allocated so that the arrays are never empty). */
static void oracle_boundary_scores(const double *ps, const double *pe, const double *pis,
                                   const double *pie, int L, int C, double **bs_out, double **be_out)
{
    size_t n = (size_t)(L > 0 ? L : 1) * C;
    double *bs = (double *)calloc(n, sizeof(double));
    double *be = (double *)calloc(n, sizeof(double));
    for (int t = 0; t < L; ++t)
        for (int c = 0; c < C; ++c) {
            if (ps) bs[(size_t)t * C + c] = ps[(size_t)t * C + c];
            if (pe) be[(size_t)t * C + c] = pe[(size_t)t * C + c];
        }
    if (L > 0)
        for (int c = 0; c < C; ++c) {
            if (pis) bs[c] += pis[c];
            if (pie) be[(size_t)(L - 1) * C + c] += pie[c];
        }
    *bs_out = bs;
    *be_out = be;
}

/* One sequence.  All arrays are fp64.  Optional inputs and outputs may be NULL. */
static void oracle_sequence(const double *f,      /* [T,C] emissions of this sequence */
                            int L, int T, int K, int C, int center, double w,
                            const double *trans,  /* [C,C] source-major: trans[c'*C+c]; or [K,C,C] */
                            size_t tks,           /* 0, or C*C when trans has one matrix per duration */
                            const double *dur,    /* [K,C] row k-1 */
                            const double *ps,     /* [T,C] start projections or NULL */
                            const double *pe,     /* [T,C] end projections or NULL */
                            const double *pis,    /* [C] scalar start boundary or NULL */
                            const double *pie,    /* [C] scalar end boundary or NULL */
                            int inner_threads,
                            double *logz_out,
                            double *gE,           /* [T,C] */
                            double *pm,           /* [T,C] */
                            double *gTr,          /* [C,C] or [K,C,C], this sequence only, weighted by w */
                            double *gD,           /* [K,C]   this sequence only, weighted by w */
                            double *S_out,        /* [T+1,C] or NULL */
                            double *alpha_out,    /* [T+1,C] or NULL */
                            double *beta_out,     /* [T+1,C] or NULL */
                            double *gS_out,       /* [T+1,C] or NULL */
                            double *gPs,          /* [T,C] or NULL, weighted by w */
                            double *gPe,          /* [T,C] or NULL, weighted by w */
                            double *bdy)          /* [T+1] or NULL: boundary posterior */
{
    (void)inner_threads;
    size_t n1 = (size_t)(L + 1) * C;
    double *nu = (double *)calloc((size_t)C, sizeof(double));
    double *S = (double *)calloc(n1, sizeof(double));
    double *alpha = (double *)malloc(n1 * sizeof(double));
    double *beta = (double *)malloc(n1 * sizeof(double));
    double *gS = (double *)calloc(n1, sizeof(double));

    double *bs, *be;
    oracle_boundary_scores(ps, pe, pis, pie, L, C, &bs, &be);

    oracle_prefix_sums(f, L, C, center, nu, S);
    double logz = oracle_forward(S, trans, tks, dur, bs, be, L, K, C, inner_threads, alpha);
    *logz_out = logz;

    /* Algorithm 3 recurrence with the whole table kept: beta[L,:] = 0. */
    for (int c = 0; c < C; ++c) beta[(size_t)L * C + c] = 0.0;
    for (int t = L - 1; t >= 0; --t) {
        int kmax = K < (L - t) ? K : (L - t);
#pragma omp parallel for num_threads(inner_threads) if (inner_threads > 1) schedule(static)
        for (int cp = 0; cp < C; ++cp) {
            double m = -INFINITY;
            for (int k = 1; k <= kmax; ++k)
                for (int c = 0; c < C; ++c) {
                    double x = PSI(t + k, k, c, cp) + beta[(size_t)(t + k) * C + c];
                    if (x > m) m = x;
                }
            double s = 0.0;
            if (m != -INFINITY)
                for (int k = 1; k <= kmax; ++k)
                    for (int c = 0; c < C; ++c)
                        s += exp(PSI(t + k, k, c, cp) + beta[(size_t)(t + k) * C + c] - m);
            beta[(size_t)t * C + cp] = lse_pair_guard(m, s);
        }
    }

    /* Marginals and expected sufficient statistics.  The destination label c
     * is the outer loop so that every accumulator element is owned by one c. */
    memset(gTr, 0, sizeof(double) * (tks ? (size_t)K * C * C : (size_t)C * C));
    memset(gD, 0, sizeof(double) * (size_t)K * C);
    if (gPs) memset(gPs, 0, sizeof(double) * (size_t)T * C);
    if (gPe) memset(gPe, 0, sizeof(double) * (size_t)T * C);
#pragma omp parallel for num_threads(inner_threads) if (inner_threads > 1) schedule(static)
    for (int c = 0; c < C; ++c) {
        for (int t = 0; t < L; ++t) {
            int kmax = K < (L - t) ? K : (L - t);
            for (int k = 1; k <= kmax; ++k)
                for (int cp = 0; cp < C; ++cp) {
                    double lm = alpha[(size_t)t * C + cp] + PSI(t + k, k, c, cp)
                                + beta[(size_t)(t + k) * C + c] - logz;
                    double mu = exp(lm);
                    gTr[(size_t)(k - 1) * tks + (size_t)cp * C + c] += w * mu;
                    gD[(size_t)(k - 1) * C + c] += w * mu;
                    gS[(size_t)(t + k) * C + c] += mu;
                    gS[(size_t)t * C + c] -= mu;
                    if (gPs) gPs[(size_t)t * C + c] += w * mu;
                    if (gPe) gPe[(size_t)(t + k - 1) * C + c] += w * mu;
                }
        }
    }

    /* Chain rule through the prefix sum (Eq. 2) and the centring (Eq. 1). */
    for (int c = 0; c < C; ++c) {
        double run = 0.0, tot = 0.0;
        for (int u = L - 1; u >= 0; --u) {
            run += gS[(size_t)(u + 1) * C + c];
            pm[(size_t)u * C + c] = run;
            tot += run;
        }
        double mean = (center && L > 0) ? tot / (double)L : 0.0;
        for (int u = 0; u < L; ++u) gE[(size_t)u * C + c] = w * (pm[(size_t)u * C + c] - mean);
        for (int u = L; u < T; ++u) {
            pm[(size_t)u * C + c] = 0.0;
            gE[(size_t)u * C + c] = 0.0;
        }
    }

    /* Posterior that a segment boundary falls at position t (1 at t = 0 and t = L). */
    if (bdy) {
        for (int t = 0; t <= T; ++t) bdy[t] = 0.0;
        for (int t = 0; t <= L; ++t) {
            double a = 0.0;
            for (int c = 0; c < C; ++c) a += exp(alpha[(size_t)t * C + c] + beta[(size_t)t * C + c] - logz);
            bdy[t] = a;
        }
    }

    if (S_out) {
        memcpy(S_out, S, n1 * sizeof(double));
        for (size_t i = n1; i < (size_t)(T + 1) * C; ++i) S_out[i] = 0.0;
    }
    if (alpha_out) {
        memcpy(alpha_out, alpha, n1 * sizeof(double));
        for (size_t i = n1; i < (size_t)(T + 1) * C; ++i) alpha_out[i] = 0.0;
    }
    if (beta_out) {
        memcpy(beta_out, beta, n1 * sizeof(double));
        for (size_t i = n1; i < (size_t)(T + 1) * C; ++i) beta_out[i] = 0.0;
    }
    if (gS_out) {
        memcpy(gS_out, gS, n1 * sizeof(double));
        for (size_t i = n1; i < (size_t)(T + 1) * C; ++i) gS_out[i] = 0.0;
    }
    free(nu); free(S); free(alpha); free(beta); free(gS); free(bs); free(be);
}

/*
 * Batched entry point.  Returns the number of OpenMP threads it used
 * (outer * inner), or a negative value on bad arguments.
 *
 *   emis      [B,T,C]   raw emissions (rows u >= lengths[b] are never read)
 *   lengths   [B]       true lengths, each in [0,T]; NULL means all T
 *   trans     [C,C]     trans[c'*C + c], source label first
 *   dur       [K,C]     dur[(k-1)*C + c]
 *   grad_logz [B]       upstream weights w_b; NULL means all ones
 * Outputs (caller-allocated, fp64):
 *   logz [B]; grad_emis [B,T,C]; pos_marg [B,T,C]; grad_trans [C,C];
 *   grad_dur [K,C]; optional per-sequence grad_trans_b [B,C,C], grad_dur_b
 *   [B,K,C]; optional tables S, alpha, beta, gS each [B,T+1,C].
 */
static int oracle_batch(const double *emis, const int32_t *lengths,
                                    const double *trans, int per_duration, const double *dur, const double *grad_logz,
                                    const double *proj_start, const double *proj_end,
                                    const double *pi_start, const double *pi_end,
                                    int B, int T, int K, int C, int center, int threads,
                                    double *logz, double *grad_emis, double *pos_marg,
                                    double *grad_trans, double *grad_dur,
                                    double *grad_trans_b, double *grad_dur_b,
                                    double *S_out, double *alpha_out, double *beta_out, double *gS_out,
                                    double *grad_proj_start, double *grad_proj_end,
                                    double *grad_pi_start, double *grad_pi_end, double *bdy_post)
{
    if (B < 1 || T < 1 || K < 1 || C < 1) return -1;
    int nthreads = 1;
#ifdef _OPENMP
    nthreads = threads > 0 ? threads : omp_get_max_threads();
#endif
    int outer = B < nthreads ? B : nthreads;
    int inner = nthreads / outer;
    if (inner < 1) inner = 1;
    if (inner > C) inner = C;
#ifdef _OPENMP
    omp_set_max_active_levels(2);
#endif
    size_t tks = per_duration ? (size_t)C * C : 0;
    size_t cc = per_duration ? (size_t)K * C * C : (size_t)C * C;
    size_t kc = (size_t)K * C, tc = (size_t)T * C, t1c = (size_t)(T + 1) * C;
    double *gTr_b = grad_trans_b ? grad_trans_b : (double *)malloc(sizeof(double) * cc * B);
    double *gD_b = grad_dur_b ? grad_dur_b : (double *)malloc(sizeof(double) * kc * B);
    /* the scalar-boundary gradients are read off the projection gradients */
    int own_ps = !grad_proj_start && grad_pi_start, own_pe = !grad_proj_end && grad_pi_end;
    double *gPs = own_ps ? (double *)malloc(sizeof(double) * tc * B) : grad_proj_start;
    double *gPe = own_pe ? (double *)malloc(sizeof(double) * tc * B) : grad_proj_end;

#pragma omp parallel for num_threads(outer) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        int L = lengths ? lengths[b] : T;
        if (L < 0) L = 0;
        if (L > T) L = T;
        double w = grad_logz ? grad_logz[b] : 1.0;
        oracle_sequence(emis + tc * b, L, T, K, C, center, w, trans, tks, dur,
                        proj_start ? proj_start + tc * b : NULL, proj_end ? proj_end + tc * b : NULL,
                        pi_start, pi_end, inner,
                        logz + b, grad_emis + tc * b, pos_marg + tc * b,
                        gTr_b + cc * b, gD_b + kc * b,
                        S_out ? S_out + t1c * b : NULL,
                        alpha_out ? alpha_out + t1c * b : NULL,
                        beta_out ? beta_out + t1c * b : NULL,
                        gS_out ? gS_out + t1c * b : NULL,
                        gPs ? gPs + tc * b : NULL, gPe ? gPe + tc * b : NULL,
                        bdy_post ? bdy_post + (size_t)(T + 1) * b : NULL);
    }
    /* Fixed-order sum over sequences. */
    for (size_t i = 0; i < cc; ++i) {
        double a = 0.0;
        for (int b = 0; b < B; ++b) a += gTr_b[cc * b + i];
        grad_trans[i] = a;
    }
    for (size_t i = 0; i < kc; ++i) {
        double a = 0.0;
        for (int b = 0; b < B; ++b) a += gD_b[kc * b + i];
        grad_dur[i] = a;
    }
    for (int c = 0; c < C; ++c) {
        double as = 0.0, ae = 0.0;
        for (int b = 0; b < B; ++b) {
            int L = lengths ? lengths[b] : T;
            if (L > T) L = T;
            if (L < 1) continue;
            if (grad_pi_start) as += gPs[tc * b + c];
            if (grad_pi_end) ae += gPe[tc * b + (size_t)(L - 1) * C + c];
        }
        if (grad_pi_start) grad_pi_start[c] = as;
        if (grad_pi_end) grad_pi_end[c] = ae;
    }
    if (!grad_trans_b) free(gTr_b);
    if (!grad_dur_b) free(gD_b);
    if (own_ps) free(gPs);
    if (own_pe) free(gPe);
    return outer * inner;
}

int semicrf_oracle_fwd_bwd_boundary(const double *emis, const int32_t *lengths,
                                    const double *trans, const double *dur, const double *grad_logz,
                                    const double *proj_start, const double *proj_end,
                                    const double *pi_start, const double *pi_end,
                                    int B, int T, int K, int C, int center, int threads,
                                    double *logz, double *grad_emis, double *pos_marg,
                                    double *grad_trans, double *grad_dur,
                                    double *grad_trans_b, double *grad_dur_b,
                                    double *S_out, double *alpha_out, double *beta_out, double *gS_out,
                                    double *grad_proj_start, double *grad_proj_end,
                                    double *grad_pi_start, double *grad_pi_end, double *bdy_post)
{
    return oracle_batch(emis, lengths, trans, 0, dur, grad_logz, proj_start, proj_end, pi_start, pi_end,
                        B, T, K, C, center, threads, logz, grad_emis, pos_marg, grad_trans, grad_dur,
                        grad_trans_b, grad_dur_b, S_out, alpha_out, beta_out, gS_out,
                        grad_proj_start, grad_proj_end, grad_pi_start, grad_pi_end, bdy_post);
}

/*
 * Duration-dependent transitions: trans [K,C,C], trans[((k-1)*C + c')*C + c] replaces
 * trans[c',c] in the potential, i.e. psi(t,k,c,c') = S[t,c] - S[t-k,c] + dur[k-1,c] + trans[k-1,c',c];
 * grad_trans [K,C,C] is then the duration-indexed expected count sum_b w_b sum_t mu_b(t,k,c,c')
 * (the transition gradient with a duration index of the gradient-workspace section).  No
 * boundary terms.  Everything else as above.
 */
int semicrf_oracle_fwd_bwd_durtrans(const double *emis, const int32_t *lengths,
                                    const double *trans, const double *dur, const double *grad_logz,
                                    int B, int T, int K, int C, int center, int threads,
                                    double *logz, double *grad_emis, double *pos_marg,
                                    double *grad_trans, double *grad_dur)
{
    return oracle_batch(emis, lengths, trans, 1, dur, grad_logz, NULL, NULL, NULL, NULL,
                        B, T, K, C, center, threads, logz, grad_emis, pos_marg, grad_trans, grad_dur,
                        NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL);
}

/* The three-term form of Eq. 4 (no boundary terms). */
int semicrf_oracle_fwd_bwd(const double *emis, const int32_t *lengths,
                           const double *trans, const double *dur, const double *grad_logz,
                           int B, int T, int K, int C, int center, int threads,
                           double *logz, double *grad_emis, double *pos_marg,
                           double *grad_trans, double *grad_dur,
                           double *grad_trans_b, double *grad_dur_b,
                           double *S_out, double *alpha_out, double *beta_out, double *gS_out)
{
    return semicrf_oracle_fwd_bwd_boundary(emis, lengths, trans, dur, grad_logz, NULL, NULL, NULL, NULL,
                                           B, T, K, C, center, threads, logz, grad_emis, pos_marg,
                                           grad_trans, grad_dur, grad_trans_b, grad_dur_b,
                                           S_out, alpha_out, beta_out, gS_out, NULL, NULL, NULL, NULL, NULL);
}

/*
 * Forward only: logZ per sequence (same recurrence, same arithmetic).
 * Used for finite-difference checks, where the backward pass is not wanted.
 */
static int oracle_logz_batch(const double *emis, const int32_t *lengths,
                                 const double *trans, int per_duration, const double *dur,
                                 const double *proj_start, const double *proj_end,
                                 const double *pi_start, const double *pi_end,
                                 int B, int T, int K, int C, int center, int threads, double *logz)
{
    if (B < 1 || T < 1 || K < 1 || C < 1) return -1;
    int nthreads = 1;
#ifdef _OPENMP
    nthreads = threads > 0 ? threads : omp_get_max_threads();
#endif
    int outer = B < nthreads ? B : nthreads;
#pragma omp parallel for num_threads(outer) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        int L = lengths ? lengths[b] : T;
        if (L < 0) L = 0;
        if (L > T) L = T;
        const double *f = emis + (size_t)T * C * b;
        size_t n1 = (size_t)(L + 1) * C;
        double *nu = (double *)calloc((size_t)C, sizeof(double));
        double *S = (double *)calloc(n1, sizeof(double));
        double *alpha = (double *)malloc(n1 * sizeof(double));
        double *bs, *be;
        oracle_boundary_scores(proj_start ? proj_start + (size_t)T * C * b : NULL,
                               proj_end ? proj_end + (size_t)T * C * b : NULL, pi_start, pi_end, L, C, &bs, &be);
        oracle_prefix_sums(f, L, C, center, nu, S);
        logz[b] = oracle_forward(S, trans, per_duration ? (size_t)C * C : 0, dur, bs, be, L, K, C, 1, alpha);
        free(nu); free(S); free(alpha); free(bs); free(be);
    }
    return outer;
}

int semicrf_oracle_logz_boundary(const double *emis, const int32_t *lengths,
                                 const double *trans, const double *dur,
                                 const double *proj_start, const double *proj_end,
                                 const double *pi_start, const double *pi_end,
                                 int B, int T, int K, int C, int center, int threads, double *logz)
{
    return oracle_logz_batch(emis, lengths, trans, 0, dur, proj_start, proj_end, pi_start, pi_end,
                             B, T, K, C, center, threads, logz);
}

/* Forward only with duration-dependent transitions trans [K,C,C]. */
int semicrf_oracle_logz_durtrans(const double *emis, const int32_t *lengths,
                                 const double *trans, const double *dur,
                                 int B, int T, int K, int C, int center, int threads, double *logz)
{
    return oracle_logz_batch(emis, lengths, trans, 1, dur, NULL, NULL, NULL, NULL,
                             B, T, K, C, center, threads, logz);
}

int semicrf_oracle_logz(const double *emis, const int32_t *lengths,
                        const double *trans, const double *dur,
                        int B, int T, int K, int C, int center, int threads, double *logz)
{
    return semicrf_oracle_logz_boundary(emis, lengths, trans, dur, NULL, NULL, NULL, NULL,
                                        B, T, K, C, center, threads, logz);
}

/*
 * Viterbi decode (max semiring): the best-scoring segmentation under the same edge
 * potential psi of Eq. 4, with the same conventions as the sum recurrence (V[0,c] = 0 for
 * every label, so the first segment pays max_c' trans[c',c]; no end term).
 *     V[t,c] = max_{k <= min(K,t)} max_{c'} ( V[t-k,c'] + psi(t,k,c,c') ),   score = max_c V[L,c]
 * Full tables, (duration, source label) back-pointers, ties broken towards the smallest k, then
 * the smallest c' (strict ">" in scan order), final label = smallest argmax.  Outputs per
 * sequence: score; per token its segment's label and a flag that is 1 on the first token of a
 * segment (tokens beyond L: label -1, flag 0); the number of segments.
 */
int semicrf_oracle_viterbi(const double *emis, const int32_t *lengths,
                           const double *trans, const double *dur,
                           const double *proj_start, const double *proj_end,
                           const double *pi_start, const double *pi_end,
                           int B, int T, int K, int C, int center, int threads,
                           double *score, int32_t *labels, int32_t *starts, int32_t *nseg)
{
    const size_t tks = 0; /* one transition matrix for every duration */
    if (B < 1 || T < 1 || K < 1 || C < 1) return -1;
    int nthreads = 1;
#ifdef _OPENMP
    nthreads = threads > 0 ? threads : omp_get_max_threads();
#endif
    int outer = B < nthreads ? B : nthreads;
#pragma omp parallel for num_threads(outer) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        int L = lengths ? lengths[b] : T;
        if (L < 0) L = 0;
        if (L > T) L = T;
        const double *f = emis + (size_t)T * C * b;
        size_t n1 = (size_t)(L + 1) * C;
        double *nu = (double *)calloc((size_t)C, sizeof(double));
        double *S = (double *)calloc(n1, sizeof(double));
        double *V = (double *)malloc(n1 * sizeof(double));
        int32_t *bk = (int32_t *)calloc(n1, sizeof(int32_t));   /* best duration */
        int32_t *bc = (int32_t *)calloc(n1, sizeof(int32_t));   /* best source label */
        double *bs, *be;
        oracle_boundary_scores(proj_start ? proj_start + (size_t)T * C * b : NULL,
                               proj_end ? proj_end + (size_t)T * C * b : NULL, pi_start, pi_end, L, C, &bs, &be);
        oracle_prefix_sums(f, L, C, center, nu, S);
        for (int c = 0; c < C; ++c) V[c] = 0.0;
        for (int t = 1; t <= L; ++t) {
            int kmax = K < t ? K : t;
            for (int c = 0; c < C; ++c) {
                double best = -INFINITY;
                int kb = 0, cb = 0;
                for (int k = 1; k <= kmax; ++k)
                    for (int cp = 0; cp < C; ++cp) {
                        double x = V[(size_t)(t - k) * C + cp] + PSI(t, k, c, cp);
                        if (x > best) { best = x; kb = k; cb = cp; }
                    }
                V[(size_t)t * C + c] = best;
                bk[(size_t)t * C + c] = kb;
                bc[(size_t)t * C + c] = cb;
            }
        }
        int32_t *lab = labels + (size_t)T * b, *st = starts + (size_t)T * b;
        for (int u = 0; u < T; ++u) { lab[u] = -1; st[u] = 0; }
        int c = 0;
        double best = -INFINITY;
        for (int cc = 0; cc < C; ++cc)
            if (V[(size_t)L * C + cc] > best) { best = V[(size_t)L * C + cc]; c = cc; }
        score[b] = L > 0 ? best : 0.0;
        int ns = 0, t = L;
        while (t > 0) {
            int k = bk[(size_t)t * C + c], cp = bc[(size_t)t * C + c];
            for (int u = t - k; u < t; ++u) lab[u] = c;
            st[t - k] = 1;
            ++ns;
            t -= k;
            c = cp;
        }
        nseg[b] = ns;
        free(nu); free(S); free(V); free(bk); free(bc); free(bs); free(be);
    }
    return outer;
}

