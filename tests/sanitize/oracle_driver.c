/* Runs every entry point of the oracle on small ragged inputs; built with -fsanitize=address,undefined by
 * tests/test_sanitizers_cpu.py, which fails on any report.  Prints one line per call. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int semicrf_oracle_fwd_bwd_boundary(const double *, const int32_t *, const double *, const double *, const double *,
                                    const double *, const double *, const double *, const double *, int, int, int,
                                    int, int, int, double *, double *, double *, double *, double *, double *,
                                    double *, double *, double *, double *, double *, double *, double *, double *,
                                    double *, double *);
int semicrf_oracle_fwd_bwd(const double *, const int32_t *, const double *, const double *, const double *, int, int,
                           int, int, int, int, double *, double *, double *, double *, double *, double *, double *,
                           double *, double *, double *, double *);
int semicrf_oracle_fwd_bwd_durtrans(const double *, const int32_t *, const double *, const double *, const double *,
                                    int, int, int, int, int, int, double *, double *, double *, double *, double *);
int semicrf_oracle_logz(const double *, const int32_t *, const double *, const double *, int, int, int, int, int, int,
                        double *);
int semicrf_oracle_logz_durtrans(const double *, const int32_t *, const double *, const double *, int, int, int, int,
                                 int, int, double *);
int semicrf_oracle_viterbi(const double *, const int32_t *, const double *, const double *, const double *,
                           const double *, const double *, const double *, int, int, int, int, int, int, double *,
                           int32_t *, int32_t *, int32_t *);

static uint64_t state = 0x9E3779B97F4A7C15ull;
static double rnd(void)
{
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (double)(state >> 11) / 9007199254740992.0 - 0.5;
}
static double *vec(size_t n, double scale)
{
    /* exact size: any access past the end is a report */
    double *p = (double *)malloc((n ? n : 1) * sizeof(double));
    for (size_t i = 0; i < n; ++i) p[i] = scale * rnd();
    return p;
}

static int one(int B, int T, int K, int C, int threads)
{
    const size_t btc = (size_t)B * T * C, bt1c = (size_t)B * (T + 1) * C;
    double *emis = vec(btc, 3.0), *trans = vec((size_t)C * C, 1.0), *dur = vec((size_t)K * C, 1.0);
    double *trans3 = vec((size_t)K * C * C, 1.0), *w = vec(B, 2.0);
    double *ps = vec(btc, 1.0), *pe = vec(btc, 1.0), *pis = vec(C, 1.0), *pie = vec(C, 1.0);
    int32_t *len = (int32_t *)malloc(B * sizeof(int32_t));
    for (int b = 0; b < B; ++b) len[b] = b == 0 ? T : (b == 1 ? 0 : (int)((rnd() + 0.5) * T));
    double *logz = vec(B, 0), *gE = vec(btc, 0), *pm = vec(btc, 0), *gT = vec((size_t)C * C, 0), *gD = vec((size_t)K * C, 0);
    double *gTb = vec((size_t)B * C * C, 0), *gDb = vec((size_t)B * K * C, 0);
    double *S = vec(bt1c, 0), *al = vec(bt1c, 0), *be = vec(bt1c, 0), *gS = vec(bt1c, 0);
    double *gPs = vec(btc, 0), *gPe = vec(btc, 0), *gPis = vec(C, 0), *gPie = vec(C, 0), *bdy = vec((size_t)B * (T + 1), 0);
    double *gT3 = vec((size_t)K * C * C, 0), *score = vec(B, 0);
    int32_t *labels = (int32_t *)malloc(((size_t)B * T + 1) * sizeof(int32_t));
    int32_t *starts = (int32_t *)malloc(((size_t)B * T + 1) * sizeof(int32_t));
    int32_t *nseg = (int32_t *)malloc(B * sizeof(int32_t));
    int bad = 0;
    int rc = semicrf_oracle_fwd_bwd(emis, len, trans, dur, w, B, T, K, C, 1, threads, logz, gE, pm, gT, gD, gTb, gDb, S,
                                    al, be, gS);
    bad |= rc < 0 || !isfinite(logz[0]);
    double l0 = logz[0];
    rc = semicrf_oracle_fwd_bwd(emis, NULL, trans, dur, NULL, B, T, K, C, 0, threads, logz, gE, pm, gT, gD, NULL, NULL,
                                NULL, NULL, NULL, NULL);
    bad |= rc < 0;
    rc = semicrf_oracle_fwd_bwd_boundary(emis, len, trans, dur, w, ps, pe, pis, pie, B, T, K, C, 1, threads, logz, gE, pm,
                                         gT, gD, gTb, gDb, S, al, be, gS, gPs, gPe, gPis, gPie, bdy);
    bad |= rc < 0 || !isfinite(logz[0]);
    rc = semicrf_oracle_fwd_bwd_durtrans(emis, len, trans3, dur, w, B, T, K, C, 1, threads, logz, gE, pm, gT3, gD);
    bad |= rc < 0 || !isfinite(logz[0]);
    rc = semicrf_oracle_logz(emis, len, trans, dur, B, T, K, C, 1, threads, logz);
    bad |= rc < 0 || fabs(logz[0] - l0) > 1e-9 * fmax(1.0, fabs(l0));
    rc = semicrf_oracle_logz_durtrans(emis, len, trans3, dur, B, T, K, C, 1, threads, logz);
    bad |= rc < 0;
    rc = semicrf_oracle_viterbi(emis, len, trans, dur, ps, pe, pis, pie, B, T, K, C, 1, threads, score, labels, starts,
                                nseg);
    bad |= rc < 0 || nseg[0] < 1 || nseg[0] > T;
    printf("B=%d T=%d K=%d C=%d threads=%d logz0=%.6f nseg0=%d %s\n", B, T, K, C, threads, l0, nseg[0],
           bad ? "BAD" : "ok");
    free(emis); free(trans); free(dur); free(trans3); free(w); free(ps); free(pe); free(pis); free(pie); free(len);
    free(logz); free(gE); free(pm); free(gT); free(gD); free(gTb); free(gDb); free(S); free(al); free(be); free(gS);
    free(gPs); free(gPe); free(gPis); free(gPie); free(bdy); free(gT3); free(score); free(labels); free(starts);
    free(nseg);
    return bad;
}

int main(void)
{
    int bad = 0;
    bad |= one(3, 37, 5, 3, 1);
    bad |= one(2, 9, 12, 4, 2);   /* K > T */
    bad |= one(4, 64, 1, 7, 4);   /* K = 1 */
    bad |= one(1, 1, 1, 1, 1);
    bad |= one(5, 50, 8, 2, 8);   /* more threads than sequences: nested label threading */
    puts(bad ? "FAILED" : "ALL OK");
    return bad;
}
