// Host-side planning of a call (see plan.h).  No HIP here: this file also builds for the host alone.
#include "plan.h"

#include <math.h>

namespace semicrf_impl {

bool wave_tasks_per_cu(int K, int C, int *scan, int *interval)
{
    // bounded by the LDS windows and by registers (two scan waves per SIMD, one where the kernel needs more
    // than 256 registers; one interval wave per SIMD)
    if (C > 64) return false;
    const int CT = spec_ct_of(C);
    const int GW = 64 / pow2_ge8(CT);
    const int per_lane = (K + GW - 1) / GW;
    if (per_lane > 64) return false;
    const int NKW = per_lane <= 16 ? 16 : (per_lane <= 32 ? 32 : 64);
    const size_t lds = wave_lds_doubles(CT, NKW) * sizeof(double);
    if (lds > LDS_LIMIT) return false;
    const int fit = (int)(LDS_LIMIT / lds);
    const int scan_regs = (CT == 64 || (CT == 32 && NKW == 64)) ? 4 : 8;
    *scan = fit < scan_regs ? fit : scan_regs;
    const size_t ilds = interval_lds_doubles(CT, NKW) * sizeof(double);
    int iw = ilds <= LDS_LIMIT ? (int)(LDS_LIMIT / ilds) * interval_waves(CT, NKW) : 1;  // else the generic kernel
    *interval = iw < 4 ? iw : 4;
    return true;
}

bool spec_applies(int K, int C)
{
    if (C > 64) return false;
    const int CT = spec_ct_of(C);
    const int GW = 64 / pow2_ge8(CT);
    const int per_lane = (K + GW - 1) / GW;
    if (per_lane > 64) return false;
    const int NKW = per_lane <= 16 ? 16 : (per_lane <= 32 ? 32 : 64);
    return wave_lds_doubles(CT, NKW) * sizeof(double) <= LDS_LIMIT;
}

// Every (sequence, interval) is one single-wave task of the chunk-parallel scans (both directions, interval +
// warm-up positions each) and of the interval stage (interval positions, about 1.2x the cost per position and
// round).  Tasks run in rounds of as many as fit the chip at once (256 compute units; per compute unit 8 scan
// waves or 4 interval waves by registers, fewer when the K-deep LDS window is large), and a partly filled round
// costs a full one.  The interval is the multiple of 8 that minimises that cost, within
// [max(8, K/2), sqrt(T*K)]: below the lower end warm-ups and K-deep checkpoints dominate work and memory; the
// upper end is the spacing of Algorithm 1, so checkpoints and per-task buffers still grow like sqrt(T) for very
// long sequences.
int auto_interval(int B, int T, int K, int C)
{
    int per_scan = 0, per_int = 0;
    if (!wave_tasks_per_cu(K, C, &per_scan, &per_int)) {
        // generic kernels: sqrt(T*K) spacing scaled to spread B*T/interval tasks over 256 units
        double d = ceil(sqrt((double)T * (double)K * (double)B / 256.0));
        int di = d < 1.0 ? 1 : (d > (double)T ? T : (int)d);
        if (di >= 8) di = (di + 7) & ~7;
        return di > T ? T : di;
    }
    const double slots_scan = 256.0 * per_scan;
    const double slots_int = 256.0 * per_int;
    const double warm = (double)sum_warmup(K);
    const int dlo = K / 2 < 8 ? 8 : K / 2;
    const double dhi_d = ceil(sqrt((double)T * (double)K));
    int dhi = dhi_d > (double)T ? T : (int)dhi_d;
    if (dhi < dlo) dhi = dlo;
    int best = 0;
    double best_cost = 0.0;
    for (int n = 1; n <= 8192; ++n) {
        long long dl = (((long long)T + n - 1) / n + 7) & ~7LL;
        int d = dl > (long long)T ? T : (int)dl;
        if (d > dhi && d != T) continue;
        if (d > dhi && n > 1) continue;
        if (d < dlo && best) break;
        const double tasks = (double)B * (double)(((long long)T + d - 1) / d);
        const double cost = ceil(2.0 * tasks / slots_scan) * (warm + d) + 1.2 * ceil(tasks / slots_int) * d;
        if (!best || cost < best_cost) {
            best = d;
            best_cost = cost;
        }
        if (d <= dlo) break;
    }
    return best;
}

int low_memory_interval(int T, int K)
{
    const double d = ceil(sqrt((double)T * (double)K));
    if (d >= (double)T) return T;
    long long di = ((long long)d + 7) & ~7LL;
    return di > (long long)T ? T : (int)di;
}

int make_plan(int B, int T, int K, int C, int ckpt_interval, int want_grad, Plan *pl)
{
    if (!pl || B < 1 || T < 1 || K < 1 || C < 1 || ckpt_interval < 0) return SEMICRF_EINVAL;
    if (want_grad < 0 || (want_grad & ~(7 | PLAN_LOW_MEMORY)) || (want_grad & 7) > 3) return SEMICRF_EINVAL;
    const bool lowmem = (want_grad & PLAN_LOW_MEMORY) != 0;
    const int kind = want_grad & 7;
    if (lowmem && kind == 3) return SEMICRF_EINVAL;  // no row slots for the stored-row marginals in this plan
    if (C > 256) return SEMICRF_EUNSUPPORTED;
    if (T > (1 << 30) || (double)B * ((double)T + 1.0) * (double)C > 2.0e10) return SEMICRF_EUNSUPPORTED;
    if ((double)K * (double)C > 1.0e6) return SEMICRF_EUNSUPPORTED;  // far beyond any LDS budget; keeps the products below in range
    pl->Delta = ckpt_interval > 0 ? (ckpt_interval > T ? T : ckpt_interval)
                                  : (lowmem ? low_memory_interval(T, K) : auto_interval(B, T, K, C));
    pl->N = (int)(((long long)T + pl->Delta - 1) / pl->Delta);
    pl->NCH = T / PREP_CH + 1;
    pl->G = (NT / C) < K ? (NT / C) : K;
    pl->lds_scan = lds_doubles(K, C, pl->G, false) * sizeof(double);
    pl->lds_interval = lds_doubles(K, C, pl->G, true) * sizeof(double);
    if (pl->lds_scan > LDS_LIMIT) return SEMICRF_EUNSUPPORTED;
    if (kind && (pl->lds_interval > LDS_LIMIT || C > GRAD_CMAX)) return SEMICRF_EUNSUPPORTED;
    const size_t ntask = (size_t)B * pl->N;
    // Row slots of the interval stage: one per task where that is at most one wave per SIMD; the low-memory
    // plan keeps a few per sequence, so that the rows, like the checkpoints, grow with the interval only.
    const size_t cap = lowmem ? (size_t)LOWMEM_SLOTS_PER_SEQ * (size_t)B : (size_t)NSLOT_MAX;
    const size_t capped = cap < (size_t)NSLOT_MAX ? cap : (size_t)NSLOT_MAX;
    pl->nslot = (int)(ntask < capped ? ntask : capped);
    pl->nslot = (pl->nslot + 11) / 12 * 12;  // whole workgroups of three or four single-wave tasks
    const size_t b = (size_t)B, t1 = (size_t)T + 1, c = (size_t)C, k = (size_t)K, n = (size_t)pl->N;
    size_t *sz = pl->size;
    for (int j = 0; j < 32; ++j) sz[j] = 0, pl->off[j] = 0;
    const size_t g = kind ? 1 : 0;
    sz[PL_HDR] = b * SEQ_HDR_BYTES;
    sz[PL_NU] = b * c * 8;
    sz[PL_CHSUM] = b * pl->NCH * c * 8;
    sz[PL_CHMAX] = b * pl->NCH * 8;
    sz[PL_TABMAX] = 2 * 8;
    sz[PL_W] = k * c * 8;
    sz[PL_ETR] = c * c * 8;
    sz[PL_EI] = b * t1 * c * 16;
    sz[PL_SPEC] = 2 * b * 2 * (n + 1) * 8 + b * 2 * 4 + 256;  // spec_lr, spec_err, spec_ok
    sz[PL_NBASE] = b * t1 * c * 4;
    sz[PL_CKA] = b * (n + 1) * (k * c + c) * 8;
    sz[PL_CKB] = g * b * (n + 1) * (k * c + c) * 8;
    sz[PL_CKYA] = b * (n + 1) * 8;
    sz[PL_CKYB] = g * b * (n + 1) * 8;
    sz[PL_ALOC] = g * (size_t)pl->nslot * pl->Delta * 2 * c * 8;
    sz[PL_ALOCY] = g * (size_t)pl->nslot * pl->Delta * 8;
    sz[PL_MEAN] = g * b * FIN_SLICES * c * 8;
    sz[PL_CKA2] = b * (n + 1) * (k * c + c) * 8;
    sz[PL_CKB2] = g * b * (n + 1) * (k * c + c) * 8;
    sz[PL_CKYA2] = b * (n + 1) * 8;
    sz[PL_CKYB2] = g * b * (n + 1) * 8;
    sz[PL_OUT0] = b * c * 8;
    sz[PL_INL] = b * c * 8;
    // Marginals from the stored rows of both scans need a second set of row slots.  Measured, marginal stage
    // alone, against the interval kernels' own recurrence: K = 512, C = 8: 0.52 against 1.08 ms; K = 64, C = 24:
    // 0.18 against 0.33 ms; K = 32, C = 64: 0.09 against 0.19 ms; K = 16, C = 24, short sequences: level.  The
    // route is planned whenever every task has its slot and the sizes fit its kernels.
    const int mg_nsl = (K + MG_KS - 1) / MG_KS;
    const size_t mg_vr = (size_t)MG_TG + (size_t)MG_KS * mg_nsl + 3;
    pl->lds_mg_dur = (MG_TG * c + mg_vr * (c | 3) + MG_TG + 2 * mg_vr + 2 * (size_t)pl->Delta + k) * sizeof(double);
    pl->lds_mg_te = ((size_t)3 * MG_TE * c + pl->Delta) * sizeof(double);
    const int mg_gw = 64 / pow2_ge8(C > 64 ? 64 : C);
    const int mg_per_simd = mg_waves_per_simd(C, (K + mg_gw - 1) / mg_gw);  // of the one-wave kernel (K < 128)
    const bool rows = !lowmem && (kind == 3 || kind == 1);
    pl->rows = rows && spec_applies(K, C) && ntask <= (size_t)pl->nslot && c * mg_nsl <= 1024 &&
               pl->lds_mg_dur <= LDS_LIMIT && pl->lds_mg_te <= LDS_LIMIT;
    const size_t gr = pl->rows ? 1 : 0;
    sz[PL_BLOC] = gr * (size_t)pl->nslot * pl->Delta * 2 * c * 8;
    sz[PL_BLOCY] = gr * (size_t)pl->nslot * pl->Delta * 8;
    // With fewer intervals than the chip holds tasks of that kernel, each interval is cut into 2 or 4 equal
    // parts of at least K positions, each part a task with partial sums of its own.
    pl->msplit = 1;
    if (pl->rows && K < 128)
        while (pl->msplit < 4 && ntask * pl->msplit < (size_t)mg_per_simd * MG_SIMDS && pl->Delta % (2 * pl->msplit) == 0 &&
               pl->Delta / (2 * pl->msplit) >= (K < 32 ? 32 : K))
            pl->msplit *= 2;
    const size_t np = n * (size_t)pl->msplit;
    sz[PL_PARTD] = g * b * np * k * c * 8;
    sz[PL_PARTTR] = g * b * np * c * c * 8;
    sz[PL_TOT] = g * b * np * c * 8;
    sz[PL_SUMR] = g * b * np * c * 8;
    sz[PL_CARRY] = g * b * np * c * 8;
    sz[PL_SINK] = (size_t)SINK_DOUBLES * 8;
    pl->narrays = PL_COUNT;
    size_t off = 0;
    for (int j = 0; j < PL_COUNT; ++j) {
        pl->off[j] = off;
        off += align_up(sz[j]);
    }
    pl->total = off;
    return SEMICRF_OK;
}

int check_flags(unsigned flags)
{
    if ((flags & SEMICRF_EMIS_F16) && (flags & SEMICRF_EMIS_BF16)) return SEMICRF_EINVAL;
    if ((flags & SEMICRF_MARGINALS_ROWS) && (flags & SEMICRF_MARGINALS_INTERVAL)) return SEMICRF_EINVAL;
    if ((flags & SEMICRF_LOW_MEMORY) && (flags & SEMICRF_MARGINALS_ROWS)) return SEMICRF_EINVAL;
    return SEMICRF_OK;
}

}  // namespace semicrf_impl
