// Streaming semi-Markov CRF forward-backward for gfx950 (MI355X).
//
// Numerical design.  The paper runs the recurrences of Algorithm 1 / Algorithm 3
// in the log domain in fp32 and renormalises at checkpoints.  CDNA has a full
// fp64 vector pipeline (half the fp32 FMA rate), so here the recurrences run in the
// LINEAR (probability) domain in fp64 with explicit power-of-two scaling; there
// is no exp/log inside any scan.  With a = exp(alpha), the factorised form of
// Eq. 4 (the transition does not depend on k, the rest not on the source label)
// reads, for a sequence with centred prefix sums S (Eq. 2):
//
//   forward   x_t(c) = sum_k W[k,c] q_{t-k}(c)            W = exp(dur)
//             a_t(c) = E_t(c) x_t(c)                       E_t(c) = exp(S[t,c])
//             z_t(c) = sum_c' a_t(c') Etr[c',c]            Etr = exp(trans)
//             q_t(c) = z_t(c) / E_t(c)                     (K-deep ring of q)
//   backward  p_t(c) = (1/E_t(c)) sum_k W[k,c] v_{t+k}(c)
//             b_t(c') = sum_c Etr[c',c] p_t(c)             b = exp(beta)
//             v_t(c') = b_t(c') E_t(c')                    (K-deep ring of v)
//   marginal  sum_c' mu(t,k,c,c') = q_t(c) W[k,c] v_{t+k}(c) / Z
//
// exp(S) would overflow, so positions are grouped in blocks of J positions and
// E is stored relative to a per-block, per-label power of two:
// ES_t(c) = exp(S[t,c] - n_j(c) ln 2), n_j(c) = round(S[jJ,c]/ln 2).  Rings are kept
// relative to the block of the position last processed and to one global
// power-of-two scale Y per direction; both are changed only by exact
// multiplications by powers of two at block boundaries.  logZ = Y ln 2 +
// log(sum_c a_L(c)).
//
// Kernels (each group in its own include file, see below): k_colsum (+ the exp tables), k_prep_seq,
// k_prefix (Eq. 1-2); k_spec, k_spec_repair, k_spec_cmp, k_spec_fix (Algorithm 1 and the beta
// recurrence of Algorithm 3 as chunk-parallel scans that are verified at every chunk boundary and
// write ring checkpoints every Delta positions; k_mscan in mscan.hip runs the same tasks sixteen at
// a time on the matrix cores); k_scan_fast / k_scan (the same scans sequentially, for what the
// verification rejects); k_interval_wave / k_interval (per checkpoint interval: recompute the forward
// messages unless the scan stored them, run beta across the interval, accumulate the expected
// sufficient statistics in registers/LDS, no global atomics); k_mg_dur / k_mg_te / k_mg_wave (the
// same statistics from the rows both scans stored, without a third recurrence); k_fin_seq (+ the
// parameter gradients), k_fin_emis (fixed-order reductions).  Interval choice and workspace layout:
// plan.cpp (host only).
#include <hip/hip_runtime.h>
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <mutex>
#include <type_traits>
#include <utility>

#include "semicrf.h"
#include "common.h"

// Workspace of semicrf_fwd_bwd_static: callers that cannot allocate (HIP graph capture, serving
// loops) get the library's scratch memory from this array instead of a workspace argument.  Every
// GPU the library runs on holds its own copy until the process ends.  In host code the name is only
// a handle for hipGetSymbolAddress; kernels receive the device address obtained there.
static __device__ __align__(256) unsigned char scratch[SEMICRF_STATIC_WORKSPACE_BYTES];

namespace {

using namespace semicrf_impl;

// The kernels, stage by stage (each file is included here, inside this namespace):
#include "prefix.inl"     // Eq. 1-2: baseline, centred prefix sums, block exponents, (ES, 1/ES)
#include "scan_seq.inl"   // sequential scans (fallback of the chunk-parallel ones)
#include "interval.inl"   // Algorithm 3 body: per-interval recompute + marginals; one-wave window geometry
#include "spec.inl"       // chunk-parallel scans with warm-up, repair and verification
#include "spec2.inl"      // the same scan tasks with two waves per task (tip + helper)
#include "viterbi.inl"    // max-semiring decode and trace-back
#include "finalise.inl"   // fixed-order reductions of the gradient formulas
#include "durtrans.inl"   // duration-dependent transitions
#include "marg.inl"       // marginals from the stored rows of both scans

// ---------------------------------------------------------------------------
// Host side: workspace carving, launches, the entry points.
// ---------------------------------------------------------------------------

void bind_workspace(Params &p, const Plan &pl, void *ws)
{
    char *w = (char *)ws;
    p.hdr = (SeqHdr *)(w + pl.off[0]);
    p.nu = (double *)(w + pl.off[1]);
    p.chsum = (double *)(w + pl.off[2]);
    p.chmax = (double *)(w + pl.off[3]);
    p.tabmax = (double *)(w + pl.off[4]);
    p.W = (double *)(w + pl.off[5]);
    p.Etr = (double *)(w + pl.off[6]);
    p.EI = (double2 *)(w + pl.off[7]);
    p.nbase = (int *)(w + pl.off[9]);
    p.ckA = (double *)(w + pl.off[10]);
    p.ckB = (double *)(w + pl.off[11]);
    p.ckYA = (double *)(w + pl.off[12]);
    p.ckYB = (double *)(w + pl.off[13]);
    p.aloc = (double *)(w + pl.off[14]);
    p.alocY = (double *)(w + pl.off[15]);
    p.NP = pl.N * pl.msplit;  // partial sums per sequence
    p.msplit = 1;             // parts per interval: set by the call that takes the one-wave stored-row marginals
    p.partD = (double *)(w + pl.off[16]);
    p.partTr = (double *)(w + pl.off[17]);
    p.tot = (double *)(w + pl.off[18]);
    p.sumR = (double *)(w + pl.off[19]);
    p.carry = (double *)(w + pl.off[20]);
    p.mean = (double *)(w + pl.off[21]);
    p.ckA2 = (double *)(w + pl.off[22]);
    p.ckB2 = (double *)(w + pl.off[23]);
    p.ckYA2 = (double *)(w + pl.off[24]);
    p.ckYB2 = (double *)(w + pl.off[25]);
    p.out0 = (double *)(w + pl.off[26]);
    p.inL = (double *)(w + pl.off[27]);
    p.bloc = (double *)(w + pl.off[28]);
    p.blocY = (double *)(w + pl.off[29]);
    p.sink = (double *)(w + pl.off[30]);
    p.spec_lr = (double *)(w + pl.off[8]);
    p.spec_err = p.spec_lr + (size_t)p.B * 2 * (pl.N + 1);
    p.spec_ok = (int *)(p.spec_err + (size_t)p.B * 2 * (pl.N + 1));
}

int check_launch()
{
    return hipGetLastError() == hipSuccess ? SEMICRF_OK : SEMICRF_ELAUNCH;
}

// prefix stage shared by all entry points
template <int ET>
int launch_prep_et(const Params &p, hipStream_t st)
{
    hipLaunchKernelGGL(k_colsum<ET>, dim3(1 + p.NCH * p.B), dim3(NT), 0, st, p);
    hipLaunchKernelGGL(k_prep_seq, dim3(p.B), dim3(PREP_NT), 0, st, p);
    if (p.logpair || p.proj_start || p.proj_end || p.pi_start || p.pi_end)
        hipLaunchKernelGGL((k_prefix<true, ET>), dim3(p.NCH, p.B), dim3(NT), 0, st, p);
    else
        hipLaunchKernelGGL((k_prefix<false, ET>), dim3(p.NCH, p.B), dim3(NT), 0, st, p);
    return check_launch();
}

int launch_prep(const Params &p, hipStream_t st)
{
    if (p.emis_type == 1) return launch_prep_et<1>(p, st);
    if (p.emis_type == 2) return launch_prep_et<2>(p, st);
    return launch_prep_et<0>(p, st);
}

// Chooses the latency-oriented scan when the helper lanes can cover the durations,
// else the generic one.  Returns 1 when the fast path does not apply.
template <int CT, int NHR>
int launch_scan_fast(const Params &p, hipStream_t st, bool both)
{
    const size_t lds = fast_lds_doubles(p.K, pow2_ge8(CT), NHR) * sizeof(double);
    if (lds > LDS_LIMIT) return 1;
    if (hipFuncSetAttribute((const void *)k_scan_fast<CT, NHR>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
        return SEMICRF_ELAUNCH;
    hipLaunchKernelGGL((k_scan_fast<CT, NHR>), dim3(both ? 2 * p.B : p.B), dim3(64 * (NHR + 1)), lds,
                       st, p, both ? 1 : 0);
    return check_launch();
}

template <int CT>
int launch_scan_ct(const Params &p, hipStream_t st, bool both)
{
    constexpr int GW = 64 / pow2_ge8(CT);
    const int terms = p.K > 3 ? p.K - 3 : 0;  // durations k >= 4 go to the helpers
    if (terms <= 1 * GW * NKL) return launch_scan_fast<CT, 1>(p, st, both);
    if (terms <= 2 * GW * NKL) return launch_scan_fast<CT, 2>(p, st, both);
    if (CT < 64 && terms <= 4 * GW * NKL)
        return launch_scan_fast<CT, (CT < 64 ? 4 : 2)>(p, st, both);
    return 1;
}

int launch_scan(const Params &p, const Plan &pl, hipStream_t st, bool both)
{
    const int C = p.C;
    int rc = 1;
    if (C <= 8) rc = launch_scan_ct<8>(p, st, both);
    else if (C <= 16) rc = launch_scan_ct<16>(p, st, both);
    else if (C <= 24) rc = launch_scan_ct<24>(p, st, both);
    else if (C <= 32) rc = launch_scan_ct<32>(p, st, both);
    else if (C <= 64) rc = launch_scan_ct<64>(p, st, both);
    if (rc != 1) return rc;
    if (hipFuncSetAttribute((const void *)k_scan, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)pl.lds_scan) != hipSuccess)
        return SEMICRF_ELAUNCH;
    hipLaunchKernelGGL(k_scan, dim3(both ? 2 * p.B : p.B), dim3(NT), pl.lds_scan, st, p, both ? 1 : 0);
    return check_launch();
}

// One wave per task when the duration strips fit the registers, else the generic kernel.
template <int CT, int NKW>
int launch_interval_wave(const Params &p, const Plan &pl, hipStream_t st)
{
    constexpr int IW = interval_waves(CT, NKW);
    const size_t lds = interval_lds_doubles(CT, NKW) * sizeof(double);
    if (lds > LDS_LIMIT) return 1;
    if (hipFuncSetAttribute((const void *)k_interval_wave<CT, NKW>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
        return SEMICRF_ELAUNCH;
    hipLaunchKernelGGL((k_interval_wave<CT, NKW>), dim3((pl.nslot + IW - 1) / IW), dim3(64 * IW), lds, st, p);
    return check_launch();
}

template <int CT>
int launch_interval_ct(const Params &p, const Plan &pl, hipStream_t st)
{
    constexpr int GW = 64 / pow2_ge8(CT);
    const int per_lane = (p.K + GW - 1) / GW;
    // longer strips would not fit the register file of one wave
    if (per_lane <= 16) return launch_interval_wave<CT, 16>(p, pl, st);
    if (per_lane <= 32) return launch_interval_wave<CT, 32>(p, pl, st);
    if (per_lane <= 64) return launch_interval_wave<CT, 64>(p, pl, st);
    return 1;
}

int launch_interval(const Params &p, const Plan &pl, hipStream_t st)
{
    const int C = p.C;
    int rc = 1;
    if (C <= 8) rc = launch_interval_ct<8>(p, pl, st);
    else if (C <= 16) rc = launch_interval_ct<16>(p, pl, st);
    else if (C <= 24) rc = launch_interval_ct<24>(p, pl, st);
    else if (C <= 32) rc = launch_interval_ct<32>(p, pl, st);
    else if (C <= 64) rc = launch_interval_ct<64>(p, pl, st);
    if (rc != 1) return rc;
    if (hipFuncSetAttribute((const void *)k_interval, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)pl.lds_interval) != hipSuccess)
        return SEMICRF_ELAUNCH;
    hipLaunchKernelGGL(k_interval, dim3(pl.nslot), dim3(NT), pl.lds_interval, st, p);
    return check_launch();
}

// Chunk-parallel scan: returns 1 when it does not apply to these sizes.
template <int CT, int NKW>
int launch_spec_k(const Params &p, hipStream_t st, bool both, int warm, int tier)
{
    const size_t lds = wave_lds_doubles(CT, NKW) * sizeof(double);
    if (lds > LDS_LIMIT) return 1;
    if (hipFuncSetAttribute((const void *)k_spec<CT, NKW>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds) != hipSuccess ||
        hipFuncSetAttribute((const void *)k_spec_repair<CT, NKW>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds) != hipSuccess)
        return SEMICRF_ELAUNCH;
    const int ndir = both ? 2 : 1;
    int rest = 0;
    if (warm > 0 && p.mscan && mscan_applies(p.K, p.C, p.Delta) && (double)p.B * ((double)p.T + 1.0) * (double)p.C < 134217728.0) {
        const int rc = launch_mscan(p, st, both, warm, tier);
        if (rc != SEMICRF_OK) return rc;
        rest = 1;
    }
    const size_t lds2 = spec2_lds_doubles<CT, NKW>() * sizeof(double);
    // two waves per task where the window or the transition product is long next to a position's dependent chain
    // (measured: longgen scans 1.27 -> 0.85 ms, speech 0.30 -> 0.25 ms; genomic 0.37 -> 0.41 ms, so not there)
    const bool two = p.spec2 == 1 || (p.spec2 == 0 && (NKW == 64 || CT == 64));
    if (warm > 0 && two && lds2 <= LDS_LIMIT) {
        if (hipFuncSetAttribute((const void *)k_spec2<CT, NKW>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds2) != hipSuccess)
            return SEMICRF_ELAUNCH;
        hipLaunchKernelGGL((k_spec2<CT, NKW>), dim3(p.B * p.N * ndir), dim3(128), lds2, st, p, both ? 1 : 0,
                           warm, tier, rest);
    } else if (warm > 0)
        hipLaunchKernelGGL((k_spec<CT, NKW>), dim3(p.B * p.N * ndir), dim3(64), lds, st, p, both ? 1 : 0,
                           warm, tier, rest);
    else
        hipLaunchKernelGGL((k_spec_repair<CT, NKW>), dim3(p.B * p.N * ndir), dim3(64), lds, st, p, both ? 1 : 0);
    hipLaunchKernelGGL(k_spec_cmp, dim3(p.N, p.B, ndir), dim3(NT), 0, st, p, tier);
    hipLaunchKernelGGL(k_spec_fix, dim3(p.B, 2), dim3(64), 0, st, p, ndir, tier, tier == 0 ? 1 : (warm == 0 ? 2 : 3));
    return check_launch();
}

template <int CT>
int launch_spec_ct(const Params &p, hipStream_t st, bool both, int warm, int tier)
{
    constexpr int GW = 64 / pow2_ge8(CT);
    const int per_lane = (p.K + GW - 1) / GW;
    if (per_lane <= 16) return launch_spec_k<CT, 16>(p, st, both, warm, tier);
    if (per_lane <= 32) return launch_spec_k<CT, 32>(p, st, both, warm, tier);
    if (per_lane <= 64) return launch_spec_k<CT, 64>(p, st, both, warm, tier);
    return 1;
}

int launch_spec(const Params &p, hipStream_t st, bool both, int warm, int tier)
{
    const int C = p.C;
    if (C <= 8) return launch_spec_ct<8>(p, st, both, warm, tier);
    if (C <= 16) return launch_spec_ct<16>(p, st, both, warm, tier);
    if (C <= 24) return launch_spec_ct<24>(p, st, both, warm, tier);
    if (C <= 32) return launch_spec_ct<32>(p, st, both, warm, tier);
    if (C <= 64) return launch_spec_ct<64>(p, st, both, warm, tier);
    return 1;
}

// Optional per-stage timing: events are recorded on the caller's stream around
// the four stages (prefix sums, scans, intervals, finalisation).
struct StageTimer {
    hipEvent_t ev[5];
    int n = 0;
    bool on = false;
    hipStream_t st = nullptr;
    void mark()
    {
        if (on && n < 5) (void)hipEventRecord(ev[n++], st);
    }
};

// Marginals from the stored rows of both scans: one wave per (sequence, interval).
template <int CT, int NKW>
int launch_mg_k(const Params &p, hipStream_t st)
{
    const size_t lds = (wave_lds_doubles(CT, NKW) + 64) * sizeof(double);
    if (lds > LDS_LIMIT) return SEMICRF_EUNSUPPORTED;
    if (hipFuncSetAttribute((const void *)k_mg_wave<CT, NKW>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds) != hipSuccess)
        return SEMICRF_ELAUNCH;
    hipLaunchKernelGGL((k_mg_wave<CT, NKW>), dim3(p.B * p.N * p.msplit), dim3(64), lds, st, p);
    return SEMICRF_OK;
}

template <int CT>
int launch_mg_ct(const Params &p, hipStream_t st)
{
    const int GW = 64 / pow2_ge8(CT);
    const int per_lane = (p.K + GW - 1) / GW;
    if (per_lane <= 16) return launch_mg_k<CT, 16>(p, st);
    if (per_lane <= 32) return launch_mg_k<CT, 32>(p, st);
    if (per_lane <= 64) return launch_mg_k<CT, 64>(p, st);
    return SEMICRF_EUNSUPPORTED;  // the plan has row slots only where the chunk-parallel scans apply
}

int launch_mg(const Params &p, hipStream_t st)
{
    const int C = p.C;
    if (C <= 8) return launch_mg_ct<8>(p, st);
    if (C <= 16) return launch_mg_ct<16>(p, st);
    if (C <= 24) return launch_mg_ct<24>(p, st);
    if (C <= 32) return launch_mg_ct<32>(p, st);
    if (C <= 64) return launch_mg_ct<64>(p, st);
    return SEMICRF_EUNSUPPORTED;
}

int run(Params p, int ckpt_interval, void *workspace, size_t workspace_bytes, hipStream_t st,
        int mode /*0 cum, 1 logz, 2 fwd_bwd*/, StageTimer *tm = nullptr)
{
    StageTimer none;
    StageTimer &T = tm ? *tm : none;
    Plan pl;
    const int kind = mode != 2 ? 0 : (p.marg_route == 1 ? 3 : (p.marg_route == 2 ? 2 : 1));
    int rc = make_plan(p.B, p.T, p.K, p.C, ckpt_interval, kind | (p.lowmem ? PLAN_LOW_MEMORY : 0), &pl);
    if (rc != SEMICRF_OK) return rc;
    if (!workspace || ((uintptr_t)workspace & 255) != 0 || workspace_bytes < pl.total)
        return SEMICRF_EWORKSPACE;
    p.Delta = pl.Delta;
    p.N = pl.N;
    p.NCH = pl.NCH;
    p.nslot = pl.nslot;
    p.want_grad = mode == 2;
    bind_workspace(p, pl, workspace);
    // warm-up lengths of the chunk-parallel scan: one and a half maximal segment lengths first,
    // eight for the (sequence, direction) pairs that fails for, the sequential scan for the rest
    int warm[2] = {sum_warmup(p.K), 8 * p.K < 64 ? 64 : 8 * p.K};
    if (p.warm0 > 0) warm[0] = p.warm0, warm[1] = 4 * p.warm0;  // the caller's first warm-up length (flags bits 16..31)
    p.spec = p.spec && mode != 0 && spec_applies(p.K, p.C);
    p.mscan = p.mscan && p.spec;
    p.fuse = p.spec && mode == 2 && (size_t)p.B * pl.N <= (size_t)pl.nslot;  // one slot per task
    // Marginals from the stored rows of both scans: where the plan has the row slots and no
    // boundary-term output is asked for (those come from the interval kernels).
    // Their emission sums are formed from the stored pairs with ES * (1/ES) = 1, which start / end projections
    // break; calls with boundary inputs or outputs go through the one-wave interval kernel.
    const bool bterms = p.proj_start || p.proj_end || p.pi_start || p.pi_end || p.g_proj_start || p.g_proj_end ||
                        p.g_pi_start || p.g_pi_end || p.bdy_post;
    p.marg = pl.rows && p.fuse && !bterms;
    if (p.K < 128 && ((double)p.T + 1.0) * (double)p.C >= 2147483648.0)
        p.marg = 0;  // the one-wave kernel indexes a sequence's rows with 32 bits
    // (the partial-sum arrays are planned for N * pl.msplit either way; a part holds at least K positions)
    if (p.marg && p.K < 128 && pl.Delta / pl.msplit >= p.K) p.msplit = pl.msplit;
    T.mark();
    rc = launch_prep(p, st);
    T.mark();
    if (rc != SEMICRF_OK || mode == 0) return rc;
    if (p.spec) {
        // Every interval after a short warm-up; then, for what did not verify, the intervals whose start disagreed
        // restart from the state their neighbour reached (warm-up 0 selects that); then everything that is still
        // open once more after a long warm-up.  The sequential scan takes the rest.
        const int attempt[3] = {warm[0], 0, warm[1]};
        for (int tier = 0; tier < 3; ++tier) {
            rc = launch_spec(p, st, mode == 2, attempt[tier], tier);
            if (rc != SEMICRF_OK) return rc;
        }
    } else {
        hipLaunchKernelGGL(k_spec_clear, dim3((2 * p.B + 63) / 64), dim3(64), 0, st, p);
    }
    // sequential scans: the whole job without the chunk-parallel scan, else only the
    // (sequence, direction) pairs it rejected (the others return at once)
    rc = launch_scan(p, pl, st, mode == 2);
    if (rc != SEMICRF_OK) return rc;
    T.mark();
    rc = check_launch();
    if (rc != SEMICRF_OK || mode == 1) return rc;
    if (p.marg && p.K < 128) {
        // one wave per (sequence, interval): measured 0.29 ms against 0.31 ms for the two kernels below at
        // K = 64, C = 24 (1024 tasks), 0.65 ms against 0.39 ms at K = 512, C = 8 (511 tasks: half the chip idle)
        rc = launch_mg(p, st);
        if (rc != SEMICRF_OK) return rc;
    } else if (p.marg) {
        const int mg_nsl = (p.K + MG_KS - 1) / MG_KS;
        if (hipFuncSetAttribute((const void *)k_mg_dur, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)pl.lds_mg_dur) != hipSuccess)
            return SEMICRF_ELAUNCH;
        int ntd = (p.C * mg_nsl + 63) / 64 * 64;
        if (ntd < NT) ntd = NT;  // the extra threads help staging the rows
        if (hipFuncSetAttribute((const void *)k_mg_te, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)pl.lds_mg_te) != hipSuccess)
            return SEMICRF_ELAUNCH;
        hipLaunchKernelGGL(k_mg_dur, dim3(p.B * p.N), dim3(ntd), pl.lds_mg_dur, st, p);
        hipLaunchKernelGGL(k_mg_te, dim3(p.B * p.N), dim3(NT), pl.lds_mg_te, st, p);
    }
    // the interval kernels: everything without the stored rows, else only what those kernels left
    rc = launch_interval(p, pl, st);
    if (rc != SEMICRF_OK) return rc;
    T.mark();
    hipLaunchKernelGGL(k_fin_seq, dim3(p.B * FIN_FS + (p.C * p.C + p.K * p.C + FIN_PO - 1) / FIN_PO + ((p.g_pi_start || p.g_pi_end) ? 1 : 0)),
                       dim3(NT), 0, st, p);
    launch_fin_emis(p, st);
    T.mark();
    return check_launch();
}

// Viterbi workspace beyond the prefix-stage plan: (V, r) pairs, best final labels, back-pointers,
// two pointer arrays and the path marks.
struct VitLayout {
    size_t vr, vbest, vbp, vpar0, vpar1, vexit, vmark, total;
};

VitLayout viterbi_layout(int B, int T, int C)
{
    const size_t nodes = (size_t)B * ((size_t)T + 1) * C;
    VitLayout l;
    size_t off = 0;
    l.vr = off; off += align_up(nodes * sizeof(double2));
    l.vbest = off; off += align_up((size_t)B * sizeof(int));
    l.vbp = off; off += align_up(nodes * sizeof(int));
    l.vpar0 = off; off += align_up(nodes * sizeof(int));
    l.vpar1 = off; off += align_up(nodes * sizeof(int));
    l.vexit = off; off += align_up(nodes * sizeof(int));
    l.vmark = off; off += align_up(nodes);
    l.total = off;
    return l;
}

template <int CT, int NKW>
int launch_viterbi_k(const Params &p, hipStream_t st)
{
    const size_t lds = wave_lds_doubles(CT, NKW) * sizeof(double);
    if (lds > LDS_LIMIT) return SEMICRF_EUNSUPPORTED;
    if (hipFuncSetAttribute((const void *)k_viterbi<CT, NKW>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds) != hipSuccess ||
        hipFuncSetAttribute((const void *)k_vit_spec<CT, NKW>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds) != hipSuccess)
        return SEMICRF_ELAUNCH;
    if (p.spec) {
        // chunk-parallel scan with two warm-up lengths, as for the sum recurrences
        int warm[2] = {2 * p.K < 32 ? 32 : 2 * p.K, 8 * p.K < 64 ? 64 : 8 * p.K};
        if (p.warm0 > 0) warm[0] = p.warm0, warm[1] = 4 * p.warm0;  // the caller's first warm-up length
        for (int tier = 0; tier < 2; ++tier) {
            hipLaunchKernelGGL((k_vit_spec<CT, NKW>), dim3(p.B * p.N), dim3(64), lds, st, p, warm[tier], tier);
            hipLaunchKernelGGL(k_vit_cmp, dim3(p.N, p.B), dim3(64), 0, st, p, tier);
            hipLaunchKernelGGL(k_vit_fix, dim3(p.B), dim3(64), 0, st, p, tier);
        }
    } else {
        hipLaunchKernelGGL(k_spec_clear, dim3((2 * p.B + 63) / 64), dim3(64), 0, st, p);
    }
    // sequential scan for what the verification rejected (returns at once otherwise)
    hipLaunchKernelGGL((k_viterbi<CT, NKW>), dim3(p.B), dim3(64), lds, st, p);
    return check_launch();
}

template <int CT>
int launch_viterbi_ct(const Params &p, hipStream_t st)
{
    constexpr int GW = 64 / pow2_ge8(CT);
    const int per_lane = (p.K + GW - 1) / GW;
    if (per_lane <= 16) return launch_viterbi_k<CT, 16>(p, st);
    if (per_lane <= 32) return launch_viterbi_k<CT, 32>(p, st);
    if (per_lane <= 64) return launch_viterbi_k<CT, 64>(p, st);
    return SEMICRF_EUNSUPPORTED;
}

// Viterbi: prefix stage with the log-domain pair, one scan wave per sequence, trace-back.
int run_viterbi(Params p, void *workspace, size_t workspace_bytes, hipStream_t st)
{
    Plan pl;
    int rc = make_plan(p.B, p.T, p.K, p.C, 0, 0, &pl);
    if (rc != SEMICRF_OK) return rc;
    if (p.C > 64 || !spec_applies(p.K, p.C)) return SEMICRF_EUNSUPPORTED;
    if (((size_t)p.T + 1) * p.C >= ((size_t)1 << 31)) return SEMICRF_EUNSUPPORTED;  // node ids are 32-bit
    if (2 * (size_t)(p.K + VBP_TILE) * p.C * sizeof(double) > LDS_LIMIT) return SEMICRF_EUNSUPPORTED;  // back-pointer tiles
    const VitLayout vl = viterbi_layout(p.B, p.T, p.C);
    const size_t total = pl.total + vl.total;
    if (!workspace || ((uintptr_t)workspace & 255) != 0 || workspace_bytes < total) return SEMICRF_EWORKSPACE;
    p.Delta = pl.Delta;
    p.N = pl.N;
    p.NCH = pl.NCH;
    p.nslot = pl.nslot;
    bind_workspace(p, pl, workspace);
    char *vw = (char *)workspace + pl.total;
    p.vr = (double2 *)(vw + vl.vr);
    p.vbest = (int *)(vw + vl.vbest);
    p.vbp = (int *)(vw + vl.vbp);
    p.vpar[0] = (int *)(vw + vl.vpar0);
    p.vpar[1] = (int *)(vw + vl.vpar1);
    p.vexit = (int *)(vw + vl.vexit);
    p.vmark = (unsigned char *)(vw + vl.vmark);
    p.logpair = 1;
    p.spec = p.spec ? 1 : 0;
    rc = launch_prep(p, st);
    if (rc != SEMICRF_OK) return rc;
    const int C = p.C;
    if (C <= 8) rc = launch_viterbi_ct<8>(p, st);
    else if (C <= 16) rc = launch_viterbi_ct<16>(p, st);
    else if (C <= 24) rc = launch_viterbi_ct<24>(p, st);
    else if (C <= 32) rc = launch_viterbi_ct<32>(p, st);
    else rc = launch_viterbi_ct<64>(p, st);
    if (rc != SEMICRF_OK) return rc;
    {
        const size_t lds = 2 * (size_t)(p.K + VBP_TILE) * p.C * sizeof(double);  // checked before the first launch
        if (hipFuncSetAttribute((const void *)k_vit_bp, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) !=
            hipSuccess)
            return SEMICRF_ELAUNCH;
        hipLaunchKernelGGL(k_vit_bp, dim3(p.T / VBP_TILE + 1, p.B), dim3(NT), lds, st, p);
    }
    const size_t lds_iv = (size_t)p.Delta * p.C * 5 + 16;  // parents (int) and path marks (byte) of one interval
    if (lds_iv <= LDS_LIMIT && !p.vit_global) {
        // trace-back by interval: local pointer jumping in LDS, doubling over the window nodes only
        if (hipFuncSetAttribute((const void *)k_vit_local, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds_iv) != hipSuccess ||
            hipFuncSetAttribute((const void *)k_vit_walk, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds_iv) != hipSuccess)
            return SEMICRF_ELAUNCH;
        hipLaunchKernelGGL(k_vit_local, dim3(p.N, p.B), dim3(NT), lds_iv, st, p);
        int hops = 1;  // after round i the marks reach the exit nodes fewer than 2^(i+1) intervals down
        while ((1 << hops) < p.N + 1) ++hops;
        const unsigned wblk = (unsigned)(((size_t)p.N * p.K * p.C + NT - 1) / NT);
        for (int i = 0; i < hops; ++i)
            hipLaunchKernelGGL(k_vit_hop, dim3(wblk, p.B), dim3(NT), 0, st, p, i & 1, i == 0 ? 1 : 0);
        hipLaunchKernelGGL(k_vit_walk, dim3(p.N, p.B), dim3(NT), lds_iv, st, p);
        return check_launch();
    }
    const size_t nn = ((size_t)p.T + 1) * p.C;
    const unsigned nblk = (unsigned)((nn + NT - 1) / NT);
    int rounds = 1;
    while (((size_t)1 << rounds) < (size_t)p.T + 1) ++rounds;
    for (int i = 0; i < rounds; ++i)
        hipLaunchKernelGGL(k_vit_round, dim3(nblk, p.B), dim3(NT), 0, st, p, i & 1, i == 0 ? 1 : 0);
    hipLaunchKernelGGL(k_vit_emit, dim3(nblk, p.B), dim3(NT), 0, st, p);
    hipLaunchKernelGGL(k_vit_count, dim3((p.T + VCNT_TOK - 1) / VCNT_TOK, p.B), dim3(NT), 0, st, p);
    return check_launch();
}


// ---------------------------------------------------------------------------
// Duration-dependent transitions: launch geometry, workspace and driver.
// ---------------------------------------------------------------------------
struct DtGeom {
    int kptf, ntf;        // forward kernel: durations per thread, threads
    int kpt, ntb;         // backward kernel: durations per thread, threads
    int ks, nta;          // marginal kernel: durations per workgroup, threads
    size_t lds_f, lds_b, lds_a;  // dynamic LDS bytes
};

// False when the sizes do not fit the kernels: the backward and marginal kernels hold one
// label pair per thread.
bool dt_geometry(int K, int C, DtGeom *g)
{
    if (C > 32) return false;
    const int nksf = K < 1024 / C ? K : 1024 / C;
    const int kptf = (K + nksf - 1) / nksf;
    if (kptf > 8) return false;
    g->kptf = kptf <= 1 ? 1 : (kptf <= 2 ? 2 : (kptf <= 4 ? 4 : 8));
    g->ntf = (C * nksf + 63) / 64 * 64;
    g->lds_f = ((size_t)K * C + (size_t)(DT_MB + 2) * C + (size_t)(DT_MB - 1) * C * C) * sizeof(double);
    const int CC = C * C;
    g->kpt = 0;
    for (int kpt = 8; kpt <= 64; kpt *= 2) {
        const int nks = (K + kpt - 1) / kpt;
        if ((size_t)CC * nks <= 1024) {
            g->kpt = kpt;
            g->ntb = (CC * nks + 63) / 64 * 64;
            g->lds_b = ((size_t)2 * K * C + (size_t)nks * C * (C | 1) + (size_t)(DT_MB + 2) * C + (size_t)(DT_MB - 1) * CC) * sizeof(double);
            break;
        }
    }
    if (!g->kpt) return false;
    g->ks = 16;
    g->nta = (CC + 63) / 64 * 64;
    g->lds_a = (size_t)(2 * DT_TG + DT_TG + g->ks + 3) * C * sizeof(double);
    return g->lds_f <= LDS_LIMIT && g->lds_b <= LDS_LIMIT;
}

// Automatic checkpoint interval of the duration-dependent path: every (sequence, interval) is one
// workgroup-sized task of the forward and of the backward scan (interval + warm-up positions
// each); tasks run in rounds of as many workgroups as the chip holds (by threads, and about five
// waves per SIMD by registers) and a partly filled round costs a full one.  The multiple of 8
// that minimises rounds * (warm-up + interval), at least max(8, K/2).
int dt_auto_interval(int B, int T, int K, const DtGeom &g)
{
    const int waves = g.ntb / 64;
    int per_cu = 2048 / g.ntb < 20 / waves ? 2048 / g.ntb : 20 / waves;
    if (per_cu < 1) per_cu = 1;
    const double slots = 256.0 * per_cu;
    const double warm = (double)sum_warmup(K);
    const int dlo = K / 2 < 8 ? 8 : K / 2;
    int best = 0;
    double best_cost = 0.0;
    for (int n = 1; n <= 8192; ++n) {
        int d = ((T + n - 1) / n + 7) & ~7;
        if (d > T) d = T;
        if (d < dlo && best) break;
        const double tasks = (double)B * (double)(((long long)T + d - 1) / d);
        const double cost = ceil(tasks / slots) * (warm + d);
        if (!best || cost < best_cost) {
            best = d;
            best_cost = cost;
        }
        if (d <= dlo) break;
    }
    return best;
}

constexpr int DT_NWG = 256;  // most persistent workgroups (per group of 16 durations) of the marginal kernel

struct DtLayout {
    size_t g3, dta, dty, dtv, dtd, dtyb, partg, sumg, total;
    int nwg;
};

DtLayout dt_layout(int B, int T, int K, int C, int N, int want_grad)
{
    DtLayout l;
    const size_t kcc = (size_t)K * C * C, t1 = (size_t)T + 1;
    const size_t ntask = (size_t)B * N;
    l.nwg = (int)(ntask < (size_t)DT_NWG ? ntask : (size_t)DT_NWG);
    size_t off = 0;
    l.g3 = off; off += align_up(kcc * 8);
    l.dta = off; off += align_up((size_t)B * t1 * C * 8);
    l.dty = off; off += align_up((size_t)B * t1 * 8);
    l.dtv = off; off += want_grad ? align_up((size_t)B * t1 * C * 8) : 0;
    l.dtd = off; off += want_grad ? align_up((size_t)B * t1 * C * 8) : 0;
    l.dtyb = off; off += want_grad ? align_up((size_t)B * t1 * 8) : 0;
    l.partg = off; off += want_grad ? align_up((size_t)l.nwg * kcc * 8) : 0;
    l.sumg = off; off += want_grad ? align_up(kcc * 8) : 0;
    l.total = off;
    return l;
}

template <int KPTF>
int launch_dt_fwd(const Params &p, const DtGeom &g, hipStream_t st, int grid, int warm, int tier, int whole)
{
    if (hipFuncSetAttribute((const void *)k_dt_fwd<KPTF>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)g.lds_f) != hipSuccess)
        return SEMICRF_ELAUNCH;
    hipLaunchKernelGGL((k_dt_fwd<KPTF>), dim3(grid), dim3(g.ntf), g.lds_f, st, p, warm, tier, whole);
    return SEMICRF_OK;
}

int launch_dt_fwd_any(const Params &p, const DtGeom &g, hipStream_t st, int grid, int warm, int tier, int whole)
{
    switch (g.kptf) {
    case 1: return launch_dt_fwd<1>(p, g, st, grid, warm, tier, whole);
    case 2: return launch_dt_fwd<2>(p, g, st, grid, warm, tier, whole);
    case 4: return launch_dt_fwd<4>(p, g, st, grid, warm, tier, whole);
    default: return launch_dt_fwd<8>(p, g, st, grid, warm, tier, whole);
    }
}

template <int KPT>
int launch_dt_bwd(const Params &p, const DtGeom &g, hipStream_t st, int grid, int warm, int tier, int mode)
{
    if (hipFuncSetAttribute((const void *)k_dt_bwd<KPT, DT_MB>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)g.lds_b) != hipSuccess)
        return SEMICRF_ELAUNCH;
    hipLaunchKernelGGL((k_dt_bwd<KPT, DT_MB>), dim3(grid), dim3(g.ntb), g.lds_b, st, p, warm, tier, mode);
    return SEMICRF_OK;
}

int launch_dt_bwd_any(const Params &p, const DtGeom &g, hipStream_t st, int grid, int warm, int tier, int mode)
{
    switch (g.kpt) {
    case 8: return launch_dt_bwd<8>(p, g, st, grid, warm, tier, mode);
    case 16: return launch_dt_bwd<16>(p, g, st, grid, warm, tier, mode);
    case 32: return launch_dt_bwd<32>(p, g, st, grid, warm, tier, mode);
    default: return launch_dt_bwd<64>(p, g, st, grid, warm, tier, mode);
    }
}

int run_durtrans(Params p, int ckpt_interval, void *workspace, size_t workspace_bytes, hipStream_t st, bool grad)
{
    if (p.B < 1 || p.T < 1 || p.K < 1 || p.C < 1 || ckpt_interval < 0) return SEMICRF_EINVAL;
    DtGeom g;
    if (!dt_geometry(p.K, p.C, &g)) return SEMICRF_EUNSUPPORTED;
    if (ckpt_interval == 0) ckpt_interval = dt_auto_interval(p.B, p.T, p.K, g);
    Plan pl;
    int rc = make_plan(p.B, p.T, p.K, p.C, ckpt_interval, grad ? 2 : 0, &pl);
    if (rc != SEMICRF_OK) return rc;
    const DtLayout dl = dt_layout(p.B, p.T, p.K, p.C, pl.N, grad ? 1 : 0);
    if (!workspace || ((uintptr_t)workspace & 255) != 0 || workspace_bytes < pl.total + dl.total)
        return SEMICRF_EWORKSPACE;
    p.Delta = pl.Delta;
    p.N = pl.N;
    p.NCH = pl.NCH;
    p.nslot = pl.nslot;
    p.want_grad = grad ? 1 : 0;
    bind_workspace(p, pl, workspace);
    char *dw = (char *)workspace + pl.total;
    p.G3 = (double *)(dw + dl.g3);
    p.dtA = (double *)(dw + dl.dta);
    p.dtY = (double *)(dw + dl.dty);
    p.dtV = (double *)(dw + dl.dtv);
    p.dtD = (double *)(dw + dl.dtd);
    p.dtYb = (double *)(dw + dl.dtyb);
    p.partG = (double *)(dw + dl.partg);
    p.sumG = (double *)(dw + dl.sumg);
    p.dt_nwg = dl.nwg;
    rc = launch_prep(p, st);
    if (rc != SEMICRF_OK) return rc;
    const size_t kcc = (size_t)p.K * p.C * p.C;
    hipLaunchKernelGGL(k_dt_tables, dim3((unsigned)((kcc + NT - 1) / NT)), dim3(NT), 0, st, p);
    const int ndir = grad ? 2 : 1;
    if (p.spec) {
        const int warm[2] = {sum_warmup(p.K), 8 * p.K < 64 ? 64 : 8 * p.K};
        for (int tier = 0; tier < 2; ++tier) {
            rc = launch_dt_fwd_any(p, g, st, p.B * p.N, warm[tier], tier, 0);
            if (rc != SEMICRF_OK) return rc;
            if (grad) {
                rc = launch_dt_bwd_any(p, g, st, p.B * p.N, warm[tier], tier, 0);
                if (rc != SEMICRF_OK) return rc;
            }
            hipLaunchKernelGGL(k_spec_cmp, dim3(p.N, p.B, ndir), dim3(NT), 0, st, p, tier);
            hipLaunchKernelGGL(k_spec_fix, dim3(p.B, 2), dim3(64), 0, st, p, ndir, tier, tier == 0 ? 1 : 3);
        }
    } else {
        hipLaunchKernelGGL(k_spec_clear, dim3((2 * p.B + 63) / 64), dim3(64), 0, st, p);
    }
    // whole-sequence scans for what the verification rejected (return at once otherwise)
    rc = launch_dt_fwd_any(p, g, st, p.B, 0, 0, 1);
    if (rc != SEMICRF_OK) return rc;
    if (!grad) return check_launch();
    rc = launch_dt_bwd_any(p, g, st, p.B, 0, 0, 1);
    if (rc != SEMICRF_OK) return rc;
    hipLaunchKernelGGL(k_dt_emis, dim3(p.B * p.N), dim3(64), 0, st, p);
    hipLaunchKernelGGL((k_dt_acc<16>), dim3(dl.nwg, (p.K + 15) / 16), dim3(g.nta), g.lds_a, st, p);
    hipLaunchKernelGGL(k_dt_fin, dim3(p.B * FIN_FS + (unsigned)((kcc + NT - 1) / NT)), dim3(NT), 0, st, p);
    hipLaunchKernelGGL(k_dt_fin_dur, dim3((p.K * p.C + NT - 1) / NT), dim3(NT), 0, st, p);
    launch_fin_emis(p, st);
    return check_launch();
}

// Fields every entry point fills the same way.  SEMICRF_EINVAL for flag combinations that make no sense.
int common_params(Params &p, const float *emis, const int32_t *lengths, const float *dur, int B, int T, int K, int C,
                  unsigned flags)
{
    if (int rc = check_flags(flags)) return rc;
    p.emis = emis;
    p.lengths = lengths;
    p.dur = dur;
    p.B = B; p.T = T; p.K = K; p.C = C;
    p.center = (flags & SEMICRF_CENTER) ? 1 : 0;
    p.emis_type = (flags & SEMICRF_EMIS_F16) ? 1 : ((flags & SEMICRF_EMIS_BF16) ? 2 : 0);
    p.spec = (flags & SEMICRF_SEQUENTIAL_SCAN) ? 0 : 1;
    p.mscan = (flags & SEMICRF_MATRIX_SCAN) ? 1 : 0;
    p.lowmem = (flags & SEMICRF_LOW_MEMORY) ? 1 : 0;
    if ((flags & SEMICRF_TWO_WAVE_SCAN) && (flags & SEMICRF_ONE_WAVE_SCAN)) return SEMICRF_EINVAL;
    p.spec2 = (flags & SEMICRF_TWO_WAVE_SCAN) ? 1 : ((flags & SEMICRF_ONE_WAVE_SCAN) ? 2 : 0);
    p.marg_route = (flags & SEMICRF_MARGINALS_ROWS) ? 1 : ((flags & SEMICRF_MARGINALS_INTERVAL) ? 2 : 0);
    p.vit_global = (flags & SEMICRF_VITERBI_GLOBAL_TRACE) ? 1 : 0;
    p.warm0 = (int)(flags >> 16);
    return SEMICRF_OK;
}

// Device address of this GPU's copy of the static scratch array, looked up once per device with
// that device current and kept for the life of the process.
constexpr int STATIC_MAX_DEVICES = 64;
std::mutex static_mu;
void *static_ptr[STATIC_MAX_DEVICES] = {};

int static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= STATIC_MAX_DEVICES) return SEMICRF_ELAUNCH;
    std::lock_guard<std::mutex> lock(static_mu);
    if (!static_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return SEMICRF_ELAUNCH;
        if (((uintptr_t)p & 255) != 0) return SEMICRF_ELAUNCH;
        static_ptr[dev] = p;
    }
    *out = static_ptr[dev];
    return SEMICRF_OK;
}

}  // namespace

extern "C" {

int semicrf_version(void) { return 1; }

const char *semicrf_strerror(int status)
{
    switch (status) {
        case SEMICRF_OK: return "ok";
        case SEMICRF_EINVAL: return "invalid argument";
        case SEMICRF_EWORKSPACE: return "workspace too small or misaligned";
        case SEMICRF_EUNSUPPORTED: return "sizes not supported (C > 256, C > 64 with gradients, or K*C exceeds the LDS budget)";
        case SEMICRF_ELAUNCH: return "HIP launch failure";
        default: return "unknown status";
    }
}

int semicrf_workspace_bytes(int B, int T, int K, int C, int ckpt_interval, int want_grad,
                            size_t *bytes)
{
    if (!bytes) return SEMICRF_EINVAL;
    Plan pl;
    int rc = make_plan(B, T, K, C, ckpt_interval, want_grad, &pl);
    if (rc != SEMICRF_OK) return rc;
    *bytes = pl.total;
    return SEMICRF_OK;
}

int semicrf_ckpt_interval(int B, int T, int K, int C, int ckpt_interval, int *interval)
{
    if (!interval) return SEMICRF_EINVAL;
    Plan pl;
    int rc = make_plan(B, T, K, C, ckpt_interval, 0, &pl);
    if (rc != SEMICRF_OK) return rc;
    *interval = pl.Delta;
    return SEMICRF_OK;
}

int semicrf_ckpt_interval_low_memory(int B, int T, int K, int C, int ckpt_interval, int *interval)
{
    if (!interval) return SEMICRF_EINVAL;
    Plan pl;
    int rc = make_plan(B, T, K, C, ckpt_interval, PLAN_LOW_MEMORY, &pl);
    if (rc != SEMICRF_OK) return rc;
    *interval = pl.Delta;
    return SEMICRF_OK;
}

int semicrf_cum_scores(const float *emis, const int32_t *lengths, int B, int T, int C,
                       unsigned flags, void *workspace, size_t workspace_bytes, double *cum,
                       void *stream)
{
    if (!emis || !cum) return SEMICRF_EINVAL;
    Params p = {};
    if (int rc = common_params(p, emis, lengths, nullptr, B, T, 1, C, flags)) return rc;
    p.cum = cum;
    return run(p, 0, workspace, workspace_bytes, (hipStream_t)stream, 0);
}

int semicrf_logz_fwd(const float *emis, const int32_t *lengths, const float *trans,
                     const float *dur, int B, int T, int K, int C, int ckpt_interval,
                     unsigned flags, void *workspace, size_t workspace_bytes, float *logz,
                     void *stream)
{
    if (!emis || !trans || !dur || !logz) return SEMICRF_EINVAL;
    Params p = {};
    if (int rc = common_params(p, emis, lengths, dur, B, T, K, C, flags)) return rc;
    p.trans = trans;
    p.logz = logz;
    return run(p, ckpt_interval, workspace, workspace_bytes, (hipStream_t)stream, 1);
}

int semicrf_fwd_bwd(const float *emis, const int32_t *lengths, const float *trans,
                    const float *dur, const float *grad_logz, int B, int T, int K, int C,
                    int ckpt_interval, unsigned flags, void *workspace, size_t workspace_bytes,
                    float *logz, float *grad_emis, float *grad_trans, float *grad_dur,
                    float *pos_marg, void *stream)
{
    if (!emis || !trans || !dur || !logz || !grad_emis || !grad_trans || !grad_dur)
        return SEMICRF_EINVAL;
    Params p = {};
    if (int rc = common_params(p, emis, lengths, dur, B, T, K, C, flags)) return rc;
    p.trans = trans; p.grad_logz = grad_logz;
    p.logz = logz; p.grad_emis = grad_emis; p.grad_trans = grad_trans; p.grad_dur = grad_dur;
    p.pos_marg = pos_marg;
    return run(p, ckpt_interval, workspace, workspace_bytes, (hipStream_t)stream, 2);
}

int semicrf_fwd_bwd_static(const float *emis, const int32_t *lengths, const float *trans, const float *dur,
                           const float *grad_logz, int B, int T, int K, int C, int ckpt_interval,
                           unsigned flags, float *logz, float *grad_emis, float *grad_trans,
                           float *grad_dur, float *pos_marg, void *stream)
{
    // sizes first: nothing is touched when the plan does not fit the static array
    size_t need = 0;
    int rc = check_flags(flags);
    if (rc != SEMICRF_OK) return rc;
    const int kind = ((flags & SEMICRF_MARGINALS_ROWS) ? 3 : ((flags & SEMICRF_MARGINALS_INTERVAL) ? 2 : 1)) |
                     ((flags & SEMICRF_LOW_MEMORY) ? PLAN_LOW_MEMORY : 0);
    rc = semicrf_workspace_bytes(B, T, K, C, ckpt_interval, kind, &need);
    if (rc != SEMICRF_OK) return rc;
    if (need > (size_t)SEMICRF_STATIC_WORKSPACE_BYTES) return SEMICRF_EWORKSPACE;
    void *ws = nullptr;
    rc = static_scratch(&ws);
    if (rc != SEMICRF_OK) return rc;
    return semicrf_fwd_bwd(emis, lengths, trans, dur, grad_logz, B, T, K, C, ckpt_interval, flags, ws,
                           (size_t)SEMICRF_STATIC_WORKSPACE_BYTES, logz, grad_emis, grad_trans, grad_dur,
                           pos_marg, stream);
}

int semicrf_fwd_bwd_profiled(const float *emis, const int32_t *lengths, const float *trans,
                             const float *dur, const float *grad_logz, int B, int T, int K, int C,
                             int ckpt_interval, unsigned flags, void *workspace,
                             size_t workspace_bytes, float *logz, float *grad_emis,
                             float *grad_trans, float *grad_dur, float *pos_marg, void *stream,
                             void *const *stage_events)
{
    if (!emis || !trans || !dur || !logz || !grad_emis || !grad_trans || !grad_dur || !stage_events)
        return SEMICRF_EINVAL;
    Params p = {};
    if (int rc = common_params(p, emis, lengths, dur, B, T, K, C, flags)) return rc;
    p.trans = trans; p.grad_logz = grad_logz;
    p.logz = logz; p.grad_emis = grad_emis; p.grad_trans = grad_trans; p.grad_dur = grad_dur;
    p.pos_marg = pos_marg;
    StageTimer tm;
    tm.on = true;
    tm.st = (hipStream_t)stream;
    for (int i = 0; i < 5; ++i) {
        if (!stage_events[i]) return SEMICRF_EINVAL;
        tm.ev[i] = (hipEvent_t)stage_events[i];
    }
    return run(p, ckpt_interval, workspace, workspace_bytes, tm.st, 2, &tm);
}

int semicrf_logz_fwd_boundary(const float *emis, const int32_t *lengths, const float *trans,
                              const float *dur, const float *proj_start, const float *proj_end,
                              const float *pi_start, const float *pi_end, int B, int T, int K, int C,
                              int ckpt_interval, unsigned flags, void *workspace, size_t workspace_bytes,
                              float *logz, void *stream)
{
    if (!emis || !trans || !dur || !logz) return SEMICRF_EINVAL;
    Params p = {};
    if (int rc = common_params(p, emis, lengths, dur, B, T, K, C, flags)) return rc;
    p.trans = trans;
    p.proj_start = proj_start; p.proj_end = proj_end; p.pi_start = pi_start; p.pi_end = pi_end;
    p.logz = logz;
    return run(p, ckpt_interval, workspace, workspace_bytes, (hipStream_t)stream, 1);
}

int semicrf_fwd_bwd_boundary(const float *emis, const int32_t *lengths, const float *trans,
                             const float *dur, const float *grad_logz, const float *proj_start,
                             const float *proj_end, const float *pi_start, const float *pi_end, int B, int T,
                             int K, int C, int ckpt_interval, unsigned flags, void *workspace,
                             size_t workspace_bytes, float *logz, float *grad_emis, float *grad_trans,
                             float *grad_dur, float *pos_marg, float *grad_proj_start, float *grad_proj_end,
                             float *grad_pi_start, float *grad_pi_end, float *bdy_post, void *stream)
{
    if (!emis || !trans || !dur || !logz || !grad_emis || !grad_trans || !grad_dur)
        return SEMICRF_EINVAL;
    Params p = {};
    if (int rc = common_params(p, emis, lengths, dur, B, T, K, C, flags)) return rc;
    p.trans = trans; p.grad_logz = grad_logz;
    p.proj_start = proj_start; p.proj_end = proj_end; p.pi_start = pi_start; p.pi_end = pi_end;
    p.logz = logz; p.grad_emis = grad_emis; p.grad_trans = grad_trans; p.grad_dur = grad_dur;
    p.pos_marg = pos_marg;
    p.g_proj_start = grad_proj_start; p.g_proj_end = grad_proj_end;
    p.g_pi_start = grad_pi_start; p.g_pi_end = grad_pi_end; p.bdy_post = bdy_post;
    return run(p, ckpt_interval, workspace, workspace_bytes, (hipStream_t)stream, 2);
}

int semicrf_entropies(const float *pos_marg, const float *bdy_post, const int32_t *lengths, int B, int T,
                      int C, float *h_pos, float *h_bdy, void *stream)
{
    if (B < 1 || T < 1 || C < 1) return SEMICRF_EINVAL;
    if ((!h_pos && !h_bdy) || (h_pos && !pos_marg) || (h_bdy && !bdy_post)) return SEMICRF_EINVAL;
    hipLaunchKernelGGL(k_entropies, dim3(B), dim3(NT), 0, (hipStream_t)stream, pos_marg, bdy_post, lengths, T,
                       C, h_pos, h_bdy);
    return check_launch();
}

int semicrf_viterbi_workspace_bytes(int B, int T, int K, int C, size_t *bytes)
{
    if (!bytes) return SEMICRF_EINVAL;
    Plan pl;
    int rc = make_plan(B, T, K, C, 0, 0, &pl);
    if (rc != SEMICRF_OK) return rc;
    if (C > 64 || !spec_applies(K, C)) return SEMICRF_EUNSUPPORTED;
    if (((size_t)T + 1) * C >= ((size_t)1 << 31)) return SEMICRF_EUNSUPPORTED;
    *bytes = pl.total + viterbi_layout(B, T, C).total;
    return SEMICRF_OK;
}

int semicrf_viterbi(const float *emis, const int32_t *lengths, const float *trans, const float *dur,
                    const float *proj_start, const float *proj_end, const float *pi_start,
                    const float *pi_end, int B, int T, int K, int C, unsigned flags, void *workspace,
                    size_t workspace_bytes, float *score, int32_t *labels, int32_t *starts, int32_t *nseg,
                    void *stream)
{
    if (!emis || !trans || !dur || !score || !labels || !starts || !nseg) return SEMICRF_EINVAL;
    Params p = {};
    if (flags & SEMICRF_LOW_MEMORY) return SEMICRF_EINVAL;  // the low-memory plan exists for the factorised sums only
    if (int rc = common_params(p, emis, lengths, dur, B, T, K, C, flags)) return rc;
    p.trans = trans;
    p.proj_start = proj_start; p.proj_end = proj_end; p.pi_start = pi_start; p.pi_end = pi_end;
    p.vscore = score; p.vlabels = labels; p.vstarts = starts; p.vnseg = nseg;
    return run_viterbi(p, workspace, workspace_bytes, (hipStream_t)stream);
}

int semicrf_durtrans_workspace_bytes(int B, int T, int K, int C, int ckpt_interval, int want_grad,
                                     size_t *bytes)
{
    if (!bytes) return SEMICRF_EINVAL;
    if (B < 1 || T < 1 || K < 1 || C < 1 || ckpt_interval < 0) return SEMICRF_EINVAL;
    DtGeom g;
    if (!dt_geometry(K, C, &g)) return SEMICRF_EUNSUPPORTED;
    if (ckpt_interval == 0) ckpt_interval = dt_auto_interval(B, T, K, g);
    Plan pl;
    int rc = make_plan(B, T, K, C, ckpt_interval, want_grad ? 2 : 0, &pl);
    if (rc != SEMICRF_OK) return rc;
    *bytes = pl.total + dt_layout(B, T, K, C, pl.N, want_grad ? 1 : 0).total;
    return SEMICRF_OK;
}

int semicrf_durtrans_ckpt_interval(int B, int T, int K, int C, int ckpt_interval, int *interval)
{
    if (!interval) return SEMICRF_EINVAL;
    if (B < 1 || T < 1 || K < 1 || C < 1 || ckpt_interval < 0) return SEMICRF_EINVAL;
    DtGeom g;
    if (!dt_geometry(K, C, &g)) return SEMICRF_EUNSUPPORTED;
    *interval = ckpt_interval == 0 ? dt_auto_interval(B, T, K, g) : (ckpt_interval > T ? T : ckpt_interval);
    return SEMICRF_OK;
}

int semicrf_logz_fwd_durtrans(const float *emis, const int32_t *lengths, const float *trans3,
                              const float *dur, int B, int T, int K, int C, int ckpt_interval,
                              unsigned flags, void *workspace, size_t workspace_bytes, float *logz,
                              void *stream)
{
    if (!emis || !trans3 || !dur || !logz) return SEMICRF_EINVAL;
    Params p = {};
    if (flags & SEMICRF_LOW_MEMORY) return SEMICRF_EINVAL;  // the low-memory plan exists for the factorised sums only
    if (int rc = common_params(p, emis, lengths, dur, B, T, K, C, flags)) return rc;
    p.trans3 = trans3;
    p.logz = logz;
    return run_durtrans(p, ckpt_interval, workspace, workspace_bytes, (hipStream_t)stream, false);
}

int semicrf_fwd_bwd_durtrans(const float *emis, const int32_t *lengths, const float *trans3,
                             const float *dur, const float *grad_logz, int B, int T, int K, int C,
                             int ckpt_interval, unsigned flags, void *workspace, size_t workspace_bytes,
                             float *logz, float *grad_emis, float *grad_trans3, float *grad_dur,
                             float *pos_marg, void *stream)
{
    if (!emis || !trans3 || !dur || !logz || !grad_emis || !grad_trans3 || !grad_dur) return SEMICRF_EINVAL;
    Params p = {};
    if (flags & SEMICRF_LOW_MEMORY) return SEMICRF_EINVAL;  // the low-memory plan exists for the factorised sums only
    if (int rc = common_params(p, emis, lengths, dur, B, T, K, C, flags)) return rc;
    p.trans3 = trans3; p.grad_logz = grad_logz;
    p.logz = logz; p.grad_emis = grad_emis; p.grad_trans3 = grad_trans3; p.grad_dur = grad_dur;
    p.pos_marg = pos_marg;
    return run_durtrans(p, ckpt_interval, workspace, workspace_bytes, (hipStream_t)stream, true);
}

int semicrf_seq_report(const void *workspace, size_t workspace_bytes, int B, int T, int K, int C,
                       int ckpt_interval, int want_grad, int32_t *range_exceeded, double *logz64, void *stream)
{
    Plan pl;
    int rc = make_plan(B, T, K, C, ckpt_interval, report_plan_kind(want_grad), &pl);
    if (rc != SEMICRF_OK) return rc;
    if (!range_exceeded && !logz64) return SEMICRF_EINVAL;
    if (!workspace || ((uintptr_t)workspace & 255) != 0 || workspace_bytes < pl.total)
        return SEMICRF_EWORKSPACE;
    Params p = {};
    p.B = B; p.T = T; p.K = K; p.C = C;
    p.N = pl.N;
    bind_workspace(p, pl, const_cast<void *>(workspace));
    hipLaunchKernelGGL(k_seq_report, dim3((B + 63) / 64), dim3(64), 0, (hipStream_t)stream, p, range_exceeded,
                       logz64);
    return check_launch();
}

int semicrf_scan_report(const void *workspace, size_t workspace_bytes, int B, int T, int K, int C,
                        int ckpt_interval, int want_grad, int32_t *accepted, double *mismatch,
                        void *stream)
{
    Plan pl;
    int rc = make_plan(B, T, K, C, ckpt_interval, report_plan_kind(want_grad), &pl);
    if (rc != SEMICRF_OK) return rc;
    if (!accepted && !mismatch) return SEMICRF_EINVAL;
    if (!workspace || ((uintptr_t)workspace & 255) != 0 || workspace_bytes < pl.total)
        return SEMICRF_EWORKSPACE;
    Params p = {};
    p.B = B; p.T = T; p.K = K; p.C = C;
    p.N = pl.N;
    bind_workspace(p, pl, const_cast<void *>(workspace));
    hipLaunchKernelGGL(k_spec_report, dim3((2 * B + 63) / 64), dim3(64), 0, (hipStream_t)stream, p,
                       accepted, mismatch);
    return check_launch();
}

}  // extern "C"
