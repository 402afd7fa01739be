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
// Kernels: k_colsum (+ the exp tables), k_prep_seq, k_prefix (Eq. 1-2); k_spec, k_spec_cmp,
// k_spec_fix (Algorithm 1 and the beta recurrence of Algorithm 3 as chunk-parallel scans
// that are verified at every chunk boundary and write ring checkpoints every Delta
// positions); k_scan_fast / k_scan (the same scans sequentially, for what the verification
// rejects); k_interval_wave / k_interval (per checkpoint interval: recompute the forward
// messages unless the scan stored them, run beta across the interval, accumulate the
// expected sufficient statistics in registers/LDS, no global atomics); k_mg_dur / k_mg_te
// (the same statistics as position-local products of the rows both scans stored, for long
// maximal durations); k_fin_seq (+ the parameter gradients), k_fin_emis (fixed-order reductions).
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

// ---------------------------------------------------------------------------
// exp(dur), exp(trans) in fp64 and the maxima that bound per-step growth.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void tables_body(const Params &p)
{
    __shared__ double red[NT];
    const int tid = threadIdx.x;
    const int KC = p.K * p.C, CC = p.C * p.C;
    if (!p.dur || (!p.trans && !p.trans3)) {  // prefix sums only: growth is bounded by the emissions alone
        if (tid < 2) p.tabmax[tid] = 0.0;
        return;
    }
    double mxd = -DBL_MAX, mxt = -DBL_MAX;
    if (p.trans3) {  // one transition matrix per duration: only the maxima are needed here
        for (int i = tid; i < KC; i += NT) mxd = fmax(mxd, (double)p.dur[i]);
        for (int i = tid; i < p.K * CC; i += NT) mxt = fmax(mxt, (double)p.trans3[i]);
    } else {
        for (int i = tid; i < KC; i += NT) {
            double v = (double)p.dur[i];
            p.W[i] = exp(v);
            mxd = fmax(mxd, v);
        }
        for (int i = tid; i < CC; i += NT) {
            double v = (double)p.trans[i];
            p.Etr[i] = exp(v);
            mxt = fmax(mxt, v);
        }
    }
    red[tid] = mxd;
    __syncthreads();
    if (tid == 0) {
        double m = red[0];
        for (int i = 1; i < NT; ++i) m = fmax(m, red[i]);
        p.tabmax[0] = m;
    }
    __syncthreads();
    red[tid] = mxt;
    __syncthreads();
    if (tid == 0) {
        double m = red[0];
        for (int i = 1; i < NT; ++i) m = fmax(m, red[i]);
        p.tabmax[1] = m;
    }
}

// ---------------------------------------------------------------------------
// Eq. 1, stage 1: per-chunk column sums (fp64) and |f| maxima.  grid (NCH, B).
// ---------------------------------------------------------------------------
template <int ET>
__device__ __forceinline__ void colsum_body(const Params &p, const int b, const int ch)
{
    __shared__ double red[NT];
    __shared__ double redm[NT];
    const int tid = threadIdx.x;
    const int C = p.C, L = seq_len(p, b);
    const int u0 = ch * PREP_CH;
    const int u1 = min(u0 + PREP_CH, L);
    const int R = NT / C;  // rows handled per pass
    const int r = tid / C, c = tid % C;
    double acc = 0.0, mx = 0.0;
    if (r < R) {
        const size_t f0 = ((size_t)b * p.T) * C;
#pragma unroll 8
        for (int u = u0 + r; u < u1; u += R) {
            double v = emis_at<ET>(p, f0 + (size_t)u * C + c);
            acc += v;
            mx = fmax(mx, fabs(v));
        }
    }
    // the boundary projections move a message like an emission does: their maxima are added
    double mps = 0.0, mpe = 0.0;
    if (r < R && (p.proj_start || p.proj_end)) {
        const size_t o = ((size_t)b * p.T) * C;
        for (int u = u0 + r; u < u1; u += R) {
            if (p.proj_start) mps = fmax(mps, fabs((double)p.proj_start[o + (size_t)u * C + c]));
            if (p.proj_end) mpe = fmax(mpe, fabs((double)p.proj_end[o + (size_t)u * C + c]));
        }
    }
    __shared__ double redp[NT];
    red[tid] = acc;
    redm[tid] = mx;
    redp[tid] = mps + mpe;
    __syncthreads();
    if (tid < C) {
        double s = 0.0;
        for (int i = 0; i < R; ++i) s += red[i * C + tid];
        p.chsum[((size_t)b * p.NCH + ch) * C + tid] = s;
    }
    if (tid == 0) {
        double m = 0.0, mp = 0.0;
        for (int i = 0; i < R * C; ++i) m = fmax(m, redm[i]);
        if (p.proj_start || p.proj_end)
            for (int i = 0; i < R * C; ++i) mp = fmax(mp, redp[i]);
        p.chmax[(size_t)b * p.NCH + ch] = m + 2.0 * mp;  // |start| + |end| bounded by twice the larger sum
    }
}

// One launch for both: workgroup 0 builds the tables, workgroup 1 + b*NCH + ch sums a chunk.
template <int ET>
__global__ __launch_bounds__(NT) void k_colsum(Params p)
{
    if (blockIdx.x == 0) {
        tables_body(p);
        return;
    }
    const int id = blockIdx.x - 1;
    colsum_body<ET>(p, id / p.NCH, id % p.NCH);
}

// ---------------------------------------------------------------------------
// Eq. 1, stage 2: nu = mean over valid positions; chunk sums -> exclusive
// offsets of the centred prefix sum; scaling block length J.  grid B.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(NT) void k_prep_seq(Params p)
{
    // The chunks are split into G = NT/C contiguous ranges, one per thread group; range sums
    // are combined in range order (a fixed order for a given problem).
    __shared__ double gsum[NT];
    __shared__ double red[NT];
    __shared__ double nu_s[NT];
    const int b = blockIdx.x, tid = threadIdx.x;
    const int C = p.C, L = seq_len(p, b), NCH = p.NCH;
    const int G = NT / C;
    const int g = tid / C, c = tid % C;
    const bool act = g < G;
    const int per = (NCH + G - 1) / G;
    const int c0 = min(g * per, NCH), c1 = min(c0 + per, NCH);
    double *cs = p.chsum + ((size_t)b * NCH) * C + c;
    double loc = 0.0;
    if (act) {
#pragma unroll 8
        for (int ch = c0; ch < c1; ++ch) loc += cs[(size_t)ch * C];
    }
    gsum[tid] = loc;
    __syncthreads();
    if (tid < C) {
        double total = 0.0;
        for (int gg = 0; gg < G; ++gg) total += gsum[gg * C + tid];
        const double nu = (p.center && L > 0) ? total / (double)L : 0.0;
        p.nu[(size_t)b * C + tid] = nu;
        nu_s[tid] = nu;
    }
    __syncthreads();
    if (act) {
        const double mynu = nu_s[c];
        double pref = 0.0;  // raw prefix sum at the start of this range
        for (int gg = 0; gg < g; ++gg) pref += gsum[gg * C + c];
#pragma unroll 8
        for (int ch = c0; ch < c1; ++ch) {
            const double sum = cs[(size_t)ch * C];
            const int nvalid = min(ch * PREP_CH, L);
            cs[(size_t)ch * C] = pref - (double)nvalid * mynu;
            pref += sum;
        }
    }
    // bound on |f - nu|
    double fm = 0.0;
#pragma unroll 4
    for (int ch = tid; ch < NCH; ch += NT) fm = fmax(fm, p.chmax[(size_t)b * NCH + ch]);
    red[tid] = fm;
    __syncthreads();
    if (tid == 0) {
        fm = 0.0;
        for (int i = 0; i < NT; ++i) fm = fmax(fm, red[i]);
        double nm = 0.0, npi = 0.0;
        for (int i = 0; i < C; ++i) {
            nm = fmax(nm, fabs(nu_s[i]));
            if (p.pi_start) npi = fmax(npi, fabs((double)p.pi_start[i]));
            if (p.pi_end) npi = fmax(npi, fabs((double)p.pi_end[i]));
        }
        fm += nm + 2.0 * npi;
        double dmax = p.tabmax[0], tmax = p.tabmax[1];
        double grow = fm + fmax(dmax, 0.0) + fmax(tmax, 0.0) + log((double)p.K * (double)C);
        double shrink = fm + fmax(-dmax, 0.0) + fmax(-tmax, 0.0);
        double r = fmax(fmax(grow, shrink), 1e-9);
        int J = 1, flags = 0;
        if (!(r <= RANGE_NATS)) flags = 1;  // also catches NaN
        while (J < JMAX && (double)(2 * J) * r <= RANGE_NATS) J *= 2;
        SeqHdr h;
        h.L = L; h.J = J; h.flags = flags; h.pad = 0; h.logZ = 0.0; h.logZb = 0.0;
        p.hdr[b] = h;
    }
}

// ---------------------------------------------------------------------------
// Eq. 2: centred prefix sums S[t,c] (fp64), the per-block exponents n_j(c) and the pair
// (ES, 1/ES), ES = exp(S - n ln2).  grid (NCH,B), 256 threads: a chunk of PREP_CH
// positions is cut into 8 segments of 32 (a multiple of every scaling block length), thread
// (segment, label) first sums its segment, the segment sums are combined in segment order,
// then the thread walks its segment again and writes.  Labels beyond 32 take further turns.
// ---------------------------------------------------------------------------
constexpr int PREP_SEG = 32;
static_assert(PREP_CH == 8 * PREP_SEG && JMAX <= PREP_SEG && NT == 256, "k_prefix geometry");

template <bool BTERMS, int ET>  // any boundary term of Eq. 4 present; emission storage type
__global__ __launch_bounds__(NT) void k_prefix(Params p)
{
    __shared__ double segsum[8][PREP_SEG + 1];
    const int b = blockIdx.y, ch = blockIdx.x;
    const int seg = threadIdx.x >> 5, cl = threadIdx.x & 31;
    const int C = p.C;
    const SeqHdr h = p.hdr[b];
    const int L = h.L, J = h.J;
    const int t0 = ch * PREP_CH + seg * PREP_SEG;
    const int tend = min(t0 + PREP_SEG, p.T + 1);
    const size_t row0 = (size_t)b * (p.T + 1);
    for (int cb = 0; cb < C; cb += 32) {
        const int c = cb + cl;
        const bool valid = c < C;
        const size_t f0 = ((size_t)b * p.T) * C + (valid ? c : 0);
        const double nu = valid ? p.nu[(size_t)b * C + c] : 0.0;
        double sum = 0.0;
        if (valid)
            for (int t = t0; t < min(tend, L); ++t) sum += emis_at<ET>(p, f0 + (size_t)t * C) - nu;
        segsum[seg][cl] = sum;
        __syncthreads();
        double S = valid ? p.chsum[((size_t)b * p.NCH + ch) * C + c] : 0.0;
        for (int s2 = 0; s2 < seg; ++s2) S += segsum[s2][cl];
        __syncthreads();
        if (!valid) continue;
        double base = 0.0;
        for (int t = t0; t < tend; ++t) {
            if (t <= L) {
                if ((t % J) == 0) {
                    const double n = rint(S * LOG2E);
                    p.nbase[(row0 + (size_t)(t / J)) * C + c] = (int)n;
                    base = n * LN2;
                }
                const double x = S - base;
                double2 pr;
                if (!BTERMS) {
                    const double es = exp(x);
                    pr = make_double2(es, 1.0 / es);
                } else {
                    // (ES * exp(end score of token t-1), exp(start score of token t) / ES): every message
                    // that arrives at position t is multiplied by the first, every one that leaves by the second
                    double xs = 0.0, xe = 0.0;
                    if (t < L) {
                        if (p.proj_start) xs = (double)p.proj_start[((size_t)b * p.T + t) * C + c];
                        if (t == 0 && p.pi_start) xs += (double)p.pi_start[c];
                    }
                    if (t >= 1) {
                        if (p.proj_end) xe = (double)p.proj_end[((size_t)b * p.T + t - 1) * C + c];
                        if (t == L && p.pi_end) xe += (double)p.pi_end[c];
                    }
                    // max semiring: the same pair in the log domain, (S + end score, start score - S)
                    pr = p.logpair ? make_double2(S + xe, xs - S) : make_double2(exp(x + xe), exp(xs - x));
                }
                p.EI[(row0 + t) * C + c] = pr;
                if (p.cum) p.cum[(row0 + t) * C + c] = S;
                if (t < L) S += emis_at<ET>(p, f0 + (size_t)t * C) - nu;
            } else if (p.cum) {
                p.cum[(row0 + t) * C + c] = 0.0;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Shared pieces of the scans.  LDS layout (doubles), CP1 = C|1 (odd row stride
// so that both orientations of the transition product are bank-conflict free):
//   ring[K*C]  Wl[K*C]  El[C*CP1]  red[G*C]  yv[C]  zv[C]  av[C]  qv[C]  sc[C](int)
//   (interval kernel only) accD[K*C]
// ---------------------------------------------------------------------------
struct Lds {
    double *ring, *Wl, *El, *red, *yv, *zv, *av, *qv, *accD;
    int *sc;
};

__device__ __forceinline__ Lds carve(double *base, int K, int C, int G, bool interval)
{
    Lds l;
    const int CP1 = C | 1;
    double *q = base;
    l.ring = q; q += K * C;
    l.Wl = q;   q += K * C;
    l.El = q;   q += C * CP1;
    l.red = q;  q += G * C;
    l.yv = q;   q += C;
    l.zv = q;   q += C;
    l.av = q;   q += C;
    l.qv = q;   q += C;
    l.sc = (int *)q; q += C;
    l.accD = interval ? q : nullptr;
    return l;
}

__device__ __forceinline__ void load_tables(const Params &p, const Lds &l, int tid)
{
    const int KC = p.K * p.C, C = p.C, CP1 = C | 1;
    for (int i = tid; i < KC; i += NT) l.Wl[i] = p.W[i];
    for (int i = tid; i < C * C; i += NT) l.El[(i / C) * CP1 + (i % C)] = p.Etr[i];
}

// sum of a C-vector in LDS, computed redundantly by every thread in index order
// (uniform result).  Its exponent is the power-of-two scale reference of the scans.
__device__ __forceinline__ double vec_sum(const double *v, int C)
{
    double m = 0.0;
    for (int i = 0; i < C; ++i) m += v[i];
    return m;
}


// Rescale the ring when the scan enters scaling block jnew from block jold:
// every entry of label c is multiplied by 2^(sgn*(n_new-n_old) - e), e being the
// exponent of the sum of the previous step's message vector (a_t going forward,
// p_t going backward).  Returns e.
__device__ __forceinline__ int rebase_ring(const Params &p, const Lds &l, const int *nb,
                                           int jnew, int jold, int sgn, double prevsum, int tid)
{
    const int C = p.C, KC = p.K * p.C;
    const int e = safe_exponent(prevsum);
    if (tid < C) l.sc[tid] = sgn * (nb[(size_t)jnew * C + tid] - nb[(size_t)jold * C + tid]) - e;
    __syncthreads();
    for (int i = tid; i < KC; i += NT) {
        double v = ldexp(l.ring[i], l.sc[i % C]);
        l.ring[i] = fmin(v, DBL_MAX);
    }
    __syncthreads();
    return e;
}

// sum_k W[k,c] * ring[(t -/+ k) mod K][c] over this thread's strip of k.
template <bool BWD>
__device__ __forceinline__ double strip_sum(const Lds &l, int K, int C, int G, int g, int c, int s0)
{
    double acc = 0.0;
    for (int k = g + 1; k <= K; k += G) {
        int slot = BWD ? s0 + k : s0 - k;
        if (BWD) { if (slot >= K) slot -= K; } else { if (slot < 0) slot += K; }
        acc = fma(l.Wl[(k - 1) * C + c], l.ring[slot * C + c], acc);
    }
    return acc;
}

// One forward step at position t (Algorithm 1 body in the linear domain).
// On exit yv = a_t (scaled), ring[t mod K] = q_t.  Two barriers inside, one at exit.
__device__ __forceinline__ void fwd_step(const Params &p, const Lds &l, int G, int tid, int t,
                                         const double2 *EIrow)
{
    const int K = p.K, C = p.C, CP1 = C | 1;
    const int g = tid / C, c = tid % C;
    const int s0 = t % K;
    if (g < G) l.red[g * C + c] = strip_sum<false>(l, K, C, G, g, c, s0);
    __syncthreads();
    if (tid < C) {
        double x = 0.0;
        for (int i = 0; i < G; ++i) x += l.red[i * C + tid];
        l.yv[tid] = x * EIrow[tid].x;
    }
    __syncthreads();
    if (tid < C) {
        double z = 0.0;
        for (int cp = 0; cp < C; ++cp) z = fma(l.yv[cp], l.El[cp * CP1 + tid], z);
        l.ring[s0 * C + tid] = z * EIrow[tid].y;
    }
    __syncthreads();
}

// ---------------------------------------------------------------------------
// The two sequential scans.  grid = B (forward only) or 2B (blockIdx&1 = direction).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(NT) void k_scan(Params p, int both)
{
    extern __shared__ double lds_raw[];
    const int tid = threadIdx.x;
    const int b = both ? (int)(blockIdx.x >> 1) : (int)blockIdx.x;
    const int dir = both ? (int)(blockIdx.x & 1) : 0;
    if (p.spec && p.spec_ok[b * 2 + dir]) return;  // the chunk-parallel scan was accepted
    const int K = p.K, C = p.C, KC = K * C, CP1 = C | 1;
    const int G = min(NT / C, K);
    const Lds l = carve(lds_raw, K, C, G, false);
    const SeqHdr h = p.hdr[b];
    const int L = h.L, J = h.J, Delta = p.Delta;
    const size_t row0 = (size_t)b * (p.T + 1);
    const double2 *EI = p.EI + row0 * C;
    const int *nb = p.nbase + row0 * C;
    const size_t ckstride = (size_t)KC + C;

    load_tables(p, l, tid);
    for (int i = tid; i < KC; i += NT) l.ring[i] = 0.0;
    __syncthreads();

    double Y = 0.0;
    if (dir == 0) {
        // ---- t = 0: a_0 = 1, q_0 = (sum_c' Etr[c',c]) / E_0(c)
        if (tid < C) {
            l.yv[tid] = 1.0;
            double z = 0.0;
            for (int cp = 0; cp < C; ++cp) z += l.El[cp * CP1 + tid];
            l.ring[tid] = z * EI[tid].y;
        }
        __syncthreads();
        if (p.want_grad) {
            double *ck = p.ckA + ((size_t)b * (p.N + 1)) * ckstride;
            for (int i = tid; i < KC; i += NT) ck[i] = l.ring[i];
            if (tid < C) ck[KC + tid] = l.yv[tid];
            if (tid == 0) p.ckYA[(size_t)b * (p.N + 1)] = 0.0;
        }
        for (int t = 1; t <= L; ++t) {
            if ((t % J) == 0) {
                double pm = vec_sum(l.yv, C);
                Y += (double)rebase_ring(p, l, nb, t / J, t / J - 1, +1, pm, tid);
            }
            fwd_step(p, l, G, tid, t, EI + (size_t)t * C);
            if (p.want_grad && (t % Delta) == 0) {
                const int i = t / Delta;
                double *ck = p.ckA + ((size_t)b * (p.N + 1) + i) * ckstride;
                for (int j = tid; j < KC; j += NT) ck[j] = l.ring[j];
                if (tid < C) ck[KC + tid] = l.yv[tid];
                if (tid == 0) p.ckYA[(size_t)b * (p.N + 1) + i] = Y;
            }
        }
        if (tid == 0) {
            double s = 0.0;
            for (int c = 0; c < C; ++c) s += l.yv[c];
            double lz = Y * LN2 + log(s);
            p.hdr[b].logZ = lz;
            p.logz[b] = (float)lz;
            for (int c = 0; c < C; ++c) p.inL[(size_t)b * C + c] = l.yv[c] / s;  // a_L(c) / Z
        }
    } else {
        // ---- t = L: b_L = 1, v_L = E_L; the scale reference starts at sum = 1
        if (tid < C) {
            l.zv[tid] = 1.0;
            l.yv[tid] = tid == 0 ? 1.0 : 0.0;
            l.ring[(L % K) * C + tid] = EI[(size_t)L * C + tid].x;
        }
        __syncthreads();
        for (int t = L - 1; t >= 0; --t) {
            if (((t + 1) % J) == 0) {
                double pm = vec_sum(l.yv, C);
                Y += (double)rebase_ring(p, l, nb, t / J, t / J + 1, -1, pm, tid);
            }
            const int g = tid / C, c = tid % C;
            const int s0 = t % K;
            if (g < G) l.red[g * C + c] = strip_sum<true>(l, K, C, G, g, c, s0);
            __syncthreads();
            if (tid < C) {
                double x = 0.0;
                for (int i = 0; i < G; ++i) x += l.red[i * C + tid];
                l.yv[tid] = x * EI[(size_t)t * C + tid].y;
            }
            __syncthreads();
            if (tid < C) {
                double z = 0.0;
                for (int cc = 0; cc < C; ++cc) z = fma(l.El[tid * CP1 + cc], l.yv[cc], z);
                l.zv[tid] = z;
                l.ring[s0 * C + tid] = z * EI[(size_t)t * C + tid].x;
            }
            __syncthreads();
            if (t > 0 && (t % Delta) == 0) {
                const int i = t / Delta;
                double *ck = p.ckB + ((size_t)b * (p.N + 1) + i) * ckstride;
                for (int j = tid; j < KC; j += NT) ck[j] = l.ring[j];
                if (tid < C) ck[KC + tid] = l.yv[tid];
                if (tid == 0) p.ckYB[(size_t)b * (p.N + 1) + i] = Y;
            }
        }
        if (tid == 0) {
            double s = 0.0;
            for (int c = 0; c < C; ++c) s += l.zv[c];
            p.hdr[b].logZb = Y * LN2 + log(s);
        }
    }
}

// ---------------------------------------------------------------------------
// Latency-oriented scan (C <= 64).  A lone wave issues about one VALU/LDS
// instruction per 8 clocks on this hardware, so the time of a step is the number
// of instructions on the dependent chain; the kernel is organised to keep that
// number small.  One workgroup per (sequence, direction):
//   wave 0 ("tip") owns the dependent chain of a step: the k = 1, 2, 3 terms
//     (its last three ring entries stay in registers), the emission factor, the
//     transition product (its part of the Etr row/column lives in registers; for
//     C <= 32 the two 32-lane halves of the wave each take half of the source
//     labels and are combined with one lane-swap) and the ring write;
//   waves 1.. ("helpers") pre-reduce, two steps ahead, the k >= 4 terms of a
//     later position from the LDS ring and leave one partial per wave and label;
//     the tip adds them in wave order one step before it needs them.  Because the
//     helpers never touch the entry the tip wrote in the step just finished, the
//     tip does not have to wait for its ring write before the step barrier: the
//     write is known to have landed one barrier later (LDS serves a wave in order
//     and the tip has since waited on younger reads).
// The LDS ring is stored twice (slots s and s+K) with a compile-time row stride,
// so a helper lane reads its NKL consecutive durations at immediate offsets from
// one base address, without wrap-around arithmetic.
// One LDS-only barrier per step (outstanding global prefetches are not drained);
// the tip prefetches the (ES, 1/ES) rows PF steps ahead into registers.
// ---------------------------------------------------------------------------
constexpr int PF = 8;        // prefetch distance of the emission factors, in steps
constexpr int NH_MAX = 4;    // most helper waves
constexpr int NKL = 16;      // consecutive durations per helper lane

struct FastGeom {
    int RSLOTS;  // ring slots: both copies plus front padding
    int XP;      // front padding slots (forward direction only)
};

__host__ __device__ inline FastGeom fast_geom(int K, int CTP, int NH)
{
    const int GW = 64 / CTP;
    const int kmaxpad = 3 + NH * GW * NKL;  // largest duration index any helper lane touches
    FastGeom g;
    g.XP = kmaxpad > K ? kmaxpad - K : 0;
    g.RSLOTS = 2 * K + g.XP;
    return g;
}

__host__ __device__ inline size_t fast_lds_doubles(int K, int CTP, int NH)
{
    return (size_t)fast_geom(K, CTP, NH).RSLOTS * CTP + 2 * (size_t)NH_MAX * CTP + 2 * (size_t)CTP;  // yv + 2 int arrays
}

template <int CT, int NHR, bool BWD>
__device__ __forceinline__ void scan_fast_body(const Params &p, double *lds, const int b)
{
    constexpr int CTP = pow2_ge8(CT);       // lanes per label group in a helper wave, LDS row stride
    constexpr int RS = CTP;
    constexpr int GW = 64 / CTP;
    constexpr int H = CT <= 32 ? 2 : 1;     // tip: lane halves sharing the transition product
    constexpr int HC = CT / H;              // source labels per tip lane
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nthreads = blockDim.x;
    const int NH = (nthreads >> 6) - 1;
    const int K = p.K, C = p.C, KC = K * C;
    const FastGeom geo = fast_geom(K, CTP, NH);
    const int XPf = BWD ? 0 : geo.XP;
    const int RTOT = geo.RSLOTS * RS;
    double *ring = lds;                           // [RSLOTS][RS]
    double *part = ring + RTOT;                   // [2][NH_MAX][CTP]
    double *yv = part + 2 * (size_t)NH_MAX * CTP; // [CTP]
    int *sc = (int *)(yv + CTP);                  // [CTP] shift applied at the current boundary
    int *sc_dn = sc + CTP;                        // [CTP] block-exponent delta of the next boundary
    const SeqHdr h = p.hdr[b];
    const int L = h.L, J = h.J, Jm = J - 1, Delta = p.Delta;
    const size_t row0 = (size_t)b * (p.T + 1);
    const double2 *EI = p.EI + row0 * C;
    const int *nb = p.nbase + row0 * C;
    const size_t ckstride = (size_t)KC + C;
    double *ckbase = (BWD ? p.ckB : p.ckA) + ((size_t)b * (p.N + 1)) * ckstride;
    double *ckY = (BWD ? p.ckYB : p.ckYA) + (size_t)b * (p.N + 1);
    const bool tip = wave == 0;
    const int hh = H == 2 ? (lane >> 5) : 0;                    // tip: which half of the source labels
    const int c = lane % CTP;  // label of this lane (tip: both halves; helper: every lane group)
    const bool cval = c < C;
    const int cc = cval ? c : 0;

    // ---- one register array, two meanings: the tip's part of Etr, a helper's W strip
    constexpr int NREG = HC > NKL ? HC : NKL;
    double treg[NREG];
    double *const Ereg = treg;
    double *const wreg = treg;
    double W1 = 0.0, W2 = 0.0, W3 = 0.0;
    const int g = lane / CTP;
    // helper lane (wave, g): durations k0, k0 + GW, k0 + 2 GW, ... so that the 64 lanes of a
    // wave read 64 consecutive doubles of the ring for every term (no LDS bank conflicts)
    const int k0 = 4 + (wave - 1) * GW * NKL + g;
#pragma unroll
    for (int i = 0; i < NREG; ++i) treg[i] = 0.0;
    if (tip) {
        if (cval) {
#pragma unroll
            for (int i = 0; i < HC; ++i) {
                const int o = hh * HC + i;  // the other label of the transition
                if (o < C) Ereg[i] = BWD ? p.Etr[(size_t)c * C + o] : p.Etr[(size_t)o * C + c];
            }
            W1 = p.W[c];
            if (K >= 2) W2 = p.W[(size_t)C + c];
            if (K >= 3) W3 = p.W[(size_t)2 * C + c];
        }
    } else if (cval) {
#pragma unroll
        for (int j = 0; j < NKL; ++j) {
            // forward lanes read their strip from the lowest address up, i.e. longest duration first
            const int k = BWD ? k0 + j * GW : k0 + (NKL - 1 - j) * GW;
            if (k <= K) wreg[j] = p.W[(size_t)(k - 1) * C + c];
        }
    }
    for (int i = tid; i < RTOT; i += nthreads) ring[i] = 0.0;
    for (int i = tid; i < 2 * NH_MAX * CTP; i += nthreads) part[i] = 0.0;
    if (tid < CTP) {
        yv[tid] = 0.0;
        sc[tid] = 0;
    }
    lds_barrier();

    // ---- first position (t = 0 forward, t = L backward)
    double q1 = 0.0, q2 = 0.0, q3 = 0.0, Y = 0.0, prevsum = BWD ? 1.0 : (double)C;
    int slot = BWD ? L % K : 0;  // ring slot (lower copy) of the position just processed
    if (tip && cval) {
        if (!BWD) {
            yv[c] = 1.0;
            double z = 0.0;
#pragma unroll
            for (int i = 0; i < HC; ++i) z += Ereg[i];
            if (H == 2) z = add_across_32(z);
            q1 = z * EI[c].y;
        } else {
            yv[c] = c == 0 ? 1.0 : 0.0;
            q1 = EI[(size_t)L * C + c].x;
        }
        ring[(XPf + slot) * RS + c] = q1;
        ring[(XPf + slot + K) * RS + c] = q1;
    }
    // Block-exponent deltas are staged through LDS by helper wave 1, one boundary ahead, so
    // that no global load is ever pending in a tip register (a wait on it would also
    // drain the tip's emission-factor prefetch queue, the counter being in-order).
    // sc_dn holds n_new(c) - n_old(c) of the next boundary; dn_from/dn_to are the pending loads
    // of n(c) on both sides of the boundary after it.
    int dn_from = 0, dn_to = 0;
    const int jlast = L / J;
    auto block_after = [&](int j) { return BWD ? max(j - 1, 0) : min(j + 1, jlast); };
    if (wave == 1) {
        const int j0 = BWD ? jlast : 0, j1 = block_after(j0), j2 = block_after(j1);
        if (lane < CTP) sc_dn[lane] = nb[(size_t)j1 * C + cc] - nb[(size_t)j0 * C + cc];
        dn_from = nb[(size_t)j1 * C + cc];
        dn_to = nb[(size_t)j2 * C + cc];
    }
    lds_barrier();
    auto write_checkpoint = [&](int i) {
        double *ck = ckbase + (size_t)i * ckstride;
        for (int q = tid; q < KC; q += nthreads) ck[q] = ring[(XPf + q / C) * RS + (q % C)];
        if (tid < C) ck[KC + tid] = yv[tid];
        if (tid == 0) ckY[i] = Y;
    };
    if (!BWD && p.want_grad) write_checkpoint(0);

    // helper: partial of sum_{k>=4} W[k,c] ring[pos -/+ k] over this lane's NKL durations,
    // for the position whose lower-copy slot is ps.
    auto helper_partial = [&](int ps, int buf) {
        const double *base = BWD ? ring + (size_t)(ps + k0) * RS + c
                                 : ring + (size_t)(XPf + ps + K - k0 - (NKL - 1) * GW) * RS + c;
        double v[NKL];
#pragma unroll
        for (int j = 0; j < NKL; ++j) v[j] = base[j * GW * RS];
        double a0 = 0.0, a1 = 0.0;
#pragma unroll
        for (int j = 0; j < NKL; j += 2) {
            a0 = fma(wreg[j], v[j], a0);
            a1 = fma(wreg[j + 1], v[j + 1], a1);
        }
        const double acc = group_sum<CTP>(a0 + a1);
        if (lane < CTP) part[((size_t)buf * NH_MAX + (wave - 1)) * CTP + lane] = acc;
    };
    auto step_slot = [&](int sl, int by) {  // slot of the position `by` steps further along the scan
        int r = BWD ? sl - by : sl + by;  // by <= 2, so two conditional wraps suffice for any K >= 1
        if (BWD) {
            if (r < 0) r += K;
            if (r < 0) r += K;
        } else {
            if (r >= K) r -= K;
            if (r >= K) r -= K;
        }
        return r;
    };

    // ---- pieces of a step that every wave runs (uniform control flow, same barriers)
    // sc[] was written by the tip before the first barrier; pbuf is the partial buffer that
    // was computed before this boundary and is still to be consumed
    auto rescale_ring = [&](int pbuf) {
        lds_barrier();
        for (int i = tid; i < RTOT; i += nthreads)
            ring[i] = fmin(ldexp(ring[i], sc[i % RS]), DBL_MAX);
        double *pb = part + (size_t)pbuf * NH_MAX * CTP;
        for (int i = tid; i < NH_MAX * CTP; i += nthreads)
            pb[i] = fmin(ldexp(pb[i], sc[i % CTP]), DBL_MAX);
        lds_barrier();
    };
    // steps left until the next checkpoint position (a positive multiple of Delta)
    int dleft = BWD ? L - ((L - 1) / Delta) * Delta : Delta;
    auto after_step = [&](int t) {
        if (__builtin_expect(--dleft == 0, 0)) {
            dleft = Delta;
            if (p.want_grad && t > 0) {
                lds_barrier();  // the tip's newest ring entry has landed (its step barrier does not wait)
                write_checkpoint(t / Delta);
                lds_barrier();
            }
        }
    };

    if (tip) {
        // All 64 lanes run the same instruction stream without masks: lanes whose label
        // index is >= C carry zeros (W1 = W2 = 0, Ereg = 0, their partials are 0).
        const double2 *EIc = EI + cc;  // this lane's column; rows are addressed by a uniform offset
        double2 qe[PF];                // emission factors of the next PF steps (aligned groups)
#pragma unroll
        for (int j = 0; j < PF; ++j) qe[j] = make_double2(0.0, 0.0);
        // Nothing lies k >= 4 behind steps 1 and 2, so their partials are the zeros
        // already in `part`.  psum is the partial of the step about to run.
        double psum = 0.0, zlast = 1.0;
        const double2 *ys = (const double2 *)__builtin_assume_aligned(yv + hh * HC, 16);
        // `kind` says which rare events a step has to look for.  Steps run in groups of 8
        // aligned on t = 0 mod 8 whenever J and Delta are multiples of 8: then a scaling
        // boundary can only precede the first step of a group and its scale reference is
        // only needed after the last one, and most steps carry no branch at all.
        //   0: any step (all checks)      1: first of a group
        //   2: middle of a group          3: last of a group
        auto tip_step = [&](auto kind_tag, const int n, const double2 e) {
            constexpr int kind = decltype(kind_tag)::value;
            const int t = BWD ? L - n : n;
            const bool boundary = kind == 0 || kind == 1 ? (BWD ? ((t + 1) & Jm) == 0 : (t & Jm) == 0) : false;
            if (__builtin_expect(boundary, 0)) {  // uniform: rescale ring, tip registers, pending partials
                const int ex = safe_exponent(prevsum);
                Y += (double)ex;
                const int sft = (BWD ? -sc_dn[c] : sc_dn[c]) - ex;
                sc[c] = sft;
                q1 = fmin(ldexp(q1, sft), DBL_MAX);
                q2 = fmin(ldexp(q2, sft), DBL_MAX);
                q3 = fmin(ldexp(q3, sft), DBL_MAX);
                psum = fmin(ldexp(psum, sft), DBL_MAX);
                rescale_ring((n + 1) & 1);
            }
            slot = step_slot(slot, 1);
            // partial of the NEXT step (finished by the helpers one barrier ago)
            const double *pp = part + (size_t)((n + 1) & 1) * NH_MAX * CTP + c;
            double pv[NHR];
#pragma unroll
            for (int w = 0; w < NHR; ++w) pv[w] = pp[w * CTP];
            const double x = fma(W1, q1, fma(W2, q2, fma(W3, q3, psum)));
            yv[c] = x * (BWD ? e.y : e.x);
            lds_wave_fence();
            double z0 = 0.0, z1 = 0.0;
#pragma unroll
            for (int i = 0; i < HC; i += 2) {
                const double2 vv = ys[i >> 1];
                z0 = fma(vv.x, Ereg[i], z0);
                z1 = fma(vv.y, Ereg[i + 1], z1);
            }
            double z = z0 + z1;
            if (H == 2) z = add_across_32(z);
            q3 = q2;
            q2 = q1;
            q1 = z * (BWD ? e.x : e.y);
            double *rw = ring + (size_t)(XPf + slot) * RS + c;
            rw[0] = q1;
            rw[(size_t)K * RS] = q1;
            double pn = pv[0];
#pragma unroll
            for (int w = 1; w < NHR; ++w) pn += pv[w];
            psum = pn;
            zlast = z;
            const bool want_sum = kind == 0 || kind == 3 ? (BWD ? (t & Jm) == 0 : ((t + 1) & Jm) == 0) : false;
            if (__builtin_expect(want_sum, 0)) {  // uniform: scale reference for the boundary that follows
                double sum = 0.0;
                for (int i = 0; i < CT; ++i) sum += yv[i];
                prevsum = sum;
            }
            // no wait for the ring write here (see the kernel comment); the tip's other LDS
            // traffic of this step has been consumed by itself already
            tip_step_barrier();
            if (kind == 0) {
                after_step(t);
            } else if (BWD ? kind == 3 : kind == 1) {
                // the only step of a group that can sit on a checkpoint position (t = 0 mod 8);
                // dleft is brought up to date for the whole group by the caller
                const int due = BWD ? 8 : 1;
                if (__builtin_expect(dleft == due, 0)) {
                    dleft = Delta + due;
                    if (p.want_grad && t > 0) {
                        lds_barrier();
                        write_checkpoint(t / Delta);
                        lds_barrier();
                    }
                }
            }
        };
        using K0 = std::integral_constant<int, 0>;
        using K1 = std::integral_constant<int, 1>;
        using K2 = std::integral_constant<int, 2>;
        using K3 = std::integral_constant<int, 3>;
        static_assert(PF == 8, "the aligned groups are 8 steps long");
        const bool grouped = (J % 8) == 0 && (Delta % 8) == 0;
        int n = 1;
        if (grouped) {
            // single steps until the next position is the first of an aligned group
            while (n <= L && ((BWD ? L - n : n) & 7) != (BWD ? 7 : 0)) {
                tip_step(K0{}, n, EIc[(size_t)(BWD ? L - n : n) * C]);
                ++n;
            }
            if (n + 7 <= L) {
#pragma unroll
                for (int j = 0; j < PF; ++j) qe[j] = EIc[(size_t)(BWD ? L - (n + j) : n + j) * C];
            }
            for (; n + 7 <= L; n += 8) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const double2 e = qe[j];
                    int n2 = n + j + 8;
                    if (n2 > L) n2 = L;
                    qe[j] = EIc[__builtin_amdgcn_readfirstlane((BWD ? L - n2 : n2) * C)];
                    if (j == 0) tip_step(K1{}, n + j, e);
                    else if (j == 7) tip_step(K3{}, n + j, e);
                    else tip_step(K2{}, n + j, e);
                }
                dleft -= 8;
            }
        } else if (n + 7 <= L) {
            // J or Delta is not a multiple of 8: same prefetch queue, every step checks everything
#pragma unroll
            for (int j = 0; j < PF; ++j) qe[j] = EIc[(size_t)(BWD ? L - (n + j) : n + j) * C];
            for (; n + 7 <= L; n += 8) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const double2 e = qe[j];
                    int n2 = n + j + 8;
                    if (n2 > L) n2 = L;
                    qe[j] = EIc[__builtin_amdgcn_readfirstlane((BWD ? L - n2 : n2) * C)];
                    tip_step(K0{}, n + j, e);
                }
            }
        }
        for (; n <= L; ++n) tip_step(K0{}, n, EIc[(size_t)(BWD ? L - n : n) * C]);
        if (BWD && L > 0) yv[c] = zlast;  // beta_0: diagnostic partition function
        lds_wave_fence();
        if (tid == 0) {
            double s = 0.0;
            for (int i = 0; i < C; ++i) s += (BWD && L == 0) ? 1.0 : yv[i];
            const double lz = Y * LN2 + log(s);
            if (BWD) {
                p.hdr[b].logZb = lz;
            } else {
                p.hdr[b].logZ = lz;
                p.logz[b] = (float)lz;
                for (int i = 0; i < C; ++i) p.inL[(size_t)b * C + i] = yv[i] / s;  // a_L(c) / Z
            }
        }
    } else {
        for (int n = 1; n <= L; ++n) {
            const int t = BWD ? L - n : n;
            const bool boundary = BWD ? ((t + 1) & Jm) == 0 : (t & Jm) == 0;
            if (__builtin_expect(boundary, 0)) {
                rescale_ring((n + 1) & 1);
                if (wave == 1) {
                    // this boundary consumed sc_dn: publish the delta of the next boundary (its
                    // loads were issued one boundary ago) and start loading the one after it
                    if (lane < CTP) sc_dn[lane] = dn_to - dn_from;
                    const int ja = block_after(t / J), jb = block_after(ja);
                    dn_from = nb[(size_t)ja * C + cc];
                    dn_to = nb[(size_t)jb * C + cc];
                }
            }
            slot = step_slot(slot, 1);
            if (n + 2 <= L) helper_partial(step_slot(slot, 2), n & 1);
            lds_barrier();
            after_step(t);
        }
    }
}

template <int CT, int NHR>
__global__ __launch_bounds__(CT == 64 ? 64 * (NHR + 1) : 320) void k_scan_fast(Params p, int both)
{
    extern __shared__ double lds_raw[];
    const int b = both ? (int)(blockIdx.x >> 1) : (int)blockIdx.x;
    const int dir = both ? (int)(blockIdx.x & 1) : 0;
    if (p.spec && p.spec_ok[b * 2 + dir]) return;  // the chunk-parallel scan was accepted
    if (dir == 0) scan_fast_body<CT, NHR, false>(p, lds_raw, b);
    else scan_fast_body<CT, NHR, true>(p, lds_raw, b);
}

// ---------------------------------------------------------------------------
// Per-interval backward work (Algorithm 3 body for one checkpoint interval):
// restore the forward ring from the checkpoint, recompute a_t and q_t for the
// interval, then run the backward recurrence across it from the backward
// checkpoint, accumulating
//   partD[k,c]  += q_t(c) W[k,c] v_{t+k}(c) / Z                (duration bias)
//   partTr[c',c] += a_t(c') p_t(c) / Z     (times Etr at the end; transitions)
//   d_t(c) = out_t(c) - in_t(c), out = z_t p_t / Z (a c-segment starts at t),
//            in = a_t b_t / Z (a c-segment ends at t); the running sum of d over
//            positions is the position marginal.
// Persistent workgroups: task = (sequence, interval).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(NT) void k_interval(Params p)
{
    extern __shared__ double lds_raw[];
    const int tid = threadIdx.x;
    const int K = p.K, C = p.C, KC = K * C, CP1 = C | 1, CC = C * C;
    const int G = min(NT / C, K);
    const Lds l = carve(lds_raw, K, C, G, true);
    const int Delta = p.Delta, N = p.N;
    const size_t ckstride = (size_t)KC + C;
    double *aloc = p.aloc + (size_t)blockIdx.x * Delta * 2 * C;
    double *alocY = p.alocY + (size_t)blockIdx.x * Delta;
    constexpr int TRP = GRAD_CMAX * GRAD_CMAX / NT;  // transition pairs per thread
    load_tables(p, l, tid);
    __syncthreads();

    const int ntask = p.B * N;
    for (int task = blockIdx.x; task < ntask; task += gridDim.x) {
        const int b = task / N, iv = task % N;
        const SeqHdr h = p.hdr[b];
        const int L = h.L, J = h.J;
        const int t0 = iv * Delta;
        if (t0 >= L) continue;  // uniform
        if (p.marg && p.spec_ok[b * 2] && p.spec_ok[b * 2 + 1]) continue;  // uniform: done from the stored rows
        const int t1 = min(t0 + Delta, L);
        const size_t row0 = (size_t)b * (p.T + 1);
        const double2 *EI = p.EI + row0 * C;
        const int *nb = p.nbase + row0 * C;
        const double logZ = h.logZ;

        // ------------------------------------------------ forward recompute
        {
            const double *ck = p.ckA + ((size_t)b * (N + 1) + iv) * ckstride;
            for (int i = tid; i < KC; i += NT) l.ring[i] = ck[i];
            if (tid < C) l.yv[tid] = ck[KC + tid];
        }
        double Y = p.ckYA[(size_t)b * (N + 1) + iv];
        __syncthreads();
        if (tid < C) {
            aloc[tid] = l.yv[tid];
            aloc[C + tid] = l.ring[(t0 % K) * C + tid];
        }
        if (tid == 0) alocY[0] = Y;
        for (int t = t0 + 1; t < t1; ++t) {
            if ((t % J) == 0) {
                double pm = vec_sum(l.yv, C);
                Y += (double)rebase_ring(p, l, nb, t / J, t / J - 1, +1, pm, tid);
            }
            fwd_step(p, l, G, tid, t, EI + (size_t)t * C);
            if (tid < C) {
                double *row = aloc + (size_t)(t - t0) * 2 * C;
                row[tid] = l.yv[tid];
                row[C + tid] = l.ring[(t % K) * C + tid];
            }
            if (tid == 0) alocY[t - t0] = Y;
        }
        __syncthreads();

        // ------------------------------------------------ backward across the interval
        double Yb;
        if (t1 == L) {
            for (int i = tid; i < KC; i += NT) l.ring[i] = 0.0;
            __syncthreads();
            if (tid < C) {
                l.yv[tid] = tid == 0 ? 1.0 : 0.0;
                l.ring[(L % K) * C + tid] = EI[(size_t)L * C + tid].x;
            }
            Yb = 0.0;
        } else {
            const int ci = t1 / Delta;
            const double *ck = p.ckB + ((size_t)b * (N + 1) + ci) * ckstride;
            for (int i = tid; i < KC; i += NT) l.ring[i] = ck[i];
            if (tid < C) l.yv[tid] = ck[KC + tid];
            Yb = p.ckYB[(size_t)b * (N + 1) + ci];
        }
        for (int i = tid; i < KC; i += NT) l.accD[i] = 0.0;
        double accTr[TRP];
#pragma unroll
        for (int j = 0; j < TRP; ++j) accTr[j] = 0.0;
        double R = 0.0, sR = 0.0;  // running suffix sum of d and its sum (threads < C)
        double kappa = 0.0, kY = -1.0e300;
        __syncthreads();

        for (int t = t1 - 1; t >= t0; --t) {
            if (((t + 1) % J) == 0) {
                double pm = vec_sum(l.yv, C);
                Yb += (double)rebase_ring(p, l, nb, t / J, t / J + 1, -1, pm, tid);
            }
            const double *row = aloc + (size_t)(t - t0) * 2 * C;
            if (tid < C) {
                l.av[tid] = row[tid];
                l.qv[tid] = row[C + tid];
            }
            const double ysum = alocY[t - t0] + Yb;
            if (ysum != kY) {  // uniform
                kY = ysum;
                kappa = exp(ysum * LN2 - logZ);
            }
            __syncthreads();
            const int g = tid / C, c = tid % C;
            const int s0 = t % K;
            if (g < G) {
                const double coef = l.qv[c] * kappa;
                double acc = 0.0;
                for (int k = g + 1; k <= K; k += G) {
                    int slot = s0 + k;
                    if (slot >= K) slot -= K;
                    double prod = l.Wl[(k - 1) * C + c] * l.ring[slot * C + c];
                    acc += prod;
                    l.accD[(k - 1) * C + c] = fma(coef, prod, l.accD[(k - 1) * C + c]);
                }
                l.red[g * C + c] = acc;
            }
            __syncthreads();
            double outv = 0.0;
            if (tid < C) {
                double x = 0.0;
                for (int i = 0; i < G; ++i) x += l.red[i * C + tid];
                l.yv[tid] = x * EI[(size_t)t * C + tid].y;
                outv = l.qv[tid] * x * kappa;
            }
            __syncthreads();
            if (tid < C) {
                double z = 0.0;
                for (int cc = 0; cc < C; ++cc) z = fma(l.El[tid * CP1 + cc], l.yv[cc], z);
                l.zv[tid] = z;
                l.ring[s0 * C + tid] = z * EI[(size_t)t * C + tid].x;
                const double inv = t >= 1 ? l.av[tid] * z * kappa : 0.0;
                p.grad_emis[((size_t)b * p.T + t) * C + tid] = (float)R;
                sR += R;
                R += outv - inv;
                // gradients of the boundary terms: a segment starts at t (first token t), ends at t (last token t-1)
                const double wb = p.grad_logz ? (double)p.grad_logz[b] : 1.0;
                if (p.g_proj_start) p.g_proj_start[((size_t)b * p.T + t) * C + tid] = (float)(wb * outv);
                if (p.g_proj_end && t >= 1) p.g_proj_end[((size_t)b * p.T + t - 1) * C + tid] = (float)(wb * inv);
                if (t == 0) p.out0[(size_t)b * C + tid] = outv;
                if (p.bdy_post) l.red[tid] = inv;
            }
            if (p.bdy_post) {  // posterior of a boundary at t: total mass of the segments that end there
                __syncthreads();
                if (tid == 0 && t >= 1) {
                    double sb = 0.0;
                    for (int i = 0; i < C; ++i) sb += l.red[i];
                    p.bdy_post[(size_t)b * (p.T + 1) + t] = (float)sb;
                }
                __syncthreads();
            }
#pragma unroll
            for (int j = 0; j < TRP; ++j) {
                const int idx = tid + j * NT;
                if (idx < CC) accTr[j] = fma(l.av[idx / C] * kappa, l.yv[idx % C], accTr[j]);
            }
            __syncthreads();
        }

        double *pD = p.partD + ((size_t)b * N + iv) * KC;
        for (int i = tid; i < KC; i += NT) pD[i] = l.accD[i];
        double *pT = p.partTr + ((size_t)b * N + iv) * CC;
#pragma unroll
        for (int j = 0; j < TRP; ++j) {
            const int idx = tid + j * NT;
            if (idx < CC) pT[idx] = accTr[j];
        }
        if (tid < C) {
            p.tot[((size_t)b * N + iv) * C + tid] = R;
            p.sumR[((size_t)b * N + iv) * C + tid] = sR;
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------
// One-wave kernels (interval stage and chunk-parallel scan): shared geometry.
//
// Window.  The last KW >= K messages of a scan live in a LINEAR LDS buffer of KW + M rows
// of exactly CT doubles: the newest row moves up (forward) or down (backward) by one per
// position, every read is base + compile-time offset, and when the buffer's end is
// reached the window is moved back (KW*CT/64 loads and stores per lane every ~M positions).
//
// Time blocking.  LDS bandwidth, not arithmetic, bounds a scan that re-reads its whole
// window at every position (8 bytes per multiply-add).  Positions are therefore taken in
// blocks of MB: lane (g, c) owns the window entries at distances d = g*NK .. g*NK+NK-1 from
// the newest message of label c, reads each ONCE per block and uses it for all MB positions
// of the block (weights W[d+1] .. W[d+MB]: a register strip of NK+MB-1 values).  What the
// block's own new messages contribute to its later positions (durations 1..MB-1) is added
// from registers while the positions are finished one after the other.
// ---------------------------------------------------------------------------
// MB positions per time block; wave_nk, lin_slack and wave_lds_doubles give the window's size (geometry.h).

// Geometry and the window operations shared by the one-wave kernels.
template <int CT, int NKW>
struct WaveWin {
    static constexpr int CTP = pow2_ge8(CT);
    static constexpr int RS = CT;
    static constexpr int GW = 64 / CTP;
    static constexpr int NK = wave_nk(CT, NKW);
    static constexpr int KW = NK * GW;
    static constexpr int M = lin_slack(KW);
    static constexpr int ROWS = KW + M;
    static constexpr int RTOT = ROWS * RS + (CTP - CT);  // lanes c >= C read (and ignore) past a row's end
    static constexpr int H = CT <= 32 ? 2 : 1;
    static constexpr int HC = CT / H;
    static constexpr int YS = CTP < 16 ? 16 : CTP;  // row stride of the MB message-vector rows
    static constexpr int TRN = (CT + 15) / 16;       // 16-label tiles of the transition gradient

    // every entry of label c times 2^sft (each lane scales its own label's column)
    static __device__ __forceinline__ void rescale(double *ring, int g, int c, bool cval, int sft)
    {
        if (cval) {
            double *q = ring + g * RS + c;
#pragma unroll 8
            for (int row = g; row < ROWS; row += GW, q += GW * RS) *q = fmin(ldexp(*q, sft), DBL_MAX);
        }
        lds_wave_fence();
    }

    // Move the live window (newest row r) back to the start of the buffer; returns the new r.
    // Chunk order keeps the sources ahead of the stores.
    template <bool BWD>
    static __device__ __forceinline__ int move(double *ring, int lane, int r)
    {
        constexpr int NCP = (KW * RS + 63) / 64;
        const int shift = (BWD ? M - r : r - (KW - 1)) * RS;  // doubles, > 0
        const int first = (BWD ? r : r - (KW - 1)) * RS;      // lowest double of the live window
        for (int u = 0; u < NCP; ++u) {
            const int i = (BWD ? NCP - 1 - u : u) * 64 + lane;
            double v = 0.0;
            if (i < KW * RS) v = ring[first + i];
            lds_wave_fence();
            if (i < KW * RS) ring[first + i + (BWD ? shift : -shift)] = v;
            lds_wave_fence();
        }
        return BWD ? M : KW - 1;
    }

    // Checkpoint layout: message of position t' at slot t' mod K.  d = distance of slot sl
    // from the newest position t.
    template <bool BWD>
    static __device__ __forceinline__ int slot_dist(int sl, int tm, int K)
    {
        int d = BWD ? sl - tm : tm - sl;
        if (d < 0) d += K;
        return d;
    }
};

// ---------------------------------------------------------------------------
// Per-interval backward work (Algorithm 3 body), throughput-oriented variant: ONE WAVE per
// task, no barriers.  The interval stage has hundreds of independent tasks, so unlike a
// sequential scan it is bound by instruction and LDS throughput, which several independent
// single-wave workgroups per compute unit fill better than one multi-wave workgroup that
// synchronises every step.  A lane (g, c) keeps its strip of W, the matching grad_dur
// accumulators, its part of the transition row/column and the matching grad_trans
// accumulators in registers for the whole task.
// ---------------------------------------------------------------------------
// With 64 labels a lane owns a whole 64-entry row or column of the transition matrix, which
// does not fit the registers next to the duration strips.  Both orientations of the matrix
// then live in LDS ([source][lane] order, conflict-free), shared by the IWAVES independent
// single-wave tasks of a workgroup.
// With the longest duration strips (NKW = 64) the strip of weights and the strip of grad_dur
// accumulators do not both fit the registers; the weights then live in LDS as well, W[m+1, c]
// at [m*CT + c] (zero beyond K), and are read once per block like the window.
// (interval_waves, interval_wtab_doubles, interval_lds_doubles: geometry.h)

template <int CT, int NKW>
__global__ __launch_bounds__(64 * interval_waves(CT, NKW)) void k_interval_wave(Params p)
{
    constexpr bool ELDS = CT == 64;
    constexpr bool WLDS = NKW == 64;
    constexpr int IW = interval_waves(CT, NKW);
    using G = WaveWin<CT, NKW>;
    constexpr int CTP = G::CTP, RS = G::RS, NK = G::NK, KW = G::KW, M = G::M, ROWS = G::ROWS;
    constexpr int RTOT = G::RTOT, H = G::H, HC = G::HC, YS = G::YS, TRN = G::TRN;
    typedef double double4_t __attribute__((ext_vector_type(4)));
    extern __shared__ double lds_raw[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int K = p.K, C = p.C, KC = K * C, CC = C * C;
    double *EtF = lds_raw;                        // [o][c] = Etr[o,c]   (forward:  z(c) = sum_o a(o) Etr[o,c])
    double *EtB = lds_raw + (ELDS ? CT * CT : 0);  // [o][c] = Etr[c,o]   (backward: b(c) = sum_o Etr[c,o] p(o))
    if (ELDS) {
        for (int i = threadIdx.x; i < CT * CT; i += 64 * IW) {
            const int o = i / CT, cl = i % CT;
            const bool ok = o < C && cl < C;
            EtF[i] = ok ? p.Etr[(size_t)o * C + cl] : 0.0;
            EtB[i] = ok ? p.Etr[(size_t)cl * C + o] : 0.0;
        }
    }
    double *Wl = lds_raw + (ELDS ? 2 * CT * CT : 0);
    constexpr int WTAB = (int)interval_wtab_doubles(CT, NKW);
    if (WLDS) {
        for (int i = threadIdx.x; i < WTAB; i += 64 * IW) {
            const int m = i / CT, col = i % CT;
            Wl[i] = (m < K && col < C) ? p.W[(size_t)m * C + col] : 0.0;
        }
    }
    if (ELDS || WLDS) __syncthreads();  // the only workgroup-wide synchronisation: the waves are independent from here
    double *ring = Wl + WTAB + (size_t)wave * (RTOT + MB * YS);  // [ROWS][RS] (+ pad)
    double *yv = ring + RTOT;        // [MB][YS]: message vector of each position of a block (row 0 outside the beta pass)
    const int Delta = p.Delta, N = p.N;
    const size_t ckstride = (size_t)KC + C;
    const int c = lane % CTP, g = lane / CTP;
    const int hh = H == 2 ? (lane >> 5) : 0;
    const bool cval = c < C;
    const int cc = cval ? c : 0;
    const bool writer = cval && g == 0;  // one lane per label
    const int slot = blockIdx.x * IW + wave;
    double2 *aloc = (double2 *)p.aloc + (size_t)slot * Delta * C;
    double *alocY = p.alocY + (size_t)slot * Delta;

    // task-invariant registers
    double wx[WLDS ? 1 : NK + MB - 1];  // W[g*NK + jj + 1, c] (register variant)
    if (!WLDS) {
#pragma unroll
        for (int jj = 0; jj < NK + MB - 1; ++jj) {
            const int k = g * NK + jj + 1;
            wx[WLDS ? 0 : jj] = (cval && k <= K) ? p.W[(size_t)(k - 1) * C + c] : 0.0;
        }
    }
    const double *wl = Wl + g * NK * CT + c;  // LDS variant: W[g*NK + m + 1, c] at wl[m*CT]
    double wn[MB - 1];       // W[1..MB-1, c]: durations inside a block
#pragma unroll
    for (int jj = 0; jj < MB - 1; ++jj) wn[jj] = (cval && jj + 1 <= K) ? p.W[(size_t)jj * C + c] : 0.0;
    double Ereg[ELDS ? 2 : HC];  // this lane's part of the transition column (forward) / row (backward)
    const double *et = EtF + c;  // LDS variant: coefficient of source o at et[o * CT]
    auto load_etr = [&](bool backward) {
        if (ELDS) {
            et = (backward ? EtB : EtF) + c;
            return;
        }
#pragma unroll
        for (int i = 0; i < HC; ++i) {
            const int o = hh * HC + i;
            const bool ok = cval && o < C;
            // forward: z(c) = sum_o a(o) Etr[o,c];  backward: b(c) = sum_o Etr[c,o] p(o)
            Ereg[i] = ok ? (backward ? p.Etr[(size_t)c * C + o] : p.Etr[(size_t)o * C + c]) : 0.0;
        }
    };
    const double2 *ys = (const double2 *)__builtin_assume_aligned(yv + hh * HC, 16);
    auto yv_sum = [&](const int row) {
        double s = 0.0;
        for (int i = 0; i < CT; ++i) s += yv[row * YS + i];
        return s;
    };

    const int ntask = p.B * N;
    for (int task = slot; task < ntask; task += gridDim.x * IW) {
        const int b = task / N, iv = task % N;
        const SeqHdr h = p.hdr[b];
        const int L = h.L, J = h.J, Jm = J - 1;
        const int t0 = iv * Delta;
        if (t0 >= L) continue;
        if (p.marg && p.spec_ok[b * 2] && p.spec_ok[b * 2 + 1]) continue;  // done from the stored rows of both scans
        const int t1 = min(t0 + Delta, L);
        const size_t row0 = (size_t)b * (p.T + 1);
        const double2 *EIc = p.EI + row0 * C + cc;
        const int *nbc = p.nbase + row0 * C + cc;
        const double logZ = h.logZ;
        // exponent step n_j(c) - n_{j-1}(c) of the lane's label at the scaling-block boundary j*J
        auto nbdelta = [&](const int j) {
            return (j >= 1 && (long)j * J <= (long)L) ? nbc[(size_t)j * C] - nbc[(size_t)(j - 1) * C] : 0;
        };

        // ============================ forward recompute over (t0, t1) ============================
        // Scale of the interval's first position; the stored per-position scales are relative to it.
        const double Y0 = p.ckYA[(size_t)b * (N + 1) + iv];
        // An accepted chunk-parallel forward scan has already stored this interval's rows.
        const bool stored = p.fuse && p.spec_ok[b * 2];
        int r = KW - 1;  // row of the newest message
        if (!stored) {
        load_etr(false);
        for (int i = lane; i < RTOT; i += 64) ring[i] = 0.0;
        for (int i = lane; i < MB * YS; i += 64) yv[i] = 0.0;
        lds_wave_fence();
        {
            const double *ck = p.ckA + ((size_t)b * (N + 1) + iv) * ckstride;
            const int tm = t0 % K;
            for (int i = lane; i < KC; i += 64) {
                const int sl = i / C, col = i % C;
                ring[(r - G::template slot_dist<false>(sl, tm, K)) * RS + col] = ck[i];
            }
            if (lane < C) yv[lane] = ck[KC + lane];
        }
        lds_wave_fence();
        double Y = 0.0;
        if (writer) aloc[c] = make_double2(yv[c], ring[r * RS + c]);
        if (lane == 0) alocY[0] = Y;
        {
            const int tend = t1 - 1;  // alpha of position t1 belongs to the next interval
            const int rdoff = -(g * NK + NK - 1) * RS + c;
            int t = t0;
            auto load_rows = [&](double2 (&e)[MB], const int tfrom) {
#pragma unroll
                for (int i = 0; i < MB; ++i) e[i] = EIc[(size_t)min(tfrom + 1 + i, L) * C];
            };
            double2 e[MB];
            load_rows(e, t);
            int jnx = t0 / J + 1;      // next scaling-block boundary ahead (position jnx*J) ...
            int dnx = nbdelta(jnx);    // ... and its exponent step, loaded one block of J early
            while (t < tend) {
                int nb = min(tend - t, MB);
                nb = min(nb, J - ((t + 1) & Jm));  // only a block's first position may cross a scaling boundary
                if (__builtin_expect(((t + 1) & Jm) == 0, 0)) {
                    const int ex = safe_exponent(yv_sum(0));
                    Y += (double)ex;
                    G::rescale(ring, g, c, cval, dnx - ex);
                    dnx = nbdelta(++jnx);
                }
                if (__builtin_expect(r + MB > ROWS - 1, 0)) r = G::template move<false>(ring, lane, r);
                const double *base = ring + r * RS + rdoff;
                double acc[MB];
#pragma unroll
                for (int i = 0; i < MB; ++i) acc[i] = 0.0;
                if (WLDS) {
                    double v[NK];
#pragma unroll
                    for (int m = 0; m < NK + MB - 1; ++m) {
                        const double w = wl[m * CT];
                        if (m < NK) v[m] = base[(NK - 1 - m) * RS];
#pragma unroll
                        for (int i = 0; i < MB; ++i)
                            if (m - i >= 0 && m - i < NK) acc[i] = fma(w, v[m - i], acc[i]);
                    }
                } else {
#pragma unroll
                    for (int jj = 0; jj < NK; ++jj) {
                        const double v = base[(NK - 1 - jj) * RS];  // distance g*NK + jj from the newest
#pragma unroll
                        for (int i = 0; i < MB; ++i) acc[i] = fma(wx[WLDS ? 0 : jj + i], v, acc[i]);
                    }
                }
#pragma unroll
                for (int i = 0; i < MB; ++i) acc[i] = group_sum<CTP>(acc[i]);
                double qn[MB];
#pragma unroll
                for (int i = 0; i < MB; ++i) {
                    if (i < nb) {
                        double x = acc[i];
#pragma unroll
                        for (int jn = 0; jn < i; ++jn) x = fma(wn[i - 1 - jn], qn[jn], x);
                        const double y = x * e[i].x;
                        if (cval) yv[c] = y;
                        lds_wave_fence();
                        double z0 = 0.0, z1 = 0.0;
#pragma unroll
                        for (int o = 0; o < HC; o += 2) {
                            const double2 vv = ys[o >> 1];
                            z0 = fma(vv.x, ELDS ? et[o * CT] : Ereg[ELDS ? 0 : o], z0);
                            z1 = fma(vv.y, ELDS ? et[(o + 1) * CT] : Ereg[ELDS ? 1 : o + 1], z1);
                        }
                        double z = z0 + z1;
                        if (H == 2) z = add_across_32(z);
                        const double q = z * e[i].y;
                        qn[i] = q;
                        ++r;
                        if (writer) {
                            ring[r * RS + c] = q;
                            aloc[(size_t)(t + 1 + i - t0) * C + c] = make_double2(y, q);
                        }
                        if (lane == 0) alocY[t + 1 + i - t0] = Y;
                        lds_wave_fence();
                    } else {
                        qn[i] = 0.0;
                    }
                }
                t += nb;
                load_rows(e, t);  // the next block's rows (first use a block's window pass later)
            }
        }
        }  // !stored

        // ============================ backward pass over [t0, t1) ============================
        __threadfence_block();  // this wave's aloc / alocY rows are read back by all of its lanes
        load_etr(true);
        for (int i = lane; i < RTOT; i += 64) ring[i] = 0.0;
        for (int i = lane; i < MB * YS; i += 64) yv[i] = 0.0;
        lds_wave_fence();
        r = M;
        double Yb;
        if (t1 == L) {  // beta_L = 1: v_L = E_L, scale reference sum = 1
            if (writer) ring[r * RS + c] = EIc[(size_t)L * C].x;
            if (lane == 0) yv[0] = 1.0;
            Yb = 0.0;
        } else {
            const int ci = t1 / Delta;
            const double *ck = p.ckB + ((size_t)b * (N + 1) + ci) * ckstride;
            const int tm = t1 % K;
            for (int i = lane; i < KC; i += 64) {
                const int sl = i / C, col = i % C;
                ring[(r + G::template slot_dist<true>(sl, tm, K)) * RS + col] = ck[i];
            }
            if (lane < C) yv[lane] = ck[KC + lane];
            Yb = p.ckYB[(size_t)b * (N + 1) + ci];
        }
        lds_wave_fence();
        double dx[NK + MB - 1];  // sum_t coef_t(c) v_{t+k}(c), k = g*NK + jj + 1 (times W[k,c] at the end)
        double dn[MB - 1];       // the same for k = 1..MB-1 from inside the blocks (lanes g == 0)
        // grad_trans[c',c] = Etr[c',c] sum_t a_t(c') kappa_t p_t(c) is a dense [C x T][T x C] product:
        // accumulated on the matrix cores, four positions (one block) per instruction, in
        // 16x16 tiles.  Operand A (a_t kappa) is loaded from the stored forward rows directly in
        // the instruction's layout (lane l: label l mod 16 of the tile, position l/16 of the
        // block); operand B (p_t) is read back from the block's message-vector rows in LDS.
        double4_t accT[TRN][TRN];
#pragma unroll
        for (int jj = 0; jj < NK + MB - 1; ++jj) dx[jj] = 0.0;
#pragma unroll
        for (int jj = 0; jj < MB - 1; ++jj) dn[jj] = 0.0;
#pragma unroll
        for (int i = 0; i < TRN; ++i)
#pragma unroll
            for (int o = 0; o < TRN; ++o) accT[i][o] = double4_t{0.0, 0.0, 0.0, 0.0};
        int yrow = 0;  // row of yv that holds the newest message vector
        double R = 0.0, sR = 0.0;
        const bool bterms = p.g_proj_start || p.g_proj_end || p.bdy_post;
        const double wb = p.grad_logz ? (double)p.grad_logz[b] : 1.0;
        double kappa = exp((Y0 + alocY[t1 - 1 - t0] + Yb) * LN2 - logZ);
        {
            const int rdoff = g * NK * RS + c;
            float *gout = p.grad_emis + ((size_t)b * p.T) * C + cc;
            int t = t1;
            double aA[TRN];  // a of (position block index lane/16, label 16*tile + lane%16)
            auto load_rows = [&](double2 (&e)[MB], double2 (&aq)[MB], const int tfrom) {
#pragma unroll
                for (int i = 0; i < MB; ++i) {
                    const int tt = max(tfrom - 1 - i, t0);
                    e[i] = EIc[(size_t)tt * C];
                    aq[i] = aloc[(size_t)(tt - t0) * C + cc];
                }
                const int tt = max(tfrom - 1 - (lane >> 4), t0);
#pragma unroll
                for (int tr = 0; tr < TRN; ++tr) {
                    const int cp = tr * 16 + (lane & 15);
                    aA[tr] = cp < C ? aloc[(size_t)(tt - t0) * C + cp].x : 0.0;
                }
            };
            double2 e[MB], aq[MB];
            load_rows(e, aq, t);
            // next scaling-block boundary below (position jnx*J), its exponent step and the forward
            // scale just below it, loaded one block of J early
            auto ybelow = [&](const int j) { return (long)j * J - 1 >= (long)t0 ? alocY[j * J - 1 - t0] : 0.0; };
            int jnx = t1 / J;
            int dnx = nbdelta(jnx);
            double aynx = ybelow(jnx);
            while (t > t0) {
                int nb = min(t - t0, MB);
                nb = min(nb, ((t - 1) & Jm) + 1);
                if (__builtin_expect((t & Jm) == 0, 0)) {
                    const int ex = safe_exponent(yv_sum(yrow));
                    Yb += (double)ex;
                    G::rescale(ring, g, c, cval, dnx - ex);
                    kappa = exp((Y0 + aynx + Yb) * LN2 - logZ);
                    --jnx;
                    dnx = nbdelta(jnx);
                    aynx = ybelow(jnx);
                }
                if (__builtin_expect(r < MB, 0)) r = G::template move<true>(ring, lane, r);
                double coef[MB], ak[MB];
#pragma unroll
                for (int i = 0; i < MB; ++i) {
                    const bool on = cval && i < nb;
                    coef[i] = on ? aq[i].y * kappa : 0.0;  // q_t(c) kappa
                    ak[i] = on ? aq[i].x * kappa : 0.0;    // a_t(c) kappa
                }
                // x_i(c) = sum_k W[k,c] v_{t_i+k}(c); every product is also a duration marginal
                const double *base = ring + r * RS + rdoff;
                double acc[MB];
#pragma unroll
                for (int i = 0; i < MB; ++i) acc[i] = 0.0;
                if (WLDS) {
                    double v[NK];
#pragma unroll
                    for (int m = 0; m < NK + MB - 1; ++m) {
                        const double w = wl[m * CT];
                        if (m < NK) v[m] = base[m * RS];  // distance g*NK + m from the newest
#pragma unroll
                        for (int i = 0; i < MB; ++i) {
                            if (m - i >= 0 && m - i < NK) {
                                acc[i] = fma(w, v[m - i], acc[i]);
                                dx[m] = fma(coef[i], v[m - i], dx[m]);
                            }
                        }
                    }
                } else {
#pragma unroll
                    for (int jj = 0; jj < NK; ++jj) {
                        const double v = base[jj * RS];  // distance g*NK + jj from the newest
#pragma unroll
                        for (int i = 0; i < MB; ++i) {
                            acc[i] = fma(wx[WLDS ? 0 : jj + i], v, acc[i]);
                            dx[jj + i] = fma(coef[i], v, dx[jj + i]);
                        }
                    }
                }
#pragma unroll
                for (int i = 0; i < MB; ++i) acc[i] = group_sum<CTP>(acc[i]);
                double qn[MB];
#pragma unroll
                for (int i = 0; i < MB; ++i) {
                    if (i < nb) {
                        const int tt = t - 1 - i;
                        double x = acc[i];
                        const double cg = g == 0 ? coef[i] : 0.0;
#pragma unroll
                        for (int jn = 0; jn < i; ++jn) {
                            x = fma(wn[i - 1 - jn], qn[jn], x);
                            dn[i - 1 - jn] = fma(cg, qn[jn], dn[i - 1 - jn]);
                        }
                        const double y = x * e[i].y;  // p_t(c)
                        if (cval) yv[i * YS + c] = y;
                        lds_wave_fence();
                        double z0 = 0.0, z1 = 0.0;
#pragma unroll
                        for (int o = 0; o < HC; o += 2) {
                            const double2 vv = ys[(i * YS + o) >> 1];
                            z0 = fma(vv.x, ELDS ? et[o * CT] : Ereg[ELDS ? 0 : o], z0);
                            z1 = fma(vv.y, ELDS ? et[(o + 1) * CT] : Ereg[ELDS ? 1 : o + 1], z1);
                        }
                        double z = z0 + z1;
                        if (H == 2) z = add_across_32(z);
                        const double q = z * e[i].x;  // v_t(c) = b_t(c) E_t(c)
                        qn[i] = q;
                        --r;
                        if (writer) {
                            ring[r * RS + c] = q;
                            gout[(size_t)tt * C] = (float)R;
                        }
                        lds_wave_fence();
                        const double outv = coef[i] * x;
                        const double inv = tt >= 1 ? ak[i] * z : 0.0;
                        sR += R;
                        R += outv - inv;
                        // gradients of the boundary terms: a segment starts at tt (first token tt) / ends at tt (last token tt-1)
                        if (__builtin_expect(bterms, 0)) {
                            if (writer) {
                                if (p.g_proj_start) p.g_proj_start[((size_t)b * p.T + tt) * C + c] = (float)(wb * outv);
                                if (p.g_proj_end && tt >= 1)
                                    p.g_proj_end[((size_t)b * p.T + tt - 1) * C + c] = (float)(wb * inv);
                            }
                            if (p.bdy_post) {  // posterior of a boundary at tt: total mass of the segments that end there
                                double sb = writer ? inv : 0.0;
#pragma unroll
                                for (int off = 1; off < 64; off <<= 1) sb += __shfl_xor(sb, off);
                                if (lane == 0 && tt >= 1) p.bdy_post[(size_t)b * (p.T + 1) + tt] = (float)sb;
                            }
                        }
                        if (tt == 0 && writer) p.out0[(size_t)b * C + c] = outv;
                    } else {
                        qn[i] = 0.0;
                    }
                }
                // transition-gradient tiles of this block (rows of yv beyond nb are stale: A is 0 there)
                {
                    const bool on = (lane >> 4) < nb;
                    double bB[TRN];
#pragma unroll
                    for (int tc = 0; tc < TRN; ++tc) bB[tc] = yv[(lane >> 4) * YS + tc * 16 + (lane & 15)];
#pragma unroll
                    for (int tr = 0; tr < TRN; ++tr) {
                        const double a = on ? aA[tr] * kappa : 0.0;
#pragma unroll
                        for (int tc = 0; tc < TRN; ++tc)
                            accT[tr][tc] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, bB[tc], accT[tr][tc], 0, 0, 0);
                    }
                }
                yrow = nb - 1;
                t -= nb;
                load_rows(e, aq, t);
            }
        }
        // ---- partials of this task.  Duration sums: the strips of neighbouring lane groups
        // overlap by MB-1 durations; they are combined through LDS in a fixed order (own strip,
        // then the neighbour's overlap, then the in-block terms) and scaled by W[k,c].
        lds_wave_fence();
        double *tmp = ring;  // [KW + MB - 1][CT], row m = duration m + 1
        {
            double *tl = tmp + g * NK * CT + c;
            if (cval) {
#pragma unroll
                for (int jj = 0; jj < NK; ++jj) tl[jj * CT] = dx[jj];
            }
            if (cval && g == G::GW - 1) {
#pragma unroll
                for (int jj = NK; jj < NK + MB - 1; ++jj) tl[jj * CT] = 0.0;
            }
            lds_wave_fence();
            if (cval) {
#pragma unroll
                for (int jj = NK; jj < NK + MB - 1; ++jj) tl[jj * CT] += dx[jj];
            }
            lds_wave_fence();
            if (writer) {
#pragma unroll
                for (int jj = 0; jj < MB - 1; ++jj) tl[jj * CT] += dn[jj];
            }
            lds_wave_fence();
        }
        double *pD = p.partD + ((size_t)b * N + iv) * KC;
        for (int i = lane; i < KC; i += 64) pD[i] = p.W[i] * tmp[(i / C) * CT + i % C];
        lds_wave_fence();
        double *pT = p.partTr + ((size_t)b * N + iv) * CC;
#pragma unroll
        for (int tr = 0; tr < TRN; ++tr)
#pragma unroll
            for (int tc = 0; tc < TRN; ++tc)
#pragma unroll
                for (int v = 0; v < 4; ++v) {  // tile element (4v + lane/16, lane%16)
                    const int src = tr * 16 + 4 * v + (lane >> 4), dst = tc * 16 + (lane & 15);
                    if (src < C && dst < C) pT[(size_t)src * C + dst] = accT[tr][tc][v];
                }
        if (lane < C) {
            p.tot[((size_t)b * N + iv) * C + lane] = R;
            p.sumR[((size_t)b * N + iv) * C + lane] = sR;
        }
    }
}

// ---------------------------------------------------------------------------
// Chunk-parallel scan.  A sequential scan of one sequence occupies one compute unit
// for T dependent steps.  The recurrences are positive linear maps, and products of
// positive maps forget their starting vector (up to scale) geometrically fast, so the
// ring state at a checkpoint position can instead be obtained by a short WARM-UP: start
// W positions earlier from the state a sequence beginning there would have, and run.
// Every checkpoint interval ("chunk") is then an independent task:
//   forward task j:  warm up over (j*Delta - W, j*Delta], record the state at j*Delta
//                    (-> ckA[j]), run the chunk, record the state at its end (-> ckA2[j+1]);
//   backward task j: the mirror image from above (-> ckB[j+1], ckB2[j]).
// Nothing is taken on trust: k_spec_cmp compares, for every chunk boundary, the state
// the previous chunk actually reached with the warm-up state the next chunk started
// from, entry by entry, after removing their common scale factor.  If all boundaries of
// a (sequence, direction) agree to SPEC_TOL the warm-up states ARE the sequential
// states to that relative accuracy (perturbations of the start do not grow: the maps
// are non-expansive in the projective metric); k_spec_fix then chains the scale
// factors into the checkpoint scales and logZ.  Otherwise the flag stays 0 and the
// sequential scan kernel, which is launched afterwards and returns at once for
// accepted (sequence, direction) pairs, recomputes that pair from scratch.
// One wave per task, no barriers, same register/LDS organisation as k_interval_wave.
// ---------------------------------------------------------------------------
constexpr double SPEC_TOL = 1e-10;
constexpr int SPEC_RUN_MAX = 2;  // intervals one wave mends in a row in the repair attempt

// One scan task of the chunk-parallel scan, one wave (window and time blocking as above).
// repair: the task restarts from the state its neighbour in scan order REACHED at their common boundary (no
// warm-up: exact if the neighbour's own start was); k_spec decides which tasks do that.
template <int CT, int NKW, bool BWD, bool repair>
__device__ __forceinline__ void spec_task(const Params &p, double *lds_raw, const int b, const int j,
                                          const int warm)
{
    using G = WaveWin<CT, NKW>;
    constexpr int CTP = G::CTP, RS = G::RS, NK = G::NK, KW = G::KW, M = G::M, ROWS = G::ROWS;
    constexpr int RTOT = G::RTOT, H = G::H, HC = G::HC;
    const int lane = threadIdx.x;
    const int K = p.K, C = p.C, KC = K * C;
    double *ring = lds_raw;          // [ROWS][RS] (+ pad)
    double *yv = ring + RTOT;        // [CTP]
    const int Delta = p.Delta, N = p.N;
    const size_t ckstride = (size_t)KC + C;
    const int c = lane % CTP, g = lane / CTP;
    const int hh = H == 2 ? (lane >> 5) : 0;
    const bool cval = c < C;
    const int cc = cval ? c : 0;
    const SeqHdr h = p.hdr[b];
    const int L = h.L, J = h.J, Jm = J - 1;
    const int lo = j * Delta;
    if (lo >= L) return;
    const int hi = min(lo + Delta, L);
    const size_t row0 = (size_t)b * (p.T + 1);
    const double2 *EIc = p.EI + row0 * C + cc;
    const int *nbc = p.nbase + row0 * C + cc;

    double wx[NK + MB - 1];  // W[g*NK + jj + 1, c]
#pragma unroll
    for (int jj = 0; jj < NK + MB - 1; ++jj) {
        const int k = g * NK + jj + 1;
        wx[jj] = (cval && k <= K) ? p.W[(size_t)(k - 1) * C + c] : 0.0;
    }
    double wn[MB - 1];       // W[1..MB-1, c]: durations inside a block
#pragma unroll
    for (int jj = 0; jj < MB - 1; ++jj) wn[jj] = (cval && jj + 1 <= K) ? p.W[(size_t)jj * C + c] : 0.0;
    double Ereg[HC];
#pragma unroll
    for (int i = 0; i < HC; ++i) {
        const int o = hh * HC + i;
        const bool ok = cval && o < C;
        Ereg[i] = ok ? (BWD ? p.Etr[(size_t)c * C + o] : p.Etr[(size_t)o * C + c]) : 0.0;
    }
    const double2 *ys = (const double2 *)__builtin_assume_aligned(yv + hh * HC, 16);

    // ---- start: the state of a sequence that begins (forward) / ends (backward) at s0
    const int s0 = repair ? (BWD ? hi : lo) : (BWD ? min(hi + warm, L) : max(lo - warm, 0));
    for (int i = lane; i < RTOT; i += 64) ring[i] = 0.0;
    if (lane < CTP) yv[lane] = 0.0;
    lds_wave_fence();
    int r = BWD ? M : KW - 1;  // row of the newest message
    double Y = 0.0;
    if (repair) {
        // the reached state at the boundary: K-deep window in slot order, message vector, scale
        const int bs = BWD ? j + 1 : j;
        const double *src = (BWD ? p.ckB2 : p.ckA2) + ((size_t)b * (N + 1) + bs) * ((size_t)KC + C);
        const int tm = s0 % K;
        for (int i = lane; i < KC; i += 64) {
            const int sl = i / C, col = i % C;
            const int d = G::template slot_dist<BWD>(sl, tm, K);
            ring[(BWD ? r + d : r - d) * RS + col] = src[i];
        }
        if (lane < C) yv[lane] = src[KC + lane];
        Y = ((BWD ? p.ckYB2 : p.ckYA2) + (size_t)b * (N + 1))[bs];
    } else {
        double q;
        if (!BWD) {
            double z = 0.0;
#pragma unroll
            for (int i = 0; i < HC; ++i) z += Ereg[i];
            if (H == 2) z = add_across_32(z);
            q = z * EIc[(size_t)s0 * C].y;
            if (lane < C) yv[lane] = 1.0;
        } else {
            q = EIc[(size_t)s0 * C].x;
            if (lane == 0) yv[0] = 1.0;
        }
        if (cval && g == 0) ring[r * RS + c] = q;
    }
    lds_wave_fence();
    // checkpoint layout: message of position t' at slot t' mod K
    auto record = [&](const int t, double *ck, double *ckY) {
        const int tm = t % K;
        for (int i = lane; i < KC; i += 64) {
            const int sl = i / C, col = i % C;
            const int d = G::template slot_dist<BWD>(sl, tm, K);
            ck[i] = ring[(BWD ? r + d : r - d) * RS + col];
        }
        if (lane < C) ck[KC + lane] = yv[lane];
        if (lane == 0) *ckY = Y;
    };
    double *ck1 = (BWD ? p.ckB : p.ckA) + ((size_t)b * (N + 1)) * ckstride;
    double *ck2 = (BWD ? p.ckB2 : p.ckA2) + ((size_t)b * (N + 1)) * ckstride;
    double *ckY1 = (BWD ? p.ckYB : p.ckYA) + (size_t)b * (N + 1);
    double *ckY2 = (BWD ? p.ckYB2 : p.ckYA2) + (size_t)b * (N + 1);
    const int tstart = BWD ? hi : lo;   // where the chunk proper begins (state -> ck1)
    const int tend = BWD ? lo : hi;
    const int istart = BWD ? j + 1 : j, iend = BWD ? j : j + 1;
    // Forward tasks also leave the rows the interval stage needs, (a_t, q_t) and the scale relative
    // to the chunk's first position, for t = lo .. hi-1, in the task's own slot (the interval
    // stage then skips its forward recompute for accepted sequences).
    // Backward tasks do the same with (p_t, v_t) and the scale relative to the chunk's upper end,
    // for t = hi-1 .. lo, when the marginals are formed from the stored rows of both scans.
    const bool keep = BWD ? p.marg != 0 : p.fuse != 0;
    const bool writer = cval && g == 0;
    double2 *aloc = (double2 *)(BWD ? p.bloc : p.aloc) + ((size_t)b * N + j) * Delta * C;
    double *alocY = (BWD ? p.blocY : p.alocY) + ((size_t)b * N + j) * Delta;
    double Yrec = 0.0;  // scale at the chunk's first position (forward) / upper end (backward)
    auto start_rows = [&]() {
        Yrec = Y;
        if (BWD) return;
        if (keep && writer) aloc[c] = make_double2(yv[c], ring[r * RS + c]);
        if (keep && lane == 0) alocY[0] = 0.0;
    };
    if (s0 == tstart && !(BWD && tstart == L)) {
        record(s0, ck1 + (size_t)istart * ckstride, ckY1 + istart);
        start_rows();
    }

    // this lane's lowest window address relative to the newest row
    const int rdoff = BWD ? g * NK * RS + c : -(g * NK + NK - 1) * RS + c;
    int t = s0;
    auto load_rows = [&](double2 (&e)[MB], const int tfrom) {  // rows of the MB positions after tfrom
#pragma unroll
        for (int i = 0; i < MB; ++i) {
            const int tt = BWD ? max(tfrom - 1 - i, tend) : min(tfrom + 1 + i, tend);
            e[i] = EIc[(size_t)tt * C];
        }
    };
    auto block_len = [&](const int tcur) {  // positions the block starting after tcur may take
        int nb = BWD ? tcur - tend : tend - tcur;
        nb = min(nb, MB);
        // only the first position of a block may cross a scaling-block boundary
        nb = min(nb, BWD ? ((tcur - 1) & Jm) + 1 : J - ((tcur + 1) & Jm));
        // the position where the chunk proper starts ends its block (its state is recorded)
        if (BWD ? tcur > tstart : tcur < tstart) nb = min(nb, BWD ? tcur - tstart : tstart - tcur);
        return nb;
    };
    double2 e[MB];
    load_rows(e, t);
    // exponent step n_j(c) - n_{j-1}(c) of the lane's label at the scaling-block boundary j*J; the
    // one of the next boundary in the scan's direction is loaded one block of J early
    auto nbdelta = [&](const int jb) {
        return (jb >= 1 && (long)jb * J <= (long)L) ? nbc[(size_t)jb * C] - nbc[(size_t)(jb - 1) * C] : 0;
    };
    int jnx = BWD ? s0 / J : s0 / J + 1;
    int dnx = nbdelta(jnx);
    while (t != tend) {
        const int nb = block_len(t);
        const int tn = BWD ? t - nb : t + nb;
        // the next block's rows, requested before this block's stores: loads and stores retire in
        // order, so a load issued after a store could not be waited for without the store
        double2 en[MB];
        load_rows(en, tn);
        const int t1 = BWD ? t - 1 : t + 1;
        const bool inchunk = keep && (BWD ? t <= tstart : t >= tstart);  // blocks end at tstart: holds for the whole block
        const bool boundary = BWD ? (t & Jm) == 0 : (t1 & Jm) == 0;
        if (__builtin_expect(boundary, 0)) {
            double prevsum = 0.0;
            for (int i = 0; i < CT; ++i) prevsum += yv[i];
            const int ex = safe_exponent(prevsum);
            Y += (double)ex;
            G::rescale(ring, g, c, cval, dnx - ex);
            jnx += BWD ? -1 : 1;
            dnx = nbdelta(jnx);
        }
        if (__builtin_expect(BWD ? r < MB : r + MB > ROWS - 1, 0)) r = G::template move<BWD>(ring, lane, r);
        // ---- what the window contributes to the MB positions of the block
        const double *base = ring + r * RS + rdoff;
        double acc[MB];
#pragma unroll
        for (int i = 0; i < MB; ++i) acc[i] = 0.0;
#pragma unroll
        for (int jj = 0; jj < NK; ++jj) {
            const double v = base[(BWD ? jj : NK - 1 - jj) * RS];  // distance g*NK + jj from the newest
#pragma unroll
            for (int i = 0; i < MB; ++i) acc[i] = fma(wx[jj + i], v, acc[i]);
        }
#pragma unroll
        for (int i = 0; i < MB; ++i) acc[i] = group_sum<CTP>(acc[i]);
        // ---- the positions one after the other
        double qn[MB];
#pragma unroll
        for (int i = 0; i < MB; ++i) {
            if (i < nb) {
                double x = acc[i];
#pragma unroll
                for (int jn = 0; jn < i; ++jn) x = fma(wn[i - 1 - jn], qn[jn], x);
                const double y = x * (BWD ? e[i].y : e[i].x);
                if (cval) yv[c] = y;
                lds_wave_fence();
                double z0 = 0.0, z1 = 0.0;
#pragma unroll
                for (int o = 0; o < HC; o += 2) {
                    const double2 vv = ys[o >> 1];
                    z0 = fma(vv.x, Ereg[o], z0);
                    z1 = fma(vv.y, Ereg[o + 1], z1);
                }
                double z = z0 + z1;
                if (H == 2) z = add_across_32(z);
                const double q = z * (BWD ? e[i].x : e[i].y);
                qn[i] = q;
                r += BWD ? -1 : 1;
                if (writer) ring[r * RS + c] = q;
                if (!BWD && inchunk && t + 1 + i < hi) {
                    if (writer) aloc[(size_t)(t + 1 + i - lo) * C + c] = make_double2(y, q);
                    if (lane == 0) alocY[t + 1 + i - lo] = Y - Yrec;
                }
                if (BWD && inchunk) {  // position t - 1 - i of [lo, hi)
                    if (writer) aloc[(size_t)(t - 1 - i - lo) * C + c] = make_double2(y, q);
                    if (lane == 0) alocY[t - 1 - i - lo] = Y - Yrec;
                }
                lds_wave_fence();
            } else {
                qn[i] = 0.0;
            }
        }
        t = tn;
#pragma unroll
        for (int i = 0; i < MB; ++i) e[i] = en[i];
        if (__builtin_expect(t == tstart, 0)) {
            record(t, ck1 + (size_t)istart * ckstride, ckY1 + istart);
            start_rows();
        }
    }
    record(tend, ck2 + (size_t)iend * ckstride, ckY2 + iend);
}

// rest: only the sequences the lock-step kernel (k_mscan, launched before) leaves out
template <int CT, int NKW>
__global__ __launch_bounds__(64) void k_spec(Params p, int both, int warm, int tier, int rest)
{
    extern __shared__ double lds_raw[];
    const int ndir = both ? 2 : 1;
    const int dir = blockIdx.x % ndir;
    const int task = blockIdx.x / ndir;
    const int b = task / p.N, j = task % p.N;
    if (tier > 0 && p.spec_ok[b * 2 + dir]) return;  // accepted by an earlier attempt
    if (rest && p.hdr[b].J >= MS_JMIN) return;
    if (dir == 0) spec_task<CT, NKW, false, false>(p, lds_raw, b, j, warm);
    else spec_task<CT, NKW, true, false>(p, lds_raw, b, j, warm);
}

// The repair attempt of the chunk-parallel scans, for the (sequence, direction) pairs that are still open.
template <int CT, int NKW>
__global__ __launch_bounds__(64) void k_spec_repair(Params p, int both)
{
    extern __shared__ double lds_raw[];
    const int ndir = both ? 2 : 1;
    const int dir = blockIdx.x % ndir;
    const int task = blockIdx.x / ndir;
    const int b = task / p.N, j = task % p.N;
    if (p.spec_ok[b * 2 + dir]) return;
    // A run of adjacent boundaries that disagreed is taken by ONE wave, the task that starts at the first of them
    // in scan order (its neighbour started from a verified or exact state, so what that neighbour reached is
    // right): it restarts from the reached state and goes on through the run's intervals one after the other,
    // at most SPEC_RUN_MAX of them; a longer run stays open for the next attempt.  Every other task returns at
    // once and keeps what it has.  Nothing in this kernel writes spec_err.
    const int L = p.hdr[b].L;
    const int nint = (L + p.Delta - 1) / p.Delta;
    const double *err = p.spec_err + ((size_t)b * 2 + dir) * (p.N + 1);
    // Mending is sequential work, one wave per run: it pays for a few isolated disagreements (a stretch of
    // uninformative input), not for a model that forgets slowly everywhere; that goes to the long warm-up.
    if (p.spec_lr[((size_t)b * 2 + dir) * (p.N + 1)] > (double)max(2, nint / 16)) return;
    auto bad = [&](const int m) { return m >= 1 && m <= nint - 1 && !(err[m] <= SPEC_TOL); };
    if (!bad(dir ? j + 1 : j) || bad(dir ? j + 2 : j - 1)) return;
    int jj = j;
    for (int n = 0; n < SPEC_RUN_MAX; ++n) {
        if (dir == 0) spec_task<CT, NKW, false, true>(p, lds_raw, b, jj, 0);
        else spec_task<CT, NKW, true, true>(p, lds_raw, b, jj, 0);
        const int nx = dir ? jj - 1 : jj + 1;              // the next task in scan order ...
        if (nx < 0 || nx >= nint || !bad(dir ? nx + 1 : nx)) break;  // ... starts where this one ended
        __threadfence();  // the reached state this wave has just written is what it restarts from
        jj = nx;
    }
}

// One workgroup per (chunk boundary j, sequence, direction): compare the state chunk j-1
// (forward) / chunk j (backward) reached at position j*Delta with the warm-up state the
// neighbouring chunk started from.
__global__ __launch_bounds__(NT) void k_spec_cmp(Params p, int tier)
{
    __shared__ double part[NT / 64];
    const int j = blockIdx.x, b = blockIdx.y, dir = blockIdx.z, tid = threadIdx.x;
    const int lane = tid & 63, wv = tid >> 6;
    if (tier > 0 && p.spec_ok[b * 2 + dir]) return;
    const int L = p.hdr[b].L;
    const int nint = (L + p.Delta - 1) / p.Delta;
    if (j < 1 || j >= nint) return;
    const int KC = p.K * p.C, C = p.C, N = p.N;
    const size_t ckstride = (size_t)KC + C;
    const double *A = (dir ? p.ckB : p.ckA) + ((size_t)b * (N + 1) + j) * ckstride;    // warm-up state
    const double *A2 = (dir ? p.ckB2 : p.ckA2) + ((size_t)b * (N + 1) + j) * ckstride;  // reached state
    const double Y = (dir ? p.ckYB : p.ckYA)[(size_t)b * (N + 1) + j];
    const double Y2 = (dir ? p.ckYB2 : p.ckYA2)[(size_t)b * (N + 1) + j];
    // sums of the two message vectors (their ratio is the common scale factor); C <= 64 here:
    // every wave forms them, in lane order
    double s1 = lane < C ? A[KC + lane] : 0.0, s2 = lane < C ? A2[KC + lane] : 0.0;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        s1 += __shfl_xor(s1, off);
        s2 += __shfl_xor(s2, off);
    }
    const double f = s2 / s1;  // reached = f * 2^(Y2-Y) * warm-up, entry by entry, if they agree
    double err = 0.0;
    if (!(s1 > 0.0) || !(s2 > 0.0) || !(f > 0.0) || !(f < DBL_MAX)) err = DBL_MAX;
#pragma unroll 8
    for (int i = tid; i < KC + C; i += NT) {
        const double x = A2[i], y = A[i] * f;
        const double m = fmax(fabs(x), fabs(y));
        if (m > 1e-290) err = fmax(err, fabs(x - y) / m);
        if (!(m < DBL_MAX)) err = DBL_MAX;
    }
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) err = fmax(err, __shfl_xor(err, off));
    if (lane == 0) part[wv] = err;
    __syncthreads();
    if (tid == 0) {
        for (int i = 1; i < NT / 64; ++i) err = fmax(err, part[i]);
        const size_t o = ((size_t)b * 2 + dir) * (N + 1) + j;
        p.spec_err[o] = err;
        p.spec_lr[o] = (Y2 - Y) + log2(f);
    }
}

// Accept or reject each (sequence, direction); chain the scale factors.  grid (B, 2), one
// wave: lane l owns a contiguous run of boundaries in scan order, the running log2 factor
// is a fixed-order prefix sum (per lane, then across lanes).
__global__ __launch_bounds__(64) void k_spec_fix(Params p, int ndir, int tier, int code)
{
    const int b = blockIdx.x, dir = blockIdx.y, lane = threadIdx.x;
    if (tier > 0 && p.spec_ok[b * 2 + dir]) return;
    const int L = p.hdr[b].L, N = p.N, C = p.C, KC = p.K * C;
    const int nint = (L + p.Delta - 1) / p.Delta;
    const size_t so = ((size_t)b * 2 + dir) * (N + 1);
    if (dir >= ndir) {  // direction not run in this call
        if (lane == 0) {
            p.spec_ok[b * 2 + dir] = 0;
            p.spec_err[so] = -1.0;
        }
        return;
    }
    const int nb = nint > 1 ? nint - 1 : 0;  // boundaries 1 .. nint-1
    const int per = (nb + 63) / 64;
    const int i0 = min(lane * per, nb), i1 = min(i0 + per, nb);
    // i-th boundary in scan order: ascending for the forward scan, descending for the backward one
    auto jof = [&](int i) { return dir == 0 ? 1 + i : nint - 1 - i; };
    double s = 0.0, worst = 0.0;
    int nbad = 0;  // boundaries that disagreed
    for (int i = i0; i < i1; ++i) {
        s += p.spec_lr[so + jof(i)];
        const double e = p.spec_err[so + jof(i)];
        worst = fmax(worst, e);
        nbad += !(e <= SPEC_TOL);
    }
    double inc = s;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const double v = __shfl_up(inc, off);
        if (lane >= off) inc += v;
    }
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        worst = fmax(worst, __shfl_xor(worst, off));
        nbad += __shfl_xor(nbad, off);
    }
    const double total = __shfl(inc, 63);
    // accepted or not (the same in every lane): every boundary within the bound, and a finite logZ
    bool ok = worst <= SPEC_TOL;
    double lz = 0.0, sumL = 1.0, vL = 0.0;
    if (dir == 0) {
        if (nint == 0) {
            lz = log((double)C);
        } else {
            // a_L(c) / Z: mass of the segments that end at L with label c
            const double *e = p.ckA2 + ((size_t)b * (N + 1) + nint) * ((size_t)KC + C);
            vL = lane < C ? e[KC + lane] : 0.0;
            sumL = vL;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) sumL += __shfl_xor(sumL, off);
            lz = (p.ckYA2[(size_t)b * (N + 1) + nint] + total) * LN2 + log(sumL);
            ok = ok && sumL > 0.0 && lz == lz;
        }
    }
    if (ok) {
        // Chain the scale factors into the checkpoint scales.  Only on acceptance: a later attempt that rewrites
        // some of the checkpoints must find the others as their tasks left them.
        double *ckY = (dir ? p.ckYB : p.ckYA) + (size_t)b * (N + 1);
        double acc = inc - s;  // log2 of the factor between the true state and the warm-up state
        for (int i = i0; i < i1; ++i) {
            acc += p.spec_lr[so + jof(i)];
            ckY[jof(i)] += acc;
        }
        if (dir == 0 && nint > 0 && lane < C) p.inL[(size_t)b * C + lane] = vL / sumL;
    }
    if (lane != 0) return;
    p.spec_err[so] = worst;  // entry 0 is no boundary: it carries the report value,
    p.spec_lr[so] = (double)nbad;  // and this one the number of boundaries that disagreed (read by the repair attempt)
    if (dir == 0 && ok) {
        p.hdr[b].logZ = lz;
        p.logz[b] = (float)lz;
    }
    p.spec_ok[b * 2 + dir] = ok ? code : 0;  // which attempt verified it (1 first, 2 after repairs, 3 long warm-up)
}

// The chunk-parallel scan was not attempted: say so in the report fields.
__global__ void k_spec_clear(Params p)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= 2 * p.B) return;
    p.spec_ok[i] = 0;
    p.spec_err[(size_t)i * (p.N + 1)] = -1.0;
}

__global__ void k_spec_report(Params p, int32_t *accepted, double *mismatch)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= 2 * p.B) return;
    if (accepted) accepted[i] = p.spec_ok[i];
    if (mismatch) mismatch[i] = p.spec_err[(size_t)i * (p.N + 1)];
}

__global__ void k_seq_report(Params p, int32_t *range_exceeded, double *logz64)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= p.B) return;
    const SeqHdr h = p.hdr[b];
    if (range_exceeded) range_exceeded[b] = h.flags & 1;
    if (logz64) logz64[b] = h.logZ;
}

// The report fields sit in front of everything that differs between the gradient plans: the smallest plan of the
// caller's kind (forward only or gradients, default or low memory) locates them.
inline int report_plan_kind(int want_grad)
{
    if (want_grad < 0) return -1;
    return (want_grad & PLAN_LOW_MEMORY) | ((want_grad & 7) ? 2 : 0);
}

// ---------------------------------------------------------------------------
// Viterbi decode (max semiring) with the window / time-block organisation of the one-wave
// kernels, in the log domain (fp64 additions and maxima only; nothing needs rescaling):
//     r_s(c) = max_c' (V_s(c') + trans[c',c]) + (start score of token s) - S[s,c]        (leaves s)
//     V_t(c) = S[t,c] + (end score of token t-1) + max_k (dur[k,c] + r_{t-k}(c))          (arrives at t)
// V_0 = 0 for every label.  One wave per sequence walks the positions in order and stores
// (V_t, r_t) for every position and label; no back-pointers are kept.  The trace-back
// (k_vit_trace) finds each segment's duration and predecessor label by recomputing the
// candidates from the stored values: the same additions as in the scan, so the maxima are
// bit-identical.  Ties go to the smallest duration, then the smallest label.
// ---------------------------------------------------------------------------
__device__ __forceinline__ double max_across_32(double v)
{
    const unsigned lo = (unsigned)__double2loint(v), hi = (unsigned)__double2hiint(v);
    const auto a = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
    const auto b = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
    return fmax(__hiloint2double((int)b[0], (int)a[0]), __hiloint2double((int)b[1], (int)a[1]));
}

__device__ __forceinline__ double max_across_16(double v)
{
    const unsigned lo = (unsigned)__double2loint(v), hi = (unsigned)__double2hiint(v);
    const auto a = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
    const auto b = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
    return fmax(__hiloint2double((int)b[0], (int)a[0]), __hiloint2double((int)b[1], (int)a[1]));
}

__device__ __forceinline__ double max_across_8(double v)
{
    const int lo = __double2loint(v), hi = __double2hiint(v);
    const int lo2 = __builtin_amdgcn_update_dpp(0, lo, 0x128, 0xf, 0xf, false);
    const int hi2 = __builtin_amdgcn_update_dpp(0, hi, 0x128, 0xf, 0xf, false);
    return fmax(v, __hiloint2double(hi2, lo2));
}

// max over the 64/CTP lanes of a wave that share lane % CTP; every lane gets the result
template <int CTP>
__device__ __forceinline__ double group_max(double v)
{
    if (CTP <= 8) v = max_across_8(v);
    if (CTP <= 16) v = max_across_16(v);
    if (CTP <= 32) v = max_across_32(v);
    return v;
}

// One scan task: the whole sequence (chunk < 0: the sequential scan) or one checkpoint interval
// (lo, hi] after a warm-up over the `warm` positions before it, started as a sequence that
// begins there.  A chunk task records its window and V vector at lo (-> ckA[chunk]) and at hi
// (-> ckA2[chunk+1]) for the verification, and stores (V_t, r_t) for lo < t <= hi (and for
// position 0 if lo = 0) in ITS OWN additive unit: max-plus recurrences are invariant under adding
// a constant to every message, and a warmed-up chunk differs from the true values by exactly such
// a constant once all best paths through the warm-up have merged.
template <int CT, int NKW>
__device__ __forceinline__ void vit_task(const Params &p, double *lds_raw, const int b, const int chunk,
                                         const int warm)
{
    using G = WaveWin<CT, NKW>;
    constexpr int CTP = G::CTP, RS = G::RS, NK = G::NK, KW = G::KW, ROWS = G::ROWS;
    constexpr int RTOT = G::RTOT, H = G::H, HC = G::HC;
    const int lane = threadIdx.x;
    const int K = p.K, C = p.C, KC = K * C;
    double *ring = lds_raw;          // [ROWS][RS] (+ pad): r of the last KW positions
    double *yv = ring + RTOT;        // [CTP]: V of the current position
    const int c = lane % CTP, g = lane / CTP;
    const int hh = H == 2 ? (lane >> 5) : 0;
    const bool cval = c < C;
    const int cc = cval ? c : 0;
    const bool writer = cval && g == 0;
    const int L = p.hdr[b].L;
    const bool whole = chunk < 0;
    const int lo = whole ? 0 : chunk * p.Delta;
    if (!whole && lo >= L && !(lo == 0 && L == 0)) return;
    const int hi = whole ? L : min(lo + p.Delta, L);
    const int s0 = whole ? 0 : max(lo - warm, 0);
    const size_t row0 = (size_t)b * (p.T + 1);
    const double2 *LPc = p.EI + row0 * C + cc;  // (S + end score, start score - S)
    double2 *VR = p.vr + row0 * C;
    const double NINF = -INFINITY;

    double wd[NK + MB - 1];  // dur[g*NK + jj, c] (duration g*NK + jj + 1)
#pragma unroll
    for (int jj = 0; jj < NK + MB - 1; ++jj) {
        const int k = g * NK + jj + 1;
        wd[jj] = (cval && k <= K) ? (double)p.dur[(size_t)(k - 1) * C + c] : NINF;
    }
    double wn[MB - 1];
#pragma unroll
    for (int jj = 0; jj < MB - 1; ++jj) wn[jj] = (cval && jj + 1 <= K) ? (double)p.dur[(size_t)jj * C + c] : NINF;
    double Treg[HC];         // trans[o, c] for the lane's half of the source labels
#pragma unroll
    for (int i = 0; i < HC; ++i) {
        const int o = hh * HC + i;
        Treg[i] = (cval && o < C) ? (double)p.trans[(size_t)o * C + c] : NINF;
    }
    const double2 *ys = (const double2 *)__builtin_assume_aligned(yv + hh * HC, 16);

    for (int i = lane; i < RTOT; i += 64) ring[i] = NINF;
    if (lane < CTP) yv[lane] = lane < C ? 0.0 : NINF;  // V = 0 for every label where the (sub)sequence begins
    lds_wave_fence();
    int r = KW - 1;
    auto leave = [&]() {  // max_o (V(o) + trans[o,c]) from the V vector in yv
        double m0 = NINF, m1 = NINF;
#pragma unroll
        for (int o = 0; o < HC; o += 2) {
            const double2 vv = ys[o >> 1];
            m0 = fmax(m0, vv.x + Treg[o]);
            m1 = fmax(m1, vv.y + Treg[o + 1]);
        }
        double m = fmax(m0, m1);
        if (H == 2) m = max_across_32(m);
        return m;
    };
    // state for the verification: r of the K positions up to t (by distance), then V_t
    const size_t ckstride = (size_t)KC + C;
    auto record = [&](double *ck) {
        for (int i = lane; i < KC; i += 64) ck[i] = ring[(r - i / C) * RS + i % C];
        if (lane < C) ck[KC + lane] = yv[lane];
    };
    {
        const double q = leave() + LPc[(size_t)s0 * C].y;
        if (writer) {
            ring[r * RS + c] = q;
            if (s0 == lo) VR[(size_t)s0 * C + c] = make_double2(0.0, q);
        }
    }
    lds_wave_fence();
    if (!whole && s0 == lo) record(p.ckA + ((size_t)b * (p.N + 1) + chunk) * ckstride);
    const int rdoff = -(g * NK + NK - 1) * RS + c;
    int t = s0;
    auto load_rows = [&](double2 (&e)[MB], const int tfrom) {
#pragma unroll
        for (int i = 0; i < MB; ++i) e[i] = LPc[(size_t)min(tfrom + 1 + i, hi) * C];
    };
    double2 e[MB];
    load_rows(e, t);
    while (t < hi) {
        int nb = min(hi - t, MB);
        if (t < lo) nb = min(nb, lo - t);  // the position where the chunk proper starts ends its block
        const bool keep = t >= lo;
        double2 en[MB];
        load_rows(en, t + nb);
        if (__builtin_expect(r + MB > ROWS - 1, 0)) r = G::template move<false>(ring, lane, r);
        const double *base = ring + r * RS + rdoff;
        double acc[MB];
#pragma unroll
        for (int i = 0; i < MB; ++i) acc[i] = NINF;
#pragma unroll
        for (int jj = 0; jj < NK; ++jj) {
            const double v = base[(NK - 1 - jj) * RS];  // r of the position g*NK + jj before the newest
#pragma unroll
            for (int i = 0; i < MB; ++i) acc[i] = fmax(acc[i], wd[jj + i] + v);
        }
#pragma unroll
        for (int i = 0; i < MB; ++i) acc[i] = group_max<CTP>(acc[i]);
        double qn[MB];
#pragma unroll
        for (int i = 0; i < MB; ++i) {
            if (i < nb) {
                double x = acc[i];
#pragma unroll
                for (int jn = 0; jn < i; ++jn) x = fmax(x, wn[i - 1 - jn] + qn[jn]);
                const double y = x + e[i].x;  // V_t(c)
                if (cval) yv[c] = y;
                lds_wave_fence();
                const double q = leave() + e[i].y;
                qn[i] = q;
                ++r;
                if (writer) {
                    ring[r * RS + c] = q;
                    if (keep) VR[(size_t)(t + 1 + i) * C + c] = make_double2(y, q);
                }
                lds_wave_fence();
            } else {
                qn[i] = NINF;
            }
        }
        t += nb;
#pragma unroll
        for (int i = 0; i < MB; ++i) e[i] = en[i];
        if (!whole && t == lo) record(p.ckA + ((size_t)b * (p.N + 1) + chunk) * ckstride);
    }
    if (!whole) {
        record(p.ckA2 + ((size_t)b * (p.N + 1) + chunk + 1) * ckstride);
        return;
    }
    // best final label (smallest on ties) and score
    double best = cval ? yv[c] : NINF;
    int bl = cval ? c : 0x7fffffff;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const double ov = __shfl_xor(best, off);
        const int ol = __shfl_xor(bl, off);
        if (ov > best || (ov == best && ol < bl)) {
            best = ov;
            bl = ol;
        }
    }
    if (lane == 0) {
        p.vscore[b] = L > 0 ? (float)best : 0.f;
        p.vbest[b] = bl;
    }
}

// The sequential scan: one wave per sequence (skips sequences whose chunk-parallel scan was accepted).
template <int CT, int NKW>
__global__ __launch_bounds__(64) void k_viterbi(Params p)
{
    extern __shared__ double lds_raw[];
    if (p.spec && p.spec_ok[blockIdx.x * 2]) return;
    vit_task<CT, NKW>(p, lds_raw, blockIdx.x, -1, 0);
}

// Largest disagreement at a chunk boundary that is accepted, relative to the larger of the entry
// and the prefix sums at the boundary.
constexpr double VIT_TOL = 1e-12;

// The chunk-parallel scan: one wave per (sequence, checkpoint interval).
template <int CT, int NKW>
__global__ __launch_bounds__(64) void k_vit_spec(Params p, int warm, int tier)
{
    extern __shared__ double lds_raw[];
    const int b = blockIdx.x / p.N, chunk = blockIdx.x % p.N;
    if (tier > 0) {
        // second pass: only the chunks whose warmed-up start disagreed with what the chunk before
        // reached (chunk 0 starts exactly; by induction over the boundaries a chunk whose left
        // boundary agrees is right up to its constant, so only these can be wrong)
        if (p.spec_ok[b * 2] || chunk == 0) return;
        if (p.spec_err[((size_t)b * 2) * (p.N + 1) + chunk] <= VIT_TOL) return;
    }
    vit_task<CT, NKW>(p, lds_raw, b, chunk, warm);
}

// Per chunk boundary j (position j*Delta): the state chunk j-1 reached against the warmed-up
// state chunk j started from.  They must agree entry by entry up to ONE additive constant
// (taken from the largest V entry); -inf entries must coincide.
__global__ __launch_bounds__(64) void k_vit_cmp(Params p, int tier)
{
    const int j = blockIdx.x, b = blockIdx.y, lane = threadIdx.x;
    if (tier > 0 && p.spec_ok[b * 2]) return;
    const int L = p.hdr[b].L;
    const int nint = (L + p.Delta - 1) / p.Delta;
    if (j < 1 || j >= nint) return;
    const int KC = p.K * p.C, C = p.C, N = p.N;
    const size_t ckstride = (size_t)KC + C;
    const double *A = p.ckA + ((size_t)b * (N + 1) + j) * ckstride;    // warm-up state
    const double *A2 = p.ckA2 + ((size_t)b * (N + 1) + j) * ckstride;  // reached state
    // additive constant: at the largest reached V entry (smallest label on ties)
    double v = lane < C ? A2[KC + lane] : -INFINITY;
    int idx = lane < C ? lane : 0x7fffffff;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const double ov = __shfl_xor(v, off);
        const int oi = __shfl_xor(idx, off);
        if (ov > v || (ov == v && oi < idx)) {
            v = ov;
            idx = oi;
        }
    }
    const double delta = v - A[KC + idx];
    double err = (v > -INFINITY && delta == delta && fabs(delta) < DBL_MAX) ? 0.0 : DBL_MAX;
    // Every entry is a difference of prefix sums (r carries -S, V carries +S), so its rounding
    // error scales with |S| here, not with the entry: measure relative to the larger of the two.
    double smag = 1.0;
    if (lane < C) {
        const double2 lp = p.EI[((size_t)b * (p.T + 1) + (size_t)j * p.Delta) * C + lane];
        if (fabs(lp.x) < DBL_MAX) smag = fmax(smag, fabs(lp.x));
        if (fabs(lp.y) < DBL_MAX) smag = fmax(smag, fabs(lp.y));
    }
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) smag = fmax(smag, __shfl_xor(smag, off));
#pragma unroll 4
    for (int i = lane; i < KC + C; i += 64) {
        const double x = A2[i], y = A[i];
        if (x == -INFINITY || y == -INFINITY) {
            if (x != y) err = DBL_MAX;
        } else {
            err = fmax(err, fabs(x - (y + delta)) / fmax(smag, fmax(fabs(x), fabs(y + delta))));
        }
    }
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) err = fmax(err, __shfl_xor(err, off));
    if (lane == 0) {
        const size_t o = ((size_t)b * 2) * (N + 1) + j;
        p.spec_err[o] = err;
        p.spec_lr[o] = delta;
    }
}

// Accept or reject each sequence; chain the additive constants (ckYA[b][j] = what must be added
// to the values stored by chunk j to get the true ones); best final label and score.

__global__ __launch_bounds__(64) void k_vit_fix(Params p, int tier)
{
    const int b = blockIdx.x, lane = threadIdx.x;
    if (tier > 0 && p.spec_ok[b * 2]) return;
    const int L = p.hdr[b].L, N = p.N, C = p.C, KC = p.K * C;
    const int nint = (L + p.Delta - 1) / p.Delta;
    const size_t so = ((size_t)b * 2) * (N + 1);
    double *off = p.ckYA + (size_t)b * (N + 1);
    double worst = 0.0;
    for (int j = 1 + lane; j < nint; j += 64) worst = fmax(worst, p.spec_err[so + j]);
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) worst = fmax(worst, __shfl_xor(worst, o));
    // prefix sums of the constants in a fixed order: lane l owns boundaries 1 + l*per .. l*per + per,
    // sums them in order, the lane totals are scanned across the wave, then every lane walks its own
    double total = 0.0;
    {
        const int per = (max(nint - 1, 0) + 63) / 64;
        const int j0 = 1 + lane * per, j1 = min(j0 + per, nint);
        double mine = 0.0;
        for (int j = j0; j < j1; ++j) mine += p.spec_lr[so + j];
        double incl = mine;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const double up = __shfl_up(incl, o);
            if (lane >= o) incl += up;
        }
        double run = incl - mine;
        for (int j = j0; j < j1; ++j) {
            run += p.spec_lr[so + j];
            off[j] = run;
        }
        if (lane == 0) off[0] = 0.0;
        total = __shfl(incl, 63);
    }
    const bool ok = worst <= VIT_TOL;
    if (ok) {
        double best = -INFINITY;
        int bl = 0x7fffffff;
        if (nint > 0) {
            const double *e = p.ckA2 + ((size_t)b * (N + 1) + nint) * ((size_t)KC + C);
            if (lane < C) {
                best = e[KC + lane];
                bl = lane;
            }
        } else if (lane == 0) {
            best = 0.0;
            bl = 0;
        }
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const double ov = __shfl_xor(best, o);
            const int ol = __shfl_xor(bl, o);
            if (ov > best || (ov == best && ol < bl)) {
                best = ov;
                bl = ol;
            }
        }
        if (lane == 0) {
            p.vscore[b] = L > 0 ? (float)(best + total) : 0.f;
            p.vbest[b] = bl;
        }
    }
    if (lane == 0) {
        p.spec_ok[b * 2] = ok ? 1 : 0;
        p.spec_err[so] = worst;
    }
}

// Trace-back, in parallel.  Node (t, c) = "a segment with label c ends at position t".
// 1. k_vit_bp: for every node the duration is the smallest k that maximises
//    dur[k,c] + r_{t-k}(c), then the predecessor label the smallest c' that maximises
//    V_{t-k}(c') + trans[c',c]: the same additions as in the scan, so the maxima are the scan's,
//    bit for bit.  A tile of 32 positions per workgroup with the K + 32 rows of (V, r) it can
//    reach staged in LDS.  parent(t, c) = (t - k, c'); nodes at position 0 are their own parent.
// 2. k_vit_round, ceil(log2(T+1)) times: every marked node marks the node its current
//    pointer leads to, then every pointer is replaced by the pointer's pointer.  After round i
//    the marked nodes are the root's ancestors at distances < 2^(i+1): the best path.
// 3. k_vit_emit: every marked node writes its segment's tokens.
constexpr int VBP_TILE = 32;

__global__ __launch_bounds__(NT) void k_vit_bp(Params p)
{
    extern __shared__ double lds_raw[];
    const int b = blockIdx.y, tid = threadIdx.x;
    const int K = p.K, C = p.C, T = p.T;
    const int L = p.hdr[b].L;
    const int t0 = blockIdx.x * VBP_TILE;
    const int rows = K + VBP_TILE, sbase = t0 - K;  // LDS row i holds position sbase + i
    double *vv = lds_raw;                            // [rows][C]  V
    double *rr = lds_raw + (size_t)rows * C;         // [rows][C]  r
    const size_t nn = (size_t)(T + 1) * C;
    const double2 *VR = p.vr + (size_t)b * nn;
    // values stored by an accepted chunk-parallel scan are in their chunk's additive unit
    const bool chunked = p.spec && p.spec_ok[b * 2];
    const double *unit = p.ckYA + (size_t)b * (p.N + 1);
    for (int i = tid; i < rows * C; i += NT) {
        const int sp = sbase + i / C;
        double2 x = make_double2(-INFINITY, -INFINITY);
        if (sp >= 0 && sp <= L) {
            x = VR[(size_t)sp * C + i % C];
            if (chunked) {
                const double u = unit[sp == 0 ? 0 : (sp - 1) / p.Delta];
                x.x += u;
                x.y += u;
            }
        }
        vv[i] = x.x;
        rr[i] = x.y;
    }
    if (blockIdx.x == 0 && tid == 0) p.vnseg[b] = 0;
    __syncthreads();
    int *bp = p.vbp + (size_t)b * nn, *par = p.vpar[0] + (size_t)b * nn;
    unsigned char *mark = p.vmark + (size_t)b * nn;
    for (int j = tid; j < VBP_TILE * C; j += NT) {
        const int t = t0 + j / C, c = j % C;
        if (t > T) continue;
        const size_t n = (size_t)t * C + c;
        mark[n] = 0;
        if (t < 1 || t > L) {
            bp[n] = 0;
            par[n] = (int)n;
            continue;
        }
        const int kmax = min(K, t);
        double best = -INFINITY;
        int kb = 1;
        const double *rcol = rr + (size_t)(t - sbase) * C + c;  // r_{t-k}(c) at rcol[-k*C]
        for (int k = 1; k <= kmax; ++k) {
            const double cand = (double)p.dur[(size_t)(k - 1) * C + c] + rcol[-(k * C)];
            if (cand > best) {
                best = cand;
                kb = k;
            }
        }
        const int sp = t - kb;
        const double *vrow = vv + (size_t)(sp - sbase) * C;
        double best2 = -INFINITY;
        int cb = 0;
        for (int o = 0; o < C; ++o) {
            const double cand = vrow[o] + (double)p.trans[(size_t)o * C + c];
            if (cand > best2) {
                best2 = cand;
                cb = o;
            }
        }
        bp[n] = (kb << 8) | cb;
        par[n] = sp * C + cb;
    }
}

__global__ __launch_bounds__(NT) void k_vit_round(Params p, int src, int first)
{
    const int b = blockIdx.y;
    const size_t nn = (size_t)(p.T + 1) * p.C;
    const size_t n = (size_t)blockIdx.x * NT + threadIdx.x;
    if (n >= nn) return;
    const int *pin = p.vpar[src] + (size_t)b * nn;
    int *pout = p.vpar[src ^ 1] + (size_t)b * nn;
    unsigned char *mark = p.vmark + (size_t)b * nn;
    const int par = pin[n];
    const bool root = first && n == (size_t)p.hdr[b].L * p.C + p.vbest[b];
    if (root) mark[n] = 1;
    if (root || mark[n]) mark[par] = 1;  // a mark set earlier in this launch only arrives sooner
    pout[n] = pin[par];
}

__global__ __launch_bounds__(NT) void k_vit_emit(Params p)
{
    const int b = blockIdx.y, C = p.C, T = p.T;
    const int L = p.hdr[b].L;
    const size_t nn = (size_t)(T + 1) * C;
    const size_t n = (size_t)blockIdx.x * NT + threadIdx.x;
    if (n >= nn) return;
    const int t = (int)(n / (unsigned)C), c = (int)(n - (size_t)t * C);
    int32_t *lab = p.vlabels + (size_t)b * T, *st = p.vstarts + (size_t)b * T;
    if (c == 0 && t >= 1 && t - 1 >= L) {  // token t-1 lies beyond the sequence
        lab[t - 1] = -1;
        st[t - 1] = 0;
    }
    if (t < 1 || t > L || !p.vmark[(size_t)b * nn + n]) return;
    const int k = p.vbp[(size_t)b * nn + n] >> 8;
    for (int u = t - k; u < t; ++u) {
        lab[u] = c;
        st[u] = u == t - k ? 1 : 0;
    }
}

// nseg[b] = number of start flags (zeroed by k_vit_bp): one integer atomic per 8192 tokens, not
// one per segment, which would serialise on one address.
constexpr int VCNT_TOK = 8192;

__global__ __launch_bounds__(NT) void k_vit_count(Params p)
{
    const int b = blockIdx.y;
    const int L = p.hdr[b].L;
    const int32_t *st = p.vstarts + (size_t)b * p.T;
    const int lo = blockIdx.x * VCNT_TOK, hi = min(L, lo + VCNT_TOK);
    int cnt = 0;
    for (int u = lo + threadIdx.x; u < hi; u += NT) cnt += st[u];
#pragma unroll
    for (int off = 32; off; off >>= 1) cnt += __shfl_xor(cnt, off);
    if ((threadIdx.x & 63) == 0 && cnt) atomicAdd(&p.vnseg[b], cnt);
}

// ---------------------------------------------------------------------------
// Trace-back by checkpoint interval (used when an interval's nodes fit in LDS): pointer doubling
// over all nodes touches every node ceil(log2 T) times in HBM; here
//   k_vit_local  one workgroup per (sequence, interval): the parents of the interval's nodes
//                (positions lo < t <= hi) are loaded into LDS and jumped until every node points
//                at its EXIT node, the first node of its path at a position <= lo;
//   k_vit_hop    ceil(log2 N) + 1 launches over the window nodes only (the at most K positions
//                below each interval's upper end, where exit nodes lie): marks the path's exit
//                nodes by pointer doubling over the exit pointers, as k_vit_round does over all;
//   k_vit_walk   one workgroup per (sequence, interval): from the interval's marked entry node
//                one thread follows the parents in LDS and marks the path; all threads then
//                write the marked nodes' segments and count them.
// ---------------------------------------------------------------------------
// local parent of the interval's node i (global id n): index inside the interval, or -(id) - 1 of
// a parent at a position <= lo
__device__ __forceinline__ int vit_local_parent(const int *par, const size_t n, const int lo, const int C)
{
    const int gp = par[n];
    const int tp = gp / C;
    return tp > lo ? (tp - lo - 1) * C + (gp - tp * C) : -gp - 1;
}

__global__ __launch_bounds__(NT) void k_vit_local(Params p)
{
    extern __shared__ int lds_int[];
    const int j = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int C = p.C, L = p.hdr[b].L;
    const size_t nn = (size_t)(p.T + 1) * C;
    const int *par = p.vpar[0] + (size_t)b * nn;
    int *e0 = p.vpar[1] + (size_t)b * nn, *e1 = p.vexit + (size_t)b * nn;
    if (j == 0 && tid < C) {  // the nodes at position 0 are where every path ends
        e0[tid] = tid;
        e1[tid] = tid;
    }
    const int lo = j * p.Delta;
    if (lo >= L) return;
    const int hi = min(lo + p.Delta, L);
    const int nloc = (hi - lo) * C;
    int *lp = lds_int;
    for (int i = tid; i < nloc; i += NT) lp[i] = vit_local_parent(par, (size_t)(lo + 1) * C + i, lo, C);
    __syncthreads();
    for (;;) {  // jump until every pointer has left the interval (at most ceil(log2(hi - lo)) + 1 rounds)
        int pending = 0;
        for (int i = tid; i < nloc; i += NT) {
            const int v = lp[i];
            if (v >= 0) {
                const int w = lp[v];  // an older or a newer pointer of v: both lie on i's path
                lp[i] = w;
                pending |= w >= 0;
            }
        }
        if (!__syncthreads_or(pending)) break;
    }
    for (int i = tid; i < nloc; i += NT) {
        const int e = -lp[i] - 1;
        e0[(size_t)(lo + 1) * C + i] = e;
        e1[(size_t)(lo + 1) * C + i] = e;
    }
}

// One doubling round over the window nodes (interval j, distance d below its upper end, label c).
__global__ __launch_bounds__(NT) void k_vit_hop(Params p, int src, int first)
{
    const int b = blockIdx.y, C = p.C, K = p.K;
    const int L = p.hdr[b].L;
    const size_t nn = (size_t)(p.T + 1) * C;
    const unsigned idx = blockIdx.x * NT + threadIdx.x;
    const unsigned kc = (unsigned)K * C;
    const int j = (int)(idx / kc);
    if (j >= p.N) return;
    const int lo = j * p.Delta;
    if (lo >= L) return;
    const int hi = min(lo + p.Delta, L);
    const int r = (int)(idx - (unsigned)j * kc);
    const int t = hi - r / C;
    if (t <= lo) return;  // that position belongs to an earlier interval's window
    const size_t n = (size_t)t * C + r % C;
    const int *ein = (src ? p.vexit : p.vpar[1]) + (size_t)b * nn;
    int *eout = (src ? p.vpar[1] : p.vexit) + (size_t)b * nn;
    unsigned char *mark = p.vmark + (size_t)b * nn;
    const int e = ein[n];
    const bool root = first && n == (size_t)L * C + p.vbest[b];
    if (root) mark[n] = 1;
    if (root || mark[n]) mark[e] = 1;  // a mark set earlier in this launch only arrives sooner
    eout[n] = ein[e];
}

__global__ __launch_bounds__(NT) void k_vit_walk(Params p)
{
    extern __shared__ int lds_int[];
    __shared__ int entry, cnt;
    const int j = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int C = p.C, T = p.T, L = p.hdr[b].L;
    const size_t nn = (size_t)(T + 1) * C;
    int32_t *lab = p.vlabels + (size_t)b * T, *st = p.vstarts + (size_t)b * T;
    const int lo = j * p.Delta;
    // tokens beyond the sequence
    for (int u = max(lo, L) + tid; u < min(lo + p.Delta, T); u += NT) {
        lab[u] = -1;
        st[u] = 0;
    }
    if (lo >= L) return;
    const int hi = min(lo + p.Delta, L);
    const int nloc = (hi - lo) * C;
    const int *par = p.vpar[0] + (size_t)b * nn;
    const unsigned char *mark = p.vmark + (size_t)b * nn;
    int *lp = lds_int;
    unsigned char *lm = (unsigned char *)(lds_int + nloc);
    if (tid == 0) {
        entry = -1;
        cnt = 0;
    }
    __syncthreads();
    for (int i = tid; i < nloc; i += NT) {
        lp[i] = vit_local_parent(par, (size_t)(lo + 1) * C + i, lo, C);
        lm[i] = 0;
        if (mark[(size_t)(lo + 1) * C + i]) entry = i;  // at most one: where the best path enters the interval
    }
    __syncthreads();
    if (tid == 0) {
        for (int cur = entry; cur >= 0; cur = lp[cur]) lm[cur] = 1;
    }
    __syncthreads();
    int mine = 0;
    for (int i = tid; i < nloc; i += NT) {
        if (!lm[i]) continue;
        const int t = lo + 1 + i / C, c = i % C;
        const int k = p.vbp[(size_t)b * nn + (size_t)t * C + c] >> 8;
        for (int u = t - k; u < t; ++u) {
            lab[u] = c;
            st[u] = u == t - k ? 1 : 0;
        }
        ++mine;
    }
    if (mine) atomicAdd(&cnt, mine);
    __syncthreads();
    if (tid == 0 && cnt) atomicAdd(&p.vnseg[b], cnt);
}

// ---------------------------------------------------------------------------
// Finalisation (fixed-order reductions).
// ---------------------------------------------------------------------------
// carry[b,i,c] = sum_{i'<=i} tot[b,i',c];  mean[b,c] = (1/L) sum_u pm[b,u,c].  grid B, NT threads:
// the intervals are split into G = NT/C contiguous chunks, one per thread group; chunk sums are
// combined in chunk order, so the result does not depend on the launch shape.
__device__ __forceinline__ void fin_seq_body(const Params &p, const int b)
{
    __shared__ double gsum[NT];
    __shared__ double gtot[NT];
    const int C = p.C, N = p.N, tid = threadIdx.x;
    const int L = p.hdr[b].L;
    const int nint = (L + p.Delta - 1) / p.Delta;
    const int G = NT / C;
    const int g = tid / C, c = tid % C;
    const int per = (nint + G - 1) / G;
    const int i0 = min(g * per, nint), i1 = min(i0 + per, nint);
    const bool act = g < G;
    double loc = 0.0;
    if (act) {
#pragma unroll 8
        for (int i = i0; i < i1; ++i) loc += p.tot[((size_t)b * N + i) * C + c];
    }
    gsum[tid] = loc;
    __syncthreads();
    double run = 0.0, total = 0.0;
    if (act) {
        for (int gg = 0; gg < g; ++gg) run += gsum[gg * C + c];
#pragma unroll 8
        for (int i = i0; i < i1; ++i) {
            const size_t o = ((size_t)b * N + i) * C + c;
            run += p.tot[o];
            p.carry[o] = run;
            const int n = min(p.Delta, L - i * p.Delta);
            total += (double)n * run - p.sumR[o];
        }
    }
    gtot[tid] = total;
    __syncthreads();
    if (tid < C) {
        double t = 0.0;
        for (int gg = 0; gg < G; ++gg) t += gtot[gg * C + tid];
        p.mean[(size_t)b * C + tid] = (p.center && L > 0) ? t / (double)L : 0.0;
    }
    // boundary posterior: certain at both ends of the sequence, nothing beyond it (the interval
    // kernels wrote positions 1 .. L-1)
    if (p.bdy_post) {
        float *bd = p.bdy_post + (size_t)b * (p.T + 1);
        for (int t = tid; t <= p.T; t += NT)
            if (t == 0 || t >= L) bd[t] = (t == 0 || t == L) ? 1.f : 0.f;
    }
}

// Gradients of the scalar sequence boundaries: sums over sequences, in sequence order, of the
// mass of the segments that start at position 0 / end at position L.  One workgroup.
__device__ __forceinline__ void fin_pi_body(const Params &p)
{
    const int c = threadIdx.x;
    if (c >= p.C) return;
    double gs = 0.0, ge = 0.0;
    for (int b = 0; b < p.B; ++b) {
        if (p.hdr[b].L < 1) continue;
        const double w = p.grad_logz ? (double)p.grad_logz[b] : 1.0;
        gs = fma(w, p.out0[(size_t)b * p.C + c], gs);
        ge = fma(w, p.inL[(size_t)b * p.C + c], ge);
    }
    if (p.g_pi_start) p.g_pi_start[c] = (float)gs;
    if (p.g_pi_end) p.g_pi_end[c] = (float)ge;
}

// grad_emis / pos_marg, elementwise over (u,c) of one sequence.  grid (blocks, B).
__global__ __launch_bounds__(NT) void k_fin_emis(Params p)
{
    const int b = blockIdx.y, C = p.C;
    const int L = p.hdr[b].L;
    const double w = p.grad_logz ? (double)p.grad_logz[b] : 1.0;
    const size_t n = (size_t)p.T * C;  // elements of one sequence
    const size_t base = (size_t)b * n;
    const double *carry = p.carry + ((size_t)b * p.N) * C;
    const double *mean = p.mean + (size_t)b * C;
    auto one = [&](const size_t idx, const int u, const int c) {
        float ge = 0.f, pmv = 0.f;
        if (u < L) {
            const int i = u / p.Delta;
            const double pm = carry[(size_t)i * C + c] - (double)p.grad_emis[base + idx];
            ge = (float)(w * (pm - mean[c]));
            pmv = (float)pm;
        }
        p.grad_emis[base + idx] = ge;
        if (p.pos_marg) p.pos_marg[base + idx] = pmv;
        // boundary projections: rows beyond the sequence are zero; the last token's end score
        // belongs to the segments that end at position L
        if (p.g_proj_start && u >= L) p.g_proj_start[base + idx] = 0.f;
        if (p.g_proj_end && u >= L - 1)
            p.g_proj_end[base + idx] = u == L - 1 ? (float)(w * p.inL[(size_t)b * C + c]) : 0.f;
    };
    if (n < ((size_t)1 << 31)) {  // 32-bit index arithmetic
        const unsigned n32 = (unsigned)n, step = gridDim.x * NT;
        for (unsigned idx = blockIdx.x * NT + threadIdx.x; idx < n32; idx += step) {
            const unsigned u = idx / (unsigned)C;
            one(idx, (int)u, (int)(idx - u * (unsigned)C));
        }
    } else {
        for (size_t idx = (size_t)blockIdx.x * NT + threadIdx.x; idx < n; idx += (size_t)gridDim.x * NT)
            one(idx, (int)(idx / C), (int)(idx % C));
    }
}

// grad_trans[c',c] = Etr[c',c] * sum_b w_b sum_i partTr;  grad_dur[k,c] = sum_b w_b sum_i partD.
// One workgroup per 32 outputs; 8 thread groups take the intervals i = g, g+8, ... and their
// sums are combined in group order (fixed order for a given problem).
__device__ __forceinline__ void fin_params_body(const Params &p, const int blk)
{
    __shared__ double red[NT];
    const int C = p.C, CC = C * C, KC = p.K * C, N = p.N, tid = threadIdx.x;
    const int o = tid & 31, g = tid >> 5;
    const int idx = blk * 32 + o;
    const bool ok = idx < CC + KC;
    double acc = 0.0;
    if (ok) {
        for (int b = 0; b < p.B; ++b) {
            const int L = p.hdr[b].L;
            const int nint = (L + p.Delta - 1) / p.Delta;
            const double w = p.grad_logz ? (double)p.grad_logz[b] : 1.0;
            const size_t stride = idx < CC ? (size_t)CC : (size_t)KC;
            const double *q = idx < CC ? p.partTr + ((size_t)b * N) * CC + idx
                                       : p.partD + ((size_t)b * N) * KC + (idx - CC);
            double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
            int i = g;
            for (; i + 24 < nint; i += 32) {
                s0 += q[(size_t)i * stride];
                s1 += q[(size_t)(i + 8) * stride];
                s2 += q[(size_t)(i + 16) * stride];
                s3 += q[(size_t)(i + 24) * stride];
            }
            for (; i < nint; i += 8) s0 += q[(size_t)i * stride];
            acc = fma(w, (s0 + s1) + (s2 + s3), acc);
        }
    }
    red[tid] = acc;
    __syncthreads();
    if (ok && g == 0) {
        double t = 0.0;
        for (int gg = 0; gg < 8; ++gg) t += red[gg * 32 + o];
        if (idx < CC) p.grad_trans[idx] = (float)(t * p.Etr[idx]);
        else p.grad_dur[idx - CC] = (float)t;
    }
}

// One launch for the two independent reductions: workgroups 0..B-1 per sequence, the rest
// per 32 parameter gradients.
__global__ __launch_bounds__(NT) void k_fin_seq(Params p)
{
    const int nparam = (p.C * p.C + p.K * p.C + 31) / 32;
    if ((int)blockIdx.x < p.B) fin_seq_body(p, blockIdx.x);
    else if ((int)blockIdx.x < p.B + nparam) fin_params_body(p, blockIdx.x - p.B);
    else fin_pi_body(p);
}

// Entropies of the posteriors (the paper's boundary-entropy paragraph): per sequence,
//   h_pos = (1/L) sum_{u<L} -sum_c pm[u,c] ln pm[u,c]          (mean per-position label entropy)
//   h_bdy = -sum_{u<L} ph_u ln ph_u,  ph_u = bdy[u] / sum_{u'<L} bdy[u']   (entropy of the normalised
//           segment-start distribution; a segment starts at token u iff a boundary falls at position u)
// One workgroup per sequence; thread partial sums are combined in thread order.
__global__ __launch_bounds__(NT) void k_entropies(const float *pos_marg, const float *bdy_post,
                                                  const int32_t *lengths, int T, int C, float *h_pos,
                                                  float *h_bdy)
{
    __shared__ double red[NT];
    const int b = blockIdx.x, tid = threadIdx.x;
    int L = lengths ? lengths[b] : T;
    L = L < 0 ? 0 : (L > T ? T : L);
    auto block_sum = [&](double v) {
        red[tid] = v;
        __syncthreads();
        double s = 0.0;
        if (tid == 0)
            for (int i = 0; i < NT; ++i) s += red[i];
        __syncthreads();
        if (tid == 0) red[0] = s;
        __syncthreads();
        s = red[0];
        __syncthreads();
        return s;
    };
    if (h_pos) {
        const float *pm = pos_marg + (size_t)b * T * C;
        double acc = 0.0;
        for (size_t i = tid; i < (size_t)L * C; i += NT) {
            const double x = (double)pm[i];
            if (x > 0.0) acc -= x * log(x);
        }
        const double tot = block_sum(acc);
        if (tid == 0) h_pos[b] = L > 0 ? (float)(tot / (double)L) : 0.f;
    }
    if (h_bdy) {
        const float *bd = bdy_post + (size_t)b * (T + 1);
        double acc = 0.0;
        for (int u = tid; u < L; u += NT) acc += (double)bd[u];
        const double norm = block_sum(acc);
        acc = 0.0;
        for (int u = tid; u < L; u += NT) {
            const double x = (double)bd[u] / norm;
            if (x > 0.0) acc -= x * log(x);
        }
        const double tot = block_sum(acc);
        if (tid == 0) h_bdy[b] = L > 0 ? (float)tot : 0.f;
    }
}

// ---------------------------------------------------------------------------
// Host side: sizing, workspace carving, launches.
// ---------------------------------------------------------------------------
#include "durtrans.inl"
#include "marg.inl"

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
    hipLaunchKernelGGL(k_prep_seq, dim3(p.B), dim3(NT), 0, st, p);
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
    if (warm > 0)
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
    hipLaunchKernelGGL((k_mg_wave<CT, NKW>), dim3(p.B * p.N), dim3(64), lds, st, p);
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
    p.marg = pl.rows && p.fuse && !p.g_proj_start && !p.g_proj_end && !p.g_pi_start && !p.g_pi_end && !p.bdy_post;
    if (p.K < 128 && ((double)p.T + 1.0) * (double)p.C >= 2147483648.0)
        p.marg = 0;  // the one-wave kernel indexes a sequence's rows with 32 bits
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
    hipLaunchKernelGGL(k_fin_seq, dim3(p.B + (p.C * p.C + p.K * p.C + 31) / 32 + ((p.g_pi_start || p.g_pi_end) ? 1 : 0)),
                       dim3(NT), 0, st, p);
    {
        size_t n = (size_t)p.T * p.C;
        size_t blocks = (n + NT - 1) / NT;
        if (blocks > 16384) blocks = 16384;
        hipLaunchKernelGGL(k_fin_emis, dim3((unsigned)blocks, p.B), dim3(NT), 0, st, p);
    }
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
    hipLaunchKernelGGL(k_dt_fin, dim3(p.B + (unsigned)((kcc + NT - 1) / NT)), dim3(NT), 0, st, p);
    hipLaunchKernelGGL(k_dt_fin_dur, dim3((p.K * p.C + NT - 1) / NT), dim3(NT), 0, st, p);
    {
        size_t n = (size_t)p.T * p.C;
        size_t blocks = (n + NT - 1) / NT;
        if (blocks > 16384) blocks = 16384;
        hipLaunchKernelGGL(k_fin_emis, dim3((unsigned)blocks, p.B), dim3(NT), 0, st, p);
    }
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
    int rc = semicrf_workspace_bytes(B, T, K, C, ckpt_interval, 1, &need);
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
