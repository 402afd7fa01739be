// The sequential scans (Algorithm 1 and the beta recurrence of Algorithm 3), one workgroup per (sequence, direction).
// Included by semicrf.hip inside its anonymous namespace (after common.h); not a translation unit of its own.

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

