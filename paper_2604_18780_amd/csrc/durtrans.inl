// ---------------------------------------------------------------------------
// Duration-dependent transitions (included by semicrf.hip inside its namespace).
//
// With one transition matrix per duration, psi(t,k,c,c') = S[t,c] - S[t-k,c] + dur[k,c] +
// trans3[k,c',c] (Eq. 4 with the duration-indexed transition whose gradient the
// gradient-workspace section allocates), the transition no longer factors out of the sum
// over durations: a position costs K*C*C multiply-adds in each recurrence instead of
// K*C + C*C, against the table G[k][c'][c] = exp(dur[k,c] + trans3[k,c',c]) (K*C*C doubles,
// read from L2: it does not fit in LDS in general).  Linear domain, fp64, the same scaling
// blocks, power-of-two scales and (ES, 1/ES) pairs as the factorised kernels:
//
//   forward   a_t(c)  = ES_t(c) * X_t(c),   X_u(c) = sum_{k} IE_{u-k}(c) * sum_c' a_{u-k}(c') G[k][c'][c]
//             ("push": when a_t is known, every future position t+k receives its term; the ring
//             X holds the K partial sums of the positions t+1 .. t+K, per label, in slot u mod K)
//   backward  b_t(c') = sum_c IE_t(c) * sum_k G[k][c'][c] v_{t+k}(c),   v_t(c) = b_t(c) ES_t(c)
//             ("pull" from the ring of the last K vectors v, slot u mod K)
//   marginal  mu(t -> t+k, c', c) = a_t(c') G[k][c'][c] IE_t(c) v_{t+k}(c) / Z
//
// Both recurrences run chunk-parallel with warm-up and are verified and chained by the same
// k_spec_cmp / k_spec_fix as the factorised scans (the checkpoint format is theirs: K*C ring
// entries in slot order, then the C-vector whose sum is the scale reference); what is rejected
// is rescanned by the same kernels in whole-sequence mode.
//
// Time blocking: the table is the traffic, so positions are taken in blocks of up to DT_MB and
// every table entry is loaded once per block.  Terms between positions of the same block
// (durations < DT_MB) are added while the block's positions are finished one after the other.
// Only the first position of a block may cross a scaling-block boundary.
// The barriers inside the scans order LDS traffic only (lds_barrier): a full barrier would
// also wait for the global stores of the rows just written, a round trip per position.
// ---------------------------------------------------------------------------
constexpr int DT_MB = 4;
constexpr int DT_NB = 8;  // table loads a thread of the backward scan keeps in flight

// G[k][c'][c] = exp(dur[k,c] + trans3[k,c',c])
__global__ __launch_bounds__(NT) void k_dt_tables(Params p)
{
    const int CC = p.C * p.C;
    const size_t n = (size_t)p.K * CC;
    const size_t i = (size_t)blockIdx.x * NT + threadIdx.x;
    if (i >= n) return;
    const int k = (int)(i / CC), c = (int)(i % p.C);
    p.G3[i] = exp((double)p.dur[(size_t)k * p.C + c] + (double)p.trans3[i]);
}

// slot index into a K-row ring from an index that is off by a few rows at most
__device__ __forceinline__ int dt_wrap(int i, const int K)
{
    while (i >= K) i -= K;
    while (i < 0) i += K;
    return i;
}

// Multiply every ring entry of label c by 2^(sgn*(n_new - n_old) - e), e = exponent of the sum of
// the last message vector (in yv).  All threads of the workgroup call it; returns e.
__device__ __forceinline__ int dt_rebase(double *ring, const double *yv, int *sc, const int *nb, int KC,
                                         int C, int jnew, int jold, int sgn)
{
    lds_barrier();  // yv and the ring are complete
    double pm = 0.0;
    for (int i = 0; i < C; ++i) pm += yv[i];
    const int e = safe_exponent(pm);
    const int tid = threadIdx.x;
    if (tid < C) sc[tid] = sgn * (nb[(size_t)jnew * C + tid] - nb[(size_t)jold * C + tid]) - e;
    lds_barrier();
    for (int i = tid; i < KC; i += blockDim.x) ring[i] = fmin(ldexp(ring[i], sc[i % C]), DBL_MAX);
    lds_barrier();
    return e;
}

// ---------------------------------------------------------------------------
// Forward recurrence.  Thread (ks, c): label c, durations k = ks + 1 + kk*NKS (kk < KPTF).
// grid = B*N chunk tasks (whole = 0) or B whole sequences (whole = 1, only sequences whose
// chunk-parallel forward scan was not accepted).
// Writes a_t (dtA) and its scale relative to the interval start (dtY) for the rows it owns
// (lo < t <= hi, and t = 0), the checkpoint states at lo and hi, and in whole mode the
// absolute interval scales, logZ and a_L / Z.
// ---------------------------------------------------------------------------
template <int KPTF>
__global__ __launch_bounds__(1024) void k_dt_fwd(Params p, int warm, int tier, int whole)
{
    extern __shared__ double lds_raw[];
    const int tid = threadIdx.x;
    const int K = p.K, C = p.C, CC = C * C, KC = K * C, N = p.N, Delta = p.Delta;
    const int NKS = min(K, 1024 / C);
    const int ks = tid / C, c = tid % C;
    const bool active = ks < NKS;
    int b, chunk;
    if (whole) {
        b = blockIdx.x;
        chunk = -1;
        if (p.spec && p.spec_ok[b * 2]) return;
    } else {
        b = blockIdx.x / N;
        chunk = blockIdx.x % N;
        if (tier > 0 && p.spec_ok[b * 2]) return;
    }
    double *X = lds_raw;             // [K][C]
    double *av = X + KC;             // [DT_MB][C]
    double *yv = av + DT_MB * C;     // [C]
    int *sc = (int *)(yv + C);       // [C]
    double *Gs = yv + 2 * C;         // [DT_MB-1][C][C] table rows of the durations below DT_MB
    const int KIN = min(K, DT_MB - 1);
    const SeqHdr h = p.hdr[b];
    const int L = h.L, J = h.J;
    const int lo = whole ? 0 : chunk * Delta;
    if (!whole && lo >= L) return;
    const int hi = whole ? L : min(lo + Delta, L);
    const int s0 = whole ? 0 : max(lo - warm, 0);
    const size_t row0 = (size_t)b * (p.T + 1);
    const double2 *EI = p.EI + row0 * C;
    const int *nb = p.nbase + row0 * C;
    const size_t ckstride = (size_t)KC + C;
    double *rowA = p.dtA + row0 * C;
    double *rowY = p.dtY + row0;

    for (int i = tid; i < KC; i += blockDim.x) X[i] = 0.0;
    for (int i = tid; i < KIN * CC; i += blockDim.x) Gs[i] = p.G3[i];
    if (tid < C) yv[tid] = 1.0;
    lds_barrier();
    double Y = 0.0, Ybase = 0.0;
    auto record = [&](double *ck) {
        for (int i = tid; i < KC; i += blockDim.x) ck[i] = X[i];
        if (tid < C) ck[KC + tid] = yv[tid];
    };

    int t0 = s0;
    while (t0 <= hi) {
        int nbk = min(DT_MB, hi - t0 + 1);
        if (t0 <= lo) nbk = min(nbk, lo - t0 + 1);  // the interval's first position ends its block
        nbk = min(nbk, J - (t0 % J));               // no scaling-block boundary inside a block
        if (t0 > s0 && (t0 % J) == 0) Y += (double)dt_rebase(X, yv, sc, nb, KC, C, t0 / J, t0 / J - 1, +1);
        // emission factors of the block's positions: fetched before the dependent chain starts
        double es[DT_MB], ie[DT_MB];
#pragma unroll
        for (int i = 0; i < DT_MB; ++i) {
            es[i] = 0.0;
            ie[i] = 0.0;
            if (i < nbk) {
                if (tid < C) es[i] = EI[(size_t)(t0 + i) * C + tid].x;
                if (active) ie[i] = EI[(size_t)(t0 + i) * C + c].y;
            }
        }
        // ---- the block's positions, one after the other
#pragma unroll
        for (int i = 0; i < DT_MB; ++i) {
            if (i >= nbk) break;
            const int tt = t0 + i;
            if (tid < C) {
                const double a = tt == s0 ? 1.0 : es[i] * X[(tt % K) * C + tid];
                av[i * C + tid] = a;
                if (tt > lo || tt == 0) rowA[(size_t)tt * C + tid] = a;
            }
            if (tid == 0) {
                if (tt > lo || tt == 0) rowY[tt] = Y - Ybase;
                if (whole && (tt % Delta) == 0) p.ckYA[(size_t)b * (N + 1) + tt / Delta] = Y;
            }
            if ((whole && (tt % Delta) == 0) || tt == lo) Ybase = Y;  // uniform
            lds_barrier();
            const int kin = nbk - 1 - i;  // durations that stay inside the block
            if (kin > 0) {
                const int k = ks + 1;
                if (active && k <= kin && k <= K) {
                    const double *g = Gs + (size_t)(k - 1) * CC + c;
                    double m = 0.0;
#pragma unroll 8
                    for (int o = 0; o < C; ++o) m = fma(av[i * C + o], g[o * C], m);
                    const int slot = ((tt + k) % K) * C + c;
                    const double val = ie[i] * m;
                    X[slot] = k == K ? val : X[slot] + val;
                }
                lds_barrier();
            }
        }
        // ---- durations that leave the block: every table entry once for all its positions
        double m[KPTF][DT_MB];
#pragma unroll
        for (int kk = 0; kk < KPTF; ++kk) {
#pragma unroll
            for (int i = 0; i < DT_MB; ++i) m[kk][i] = 0.0;
        }
        if (active) {
            // source labels in chunks of four: the chunk's a values are read once (broadcast) for all
            // the thread's durations; 4 * KPTF table loads are in flight together
            unsigned gi[KPTF];
            bool kok[KPTF];
#pragma unroll
            for (int kk = 0; kk < KPTF; ++kk) {
                const int k = ks + 1 + kk * NKS;
                kok[kk] = k <= K;
                gi[kk] = (unsigned)((kok[kk] ? k - 1 : 0) * CC + c);
            }
            const double *G3 = p.G3;
            int o = 0;
            for (; o + 4 <= C; o += 4) {
                double a4[DT_MB][4], gv[KPTF][4];
#pragma unroll
                for (int kk = 0; kk < KPTF; ++kk) {
#pragma unroll
                    for (int u = 0; u < 4; ++u) gv[kk][u] = G3[gi[kk] + (unsigned)((o + u) * C)];
                }
#pragma unroll
                for (int i = 0; i < DT_MB; ++i) {
#pragma unroll
                    for (int u = 0; u < 4; ++u) a4[i][u] = av[i * C + o + u];
                }
#pragma unroll
                for (int kk = 0; kk < KPTF; ++kk) {
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
#pragma unroll
                        for (int i = 0; i < DT_MB; ++i) m[kk][i] = fma(a4[i][u], gv[kk][u], m[kk][i]);
                    }
                }
            }
            for (; o < C; ++o) {
#pragma unroll
                for (int kk = 0; kk < KPTF; ++kk) {
                    const double gv = G3[gi[kk] + (unsigned)(o * C)];
#pragma unroll
                    for (int i = 0; i < DT_MB; ++i) m[kk][i] = fma(av[i * C + o], gv, m[kk][i]);
                }
            }
        }
#pragma unroll
        for (int i = 0; i < DT_MB; ++i) {
            if (i < nbk) {  // uniform
                const int tt = t0 + i;
                if (active) {
#pragma unroll
                    for (int kk = 0; kk < KPTF; ++kk) {
                        const int k = ks + 1 + kk * NKS;
                        if (k <= K && i + k >= nbk) {
                            const int slot = ((tt + k) % K) * C + c;
                            const double val = ie[i] * m[kk][i];
                            X[slot] = k == K ? val : X[slot] + val;
                        }
                    }
                }
                lds_barrier();
            }
        }
        if (tid < C) yv[tid] = av[(nbk - 1) * C + tid];
        const int tlast = t0 + nbk - 1;
        if (!whole && tlast == lo) {
            record(p.ckA + ((size_t)b * (N + 1) + chunk) * ckstride);
            if (tid == 0) p.ckYA[(size_t)b * (N + 1) + chunk] = Y;
        }
        t0 += nbk;
    }
    if (!whole) {
        record(p.ckA2 + ((size_t)b * (N + 1) + chunk + 1) * ckstride);
        if (tid == 0) p.ckYA2[(size_t)b * (N + 1) + chunk + 1] = Y;
        return;
    }
    lds_barrier();
    if (tid == 0) {
        double s = 0.0;
        for (int i = 0; i < C; ++i) s += yv[i];
        const double lz = Y * LN2 + log(s);
        p.hdr[b].logZ = lz;
        p.logz[b] = (float)lz;
        for (int i = 0; i < C; ++i) p.inL[(size_t)b * C + i] = yv[i] / s;
    }
}

// ---------------------------------------------------------------------------
// Backward recurrence.  Thread (ks, c', c): one label pair and the KPT consecutive durations
// ks*KPT + 1 .. ks*KPT + KPT; its sum over those durations goes through a [NKS][C][C] table in
// LDS from which threads 0..C-1 form b_t (row sums) and the mass of the segments that start
// at t (column sums weighted by a_t, which the forward scan has stored).
// mode 0: grid B*N chunk tasks with warm-up (checkpoint states at both ends)
// mode 1: grid B whole sequences whose chunk-parallel backward scan was not accepted
// For the positions of its interval a task stores, in its own power-of-two scale,
//   dtV  v_t(c)                         (read by the marginal kernel)
//   dtD  out_t(c) - in_t(c), out = sum_c' a_t(c') IE_t(c) sum_k G v_{t+k}(c): segments that start at t,
//        in = a_t(c) b_t(c): segments that end at t   (times exp(scales - logZ) later)
//   dtYb the log2 scale of both relative to the interval's upper end.
// ---------------------------------------------------------------------------
template <int KPT, int MBT>
__global__ __launch_bounds__(1024) void k_dt_bwd(Params p, int warm, int tier, int mode)
{
    extern __shared__ double lds_raw[];
    const int tid = threadIdx.x;
    const int K = p.K, C = p.C, CC = C * C, KC = K * C, N = p.N, Delta = p.Delta;
    const int NKS = (K + KPT - 1) / KPT;
    const int ks = tid / CC, pair = tid % CC;
    const int c = pair % C;
    const int CP1 = C | 1, CCP = C * CP1;         // odd row stride of the pair table: rows and columns
    const int ppair = (pair / C) * CP1 + c;       // are both read without bank conflicts
    const bool active = ks < NKS;
    const int k0 = ks * KPT;  // the thread's durations are k0 + 1 .. k0 + KPT
    double *ring = lds_raw;           // [2K][C]  v_u(c) at slots u mod K and u mod K + K: K consecutive
                                      //          positions are K consecutive rows wherever they start
    double *red = ring + 2 * KC;      // [NKS][C][C|1]
    double *av = red + NKS * CCP;     // [MBT][C] a_t of the block's positions
    double *yv = av + MBT * C;        // [C]      b_t: scale reference
    int *sc = (int *)(yv + C);        // [C]
    double *Gs = yv + 2 * C;          // [MBT-1][C][C] table rows of the durations below MBT
    const int KIN = min(K, MBT - 1);
    const size_t ckstride = (size_t)KC + C;

    const int b = mode == 1 ? (int)blockIdx.x : (int)blockIdx.x / N;
    const int chunk = mode == 1 ? -1 : (int)blockIdx.x % N;
    if (mode == 0 && tier > 0 && p.spec_ok[b * 2 + 1]) return;
    if (mode == 1 && p.spec && p.spec_ok[b * 2 + 1]) return;
    const SeqHdr h = p.hdr[b];
    const int L = h.L, J = h.J;
    const int lo = mode == 1 ? 0 : chunk * Delta;
    if (mode != 1 && lo >= L) return;
    const int hi = mode == 1 ? L : min(lo + Delta, L);
    const int s1 = mode == 0 ? min(hi + warm, L) : hi;  // where this task's recurrence starts
    const size_t row0 = (size_t)b * (p.T + 1);
    const double2 *EI = p.EI + row0 * C;
    const int *nb = p.nbase + row0 * C;
    const double *rowA = p.dtA + row0 * C;
    double *rowV = p.dtV + row0 * C;
    double *rowD = p.dtD + row0 * C;
    double *rowYb = p.dtYb + row0;

    // a sequence that ends at s1 (exactly so when s1 = L): b = 1, v = ES
    for (int i = tid; i < 2 * KC; i += blockDim.x) ring[i] = 0.0;
    for (int i = tid; i < KIN * CC; i += blockDim.x) Gs[i] = p.G3[i];
    lds_barrier();
    if (tid < C) {
        yv[tid] = tid == 0 ? 1.0 : 0.0;
        const double v = EI[(size_t)s1 * C + tid].x;
        ring[(s1 % K) * C + tid] = v;
        ring[(s1 % K + K) * C + tid] = v;
        if (s1 == L) rowV[(size_t)L * C + tid] = v;
    }
    if (s1 == L && tid == 0) rowYb[L] = 0.0;
    double Yb = 0.0, Ytop = 0.0;
    lds_barrier();
    auto record = [&](double *ck) {
        for (int i = tid; i < KC; i += blockDim.x) ck[i] = ring[i];  // first copy of the ring
        if (tid < C) ck[KC + tid] = yv[tid];
    };

    int t0 = s1 - 1;
    while (t0 >= lo) {
        int nbk = min(MBT, t0 - lo + 1);
        if (t0 >= hi) nbk = min(nbk, t0 - hi + 1);         // the interval's upper end ends its block
        nbk = min(nbk, (t0 % J) + 1);                       // no scaling-block boundary inside a block
        if (mode == 1) nbk = min(nbk, (t0 % Delta) + 1);    // checkpoints are recorded at block ends
        if (((t0 + 1) % J) == 0) Yb += (double)dt_rebase(ring, yv, sc, nb, 2 * KC, C, t0 / J, t0 / J + 1, -1);
        double ie[MBT], es[MBT];
#pragma unroll
        for (int i = 0; i < MBT; ++i) {
            ie[i] = 0.0;
            es[i] = 0.0;
            if (i < nbk) {
                const int tt = t0 - i;
                if (active) ie[i] = EI[(size_t)tt * C + c].y;
                if (tid < C) {
                    es[i] = EI[(size_t)tt * C + tid].x;
                    av[i * C + tid] = rowA[(size_t)tt * C + tid];
                }
            }
        }
        // ---- durations that reach beyond the block: every table entry once for all positions
        double bs[MBT];
#pragma unroll
        for (int i = 0; i < MBT; ++i) bs[i] = 0.0;
        if (active) {
            // position t0 - i with duration k reads v of position t0 + k - i: one new ring row per
            // duration (w[0]); the rows of the later positions are the earlier durations' rows
            const double *G3 = p.G3;
            unsigned gi = (unsigned)(k0 * CC + pair);  // index of G[k0 + 1][c'][c] (the table is < 4 GB)
            const int sl = (t0 + k0 + 1) % K;          // slot of position t0 + k0 + 1
            const int nk = min(KPT, K - k0);           // this thread's durations (at least one: ks < NKS)
            const double *rp = ring + sl * C + c;      // rows sl, sl + 1, ... of the doubled ring: no wrap
            double w[MBT];
#pragma unroll
            for (int i = 1; i < MBT; ++i) w[i] = ring[dt_wrap(sl - i, K) * C + c];
            int kk = 0;
            // A duration k <= i would end inside the block, at a position not finished yet: those
            // terms are left out here and added from the fresh values below.  Only the durations
            // below MBT are affected; they are taken first, one by one.
            if (k0 == 0) {
                for (; kk < MBT - 1 && kk < nk; ++kk) {
                    const double gv = Gs[kk * CC + pair];  // the short durations' rows are in LDS
                    w[0] = *rp;
#pragma unroll
                    for (int i = 0; i < MBT; ++i) bs[i] = fma(gv, kk + 1 > i ? w[i] : 0.0, bs[i]);
#pragma unroll
                    for (int i = MBT - 1; i > 0; --i) w[i] = w[i - 1];
                    gi += CC;
                    rp += C;
                }
            }
            // the rest in batches of DT_NB table loads in flight together (no branch between them)
            for (; kk + DT_NB <= nk; kk += DT_NB) {
                double gv[DT_NB], wv[DT_NB];
#pragma unroll
                for (int u = 0; u < DT_NB; ++u) {
                    gv[u] = G3[gi + (unsigned)(u * CC)];
                    wv[u] = rp[u * C];
                }
#pragma unroll
                for (int u = 0; u < DT_NB; ++u) {
                    w[0] = wv[u];
#pragma unroll
                    for (int i = 0; i < MBT; ++i) bs[i] = fma(gv[u], w[i], bs[i]);
#pragma unroll
                    for (int i = MBT - 1; i > 0; --i) w[i] = w[i - 1];
                }
                gi += (unsigned)(DT_NB * CC);
                rp += DT_NB * C;
            }
            if (kk < nk) {  // the last, partial batch: indices clamped, surplus terms times zero (no serial loads)
                double gv[DT_NB], wv[DT_NB];
                const int left = nk - kk;
#pragma unroll
                for (int u = 0; u < DT_NB; ++u) {
                    const int uu = u < left ? u : left - 1;
                    gv[u] = G3[gi + (unsigned)(uu * CC)];
                    wv[u] = rp[uu * C];
                }
#pragma unroll
                for (int u = 0; u < DT_NB; ++u) {
                    w[0] = wv[u];
                    const double g = u < left ? gv[u] : 0.0;
#pragma unroll
                    for (int i = 0; i < MBT; ++i) bs[i] = fma(g, w[i], bs[i]);
#pragma unroll
                    for (int i = MBT - 1; i > 0; --i) w[i] = w[i - 1];
                }
            }
        }
        // ---- finish the positions one after the other
#pragma unroll
        for (int i = 0; i < MBT; ++i) {
            if (i < nbk) {  // uniform
                const int tt = t0 - i;
                if (active) {
                    // durations 1 .. i end inside the block, at positions finished just before
                    for (int k = 1; k <= i && k <= K; ++k)
                        if (k > k0 && k <= k0 + KPT)
                            bs[i] = fma(Gs[(k - 1) * CC + pair], ring[((tt + k) % K) * C + c], bs[i]);
                    red[ks * CCP + ppair] = bs[i] * ie[i];
                }
                lds_barrier();
                if (NKS > 1) {  // uniform: sum the duration groups per label pair first, in group order
                    if (tid < CC) {
                        double sq = red[ppair];
                        for (int q = 1; q < NKS; ++q) sq += red[q * CCP + ppair];
                        red[ppair] = sq;
                    }
                    lds_barrier();
                }
                if (tid < C) {
                    double bsum = 0.0, osum = 0.0;
#pragma unroll 8
                    for (int o = 0; o < C; ++o) {
                        bsum += red[tid * CP1 + o];
                        osum = fma(av[i * C + o], red[o * CP1 + tid], osum);
                    }
                    yv[tid] = bsum;
                    const double v = bsum * es[i];
                    ring[(tt % K) * C + tid] = v;
                    ring[(tt % K + K) * C + tid] = v;
                    if (tt < hi) {
                        rowV[(size_t)tt * C + tid] = v;
                        rowD[(size_t)tt * C + tid] = osum - (tt >= 1 ? av[i * C + tid] * bsum : 0.0);
                    }
                }
                if (tid == 0 && tt < hi) rowYb[tt] = Yb - Ytop;
                lds_barrier();
            }
        }
        const int tlast = t0 - nbk + 1;
        if (mode == 0 && tlast == hi && hi < L) {
            record(p.ckB + ((size_t)b * (N + 1) + hi / Delta) * ckstride);
            if (tid == 0) p.ckYB[(size_t)b * (N + 1) + hi / Delta] = Yb;
            Ytop = Yb;
        }
        if (mode == 1 && tlast > 0 && (tlast % Delta) == 0) {
            record(p.ckB + ((size_t)b * (N + 1) + tlast / Delta) * ckstride);
            if (tid == 0) p.ckYB[(size_t)b * (N + 1) + tlast / Delta] = Yb;
            Ytop = Yb;
        }
        t0 -= nbk;
    }
    if (mode == 0 && lo > 0) {
        record(p.ckB2 + ((size_t)b * (N + 1) + lo / Delta) * ckstride);
        if (tid == 0) p.ckYB2[(size_t)b * (N + 1) + lo / Delta] = Yb;
    }
    if (mode == 1 && tid == 0) {
        double s = 0.0;
        for (int i = 0; i < C; ++i) s += yv[i];
        p.hdr[b].logZb = Yb * LN2 + log(s);
    }
}

// Absolute log2 scale of the backward rows of interval j at its upper end (0 at the sequence end).
__device__ __forceinline__ double dt_ytop(const Params &p, int b, int j, int L)
{
    const int hi = min((j + 1) * p.Delta, L);
    return hi == L ? 0.0 : p.ckYB[(size_t)b * (p.N + 1) + j + 1];
}

// Running emission-gradient sums per interval, in the form k_fin_seq / k_fin_emis expect from the
// interval kernels: grad_emis[t] = sum of (out - in) over the interval's positions above t, tot and
// sumR per interval.  One wave per (sequence, interval), lane = label; rows are fetched eight
// positions at a time.
__global__ __launch_bounds__(64) void k_dt_emis(Params p)
{
    const int b = blockIdx.x / p.N, j = blockIdx.x % p.N, lane = threadIdx.x;
    const int C = p.C, Delta = p.Delta, N = p.N;
    const int L = p.hdr[b].L;
    const int lo = j * Delta;
    if (lo >= L) return;
    const int hi = min(lo + Delta, L);
    const size_t row0 = (size_t)b * (p.T + 1);
    const double *rowD = p.dtD + row0 * C;
    const double *rowY = p.dtY + row0, *rowYb = p.dtYb + row0;
    const double *ckYA = p.ckYA + (size_t)b * (N + 1);
    const double logZ = p.hdr[b].logZ;
    const double ytop = dt_ytop(p, b, j, L);
    const bool act = lane < C;
    double R = 0.0, sR = 0.0, kappa = 0.0, kY = -1.0e300;
    for (int t1 = hi; t1 > lo; t1 -= 8) {
        double d[8], y[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int tt = t1 - 1 - i;
            d[i] = 0.0;
            y[i] = 0.0;
            if (tt >= lo) {
                if (act) d[i] = rowD[(size_t)tt * C + lane];
                y[i] = ckYA[tt == 0 ? 0 : (tt - 1) / Delta] + rowY[tt] + ytop + rowYb[tt];
            }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int tt = t1 - 1 - i;
            if (tt >= lo) {
                if (y[i] != kY) {  // uniform
                    kY = y[i];
                    kappa = exp(kY * LN2 - logZ);
                }
                if (act) {
                    p.grad_emis[((size_t)b * p.T + tt) * C + lane] = (float)R;
                    sR += R;
                    R = fma(d[i], kappa, R);
                }
            }
        }
    }
    if (act) {
        p.tot[((size_t)b * p.NP + j) * C + lane] = R;
        p.sumR[((size_t)b * p.NP + j) * C + lane] = sR;
    }
}

// ---------------------------------------------------------------------------
// Marginals: sum_t w_b mu_b(t -> t+k, c', c) for every (k, c', c), from the stored rows.
//   mu = a_t(c') IE_t(c) G[k][c'][c] v_{t+k}(c) 2^(n_blk(t+k)(c) - n_blk(t)(c)) exp((YA(t) + YB(t+k)) ln2 - logZ)
// (the power of two is what the backward recurrence applies to its ring when it crosses the
// scaling blocks between t+k and t).  Thread = label pair; workgroup (x, y) = persistent over
// the (sequence, interval) tasks x, x + gridDim.x, ... for the KS durations y*KS + 1 .. y*KS + KS,
// one accumulator per duration in registers, multiplied by G once at the end.  Positions are
// taken in groups that lie in one scaling block (at most DT_TG): the group's a and IE rows and
// the v rows it can reach are staged in LDS, the latter converted to the group's frame; four
// positions share every LDS read.
// ---------------------------------------------------------------------------
constexpr int DT_TG = 32;

template <int KS>
__global__ __launch_bounds__(1024) void k_dt_acc(Params p)
{
    extern __shared__ double lds_raw[];
    const int tid = threadIdx.x;
    const int K = p.K, C = p.C, CC = C * C, N = p.N, Delta = p.Delta;
    const bool active = tid < CC;
    const int pair = active ? tid : 0;
    const int cp = pair / C, c = pair % C;
    const int kA = blockIdx.y * KS;
    constexpr int VR = DT_TG + KS + 3;   // rows of v a group can reach (+3: blocks of four positions)
    double *Arow = lds_raw;              // [DT_TG][C]  a_t(c') w_b 2^(YA(t) - YA(group))
    double *IErow = Arow + DT_TG * C;    // [DT_TG][C]
    double *Vp = IErow + DT_TG * C;      // [VR][C]
    double acc[KS];
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) acc[kk] = 0.0;

    const int ntask = p.B * N;
    for (int task = blockIdx.x; task < ntask; task += gridDim.x) {
        const int b = task / N, chunk = task % N;
        const SeqHdr h = p.hdr[b];
        const int L = h.L, J = h.J;
        const int lo = chunk * Delta;
        if (lo >= L) continue;
        const int hi = min(lo + Delta, L);
        const size_t row0 = (size_t)b * (p.T + 1);
        const double2 *EI = p.EI + row0 * C;
        const int *nb = p.nbase + row0 * C;
        const double *rowA = p.dtA + row0 * C, *rowV = p.dtV + row0 * C;
        const double *rowY = p.dtY + row0, *rowYb = p.dtYb + row0;
        const double *ckYA = p.ckYA + (size_t)b * (N + 1);
        const double logZ = h.logZ;
        const double wb = p.grad_logz ? (double)p.grad_logz[b] : 1.0;
        for (int tg0 = lo; tg0 < hi;) {
            const int tg1 = min(min(hi, (tg0 / J + 1) * J), tg0 + DT_TG);
            const int ng = tg1 - tg0, jt = tg0 / J;
            const double yA0 = ckYA[tg0 == 0 ? 0 : (tg0 - 1) / Delta] + rowY[tg0];
            __syncthreads();  // the previous group is done with the staged rows
            for (int i = tid; i < DT_TG * C; i += blockDim.x) {
                const int r = i / C, o = i % C, tt = tg0 + r;
                double a = 0.0, e = 0.0;
                if (r < ng) {
                    const double yA = ckYA[tt == 0 ? 0 : (tt - 1) / Delta] + rowY[tt];
                    a = rowA[(size_t)tt * C + o] * wb * exp2(yA - yA0);
                    e = EI[(size_t)tt * C + o].y;
                }
                Arow[i] = a;
                IErow[i] = e;
            }
            for (int i = tid; i < VR * C; i += blockDim.x) {
                const int r = i / C, o = i % C, s = tg0 + kA + 1 + r;
                double v = 0.0;
                if (s <= L && r < ng + KS) {
                    const int js = s / J;
                    const int jc = s == L ? -1 : s / Delta;  // interval whose backward task stored the row
                    const double yB = jc < 0 ? 0.0 : dt_ytop(p, b, jc, L) + rowYb[s];
                    // all exponents are combined before anything is formed, so that an empty row
                    // stays zero and nothing passes through infinity
                    const double lf = (yA0 + yB) - logZ * LOG2E;
                    const double fl = floor(lf);
                    const int sh = nb[(size_t)js * C + o] - nb[(size_t)jt * C + o];
                    const double ef = fmin(fmax(fl, -100000.0), 100000.0);
                    v = fmin(ldexp(rowV[(size_t)s * C + o] * exp2(lf - fl), sh + (int)ef), DBL_MAX);
                }
                Vp[i] = v;
            }
            __syncthreads();
            if (active) {
                for (int i0 = 0; i0 < ng; i0 += 4) {
                    double ca[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        ca[i] = i0 + i < ng ? Arow[(i0 + i) * C + cp] * IErow[(i0 + i) * C + c] : 0.0;
                    double w[KS + 3];
#pragma unroll
                    for (int q = 0; q < KS + 3; ++q) w[q] = Vp[(i0 + q) * C + c];
#pragma unroll
                    for (int kk = 0; kk < KS; ++kk) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) acc[kk] = fma(ca[i], w[kk + i], acc[kk]);
                    }
                }
            }
            tg0 = tg1;
        }
    }
    if (active) {
        double *pg = p.partG + (size_t)blockIdx.x * K * CC;
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) {
            const int k = kA + kk + 1;
            if (k <= K) pg[(size_t)(k - 1) * CC + pair] = acc[kk] * p.G3[(size_t)(k - 1) * CC + pair];
        }
    }
}

// Finalisation: FIN_FS workgroups per sequence (interval carries and means, as for the
// factorised path), the others sum the per-workgroup marginal sums in workgroup order.
__global__ __launch_bounds__(NT) void k_dt_fin(Params p)
{
    if ((int)blockIdx.x < p.B * FIN_FS) {
        fin_seq_body(p, blockIdx.x / FIN_FS, blockIdx.x % FIN_FS);
        return;
    }
    const size_t n = (size_t)p.K * p.C * p.C;
    const size_t i = (size_t)(blockIdx.x - p.B * FIN_FS) * NT + threadIdx.x;
    if (i >= n) return;
    double s = 0.0;
    for (int w = 0; w < p.dt_nwg; ++w) s += p.partG[(size_t)w * n + i];
    p.sumG[i] = s;
    p.grad_trans3[i] = (float)s;
}

// The duration bias enters the potential together with the transition: its gradient is the
// transition gradient summed over the source label (in label order).
__global__ __launch_bounds__(NT) void k_dt_fin_dur(Params p)
{
    const int C = p.C, CC = C * C;
    const int i = blockIdx.x * NT + threadIdx.x;
    if (i >= p.K * C) return;
    const int k = i / C, c = i % C;
    double s = 0.0;
    for (int o = 0; o < C; ++o) s += p.sumG[(size_t)k * CC + (size_t)o * C + c];
    p.grad_dur[i] = (float)s;
}
