// ---------------------------------------------------------------------------
// Marginals from the stored rows of both scans (included by semicrf.hip inside its namespace).
//
// When the chunk-parallel forward AND backward scans of a sequence are accepted, both have left
// their per-position rows behind -- forward (a_t, q_t), backward (p_t, v_t), each with its
// power-of-two scale relative to its interval -- and every expected statistic of the "Gradient
// Formulas" section is a position-local product of the two:
//   duration     sum_t q_t(c) W[k,c] v_{t+k}(c) 2^(n_blk(t+k)(c) - n_blk(t)(c)) kappa(t, t+k)
//   transition   Etr[c',c] sum_t a_t(c') p_t(c) kappa(t, t)
//   emission     out_t(c) - in_t(c) = (q_t ES_t p_t - a_t v_t IE_t)(c) kappa(t, t)
//   kappa(t, s) = exp((Y_alpha(t) + Y_beta(s)) ln2 - logZ)
// (the power of two is what the backward recurrence applies to its window when it crosses the
// scaling blocks between t+k and t).  No recurrence is run again: Algorithm 3's per-interval
// backward pass has already happened inside the backward scan.  Two kernels, one workgroup per
// (sequence, interval) each; they write the same partials as the interval kernels (partD,
// partTr, the running emission sums, tot, sumR), which skip the sequences handled here.
// ---------------------------------------------------------------------------

// absolute log2 scale of the forward / backward row i of interval j
__device__ __forceinline__ double mg_ya(const Params &p, const int b, const int j, const int i)
{
    return p.ckYA[(size_t)b * (p.N + 1) + j] + p.alocY[((size_t)b * p.N + j) * p.Delta + i];
}

__device__ __forceinline__ double mg_yb(const Params &p, const int b, const int j, const int i, const int L)
{
    const int hi = min((j + 1) * p.Delta, L);
    const double top = hi == L ? 0.0 : p.ckYB[(size_t)b * (p.N + 1) + j + 1];
    return top + p.blocY[((size_t)b * p.N + j) * p.Delta + i];
}

// Duration-bias statistics.  Thread (ks, c): label c, durations ks*MG_KS + 1 .. ks*MG_KS + MG_KS, one
// accumulator each.  Positions are taken in groups inside one scaling block: the group's q rows
// and the v rows it can reach are staged in LDS, the latter converted to the group's frame with
// all exponents combined before anything is formed; four positions share every LDS read.  The
// absolute scales of all rows the interval can touch are fetched into LDS once, at the start.
__global__ __launch_bounds__(1024) void k_mg_dur(Params p)
{
    extern __shared__ double lds_raw[];
    const int tid = threadIdx.x, nth = blockDim.x;
    const int K = p.K, C = p.C, N = p.N, Delta = p.Delta;
    const int b = blockIdx.x / N, iv = blockIdx.x % N;
    const SeqHdr h = p.hdr[b];
    const int L = h.L, J = h.J;
    const int lo = iv * Delta;
    if (lo >= L) return;
    if (!(p.spec_ok[b * 2] && p.spec_ok[b * 2 + 1])) return;  // the interval kernel takes this sequence
    const int hi = min(lo + Delta, L);
    const int nsl = (K + MG_KS - 1) / MG_KS;
    const bool active = tid < C * nsl;
    const int c = tid % C, kA = (tid / C) * MG_KS;
    const int VR = MG_TG + MG_KS * nsl + 3;
    double *Qrow = lds_raw;            // [MG_TG][C]
    // rows of CP = C|3 doubles: the threads of a wave read rows MG_KS apart (one per duration strip),
    // and MG_KS*C is a multiple of the 32 banks (of 8 bytes) for every C that is a multiple of 4;
    // with CP = 3 mod 4 the strips of a half-wave fall 24 banks apart instead of on top of each other
    const int CP = C | 3;
    double *Vp = Qrow + MG_TG * C;     // [VR][CP]
    double *qf = Vp + VR * CP;         // [MG_TG] per-row factors of the group
    double *vf = qf + MG_TG;           // [VR]
    int *ve = (int *)(vf + VR);        // [VR]
    int *vj = ve + VR;                 // [VR]
    double *yAs = vf + 2 * VR;         // [Delta]      absolute scale of the forward row lo + i
    double *yBs = yAs + Delta;         // [Delta + K]  absolute scale of the backward row lo + 1 + i
    const size_t row0 = (size_t)b * (p.T + 1);
    const double2 *EI = p.EI + row0 * C;
    const int *nb = p.nbase + row0 * C;
    const double2 *frow = (const double2 *)p.aloc + ((size_t)b * N) * Delta * C;  // row of position t at t*C
    const double2 *brow = (const double2 *)p.bloc + ((size_t)b * N) * Delta * C;  // (slots are consecutive)
    const double logZ = h.logZ;
    double acc[MG_KS];
#pragma unroll
    for (int kk = 0; kk < MG_KS; ++kk) acc[kk] = 0.0;
    for (int i = tid; i < hi - lo; i += blockDim.x) yAs[i] = mg_ya(p, b, iv, i);
    for (int i = tid; i < hi - lo + K; i += blockDim.x) {
        const int s = lo + 1 + i;
        yBs[i] = s < L ? mg_yb(p, b, s / Delta, s % Delta, L) : 0.0;  // b_L = 1: scale 0
    }

    for (int tg0 = lo; tg0 < hi;) {
        const int tg1 = min(min(hi, (tg0 / J + 1) * J), tg0 + MG_TG);
        const int ng = tg1 - tg0, jt = tg0 / J;
        __syncthreads();  // the previous group is done with the staged rows (first: the scales are there)
        const double yA0 = yAs[tg0 - lo];
        // per row first (uniform over the labels): the scale factor of a q row; for a v row the
        // fractional factor, the integer exponent and the scaling block it was stored in
        for (int r = tid; r < MG_TG + VR; r += blockDim.x) {
            if (r < MG_TG) {
                qf[r] = r < ng ? exp2(yAs[tg0 + r - lo] - yA0) : 0.0;
            } else {
                const int rr = r - MG_TG, s = tg0 + 1 + rr;
                double f = 0.0;
                int e = 0, js = jt;
                if (s <= L && rr < ng + K) {
                    const double lf = (yA0 + yBs[s - lo - 1]) - logZ * LOG2E;
                    const double fl = floor(lf);
                    f = exp2(lf - fl);
                    e = (int)fmin(fmax(fl, -100000.0), 100000.0);
                    js = s / J;
                }
                vf[rr] = f;
                ve[rr] = e;
                vj[rr] = js;
            }
        }
        __syncthreads();
        // v_L = ES_L; all exponents are combined before anything is formed, so that an empty row stays
        // zero and nothing passes through infinity.  Thread (row offset, label): no index divisions in
        // the loops; the loads of several rows per thread are issued together (rows beyond the
        // sequence are clamped, their factor is zero).
        {
            const int rstep = nth / C;               // rows per sweep of the workgroup
            const int o = tid % C, r0 = tid / C;     // threads with r0 >= rstep idle here
            if (r0 < rstep) {
                {
                    constexpr int UQ = 4;  // the q rows of a thread are fetched together
                    for (int rb = r0; rb < MG_TG; rb += UQ * rstep) {
                        double qv[UQ];
#pragma unroll
                        for (int u = 0; u < UQ; ++u)
                            qv[u] = frow[(size_t)(tg0 + min(rb + u * rstep, ng - 1)) * C + o].y;
#pragma unroll
                        for (int u = 0; u < UQ; ++u) {
                            const int r = rb + u * rstep;
                            if (r < MG_TG) Qrow[r * C + o] = qv[u] * qf[r];  // qf is zero beyond the group
                        }
                    }
                }
                const int nbt = nb[(size_t)jt * C + o];
                constexpr int UV = 4;
                for (int rb = r0; rb < VR; rb += UV * rstep) {
                    double vs[UV];
                    int n1[UV];
#pragma unroll
                    for (int u = 0; u < UV; ++u) {
                        const int r = min(rb + u * rstep, VR - 1);
                        const int s = min(tg0 + 1 + r, L);
                        vs[u] = s == L ? EI[(size_t)L * C + o].x : brow[(size_t)s * C + o].y;
                        n1[u] = nb[(size_t)vj[r] * C + o];
                    }
#pragma unroll
                    for (int u = 0; u < UV; ++u) {
                        const int r = rb + u * rstep;
                        if (r < VR) {
                            const double f = vf[r];
                            Vp[r * CP + o] = f != 0.0 ? fmin(ldexp(vs[u] * f, n1[u] - nbt + ve[r]), DBL_MAX) : 0.0;
                        }
                    }
                }
            }
        }
        __syncthreads();
        if (active) {
            for (int i0 = 0; i0 < ng; i0 += 4) {
                double ca[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) ca[i] = i0 + i < ng ? Qrow[(i0 + i) * C + c] : 0.0;
                double w[MG_KS + 3];
#pragma unroll
                for (int q = 0; q < MG_KS + 3; ++q) w[q] = Vp[(i0 + kA + q) * CP + c];
#pragma unroll
                for (int kk = 0; kk < MG_KS; ++kk) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) acc[kk] = fma(ca[i], w[kk + i], acc[kk]);
                }
            }
        }
        tg0 = tg1;
    }
    if (active) {
        double *pD = p.partD + ((size_t)b * p.NP + iv) * K * C;
#pragma unroll
        for (int kk = 0; kk < MG_KS; ++kk) {
            const int k = kA + kk + 1;
            if (k <= K) pD[(size_t)(k - 1) * C + c] = acc[kk] * p.W[(size_t)(k - 1) * C + c];
        }
    }
}

// Transition statistics and the running emission sums.  Groups of MG_TE positions from the
// interval's upper end downwards (the emission sums are suffix sums); per group all threads stage
// a_t kappa, p_t and (out - in) kappa (rows beyond the group are zero), then every thread adds the
// group's products for its label pairs while threads 0..C-1 walk the group for the running sums.

__global__ __launch_bounds__(NT) void k_mg_te(Params p)
{
    extern __shared__ double lds_raw[];
    const int tid = threadIdx.x;
    const int C = p.C, CC = C * C, N = p.N, Delta = p.Delta;
    const int b = blockIdx.x / N, iv = blockIdx.x % N;
    const SeqHdr h = p.hdr[b];
    const int L = h.L;
    const int lo = iv * Delta;
    if (lo >= L) return;
    if (!(p.spec_ok[b * 2] && p.spec_ok[b * 2 + 1])) return;
    const int hi = min(lo + Delta, L);
    double *AK = lds_raw;            // [MG_TE][C] a_t(c') kappa(t,t)
    double *P = AK + MG_TE * C;      // [MG_TE][C] p_t(c)
    double *D = P + MG_TE * C;       // [MG_TE][C] (out_t - in_t)(c)
    double *kp = D + MG_TE * C;      // [Delta]    kappa(t,t) of every position of the interval
    const size_t row0 = (size_t)b * (p.T + 1);
    const double2 *EI = p.EI + row0 * C;
    const double2 *frow = (const double2 *)p.aloc + ((size_t)b * N) * Delta * C;
    const double2 *brow = (const double2 *)p.bloc + ((size_t)b * N) * Delta * C;
    const double logZ = h.logZ;
    constexpr int NPAIR = GRAD_CMAX * GRAD_CMAX / NT;  // label pairs tid, tid + NT, ...
    double acc[NPAIR];
#pragma unroll
    for (int n = 0; n < NPAIR; ++n) acc[n] = 0.0;
    double R = 0.0, sR = 0.0;
    for (int i = tid; i < hi - lo; i += NT)
        kp[i] = exp((mg_ya(p, b, iv, i) + mg_yb(p, b, iv, i, L)) * LN2 - logZ);

    for (int tg1 = hi; tg1 > lo;) {
        const int tg0 = max(lo, tg1 - MG_TE);
        const int ng = tg1 - tg0;
        __syncthreads();
        {
            const int rstep = NT / C, o = tid % C, r0 = tid / C;  // thread (row offset, label): no index divisions below
            if (r0 < rstep) {
                for (int r = r0; r < MG_TE; r += rstep) {
                    const int t = tg0 + r;
                    double ak = 0.0, pp = 0.0, d = 0.0;
                    if (r < ng) {
                        const double2 fa = frow[(size_t)t * C + o], fb = brow[(size_t)t * C + o], e = EI[(size_t)t * C + o];
                        const double kap = kp[t - lo];
                        ak = fa.x * kap;
                        pp = fb.x;
                        // a segment of label o starts at t (z_t p_t, z = q ES) / ends at t (a_t b_t, b = v IE; none ends at 0)
                        d = (fa.y * e.x * fb.x - (t >= 1 ? fa.x * fb.y * e.y : 0.0)) * kap;
                    }
                    AK[r * C + o] = ak;
                    P[r * C + o] = pp;
                    D[r * C + o] = d;
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int n = 0; n < NPAIR; ++n) {
            const int pair = tid + n * NT;
            if (pair < CC) {
                const int cp = pair / C, c = pair % C;
                double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
#pragma unroll 4
                for (int r = 0; r < MG_TE; r += 4) {
                    a0 = fma(AK[r * C + cp], P[r * C + c], a0);
                    a1 = fma(AK[(r + 1) * C + cp], P[(r + 1) * C + c], a1);
                    a2 = fma(AK[(r + 2) * C + cp], P[(r + 2) * C + c], a2);
                    a3 = fma(AK[(r + 3) * C + cp], P[(r + 3) * C + c], a3);
                }
                acc[n] += (a0 + a1) + (a2 + a3);
            }
        }
        if (tid < C) {
            for (int r = ng - 1; r >= 0; --r) {
                p.grad_emis[((size_t)b * p.T + tg0 + r) * C + tid] = (float)R;
                sR += R;
                R += D[r * C + tid];
            }
        }
        tg1 = tg0;
    }
    double *pT = p.partTr + ((size_t)b * p.NP + iv) * CC;
#pragma unroll
    for (int n = 0; n < NPAIR; ++n) {
        const int pair = tid + n * NT;
        if (pair < CC) pT[pair] = acc[n];
    }
    if (tid < C) {
        p.tot[((size_t)b * p.NP + iv) * C + tid] = R;
        p.sumR[((size_t)b * p.NP + iv) * C + tid] = sR;
    }
}

// ---------------------------------------------------------------------------
// The same statistics for short maximal durations (K < 128), where the work of an interval fits single waves.
// One wave per (sequence, interval, part): an interval is cut into p.msplit parts of equal length, each its own
// task, so that the chip holds two tasks per SIMD where there are few intervals; nothing in these statistics
// depends on the position before, only the running emission sums do, and those restart with every part (the
// partial sums tot, sumR, partD, partTr are per part: index interval*msplit + part).  Lane organisation of the
// interval kernel (lane (g, c): label c, durations g*NK + 1 ..): the wave walks its part from the upper end
// downwards, as the backward scan did, but takes p_t and v_t from that scan's stored rows instead of running the
// recurrence.  The K-deep window of v rows slides through LDS in the frame of the current scaling block (rescaled
// by the same powers of two at the same positions as in the scan, read off the stored scales), so the duration
// statistics are NK multiply-adds per position and lane with every window entry read once per block of MB
// positions; the transition statistics run on the matrix cores, four positions per v_mfma_f64_16x16x4; the
// emission sums are running sums.  The rows of the next block are requested as soon as the current block's have
// been turned into the few values the multiply-adds need.
template <int CT, int NKW>
__global__ __launch_bounds__(64, mg_waves_per_simd(CT, NKW)) void k_mg_wave(Params p)
{
    using G = WaveWin<CT, NKW>;
    constexpr int CTP = G::CTP, RS = G::RS, NK = G::NK, KW = G::KW, M = G::M, RTOT = G::RTOT, TRN = G::TRN;
    typedef double double4_t __attribute__((ext_vector_type(4)));
    extern __shared__ double lds_raw[];
    double *ring = lds_raw;  // [ROWS][RS] (+ pad), then 64 doubles nobody reads
    const int lane = threadIdx.x;
    const int K = p.K, C = p.C, KC = K * C, CC = C * C, N = p.N, Delta = p.Delta;
    const int S = p.msplit, Dm = Delta / S;
    const int sub = blockIdx.x % S, b = (blockIdx.x / S) / N, iv = (blockIdx.x / S) % N;
    const SeqHdr h = p.hdr[b];
    const int L = h.L, J = h.J, Jm = J - 1;
    const int t0 = iv * Delta;      // the interval: its rows are stored relative to t0
    const int ta = t0 + sub * Dm;   // this task's positions: ta <= t < tb
    if (ta >= L) return;
    if (!(p.spec_ok[b * 2] && p.spec_ok[b * 2 + 1])) return;  // the interval kernel takes this sequence
    const int t1 = min(t0 + Delta, L);
    const int tb = min(ta + Dm, L);
    const int c = lane % CTP, g = lane / CTP;
    const bool cval = c < C;
    const int cc = cval ? c : 0;
    const bool writer = cval && g == 0;  // one lane per label
    const int pj = lane >> 4, pl = lane & 15;  // matrix-core operands: position pj of the block, label pl of the tile
    const size_t row0 = (size_t)b * (p.T + 1);
    const double2 *EIc = p.EI + row0 * C + cc;
    const int *nbc = p.nbase + row0 * C + cc;
    const size_t slot = (size_t)b * N + iv;
    const size_t part = (size_t)b * p.NP + (size_t)iv * S + sub;
    const double2 *arow = (const double2 *)p.aloc + slot * Delta * C;  // (a_t, q_t) of position t0 + i at i*C
    const double2 *brow = (const double2 *)p.bloc + slot * Delta * C;  // (p_t, v_t)
    const double *arowY = p.alocY + slot * Delta;
    const double *browY = p.blocY + slot * Delta;
    const double logZ = h.logZ;
    const double Y0 = p.ckYA[(size_t)b * (N + 1) + iv];
    const double Ytop = t1 == L ? 0.0 : p.ckYB[(size_t)b * (N + 1) + iv + 1];

    // ---- the window above the part
    for (int i = lane; i < RTOT; i += 64) ring[i] = 0.0;
    lds_wave_fence();
    int r = M;  // row of the newest (lowest) position
    double ybPrev = 0.0;  // stored scale (relative to the interval's upper end) of the frame the window is in
    if (tb == L) {  // v_L = E_L
        if (writer) ring[r * RS + c] = EIc[(size_t)L * C].x;
    } else if (tb == t1) {  // the state the backward task started from
        const double *ck = p.ckB + ((size_t)b * (N + 1) + iv + 1) * ((size_t)KC + C);
        const int tm = t1 % K;
        if (cval) {  // lane (g, c): the window rows at distances g, g + GW, ... of its label (no index divisions)
#pragma unroll 8
            for (int d = g; d < K; d += G::GW) {
                int sl = tm + d;  // checkpoint slot of the position at that distance
                sl -= sl >= K ? K : 0;
                ring[(r + d) * RS + c] = ck[(size_t)sl * C + c];
            }
        }
    } else {
        // inside the interval: the rows v_tb .. v_{tb+K-1} as the backward task stored them (a part is at least
        // K positions long, so they all belong to this interval, or are v_L), each brought from the frame of its own
        // scaling block into that of position tb: the powers of two the scan applied on its way down from there
        // and the difference of the stored scales (whole numbers).  Lane (g, c) fills its own strip, rows g*NK ..
        // of label c; everything is loaded first, so that the loads of all rows are in flight together.
        const int nbt = nbc[(size_t)(tb / J) * C];
        const double ybt = browY[tb - t0];
        const int top = min(t1 - 1, L - 1) - t0;  // last stored row of the interval
        double vr[NK], ys[NK];
        int ns[NK];
#pragma unroll
        for (int u = 0; u < NK; ++u) {
            const int i = min(tb - t0 + g * NK + u, top);  // v_L and what lies beyond are dealt with below
            vr[u] = brow[(size_t)i * C + cc].y;
            ys[u] = browY[i];
            ns[u] = nbc[(size_t)((t0 + i) / J) * C];
        }
        const double vL = EIc[(size_t)L * C].x;  // scale 0 relative to the upper end
        const int nsL = nbc[(size_t)(L / J) * C];
#pragma unroll
        for (int u = 0; u < NK; ++u) {
            const int d = g * NK + u, sp = tb + d;
            const int e = (int)fmin(fmax((sp == L ? 0.0 : ys[u]) - ybt, -100000.0), 100000.0) + (sp == L ? nsL : ns[u]) - nbt;
            const double val = fmin(ldexp(sp == L ? vL : vr[u], e), DBL_MAX);
            if (cval && d < K && sp <= L) ring[(r + d) * RS + c] = val;
        }
        ybPrev = browY[tb - t0];
    }
    lds_wave_fence();

    double dx[NK + MB - 1];  // sum_t q_t(c) kappa_t v_{t+k}(c), k = g*NK + jj + 1 (times W[k,c] at the end)
    double dn[MB - 1];       // the same for k = 1..MB-1 from inside the blocks (lanes g == 0)
    double4_t accT[TRN][TRN];
#pragma unroll
    for (int jj = 0; jj < NK + MB - 1; ++jj) dx[jj] = 0.0;
#pragma unroll
    for (int jj = 0; jj < MB - 1; ++jj) dn[jj] = 0.0;
#pragma unroll
    for (int i = 0; i < TRN; ++i)
#pragma unroll
        for (int o = 0; o < TRN; ++o) accT[i][o] = double4_t{0.0, 0.0, 0.0, 0.0};
    double R = 0.0, sR = 0.0;
    float *const sink = (float *)p.sink + lane;
    float *const gout = p.grad_emis + ((size_t)b * p.T) * C + cc;

    // The rows of one block of positions, as they come from memory.  Where a label's lanes come in pairs 32 apart
    // (CTP <= 32) the lower half of the wave fetches the block's first two positions and the upper half the
    // other two: half the row loads, which is what this kernel waits for most (the few values the other half
    // needs travel by v_permlane32_swap).  With 64 labels per lane group every lane fetches all four.
    static_assert(MB == 4, "the split of a block between the halves of the wave is written for four positions");
    constexpr bool SPLIT = CTP <= 32;
    constexpr int NPL = SPLIT ? MB / 2 : MB;  // positions of a block this lane fetches
    const int pofs = SPLIT ? (lane >> 5) * NPL : 0;  // the first of them
    double2 aq[NPL], pv[NPL], e[NPL];  // this lane's label, positions pofs .. pofs+NPL-1 below tfrom
    double aA[TRN], bB[TRN];        // operand elements: position pj of the block, label pl of tile tr
    double ya, yb;                  // stored scales of the position just below tfrom (forward, backward)
    int nd;                         // exponent step of this lane's label at the scaling-block boundary tfrom
    // Byte offsets from the (wave-uniform) starts of the interval's rows fit 32 bits: a slot has Delta*C < 2^27
    // pairs (the plan's limits), a sequence fewer than 2^31 position-label pairs (checked by the caller).
    const char *const arb = (const char *)arow, *const brb = (const char *)brow;
    const char *const eib = (const char *)(p.EI + (row0 + t0) * C);
    const unsigned C16 = (unsigned)C * 16u, cc16 = (unsigned)cc * 16u;
    unsigned cpo16[TRN];  // label pl of tile tr (clamped: what lies beyond C lands in tile rows nobody stores), less pj rows
#pragma unroll
    for (int tr = 0; tr < TRN; ++tr) cpo16[tr] = (unsigned)min(tr * 16 + pl, C - 1) * 16u;
    auto ld2 = [](const char *base, const unsigned off) { return *(const double2 *)(base + off); };
    auto ld1 = [](const char *base, const unsigned off) { return *(const double *)(base + off); };
    // the block below tfrom; rows below the part's first are replaced by that one (nobody uses them)
    auto request = [&](const int tfrom) {
#pragma unroll
        for (int l = 0; l < NPL; ++l) {
            const unsigned o = (unsigned)(max(tfrom - 1 - l - pofs, ta) - t0) * C16 + cc16;
            aq[l] = ld2(arb, o);
            pv[l] = ld2(brb, o);
            e[l] = ld2(eib, o);
        }
        const unsigned om = (unsigned)(max(tfrom - 1 - pj, ta) - t0) * C16;
#pragma unroll
        for (int tr = 0; tr < TRN; ++tr) {
            aA[tr] = ld1(arb, om + cpo16[tr]);
            bB[tr] = ld1(brb, om + cpo16[tr]);
        }
        // what a scaling-block boundary at tfrom needs, fetched with every block: a load inside the (rare)
        // boundary branch would make the wave wait there for everything in flight
        const int i0 = max(tfrom - 1 - t0, 0);
        ya = arowY[i0];
        yb = browY[i0];
        const int jb = max(tfrom / J, 1);
        const int hiE = nbc[(size_t)min(jb, L / J) * C], loE = nbc[(size_t)(jb - 1) * C];
        nd = (tfrom / J >= 1 && (long)jb * J <= (long)L) ? hiE - loE : 0;
    };
    // kappa(t,t) = exp((Y_alpha + Y_beta) ln2 - logZ) of the positions of a scaling block (they share both scales):
    // the stored scales are whole numbers, so it is one fixed factor in [1, 2) times a power of two
    const double kx = (Y0 + Ytop) - logZ * LOG2E, kxi = floor(kx);
    const double kfrac = exp2(kx - kxi);
    const int kint = (int)fmin(fmax(kxi, -100000.0), 100000.0);
    auto kappa_of = [&]() { return ldexp(kfrac, kint + (int)(ya + yb)); };

    int t = tb;
    const int rdoff = g * NK * RS + c;
    request(t);
    double kappa = kappa_of();
    float *const gseq = p.grad_emis + ((size_t)b * p.T) * C;
    while (t > ta) {
        const int nb = min(min(t - ta, MB), ((t - 1) & Jm) + 1);
        if (__builtin_expect((t & Jm) == 0, 0)) {
            // the scan stepped into a new scaling block here: same shift of the live window, read off its scales
            G::template rescale_live<true>(ring, g, c, cval, r, nd - (int)(yb - ybPrev));
            ybPrev = yb;
            kappa = kappa_of();
        }
        if (__builtin_expect(r < MB, 0)) r = G::template move<true>(ring, lane, r);
        // ---- everything the block needs from its rows; v_t(c) enters the window at once (the rows below the
        // newest are not among those the block reads)
        double coef[MB];
        const bool whole = nb == MB && t - MB >= 1;
        if (SPLIT && whole) {
            // This lane's positions of the block: pofs + l, rows t-1-pofs-l.  A whole block (nearly all are) decides
            // nothing per position: every lane works on its label cc (the lanes of one label and half hold the same
            // rows and store the same values to the same places; what lanes beyond C add up is never stored).
            double dl[NPL];
#pragma unroll
            for (int l = 0; l < NPL; ++l) {
                both_halves(aq[l].y * kappa, coef[l], coef[NPL + l]);  // q_t(c) kappa of positions l and NPL + l
                // a segment of this label starts at the position (z p, z = q ES) / ends at it (a b, b = v IE)
                dl[l] = (aq[l].y * e[l].x * pv[l].x - aq[l].x * pv[l].y * e[l].y) * kappa;
            }
            // durations 1..3 inside the block: this lane's v rows with the coefficients of the later positions
            // (lower half: positions 0, 1; upper half: 2, 3; the two halves are added up at the end)
            const bool lowh = pofs == 0;
            const double k13 = lowh ? coef[1] : coef[3], k2 = lowh ? coef[2] : 0.0, k3 = lowh ? coef[3] : 0.0;
            dn[0] = fma(k13, pv[0].y, dn[0]);
            dn[1] = fma(k2, pv[0].y, dn[1]);
            dn[2] = fma(k3, pv[0].y, dn[2]);
            dn[0] = fma(k2, pv[1].y, dn[0]);
            dn[1] = fma(k3, pv[1].y, dn[1]);
            // running emission sums: R before the block, plus what the positions before this lane's add
            double s01, s23;
            both_halves(dl[0] + dl[1], s01, s23);
            const double r0 = lowh ? R : R + s01, r1 = r0 + dl[0];
            sR += r0 + r1;
            R = (R + s01) + s23;
            float *gp = gseq + ((unsigned)(t - 1 - pofs) * (unsigned)C + (unsigned)cc);
            double *rw = ring + (r - 1 - pofs) * RS + cc;
            rw[0] = pv[0].y;
            rw[-RS] = pv[1].y;
            gp[0] = (float)r0;
            gp[-C] = (float)r1;
        } else if (SPLIT) {
            // A short block (at most two at the part's upper end, the last one, the one with position 0): the
            // positions beyond its end count nothing and their stores go to the pad and to the sink.  The lanes
            // beyond C keep label cc's running sums here too: in whole blocks they store them.
            double dl[NPL];
            bool act[NPL];
#pragma unroll
            for (int l = 0; l < NPL; ++l) {
                const int tt = t - 1 - pofs - l;
                act[l] = pofs + l < nb;
                both_halves((act[l] && cval) ? aq[l].y * kappa : 0.0, coef[l], coef[NPL + l]);
                // none ends at position 0
                dl[l] = act[l] ? (aq[l].y * e[l].x * pv[l].x - (tt >= 1 ? aq[l].x * pv[l].y * e[l].y : 0.0)) * kappa : 0.0;
            }
            const bool lowh = pofs == 0;
            const double k13 = lowh ? coef[1] : coef[3], k2 = lowh ? coef[2] : 0.0, k3 = lowh ? coef[3] : 0.0;
            dn[0] = fma(k13, pv[0].y, dn[0]);
            dn[1] = fma(k2, pv[0].y, dn[1]);
            dn[2] = fma(k3, pv[0].y, dn[2]);
            dn[0] = fma(k2, pv[1].y, dn[0]);
            dn[1] = fma(k3, pv[1].y, dn[1]);
            double s01, s23;
            both_halves(dl[0] + dl[1], s01, s23);
            const double r0 = lowh ? R : R + s01, r1 = r0 + dl[0];
            sR += (act[0] ? r0 : 0.0) + (act[1] ? r1 : 0.0);
            R = (R + s01) + s23;
#pragma unroll
            for (int l = 0; l < NPL; ++l) {
                const int i = pofs + l;
                const bool on = act[l] && cval;
                double *rdst = on ? ring + (r - 1 - i) * RS + c : ring + RTOT + lane;
                *rdst = pv[l].y;
                float *dst = on ? gout + (unsigned)(t - 1 - i) * (unsigned)C : sink;
                *dst = (float)(l == 0 ? r0 : r1);
            }
        } else if (whole) {
            // 64 labels per lane group: every lane holds all four positions of its label
            float *gp = gseq + ((unsigned)(t - 1) * (unsigned)C + (unsigned)cc);
            double *rw = ring + (r - 1) * RS + cc;
#pragma unroll
            for (int i = 0; i < NPL; ++i) {
                coef[i] = aq[i].y * kappa;
#pragma unroll
                for (int jn = 0; jn < i; ++jn) dn[i - 1 - jn] = fma(coef[i], pv[jn].y, dn[i - 1 - jn]);
                rw[-i * RS] = pv[i].y;
                const double d = (aq[i].y * e[i].x * pv[i].x - aq[i].x * pv[i].y * e[i].y) * kappa;
                gp[-i * C] = (float)R;
                sR += R;
                R += d;
            }
        } else {
#pragma unroll
            for (int i = 0; i < NPL; ++i) {
                const bool on = i < nb;
                const int tt = t - 1 - i;
                coef[i] = (cval && on) ? aq[i].y * kappa : 0.0;
                const double cg = g == 0 ? coef[i] : 0.0;
#pragma unroll
                for (int jn = 0; jn < i; ++jn) dn[i - 1 - jn] = fma(cg, pv[jn].y, dn[i - 1 - jn]);
                double *rdst = (on && writer) ? ring + (r - 1 - i) * RS + c : ring + RTOT + lane;
                *rdst = pv[i].y;
                const double d = on ? (aq[i].y * e[i].x * pv[i].x - (tt >= 1 ? aq[i].x * pv[i].y * e[i].y : 0.0)) * kappa : 0.0;
                float *dst = (on && writer) ? gout + (unsigned)tt * (unsigned)C : sink;
                *dst = (float)R;
                sR += on ? R : 0.0;
                R += d;
            }
        }
        {
            // transition statistics on the matrix cores; label rows beyond C are never stored, positions beyond a
            // short block's end must count nothing
            const bool on = whole || pj < nb;
#pragma unroll
            for (int tr = 0; tr < TRN; ++tr) {
                const double a = on ? aA[tr] * kappa : 0.0;
#pragma unroll
                for (int tc = 0; tc < TRN; ++tc)
                    accT[tr][tc] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, bB[tc], accT[tr][tc], 0, 0, 0);
            }
        }
        // ---- the next block's rows
        request(t - nb);
        // window reads in groups of four, each group requested before the multiply-adds of the one before it
        // (all NK at once would cost their registers, one group at a time would wait for every one)
        const double *base = ring + r * RS + rdoff;
        double vc[4], vn[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) vc[q] = base[q * RS];
#pragma unroll
        for (int jg = 0; jg < NK; jg += 4) {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (jg + 4 + q < NK) vn[q] = base[(jg + 4 + q) * RS];
#pragma unroll
            for (int q = 0; q < 4; ++q) {  // distance g*NK + jg + q from the newest (NK need not be a multiple of 4)
                if (jg + q < NK) {
#pragma unroll
                    for (int i = 0; i < MB; ++i) dx[jg + q + i] = fma(coef[i], vc[q], dx[jg + q + i]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int q = 0; q < 4; ++q) vc[q] = vn[q];
        }
        r -= nb;
        lds_wave_fence();
        t -= nb;
    }
    // ---- partials of this task.  Duration sums: the strips of neighbouring lane groups overlap by MB-1
    // durations; they are combined through LDS in a fixed order (own strip, then the neighbour's overlap, then
    // the in-block terms) and scaled by W[k,c].
    lds_wave_fence();
    if (SPLIT) {  // what the two halves of the wave gathered separately
#pragma unroll
        for (int jj = 0; jj < MB - 1; ++jj) dn[jj] = add_across_32(dn[jj]);
        sR = add_across_32(sR);
    }
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
    double *pD = p.partD + part * KC;
    if (cval) {
#pragma unroll 8
        for (int k = g; k < K; k += G::GW) pD[(size_t)k * C + c] = p.W[(size_t)k * C + c] * tmp[k * CT + c];
    }
    double *pT = p.partTr + part * CC;
#pragma unroll
    for (int tr = 0; tr < TRN; ++tr)
#pragma unroll
        for (int tc = 0; tc < TRN; ++tc)
#pragma unroll
            for (int v = 0; v < 4; ++v) {  // tile element (4v + lane/16, lane%16)
                const int src = tr * 16 + 4 * v + pj, dst = tc * 16 + pl;
                if (src < C && dst < C) pT[(size_t)src * C + dst] = accT[tr][tc][v];
            }
    if (lane < C) {
        p.tot[part * C + lane] = R;
        p.sumR[part * C + lane] = sR;
    }
}
