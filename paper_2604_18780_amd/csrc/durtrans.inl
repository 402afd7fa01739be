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
// ---------------------------------------------------------------------------
constexpr int DT_MB = 4;

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
    __syncthreads();  // yv and the ring are complete
    double pm = 0.0;
    for (int i = 0; i < C; ++i) pm += yv[i];
    const int e = safe_exponent(pm);
    const int tid = threadIdx.x;
    if (tid < C) sc[tid] = sgn * (nb[(size_t)jnew * C + tid] - nb[(size_t)jold * C + tid]) - e;
    __syncthreads();
    for (int i = tid; i < KC; i += blockDim.x) ring[i] = fmin(ldexp(ring[i], sc[i % C]), DBL_MAX);
    __syncthreads();
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
    if (tid < C) yv[tid] = 1.0;
    __syncthreads();
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
        // ---- the block's positions, one after the other
        for (int i = 0; i < nbk; ++i) {
            const int tt = t0 + i;
            if (tid < C) {
                const double a = tt == s0 ? 1.0 : EI[(size_t)tt * C + tid].x * X[(tt % K) * C + tid];
                av[i * C + tid] = a;
                if (tt > lo || tt == 0) rowA[(size_t)tt * C + tid] = a;
            }
            if (tid == 0) {
                if (tt > lo || tt == 0) rowY[tt] = Y - Ybase;
                if (whole && (tt % Delta) == 0) p.ckYA[(size_t)b * (N + 1) + tt / Delta] = Y;
            }
            if ((whole && (tt % Delta) == 0) || tt == lo) Ybase = Y;  // uniform
            __syncthreads();
            const int kin = nbk - 1 - i;  // durations that stay inside the block
            if (kin > 0) {
                const int k = ks + 1;
                if (active && k <= kin && k <= K) {
                    const double *g = p.G3 + (size_t)(k - 1) * CC + c;
                    double m = 0.0;
                    for (int o = 0; o < C; ++o) m = fma(av[i * C + o], g[(size_t)o * C], m);
                    const int slot = ((tt + k) % K) * C + c;
                    const double val = EI[(size_t)tt * C + c].y * m;
                    X[slot] = k == K ? val : X[slot] + val;
                }
                __syncthreads();
            }
        }
        // ---- durations that leave the block: every table entry once for all its positions
        double m[KPTF][DT_MB];
#pragma unroll
        for (int kk = 0; kk < KPTF; ++kk) {
#pragma unroll
            for (int i = 0; i < DT_MB; ++i) m[kk][i] = 0.0;
            const int k = ks + 1 + kk * NKS;
            if (active && k <= K) {
                const double *g = p.G3 + (size_t)(k - 1) * CC + c;
#pragma unroll 4
                for (int o = 0; o < C; ++o) {
                    const double gv = g[(size_t)o * C];
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
                    const double ie = EI[(size_t)tt * C + c].y;
#pragma unroll
                    for (int kk = 0; kk < KPTF; ++kk) {
                        const int k = ks + 1 + kk * NKS;
                        if (k <= K && i + k >= nbk) {
                            const int slot = ((tt + k) % K) * C + c;
                            const double val = ie * m[kk][i];
                            X[slot] = k == K ? val : X[slot] + val;
                        }
                    }
                }
                __syncthreads();
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
    __syncthreads();
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
// Backward recurrence and, with ACC, the marginals.  Thread (ks, c', c): one label pair and the
// KPT consecutive durations ks*KPT + 1 .. ks*KPT + KPT; its sum over those durations goes
// through a [NKS][C][C] table in LDS from which threads 0..C-1 form b_t (row sums) and, with
// ACC, the mass of the segments that start at t (column sums weighted by a_t).
// mode 0: grid B*N chunk tasks with warm-up (scan; checkpoint states at both ends)
// mode 1: grid B whole sequences whose chunk-parallel backward scan was not accepted
// mode 2: persistent workgroups over the (sequence, interval) tasks, restoring the state at
//         the interval's upper end from the backward checkpoints; accumulates, per thread,
//         sum_t w_b mu(t -> t+k, c', c) for its pair and durations (registers, all tasks of
//         the workgroup), and writes the running emission-gradient sums like k_interval.
// ---------------------------------------------------------------------------
template <int KPT, bool ACC, int MBT, int NTMAX>
__global__ __launch_bounds__(NTMAX) void k_dt_bwd(Params p, int warm, int tier, int mode)
{
    extern __shared__ double lds_raw[];
    const int tid = threadIdx.x;
    const int K = p.K, C = p.C, CC = C * C, KC = K * C, N = p.N, Delta = p.Delta;
    const int NKS = (K + KPT - 1) / KPT;
    const int ks = tid / CC, pair = tid % CC;
    const int cp = pair / C, c = pair % C;
    const bool active = ks < NKS;
    const int k0 = ks * KPT;  // the thread's durations are k0 + 1 .. k0 + KPT
    double *ring = lds_raw;           // [K][C]   v_u(c) at slot u mod K
    double *red = ring + KC;          // [NKS][C][C]
    double *av = red + NKS * CC;      // [MBT][C] a_t of the block's positions (ACC)
    double *yv = av + MBT * C;        // [C]      b_t: scale reference
    int *sc = (int *)(yv + C);        // [C]
    const size_t ckstride = (size_t)KC + C;

    double acc[ACC ? KPT : 1];
    if (ACC) {
#pragma unroll
        for (int kk = 0; kk < KPT; ++kk) acc[kk] = 0.0;
    }

    const int ntask = mode == 1 ? p.B : p.B * N;
    for (int task = blockIdx.x; task < ntask; task += gridDim.x) {
        const int b = mode == 1 ? task : task / N;
        const int chunk = mode == 1 ? -1 : task % N;
        if (mode == 0 && tier > 0 && p.spec_ok[b * 2 + 1]) continue;
        if (mode == 1 && p.spec && p.spec_ok[b * 2 + 1]) continue;
        const SeqHdr h = p.hdr[b];
        const int L = h.L, J = h.J;
        const int lo = mode == 1 ? 0 : chunk * Delta;
        if (mode != 1 && lo >= L) continue;
        const int hi = mode == 1 ? L : min(lo + Delta, L);
        const int s1 = mode == 0 ? min(hi + warm, L) : hi;  // where this task's recurrence starts
        const size_t row0 = (size_t)b * (p.T + 1);
        const double2 *EI = p.EI + row0 * C;
        const int *nb = p.nbase + row0 * C;
        const double *rowA = p.dtA + row0 * C;
        const double *rowY = p.dtY + row0;
        const double *ckYA = p.ckYA + (size_t)b * (N + 1);
        const double logZ = h.logZ;
        const double wb = (ACC && p.grad_logz) ? (double)p.grad_logz[b] : 1.0;

        __syncthreads();  // the previous task is done with the LDS arrays
        double Yb = 0.0;
        if (s1 == L) {  // exact: b_L = 1, v_L = ES_L
            for (int i = tid; i < KC; i += blockDim.x) ring[i] = 0.0;
            __syncthreads();
            if (tid < C) {
                yv[tid] = tid == 0 ? 1.0 : 0.0;
                ring[(L % K) * C + tid] = EI[(size_t)L * C + tid].x;
            }
        } else if (mode == 0) {  // a sequence that ends at s1
            for (int i = tid; i < KC; i += blockDim.x) ring[i] = 0.0;
            __syncthreads();
            if (tid < C) {
                yv[tid] = tid == 0 ? 1.0 : 0.0;
                ring[(s1 % K) * C + tid] = EI[(size_t)s1 * C + tid].x;
            }
        } else {  // the checkpoint at the interval's upper end
            const int ci = s1 / Delta;
            const double *ck = p.ckB + ((size_t)b * (N + 1) + ci) * ckstride;
            for (int i = tid; i < KC; i += blockDim.x) ring[i] = ck[i];
            if (tid < C) yv[tid] = ck[KC + tid];
            Yb = p.ckYB[(size_t)b * (N + 1) + ci];
        }
        double R = 0.0, sR = 0.0;  // running suffix sum of (out - in) and its sum: threads < C
        double kappa = 0.0, kY = -1.0e300;  // exp((Y_alpha + Y_beta) ln2 - logZ), recomputed when the scales move
        __syncthreads();
        auto record = [&](double *ck) {
            for (int i = tid; i < KC; i += blockDim.x) ck[i] = ring[i];
            if (tid < C) ck[KC + tid] = yv[tid];
        };

        int t0 = s1 - 1;
        while (t0 >= lo) {
            int nbk = min(MBT, t0 - lo + 1);
            if (t0 >= hi) nbk = min(nbk, t0 - hi + 1);         // the interval's upper end ends its block
            nbk = min(nbk, (t0 % J) + 1);                       // no scaling-block boundary inside a block
            if (mode == 1) nbk = min(nbk, (t0 % Delta) + 1);    // checkpoints are recorded at block ends
            if (((t0 + 1) % J) == 0) Yb += (double)dt_rebase(ring, yv, sc, nb, KC, C, t0 / J, t0 / J + 1, -1);
            // ---- per-position factors of this thread
            double ie[MBT], coef[MBT], kap[MBT];
#pragma unroll
            for (int i = 0; i < MBT; ++i) {
                ie[i] = 0.0;
                coef[i] = 0.0;
                kap[i] = 0.0;
                if (i < nbk) {
                    const int tt = t0 - i;
                    if (active) ie[i] = EI[(size_t)tt * C + c].y;
                    if (ACC) {
                        const int jr = tt == 0 ? 0 : (tt - 1) / Delta;
                        const double ysum = ckYA[jr] + rowY[tt] + Yb;
                        if (ysum != kY) {  // uniform
                            kY = ysum;
                            kappa = exp(ysum * LN2 - logZ);
                        }
                        kap[i] = kappa;
                        if (active) coef[i] = rowA[(size_t)tt * C + cp] * kap[i] * wb * ie[i];
                        if (tid < C) av[i * C + tid] = rowA[(size_t)tt * C + tid];
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
                const double *gp = p.G3 + (size_t)k0 * CC + pair;
                int sl = (t0 + k0 + 1) % K;  // slot of position t0 + k0 + 1
                double w[MBT];
#pragma unroll
                for (int i = 1; i < MBT; ++i) w[i] = ring[dt_wrap(sl - i, K) * C + c];
#pragma unroll  // fully: the accumulators must stay in registers
                for (int kk = 0; kk < KPT; ++kk) {
                    const int k = k0 + kk + 1;
                    if (k <= K) {
                        w[0] = ring[sl * C + c];
                        const double gv = *gp;
#pragma unroll
                        for (int i = 0; i < MBT; ++i) {
                            if (i < nbk && k > i) {
                                const double gu = gv * w[i];
                                bs[i] += gu;
                                if (ACC) acc[kk] = fma(coef[i], gu, acc[kk]);
                            }
                        }
#pragma unroll
                        for (int i = MBT - 1; i > 0; --i) w[i] = w[i - 1];
                        sl = sl + 1 == K ? 0 : sl + 1;
                        gp += CC;
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
                        for (int k = 1; k <= i && k <= K; ++k) {
                            if (k > k0 && k <= k0 + KPT) {
                                const double gu = p.G3[(size_t)(k - 1) * CC + pair] * ring[((tt + k) % K) * C + c];
                                bs[i] += gu;
                                if (ACC) {
#pragma unroll
                                    for (int kk = 0; kk < (KPT < MBT ? KPT : MBT - 1); ++kk)
                                        if (kk == k - 1 - k0) acc[kk] = fma(coef[i], gu, acc[kk]);
                                }
                            }
                        }
                        red[ks * CC + pair] = bs[i] * ie[i];
                    }
                    __syncthreads();
                    if (tid < C) {
                        double bsum = 0.0, osum = 0.0;
                        for (int q = 0; q < NKS; ++q) {
                            const double *rq = red + q * CC;
                            for (int o = 0; o < C; ++o) {
                                bsum += rq[tid * C + o];
                                if (ACC) osum = fma(av[i * C + o], rq[o * C + tid], osum);
                            }
                        }
                        yv[tid] = bsum;
                        ring[(tt % K) * C + tid] = bsum * EI[(size_t)tt * C + tid].x;
                        if (ACC) {
                            const double outv = osum * kap[i];
                            const double inv = tt >= 1 ? av[i * C + tid] * bsum * kap[i] : 0.0;
                            p.grad_emis[((size_t)b * p.T + tt) * C + tid] = (float)R;
                            sR += R;
                            R += outv - inv;
                            if (tt == 0) p.out0[(size_t)b * C + tid] = outv;
                        }
                    }
                    __syncthreads();
                }
            }
            const int tlast = t0 - nbk + 1;
            if (mode == 0 && tlast == hi && hi < L) {
                record(p.ckB + ((size_t)b * (N + 1) + hi / Delta) * ckstride);
                if (tid == 0) p.ckYB[(size_t)b * (N + 1) + hi / Delta] = Yb;
            }
            if (mode == 1 && tlast > 0 && (tlast % Delta) == 0) {
                record(p.ckB + ((size_t)b * (N + 1) + tlast / Delta) * ckstride);
                if (tid == 0) p.ckYB[(size_t)b * (N + 1) + tlast / Delta] = Yb;
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
        if (ACC && tid < C) {
            p.tot[((size_t)b * N + chunk) * C + tid] = R;
            p.sumR[((size_t)b * N + chunk) * C + tid] = sR;
        }
    }
    if (ACC && active) {
        double *pg = p.partG + (size_t)blockIdx.x * K * CC;
#pragma unroll
        for (int kk = 0; kk < KPT; ++kk) {
            const int k = k0 + kk + 1;
            if (k <= K) pg[(size_t)(k - 1) * CC + pair] = acc[kk];
        }
    }
}

// Finalisation: workgroups 0..B-1 per sequence (interval carries and means, as for the
// factorised path), the others sum the per-workgroup marginal sums in workgroup order.
__global__ __launch_bounds__(NT) void k_dt_fin(Params p)
{
    if ((int)blockIdx.x < p.B) {
        fin_seq_body(p, blockIdx.x);
        return;
    }
    const size_t n = (size_t)p.K * p.C * p.C;
    const size_t i = (size_t)(blockIdx.x - p.B) * NT + threadIdx.x;
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
