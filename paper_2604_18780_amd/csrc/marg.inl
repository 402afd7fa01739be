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
constexpr int MG_TG = 32;  // positions staged at a time
constexpr int MG_KS = 16;  // durations per thread of the duration kernel

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

// Duration-bias statistics.  Thread (ks, c): label c, durations ks*16 + 1 .. ks*16 + 16, one
// accumulator each.  Positions are taken in groups inside one scaling block: the group's q rows
// and the v rows it can reach are staged in LDS, the latter converted to the group's frame with
// all exponents combined before anything is formed; four positions share every LDS read.
__global__ __launch_bounds__(1024) void k_mg_dur(Params p)
{
    extern __shared__ double lds_raw[];
    const int tid = threadIdx.x;
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
    double *Vp = Qrow + MG_TG * C;     // [VR][C]
    const size_t row0 = (size_t)b * (p.T + 1);
    const double2 *EI = p.EI + row0 * C;
    const int *nb = p.nbase + row0 * C;
    const double2 *frow = (const double2 *)p.aloc + ((size_t)b * N) * Delta * C;  // row of position t at t*C
    const double2 *brow = (const double2 *)p.bloc + ((size_t)b * N) * Delta * C;  // (slots are consecutive)
    const double logZ = h.logZ;
    double acc[MG_KS];
#pragma unroll
    for (int kk = 0; kk < MG_KS; ++kk) acc[kk] = 0.0;

    for (int tg0 = lo; tg0 < hi;) {
        const int tg1 = min(min(hi, (tg0 / J + 1) * J), tg0 + MG_TG);
        const int ng = tg1 - tg0, jt = tg0 / J;
        const double yA0 = mg_ya(p, b, iv, tg0 - lo);
        __syncthreads();  // the previous group is done with the staged rows
        for (int i = tid; i < MG_TG * C; i += blockDim.x) {
            const int r = i / C, o = i % C;
            double q = 0.0;
            if (r < ng) q = frow[(size_t)(tg0 + r) * C + o].y * exp2(mg_ya(p, b, iv, tg0 + r - lo) - yA0);
            Qrow[i] = q;
        }
        for (int i = tid; i < VR * C; i += blockDim.x) {
            const int r = i / C, o = i % C, s = tg0 + 1 + r;
            double v = 0.0;
            if (s <= L && r < ng + K) {
                double vs, yB;
                if (s == L) {  // b_L = 1: v_L = ES_L, scale 0
                    vs = EI[(size_t)L * C + o].x;
                    yB = 0.0;
                } else {
                    vs = brow[(size_t)s * C + o].y;
                    yB = mg_yb(p, b, s / Delta, s % Delta, L);
                }
                const double lf = (yA0 + yB) - logZ * LOG2E;
                const double fl = floor(lf);
                const int sh = nb[(size_t)(s / J) * C + o] - nb[(size_t)jt * C + o];
                const double ef = fmin(fmax(fl, -100000.0), 100000.0);
                v = fmin(ldexp(vs * exp2(lf - fl), sh + (int)ef), DBL_MAX);
            }
            Vp[i] = v;
        }
        __syncthreads();
        if (active) {
            for (int i0 = 0; i0 < ng; i0 += 4) {
                double ca[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) ca[i] = i0 + i < ng ? Qrow[(i0 + i) * C + c] : 0.0;
                double w[MG_KS + 3];
#pragma unroll
                for (int q = 0; q < MG_KS + 3; ++q) w[q] = Vp[(i0 + kA + q) * C + c];
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
        double *pD = p.partD + ((size_t)b * N + iv) * K * C;
#pragma unroll
        for (int kk = 0; kk < MG_KS; ++kk) {
            const int k = kA + kk + 1;
            if (k <= K) pD[(size_t)(k - 1) * C + c] = acc[kk] * p.W[(size_t)(k - 1) * C + c];
        }
    }
}

// Transition statistics and the running emission sums.  Groups of positions from the interval's
// upper end downwards (the emission sums are suffix sums); per group all threads stage
// a_t kappa, p_t and (out - in) kappa, then every thread adds the group's products for its label
// pairs while threads 0..C-1 walk the group for the running sums.
__global__ __launch_bounds__(1024) void k_mg_te(Params p)
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
    double *AK = lds_raw;            // [MG_TG][C] a_t(c') kappa(t,t)
    double *P = AK + MG_TG * C;      // [MG_TG][C] p_t(c)
    double *D = P + MG_TG * C;       // [MG_TG][C] (out_t - in_t)(c)
    const size_t row0 = (size_t)b * (p.T + 1);
    const double2 *EI = p.EI + row0 * C;
    const double2 *frow = (const double2 *)p.aloc + ((size_t)b * N) * Delta * C;
    const double2 *brow = (const double2 *)p.bloc + ((size_t)b * N) * Delta * C;
    const double logZ = h.logZ;
    double acc[4] = {0.0, 0.0, 0.0, 0.0};  // label pairs tid, tid + blockDim, ... (C <= 64, >= 1024 threads then)
    double R = 0.0, sR = 0.0;

    for (int tg1 = hi; tg1 > lo;) {
        const int tg0 = max(lo, tg1 - MG_TG);
        const int ng = tg1 - tg0;
        __syncthreads();
        for (int i = tid; i < ng * C; i += blockDim.x) {
            const int r = i / C, o = i % C, t = tg0 + r;
            const double2 fa = frow[(size_t)t * C + o], fb = brow[(size_t)t * C + o], e = EI[(size_t)t * C + o];
            const double kap = exp((mg_ya(p, b, iv, t - lo) + mg_yb(p, b, iv, t - lo, L)) * LN2 - logZ);
            AK[i] = fa.x * kap;
            P[i] = fb.x;
            // a segment of label o starts at t (z_t p_t, z = q ES) / ends at t (a_t b_t, b = v IE; none ends at 0)
            D[i] = (fa.y * e.x * fb.x - (t >= 1 ? fa.x * fb.y * e.y : 0.0)) * kap;
        }
        __syncthreads();
#pragma unroll
        for (int n = 0; n < 4; ++n) {
            const int pair = tid + n * (int)blockDim.x;
            if (pair < CC) {
                const int cp = pair / C, c = pair % C;
                double a = acc[n];
                for (int r = 0; r < ng; ++r) a = fma(AK[r * C + cp], P[r * C + c], a);
                acc[n] = a;
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
    double *pT = p.partTr + ((size_t)b * N + iv) * CC;
#pragma unroll
    for (int n = 0; n < 4; ++n) {
        const int pair = tid + n * (int)blockDim.x;
        if (pair < CC) pT[pair] = acc[n];
    }
    if (tid < C) {
        p.tot[((size_t)b * N + iv) * C + tid] = R;
        p.sumR[((size_t)b * N + iv) * C + tid] = sR;
    }
}
