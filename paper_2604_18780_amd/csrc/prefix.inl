// Eq. 1 and Eq. 2: tables, per-sequence baseline, centred prefix sums, block exponents and the (ES, 1/ES) pairs.
// Included by semicrf.hip inside its anonymous namespace (after common.h); not a translation unit of its own.

// ---------------------------------------------------------------------------
// exp(dur), exp(trans) in fp64 and the maxima that bound per-step growth.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void tables_body(const Params &p)
{
    __shared__ double red[2 * (NT / 64)];
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
    // maxima: inside each wave by shuffles, then over the waves (any order)
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        mxd = fmax(mxd, __shfl_xor(mxd, off));
        mxt = fmax(mxt, __shfl_xor(mxt, off));
    }
    if ((tid & 63) == 0) {
        red[tid >> 6] = mxd;
        red[NT / 64 + (tid >> 6)] = mxt;
    }
    __syncthreads();
    if (tid < 2) {
        double m = red[tid * (NT / 64)];
        for (int i = 1; i < NT / 64; ++i) m = fmax(m, red[tid * (NT / 64) + i]);
        p.tabmax[tid] = m;
    }
}

// ---------------------------------------------------------------------------
// Eq. 1, stage 1: per-chunk column sums (fp64) and |f| maxima.  grid (NCH, B).
// ---------------------------------------------------------------------------
template <int ET>
__device__ __forceinline__ void colsum_body(const Params &p, const int b, const int ch)
{
    __shared__ double red[NT];
    __shared__ double redm[2 * (NT / 64)];
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
    // the maxima first inside each wave (threads that took no row hold zeros; a maximum does not care for order)
    double mp = mps + mpe;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        mx = fmax(mx, __shfl_xor(mx, off));
        mp = fmax(mp, __shfl_xor(mp, off));
    }
    red[tid] = acc;
    if ((tid & 63) == 0) {
        redm[tid >> 6] = mx;
        redm[NT / 64 + (tid >> 6)] = mp;
    }
    __syncthreads();
    if (tid < C) {
        double s = 0.0;
        for (int i = 0; i < R; ++i) s += red[i * C + tid];
        p.chsum[((size_t)b * p.NCH + ch) * C + tid] = s;
    }
    if (tid == 0) {
        double m = 0.0, q = 0.0;
        for (int i = 0; i < NT / 64; ++i) {
            m = fmax(m, redm[i]);
            q = fmax(q, redm[NT / 64 + i]);
        }
        p.chmax[(size_t)b * p.NCH + ch] = m + 2.0 * q;  // |start| + |end| bounded by twice the larger sum
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
constexpr int PREP_NT = 1024;  // one workgroup per sequence: as many threads as a workgroup may have
__global__ __launch_bounds__(PREP_NT) void k_prep_seq(Params p)
{
    // The chunks are split into G = PREP_NT/C contiguous ranges, one per thread group; range sums
    // are combined in range order (a fixed order for a given problem).
    __shared__ double gsum[PREP_NT];
    __shared__ double red[PREP_NT / 64];
    __shared__ double nu_s[256];  // C <= 256
    const int b = blockIdx.x, tid = threadIdx.x;
    const int C = p.C, L = seq_len(p, b), NCH = p.NCH;
    const int G = PREP_NT / C;
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
    for (int ch = tid; ch < NCH; ch += PREP_NT) fm = fmax(fm, p.chmax[(size_t)b * NCH + ch]);
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) fm = fmax(fm, __shfl_xor(fm, off));  // a maximum: any order
    if ((tid & 63) == 0) red[tid >> 6] = fm;
    __syncthreads();
    if (tid == 0) {
        fm = 0.0;
        for (int i = 0; i < PREP_NT / 64; ++i) fm = fmax(fm, red[i]);
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

