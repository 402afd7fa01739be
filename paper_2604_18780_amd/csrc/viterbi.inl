// Viterbi decode (max semiring): scan, verification, trace-back.
// Included by semicrf.hip inside its anonymous namespace (after common.h); not a translation unit of its own.

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

