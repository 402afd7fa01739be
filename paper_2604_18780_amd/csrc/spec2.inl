// The chunk-parallel scan tasks with TWO waves per task.
// Included by semicrf.hip inside its anonymous namespace (after spec.inl); not a translation unit of its own.

// ---------------------------------------------------------------------------
// A one-wave scan task (spec.inl) issues about 135 instructions per position, and how fast a
// compute unit's SIMDs issue the instructions of the few waves they hold is what bounds it.
// Here a task is a workgroup of two waves that share the task's LDS window:
//   * the TIP runs the positions' dependent chains (product with ES, transition product, division)
//     and adds what the newest MB window entries and the block's own positions contribute
//     (durations 1 .. 2MB-1, from registers);
//   * the HELPER adds up, one block AHEAD, what all older window entries contribute to the MB
//     positions of the next block (durations > MB: every entry it needs is known before the tip
//     starts the current block), and hands the MB sums per label over through LDS.
// Each wave's stream is about half as long, four waves instead of two share a SIMD, and the
// helper's work is off the tip's chain.  One LDS-only workgroup barrier per block of MB positions.
// At a scaling-block boundary the tip publishes the exponent it found and scales its own registers;
// the helper rescales the window rows (the tip only writes rows the helper does not touch).  The
// helper also moves the window back when the linear buffer's end is reached.  Both waves walk the
// same sequence of blocks, so they execute the same barriers; checkpoints, stored rows and
// verification are those of the one-wave task.
// ---------------------------------------------------------------------------
template <int CT, int NKW>
__host__ __device__ constexpr size_t spec2_lds_doubles()
{
    const int CTP = pow2_ge8(CT);
    const int KW = wave_nk(CT, NKW) * (64 / CTP);
    // window rows + MB spare rows at both ends (the helper's window starts MB rows behind the newest row),
    // the message vector, two sets of MB far sums per label, the published exponent
    return (size_t)(KW + lin_slack(KW) + 2 * MB) * CT + (size_t)(CTP - CT) + (size_t)CTP + (size_t)2 * MB * CTP + 2;
}

template <int CT, int NKW, bool BWD>
__device__ __forceinline__ void spec2_task(const Params &p, double *lds_raw, const int b, const int j,
                                           const int warm)
{
    using G = WaveWin<CT, NKW>;
    constexpr int CTP = G::CTP, RS = G::RS, NK = G::NK, KW = G::KW, M = G::M, ROWS = G::ROWS, GW = G::GW;
    constexpr int H = G::H, HC = G::HC;
    constexpr int RTOT2 = (ROWS + 2 * MB) * RS + (CTP - CT);
    const int lane = threadIdx.x & 63;
    const bool tip = threadIdx.x < 64;
    const int K = p.K, C = p.C, KC = K * C;
    double *ring = lds_raw + MB * RS;   // logical row 0 (MB spare rows below, MB above)
    double *yv = lds_raw + RTOT2;       // [CTP]
    double *farb = yv + CTP;            // [2][MB][CTP] what the older window entries add to the next block
    int *exv = (int *)(farb + 2 * MB * CTP);
    const int Delta = p.Delta, N = p.N;
    const size_t ckstride = (size_t)KC + C;
    const int c = lane % CTP, g = lane / CTP;
    const int hh = H == 2 ? (lane >> 5) : 0;
    const bool cval = c < C;
    const int cc = cval ? c : 0;
    const SeqHdr h = p.hdr[b];
    const int L = h.L, J = h.J, Jm = J - 1;
    const int lo = j * Delta;
    if (lo >= L) return;   // both waves
    const int hi = min(lo + Delta, L);
    const size_t row0 = (size_t)b * (p.T + 1);
    const int *nbc = p.nbase + row0 * C + cc;
    const int s0 = BWD ? min(hi + warm, L) : max(lo - warm, 0);
    const int tstart = BWD ? hi : lo;   // where the chunk proper begins (state -> ck1)
    const int tend = BWD ? lo : hi;

    // ---- what both waves compute alike: the sequence of blocks and the window's row
    auto block_len = [&](const int tcur) {  // positions the block starting after tcur may take
        int nb = BWD ? tcur - tend : tend - tcur;
        nb = min(nb, MB);
        // only the first position of a block may cross a scaling-block boundary
        nb = min(nb, BWD ? ((tcur - 1) & Jm) + 1 : J - ((tcur + 1) & Jm));
        // the position where the chunk proper starts ends its block (its state is recorded)
        if (BWD ? tcur > tstart : tcur < tstart) nb = min(nb, BWD ? tcur - tstart : tstart - tcur);
        return nb;
    };
    auto at_boundary = [&](const int tcur) { return BWD ? (tcur & Jm) == 0 : ((tcur + 1) & Jm) == 0; };
    auto must_move = [&](const int rcur) { return BWD ? rcur < MB : rcur + MB > ROWS - 1; };
    // exponent step n_j(c) - n_{j-1}(c) of the lane's label at the scaling-block boundary j*J; the
    // one of the next boundary in the scan's direction is loaded one block of J early
    auto nbdelta = [&](const int jb) {
        return (jb >= 1 && (long)jb * J <= (long)L) ? nbc[(size_t)jb * C] - nbc[(size_t)(jb - 1) * C] : 0;
    };

    // ---- start: the state of a sequence that begins (forward) / ends (backward) at s0
    for (int i = threadIdx.x; i < RTOT2; i += 128) lds_raw[i] = 0.0;
    for (int i = threadIdx.x; i < CTP + 2 * MB * CTP; i += 128) yv[i] = 0.0;
    lds_barrier();
    int r = BWD ? M : KW - 1;  // row of the newest message
    int t = s0;
    int jnx = BWD ? s0 / J : s0 / J + 1;
    int dnx = nbdelta(jnx);
    int nblk = 0;

    if (tip) {
        // ================================ the tip ================================
        const double2 *EIc = p.EI + row0 * C + cc;
        double wn[2 * MB - 1];   // W[1 .. 2MB-1, c]: durations inside a block and back to the MB newest entries
#pragma unroll
        for (int jj = 0; jj < 2 * MB - 1; ++jj) wn[jj] = (cval && jj + 1 <= K) ? p.W[(size_t)jj * C + c] : 0.0;
        double Ereg[HC];
#pragma unroll
        for (int i = 0; i < HC; ++i) {
            const int o = hh * HC + i;
            const bool ok = cval && o < C;
            Ereg[i] = ok ? (BWD ? p.Etr[(size_t)c * C + o] : p.Etr[(size_t)o * C + c]) : 0.0;
        }
        const double2 *ys = (const double2 *)__builtin_assume_aligned(yv + hh * HC, 16);
        double Y = 0.0;
        {
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
        auto record = [&](const int tt, double *ck, double *ckY) {
            const int tm = tt % K;
            if (cval) {  // lane (g, c): the window rows at distances g, g + GW, ... of its label (no index divisions)
#pragma unroll 4
                for (int d = g; d < K; d += G::GW) {
                    int sl = BWD ? tm + d : tm - d;  // slot of the position at that distance
                    sl += BWD ? (sl >= K ? -K : 0) : (sl < 0 ? K : 0);
                    ck[(size_t)sl * C + c] = ring[(BWD ? r + d : r - d) * RS + c];
                }
            }
            if (lane < C) ck[KC + lane] = yv[lane];
            if (lane == 0) *ckY = Y;
        };
        double *ck1 = (BWD ? p.ckB : p.ckA) + ((size_t)b * (N + 1)) * ckstride;
        double *ck2 = (BWD ? p.ckB2 : p.ckA2) + ((size_t)b * (N + 1)) * ckstride;
        double *ckY1 = (BWD ? p.ckYB : p.ckYA) + (size_t)b * (N + 1);
        double *ckY2 = (BWD ? p.ckYB2 : p.ckYA2) + (size_t)b * (N + 1);
        const int istart = BWD ? j + 1 : j, iend = BWD ? j : j + 1;
        // rows for the interval stage / the stored-row marginals, as in the one-wave task
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
        auto load_rows = [&](double2 (&e)[MB], const int tfrom) {  // rows of the MB positions after tfrom
#pragma unroll
            for (int i = 0; i < MB; ++i) {
                const int tt = BWD ? max(tfrom - 1 - i, tend) : min(tfrom + 1 + i, tend);
                e[i] = EIc[(size_t)tt * C];
            }
        };
        double2 e[MB];
        load_rows(e, t);
        lds_barrier();  // start: the helper may read the window
        while (t != tend) {
            const int nb = block_len(t);
            const int tn = BWD ? t - nb : t + nb;
            double2 en[MB];
            load_rows(en, tn);
            if (__builtin_expect(must_move(r), 0)) {
                lds_barrier();   // the helper moves the window back
                lds_barrier();
                r = BWD ? M : KW - 1;
            }
            const bool inchunk = keep && (BWD ? t <= tstart : t >= tstart);  // blocks end at tstart: holds for the whole block
            // what the window adds to this block: the helper's sums over the older entries, and the MB newest entries
            double far[MB], qp[MB];
            const double *fb = farb + (nblk & 1) * MB * CTP + c;
#pragma unroll
            for (int i = 0; i < MB; ++i) {
                far[i] = fb[i * CTP];
                qp[i] = ring[(BWD ? r + i : r - i) * RS + c];   // message of the position i before this block
            }
            if (__builtin_expect(at_boundary(t), 0)) {
                // sum of the newest message vector, one entry per lane, added up across the wave (the same value in
                // every lane; only its exponent is used, and any power of two would do: scaling is exact)
                // (a short vector is summed faster entry by entry)
                double prevsum = 0.0;
                if (CT >= 32) {
                    prevsum = lane < CT ? yv[lane] : 0.0;
#pragma unroll
                    for (int off = 1; off < 64; off <<= 1) prevsum += __shfl_xor(prevsum, off);
                } else {
                    for (int i = 0; i < CT; ++i) prevsum += yv[i];
                }
                const int ex = safe_exponent(prevsum);
                Y += (double)ex;
                if (lane == 0) exv[0] = ex;
                const int sft = dnx - ex;
#pragma unroll
                for (int i = 0; i < MB; ++i) {
                    far[i] = fmin(ldexp(far[i], sft), DBL_MAX);
                    qp[i] = fmin(ldexp(qp[i], sft), DBL_MAX);
                }
                jnx += BWD ? -1 : 1;
                dnx = nbdelta(jnx);
                lds_barrier();   // the exponent is published (and the window entries above were read before it is rescaled)
            }
            double qn[MB];
#pragma unroll
            for (int i = 0; i < MB; ++i) {
                if (i < nb) {
                    double x = far[i];
#pragma unroll
                    for (int m = 0; m < MB; ++m) x = fma(wn[i + m], qp[m], x);        // duration i + 1 + m
#pragma unroll
                    for (int jn = 0; jn < i; ++jn) x = fma(wn[i - 1 - jn], qn[jn], x);  // inside the block
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
                    if (writer) ring[(BWD ? r - 1 - i : r + 1 + i) * RS + c] = q;
                    if (!BWD && inchunk && t + 1 + i < hi) {
                        if (writer) store_row(aloc + (size_t)(t + 1 + i - lo) * C + c, y, q);
                        if (lane == 0) alocY[t + 1 + i - lo] = Y - Yrec;
                    }
                    if (BWD && inchunk) {  // position t - 1 - i of [lo, hi)
                        if (writer) store_row(aloc + (size_t)(t - 1 - i - lo) * C + c, y, q);
                        if (lane == 0) alocY[t - 1 - i - lo] = Y - Yrec;
                    }
                    lds_wave_fence();
                } else {
                    qn[i] = 0.0;
                }
            }
            lds_barrier();   // end of the block: the new window rows and the helper's sums for the next block are there
            r += BWD ? -nb : nb;
            t = tn;
            ++nblk;
#pragma unroll
            for (int i = 0; i < MB; ++i) e[i] = en[i];
            if (__builtin_expect(t == tstart, 0)) {
                record(t, ck1 + (size_t)istart * ckstride, ckY1 + istart);
                start_rows();
            }
        }
        record(tend, ck2 + (size_t)iend * ckstride, ckY2 + iend);
    } else {
        // ================================ the helper ================================
        double wx[NK + MB - 1];  // W[g*NK + jj + MB + 1, c]: entry at distance g*NK + jj behind the window's base
#pragma unroll
        for (int jj = 0; jj < NK + MB - 1; ++jj) {
            const int k = g * NK + jj + MB + 1;
            wx[jj] = (cval && k <= K) ? p.W[(size_t)(k - 1) * C + c] : 0.0;
        }
        lds_barrier();  // start
        while (t != tend) {
            const int nb = block_len(t);
            const int tn = BWD ? t - nb : t + nb;
            if (__builtin_expect(must_move(r), 0)) {
                lds_barrier();
                r = G::template move<BWD>(ring, lane, r);
                lds_barrier();
            }
            if (__builtin_expect(at_boundary(t), 0)) {
                lds_barrier();   // the tip has published the exponent and read the newest entries
                const int sft = dnx - exv[0];
                jnx += BWD ? -1 : 1;
                dnx = nbdelta(jnx);
                // the KW rows that can still contribute, each lane its own label's column; the rows the tip
                // writes in this block lie beyond r and are already in the new frame
                if (cval) {
#pragma unroll 8
                    for (int d = g; d < KW; d += GW) {
                        double *q = ring + (BWD ? r + d : r - d) * RS + c;
                        *q = fmin(ldexp(*q, sft), DBL_MAX);
                    }
                }
                lds_wave_fence();
            }
            // what the entries at least MB positions before the NEXT block's base add to its MB positions
            // (the base is the last position of this block; its newest MB predecessors are the tip's)
            {
                const int rb = BWD ? r - nb + MB : r + nb - MB;   // row of the newest entry that is the helper's
                const double *base = ring + rb * RS + (BWD ? g * NK * RS + c : -(g * NK + NK - 1) * RS + c);
                double acc[MB];
#pragma unroll
                for (int i = 0; i < MB; ++i) acc[i] = 0.0;
#pragma unroll
                for (int jj = 0; jj < NK; ++jj) {
                    const double v = base[(BWD ? jj : NK - 1 - jj) * RS];  // distance g*NK + jj behind rb
#pragma unroll
                    for (int i = 0; i < MB; ++i) acc[i] = fma(wx[jj + i], v, acc[i]);
                }
#pragma unroll
                for (int i = 0; i < MB; ++i) acc[i] = group_sum<CTP>(acc[i]);
                double *fb = farb + ((nblk + 1) & 1) * MB * CTP + c;
                if (g == 0) {
#pragma unroll
                    for (int i = 0; i < MB; ++i) fb[i * CTP] = acc[i];
                }
            }
            lds_barrier();   // end of the block
            r += BWD ? -nb : nb;
            t = tn;
            ++nblk;
        }
    }
}

// Waves per SIMD the register allocation aims at: four (two tasks) where both roles fit 128 registers.
constexpr int spec2_waves_per_simd(int CT, int NKW) { return (CT <= 32 && NKW <= 32) ? 4 : 2; }

template <int CT, int NKW>
__global__ __launch_bounds__(128, spec2_waves_per_simd(CT, NKW)) void k_spec2(Params p, int both, int warm, int tier, int rest)
{
    extern __shared__ double lds_raw[];
    const int ndir = both ? 2 : 1;
    const int dir = blockIdx.x % ndir;
    const int task = blockIdx.x / ndir;
    const int b = task / p.N, j = task % p.N;
    if (tier > 0 && p.spec_ok[b * 2 + dir]) return;  // accepted by an earlier attempt
    if (rest && p.hdr[b].J >= MS_JMIN) return;
    if (dir == 0) spec2_task<CT, NKW, false>(p, lds_raw, b, j, warm);
    else spec2_task<CT, NKW, true>(p, lds_raw, b, j, warm);
}
