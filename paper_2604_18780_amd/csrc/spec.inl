// The chunk-parallel scans: one-wave scan tasks with warm-up, the repair attempt, verification of the interval boundaries.
// Included by semicrf.hip inside its anonymous namespace (after common.h); not a translation unit of its own.

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
            // sum of the newest message vector (each half of the wave its half of the labels, as in the
            // transition product); only its exponent is used, and any power of two would do: scaling is exact
            double s0 = 0.0, s1 = 0.0;
#pragma unroll
            for (int o = 0; o < HC; o += 2) {
                const double2 vv = ys[o >> 1];
                s0 += vv.x;
                s1 += vv.y;
            }
            double prevsum = s0 + s1;
            if (H == 2) prevsum = add_across_32(prevsum);
            const int ex = safe_exponent(prevsum);
            Y += (double)ex;
            G::template rescale_live<BWD>(ring, g, c, cval, r, dnx - ex);
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
        // A whole block (nearly all are): nothing is decided per position.  The rows of a block that lies in the
        // chunk go out through one pointer per lane (the lanes that own no label store to a sink), its scale once
        // for the MB positions.  A forward block that reaches the chunk's end takes the general path (the end
        // position itself has no row).
        if (__builtin_expect(nb == MB && (BWD || !inchunk || t + MB < hi), 1)) {
            double2 *rowp = (double2 *)p.sink + lane;
            int rstep = 0;
            if (inchunk) {
                const int p0 = BWD ? t - 1 - lo : t + 1 - lo;  // slot row of the block's first position
                if (writer) {
                    rowp = aloc + (size_t)p0 * C + c;
                    rstep = BWD ? -C : C;
                }
                alocY[BWD ? p0 - (lane & (MB - 1)) : p0 + (lane & (MB - 1))] = Y - Yrec;  // every lane, the same value
            }
#pragma unroll
            for (int i = 0; i < MB; ++i) {
                double x = acc[i];
#pragma unroll
                for (int jn = 0; jn < i; ++jn) x = fma(wn[i - 1 - jn], qn[jn], x);
                const double y = x * (BWD ? e[i].y : e[i].x);
                yv[c] = y;  // both lane groups the same value; entries beyond C are zero and nobody reads them
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
                if (keep) store_row(rowp + i * rstep, y, q);
                lds_wave_fence();
            }
        } else {
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

