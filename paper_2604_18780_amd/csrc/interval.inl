// The interval stage (Algorithm 3 body): generic workgroup kernel, the geometry shared by the one-wave kernels, and the one-wave interval kernel.
// Included by semicrf.hip inside its anonymous namespace (after common.h); not a translation unit of its own.

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

        double *pD = p.partD + ((size_t)b * p.NP + iv) * KC;
        for (int i = tid; i < KC; i += NT) pD[i] = l.accD[i];
        double *pT = p.partTr + ((size_t)b * p.NP + iv) * CC;
#pragma unroll
        for (int j = 0; j < TRP; ++j) {
            const int idx = tid + j * NT;
            if (idx < CC) pT[idx] = accTr[j];
        }
        if (tid < C) {
            p.tot[((size_t)b * p.NP + iv) * C + tid] = R;
            p.sumR[((size_t)b * p.NP + iv) * C + tid] = sR;
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

    // The same for the KW live rows only (newest row r; the window lies behind it in a forward scan, above it in a
    // backward one): the slack rows hold nothing that is read before it is written again.
    template <bool BWD>
    static __device__ __forceinline__ void rescale_live(double *ring, int g, int c, bool cval, int r, int sft)
    {
        if (cval) {
            double *q = ring + ((BWD ? r : r - (KW - 1)) + g) * RS + c;
#pragma unroll 8
            for (int row = g; row < KW; row += GW, q += GW * RS) *q = fmin(ldexp(*q, sft), DBL_MAX);
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
        double *pD = p.partD + ((size_t)b * p.NP + iv) * KC;
        for (int i = lane; i < KC; i += 64) pD[i] = p.W[i] * tmp[(i / C) * CT + i % C];
        lds_wave_fence();
        double *pT = p.partTr + ((size_t)b * p.NP + iv) * CC;
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
            p.tot[((size_t)b * p.NP + iv) * C + lane] = R;
            p.sumR[((size_t)b * p.NP + iv) * C + lane] = sR;
        }
    }
}

