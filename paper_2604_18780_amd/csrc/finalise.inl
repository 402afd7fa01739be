// Fixed-order reductions of the gradient formulas: per-sequence sums, the emission gradient and the position marginals.
// Included by semicrf.hip inside its anonymous namespace (after common.h); not a translation unit of its own.

// ---------------------------------------------------------------------------
// Finalisation (fixed-order reductions).
// ---------------------------------------------------------------------------
// Positions per partial sum of sequence b: an interval, or a part of one where the one-wave stored-row marginals
// took the sequence (the condition under which that kernel works on it).
__device__ __forceinline__ int stat_delta(const Params &p, const int b)
{
    return (p.msplit > 1 && p.spec_ok[b * 2] && p.spec_ok[b * 2 + 1]) ? p.Delta / p.msplit : p.Delta;
}

// carry[b,i,c] = sum_{i'<=i} tot[b,i',c] and the sums behind mean[b,c] = (1/L) sum_u pm[b,u,c].  FIN_FS workgroups
// per sequence, each a contiguous slice of the sequence's partial sums (it first adds up, label by label, what
// lies before its slice).  Inside a workgroup the partial sums are split into G = NT/C contiguous chunks, one per
// thread group; chunk sums are combined in chunk order, so the result does not depend on the launch shape.
// mean is left as FIN_FS sums per label; k_fin_emis adds them and divides.
constexpr int FIN_FS = FIN_SLICES;
__device__ __forceinline__ void fin_seq_body(const Params &p, const int b, const int s)
{
    __shared__ double gsum[NT];
    __shared__ double gtot[NT];
    const int C = p.C, N = p.NP, tid = threadIdx.x;
    const int L = p.hdr[b].L;
    const int Ds = stat_delta(p, b);
    const int nint = (L + Ds - 1) / Ds;
    const int G = NT / C;
    const int g = tid / C, c = tid % C;
    const bool act = g < G;
    const int per_s = (nint + FIN_FS - 1) / FIN_FS;
    const int s0 = min(s * per_s, nint), s1 = min(s0 + per_s, nint);
    const double *tot = p.tot + ((size_t)b * N) * C + c;
    // what lies before the slice
    {
        const int per = (s0 + G - 1) / G;
        const int a0 = min(g * per, s0), a1 = min(a0 + per, s0);
        double pre = 0.0;
        if (act) {
#pragma unroll 8
            for (int i = a0; i < a1; ++i) pre += tot[(size_t)i * C];
        }
        gsum[tid] = pre;
    }
    __syncthreads();
    double run = 0.0;
    if (act)
        for (int gg = 0; gg < G; ++gg) run += gsum[gg * C + c];
    __syncthreads();
    // the slice
    const int per = (s1 - s0 + G - 1) / G;
    const int i0 = min(s0 + g * per, s1), i1 = min(i0 + per, s1);
    double loc = 0.0;
    if (act) {
#pragma unroll 8
        for (int i = i0; i < i1; ++i) loc += tot[(size_t)i * C];
    }
    gsum[tid] = loc;
    __syncthreads();
    double total = 0.0;
    if (act) {
        for (int gg = 0; gg < g; ++gg) run += gsum[gg * C + c];
#pragma unroll 8
        for (int i = i0; i < i1; ++i) {
            const size_t o = ((size_t)b * N + i) * C + c;
            run += p.tot[o];
            p.carry[o] = run;
            const int n = min(Ds, L - i * Ds);
            total += (double)n * run - p.sumR[o];
        }
    }
    gtot[tid] = total;
    __syncthreads();
    if (tid < C) {
        double t = 0.0;
        for (int gg = 0; gg < G; ++gg) t += gtot[gg * C + tid];
        p.mean[((size_t)b * FIN_FS + s) * C + tid] = t;
    }
    // boundary posterior: certain at both ends of the sequence, nothing beyond it (the interval
    // kernels wrote positions 1 .. L-1)
    if (p.bdy_post && s == 0) {
        float *bd = p.bdy_post + (size_t)b * (p.T + 1);
        for (int t = tid; t <= p.T; t += NT)
            if (t == 0 || t >= L) bd[t] = (t == 0 || t == L) ? 1.f : 0.f;
    }
}

// Gradients of the scalar sequence boundaries: sums over sequences, in sequence order, of the
// mass of the segments that start at position 0 / end at position L.  One workgroup.
__device__ __forceinline__ void fin_pi_body(const Params &p)
{
    const int c = threadIdx.x;
    if (c >= p.C) return;
    double gs = 0.0, ge = 0.0;
    for (int b = 0; b < p.B; ++b) {
        if (p.hdr[b].L < 1) continue;
        const double w = p.grad_logz ? (double)p.grad_logz[b] : 1.0;
        gs = fma(w, p.out0[(size_t)b * p.C + c], gs);
        ge = fma(w, p.inL[(size_t)b * p.C + c], ge);
    }
    if (p.g_pi_start) p.g_pi_start[c] = (float)gs;
    if (p.g_pi_end) p.g_pi_end[c] = (float)ge;
}

// grad_emis / pos_marg, elementwise over (u,c) of one sequence.  grid (blocks, B).
// V = 4: four labels of one position per thread as 16-byte accesses (C a multiple of 4, outputs 16-byte aligned,
// fewer than 2^31 elements per sequence, no boundary projections among the outputs); V = 1: the general form.
template <int V>
__global__ __launch_bounds__(NT) void k_fin_emis(Params p)
{
    const int b = blockIdx.y, C = p.C;
    const int L = p.hdr[b].L;
    const double w = p.grad_logz ? (double)p.grad_logz[b] : 1.0;
    const size_t n = (size_t)p.T * C;  // elements of one sequence
    const size_t base = (size_t)b * n;
    const double *carry = p.carry + ((size_t)b * p.NP) * C;
    const int Ds = stat_delta(p, b);
    __shared__ double mean[GRAD_CMAX];
    if ((int)threadIdx.x < C) {
        double t = 0.0;
        for (int s = 0; s < FIN_FS; ++s) t += p.mean[((size_t)b * FIN_FS + s) * C + threadIdx.x];
        mean[threadIdx.x] = (p.center && L > 0) ? t / (double)L : 0.0;
    }
    __syncthreads();
    if (V == 4) {
        const unsigned Cq = (unsigned)C / 4u, nq = (unsigned)(n / 4), step = gridDim.x * NT;
        float4 *ge4 = (float4 *)(p.grad_emis + base);
        float4 *pm4 = p.pos_marg ? (float4 *)(p.pos_marg + base) : nullptr;
        for (unsigned q = blockIdx.x * NT + threadIdx.x; q < nq; q += step) {
            const unsigned u = q / Cq, c = (q - u * Cq) * 4u;
            float4 ge = make_float4(0.f, 0.f, 0.f, 0.f), pmv = ge;
            if ((int)u < L) {
                const double *cr = carry + (size_t)(u / (unsigned)Ds) * C + c;
                const float4 r = ge4[q];
                const double pm0 = cr[0] - (double)r.x, pm1 = cr[1] - (double)r.y;
                const double pm2 = cr[2] - (double)r.z, pm3 = cr[3] - (double)r.w;
                ge = make_float4((float)(w * (pm0 - mean[c])), (float)(w * (pm1 - mean[c + 1])),
                                 (float)(w * (pm2 - mean[c + 2])), (float)(w * (pm3 - mean[c + 3])));
                pmv = make_float4((float)pm0, (float)pm1, (float)pm2, (float)pm3);
            }
            ge4[q] = ge;
            if (pm4) pm4[q] = pmv;
        }
        return;
    }
    auto one = [&](const size_t idx, const int u, const int c) {
        float ge = 0.f, pmv = 0.f;
        if (u < L) {
            const int i = u / Ds;
            const double pm = carry[(size_t)i * C + c] - (double)p.grad_emis[base + idx];
            ge = (float)(w * (pm - mean[c]));
            pmv = (float)pm;
        }
        p.grad_emis[base + idx] = ge;
        if (p.pos_marg) p.pos_marg[base + idx] = pmv;
        // boundary projections: rows beyond the sequence are zero; the last token's end score
        // belongs to the segments that end at position L
        if (p.g_proj_start && u >= L) p.g_proj_start[base + idx] = 0.f;
        if (p.g_proj_end && u >= L - 1)
            p.g_proj_end[base + idx] = u == L - 1 ? (float)(w * p.inL[(size_t)b * C + c]) : 0.f;
    };
    if (n < ((size_t)1 << 31)) {  // 32-bit index arithmetic
        const unsigned n32 = (unsigned)n, step = gridDim.x * NT;
        for (unsigned idx = blockIdx.x * NT + threadIdx.x; idx < n32; idx += step) {
            const unsigned u = idx / (unsigned)C;
            one(idx, (int)u, (int)(idx - u * (unsigned)C));
        }
    } else {
        for (size_t idx = (size_t)blockIdx.x * NT + threadIdx.x; idx < n; idx += (size_t)gridDim.x * NT)
            one(idx, (int)(idx / C), (int)(idx % C));
    }
}

// Launch of k_fin_emis in the form the sizes and outputs allow.
inline void launch_fin_emis(const Params &p, hipStream_t st)
{
    const size_t n = (size_t)p.T * p.C;
    const bool vec = p.C % 4 == 0 && n < ((size_t)1 << 31) && !p.g_proj_start && !p.g_proj_end &&
                     ((uintptr_t)p.grad_emis & 15) == 0 && ((uintptr_t)p.pos_marg & 15) == 0;
    size_t blocks = ((vec ? n / 4 : n) + NT - 1) / NT;
    if (blocks > 16384) blocks = 16384;
    if (vec) hipLaunchKernelGGL(k_fin_emis<4>, dim3((unsigned)blocks, p.B), dim3(NT), 0, st, p);
    else hipLaunchKernelGGL(k_fin_emis<1>, dim3((unsigned)blocks, p.B), dim3(NT), 0, st, p);
}

// grad_trans[c',c] = Etr[c',c] * sum_b w_b sum_i partTr;  grad_dur[k,c] = sum_b w_b sum_i partD.
// One workgroup per FIN_PO outputs; NT / FIN_PO thread groups take the partial sums i = g, g + groups, ... and
// their sums are combined in group order (fixed order for a given problem).
constexpr int FIN_PO = 8;  // small: the partial sums of a long sequence are many, the outputs few
__device__ __forceinline__ void fin_params_body(const Params &p, const int blk)
{
    __shared__ double red[NT];
    constexpr int NG = NT / FIN_PO;
    const int C = p.C, CC = C * C, KC = p.K * C, N = p.NP, tid = threadIdx.x;
    const int o = tid % FIN_PO, g = tid / FIN_PO;
    const int idx = blk * FIN_PO + o;
    const bool ok = idx < CC + KC;
    // The number of partial sums of a sequence is fetched once per sequence by the first threads, and the
    // sequences are taken four at a time: the first partial sum each thread group takes of each of them is loaded
    // before any is added (many short sequences would otherwise cost one memory latency each), the rest, for
    // sequences with more partial sums than thread groups, in four chains as before.  Fixed order throughout.
    constexpr int UB = 4;
    __shared__ int npart[NT];
    if (tid < p.B) {
        const int Ds = stat_delta(p, tid);
        npart[tid] = (p.hdr[tid].L + Ds - 1) / Ds;
    }
    __syncthreads();
    auto count = [&](const int b) {
        if (b < NT) return npart[b];
        const int Ds = stat_delta(p, b);
        return (p.hdr[b].L + Ds - 1) / Ds;
    };
    const size_t stride = idx < CC ? (size_t)CC : (size_t)KC;
    const double *q0 = idx < CC ? p.partTr + idx : p.partD + (idx - CC);  // partial sum i of sequence b at (b*N + i)*stride
    double acc = 0.0;
    if (ok) {
        for (int b0 = 0; b0 < p.B; b0 += UB) {
            double v[UB], w[UB];
            int nint[UB];
            bool more = false;
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                const int b = b0 + u;
                nint[u] = b < p.B ? count(b) : 0;
                w[u] = (b < p.B && p.grad_logz) ? (double)p.grad_logz[b] : 1.0;
                v[u] = g < nint[u] ? q0[((size_t)b * N + g) * stride] : 0.0;
                more = more || nint[u] > NG;
            }
            if (more) {
#pragma unroll
                for (int u = 0; u < UB; ++u) {
                    const double *q = q0 + ((size_t)(b0 + u) * N) * stride;
                    double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
                    int i = g + NG;
                    for (; i + 3 * NG < nint[u]; i += 4 * NG) {
                        s0 += q[(size_t)i * stride];
                        s1 += q[(size_t)(i + NG) * stride];
                        s2 += q[(size_t)(i + 2 * NG) * stride];
                        s3 += q[(size_t)(i + 3 * NG) * stride];
                    }
                    for (; i < nint[u]; i += NG) s0 += q[(size_t)i * stride];
                    v[u] += (s0 + s1) + (s2 + s3);
                }
            }
#pragma unroll
            for (int u = 0; u < UB; ++u) acc = fma(w[u], v[u], acc);
        }
    }
    red[tid] = acc;
    __syncthreads();
    if (ok && g == 0) {
        double t = 0.0;
        for (int gg = 0; gg < NG; ++gg) t += red[gg * FIN_PO + o];
        if (idx < CC) p.grad_trans[idx] = (float)(t * p.Etr[idx]);
        else p.grad_dur[idx - CC] = (float)t;
    }
}

// One launch for the two independent reductions: FIN_FS workgroups per sequence, the rest
// per FIN_PO parameter gradients.
__global__ __launch_bounds__(NT) void k_fin_seq(Params p)
{
    const int nparam = (p.C * p.C + p.K * p.C + FIN_PO - 1) / FIN_PO;
    const int nseq = p.B * FIN_FS;
    if ((int)blockIdx.x < nseq) fin_seq_body(p, blockIdx.x / FIN_FS, blockIdx.x % FIN_FS);
    else if ((int)blockIdx.x < nseq + nparam) fin_params_body(p, blockIdx.x - nseq);
    else fin_pi_body(p);
}

// Entropies of the posteriors (the paper's boundary-entropy paragraph): per sequence,
//   h_pos = (1/L) sum_{u<L} -sum_c pm[u,c] ln pm[u,c]          (mean per-position label entropy)
//   h_bdy = -sum_{u<L} ph_u ln ph_u,  ph_u = bdy[u] / sum_{u'<L} bdy[u']   (entropy of the normalised
//           segment-start distribution; a segment starts at token u iff a boundary falls at position u)
// One workgroup per sequence; thread partial sums are combined in thread order.
__global__ __launch_bounds__(NT) void k_entropies(const float *pos_marg, const float *bdy_post,
                                                  const int32_t *lengths, int T, int C, float *h_pos,
                                                  float *h_bdy)
{
    __shared__ double red[NT];
    const int b = blockIdx.x, tid = threadIdx.x;
    int L = lengths ? lengths[b] : T;
    L = L < 0 ? 0 : (L > T ? T : L);
    auto block_sum = [&](double v) {
        red[tid] = v;
        __syncthreads();
        double s = 0.0;
        if (tid == 0)
            for (int i = 0; i < NT; ++i) s += red[i];
        __syncthreads();
        if (tid == 0) red[0] = s;
        __syncthreads();
        s = red[0];
        __syncthreads();
        return s;
    };
    if (h_pos) {
        const float *pm = pos_marg + (size_t)b * T * C;
        double acc = 0.0;
        for (size_t i = tid; i < (size_t)L * C; i += NT) {
            const double x = (double)pm[i];
            if (x > 0.0) acc -= x * log(x);
        }
        const double tot = block_sum(acc);
        if (tid == 0) h_pos[b] = L > 0 ? (float)(tot / (double)L) : 0.f;
    }
    if (h_bdy) {
        const float *bd = bdy_post + (size_t)b * (T + 1);
        double acc = 0.0;
        for (int u = tid; u < L; u += NT) acc += (double)bd[u];
        const double norm = block_sum(acc);
        acc = 0.0;
        for (int u = tid; u < L; u += NT) {
            const double x = (double)bd[u] / norm;
            if (x > 0.0) acc -= x * log(x);
        }
        const double tot = block_sum(acc);
        if (tid == 0) h_bdy[b] = L > 0 ? (float)tot : 0.f;
    }
}

