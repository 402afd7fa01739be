// Chunk-parallel scans of Algorithm 1 and of the beta recurrence of Algorithm 3 on the matrix cores.
#include "common.h"

namespace semicrf_impl {
namespace {

// ---------------------------------------------------------------------------
// Chunk-parallel scans on the matrix cores (17 <= C <= 24 labels, K <= 64).
//
// The one-wave scan tasks of k_spec are bound by how fast one wave issues its instruction
// stream: a position costs about 125 vector instructions for 44 multiply-adds.  Both
// recurrences of Algorithm 1 / Algorithm 3 are linear in the messages with coefficients (W, Etr)
// that all tasks share, so SIXTEEN tasks that advance in lock step turn every step into dense
// products with the task index as the free dimension:
//
//   window      x[i][task] = sum_src  W[k = i - src, c] * q[src][task]          per label c:
//               [16 positions of a time block] x [4 source positions] x [16 tasks], Toeplitz in (i, src)
//   transition  z[c][task] = sum_c'   Etr[c', c]        * a[c'][task]           per position:
//               [16 labels] x [4 labels] x [16 tasks]
//
// i.e. v_mfma_f64_16x16x4_f64 with the tasks as the 16 columns: one instruction does the work of
// sixteen vector multiply-add instructions, a wave alone keeps the fp64 pipe full, and nothing
// of the window has to be read again per position (the K-deep message window is the B operand and
// lives in registers and, for its older half, in LDS).
//
// Organisation.  One workgroup = 4 waves = 16 tasks (same direction).  Wave w owns six labels
// (4w .. 4w+3 and 16+2w, 17+2w).  Two register layouts of a 64-lane register, lane = 16*row + task:
//   "label rows"     row = label (one register per position and label group):     the sequential part
//                    of a step, elementwise work and the B operand of the transition product;
//   "position rows"  row = position within a chunk of 4 (one register per label): the B operand of
//                    the window products and the rows of their accumulators.
// A 4x4 transpose over (register, row) - eight lane swaps - converts a chunk between the two.
// Time runs in blocks of 16 positions (4 chunks).  What older blocks and finished chunks contribute
// to the positions of the current and the next block is accumulated by window products that are
// issued in the shadow of the sequential steps; what the previous chunk and the chunk itself
// contribute (durations 1..7) is added by ordinary multiply-adds in the label-row layout, so a
// window product is never on a position's dependent chain.  Per position each wave forms the partial
// transition product over its own six source labels for all 24 destinations; the partials are
// exchanged through LDS (one workgroup barrier per position) and summed by the wave that owns the
// destination label, in wave order.
//
// Task geometry.  Step n = 0 .. warm + Delta of a forward task is position lo - warm + n, of a backward
// task position lo + Delta + warm - 1 - n; tasks that have less room before (after) them start later
// (their lanes carry zeros until the start position) and a forward task whose interval is cut by the
// sequence end stops early (only its last message vector is kept).  With Delta, warm = 0 mod 32 all
// tasks of a workgroup see scaling-block boundaries at block starts, the checkpoint at the interval's
// near end falls on the first position of a block (forward) or the last one (backward) and the far
// end likewise.  Outputs are exactly those of k_spec (checkpoints, reached states, stored rows), so
// verification, chaining and the interval stage are unchanged.  Sequences whose scaling blocks are
// shorter than 16 positions are left to k_spec.
// ---------------------------------------------------------------------------
typedef double mfma_d4 __attribute__((ext_vector_type(4)));

// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>): loop indices that are constant expressions,
// so that every register array below is indexed by constants by construction
template <class F, int... I>
__device__ __forceinline__ void ms_static_for_impl(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void ms_static_for(F &&f)
{
    ms_static_for_impl(f, std::make_integer_sequence<int, N>{});
}

constexpr int MS_CT = 24;        // labels the layout holds
constexpr int MS_LW = 6;         // labels per wave
constexpr int MS_WT_OFF = 7;     // entry e of a label's weight table holds W[k = e - 7, c] (0 outside 1..K)
constexpr int MS_WT_LEN = 88;    // k = -7 .. 80
#ifndef MS_PFD
#define MS_PFD 2                 // positions the (ES, 1/ES) pairs are requested ahead: 2 or 4
#endif
constexpr int MS_TASKS = 16;     // tasks per workgroup = columns of the matrix instruction

__host__ __device__ constexpr size_t ms_lds_doubles(int NBLK)
{
    return (size_t)MS_CT * MS_WT_LEN + 2 * 4 * 6 * 64 + 64 + 4 * MS_LW * 64 +
           (size_t)4 * (NBLK > 2 ? NBLK - 2 : 0) * 4 * MS_LW * 64;
}

// a.rows{2,3} <-> b.rows{0,1}  (a row is 16 lanes)
__device__ __forceinline__ void rows_swap32(double &a, double &b)
{
    const auto l = __builtin_amdgcn_permlane32_swap((unsigned)__double2loint(a), (unsigned)__double2loint(b), false, false);
    const auto h = __builtin_amdgcn_permlane32_swap((unsigned)__double2hiint(a), (unsigned)__double2hiint(b), false, false);
    a = __hiloint2double((int)h[0], (int)l[0]);
    b = __hiloint2double((int)h[1], (int)l[1]);
}

// a.rows{1,3} <-> b.rows{0,2}
__device__ __forceinline__ void rows_swap16(double &a, double &b)
{
    const auto l = __builtin_amdgcn_permlane16_swap((unsigned)__double2loint(a), (unsigned)__double2loint(b), false, false);
    const auto h = __builtin_amdgcn_permlane16_swap((unsigned)__double2hiint(a), (unsigned)__double2hiint(b), false, false);
    a = __hiloint2double((int)h[0], (int)l[0]);
    b = __hiloint2double((int)h[1], (int)l[1]);
}

// 4x4 transpose over (register index, lane row): on exit x_j holds in row r what x_r held in row j
__device__ __forceinline__ void transpose4(double &x0, double &x1, double &x2, double &x3)
{
    rows_swap32(x0, x2);
    rows_swap32(x1, x3);
    rows_swap16(x0, x1);
    rows_swap16(x2, x3);
}

// out[j] = the value s holds in lane row j, in every row
__device__ __forceinline__ void bcast_rows(const int s, int (&out)[4])
{
    unsigned x0 = (unsigned)s, x1 = (unsigned)s, x2 = (unsigned)s, x3 = (unsigned)s;
    auto a = __builtin_amdgcn_permlane32_swap(x0, x2, false, false);
    x0 = a[0]; x2 = a[1];
    a = __builtin_amdgcn_permlane32_swap(x1, x3, false, false);
    x1 = a[0]; x3 = a[1];
    a = __builtin_amdgcn_permlane16_swap(x0, x1, false, false);
    x0 = a[0]; x1 = a[1];
    a = __builtin_amdgcn_permlane16_swap(x2, x3, false, false);
    x2 = a[0]; x3 = a[1];
    out[0] = (int)x0; out[1] = (int)x1; out[2] = (int)x2; out[3] = (int)x3;
}

__device__ __forceinline__ double ms_scale(const double v, const int s) { return fmin(ldexp(v, s), DBL_MAX); }

// Window products per position of a block: pi = 4*chunk + position.  Mandatory ones first (what finished
// chunks of this block add to the current and the next block), then products with older blocks up to an
// even budget; the block's last position issues none, so that the accumulators of the next block are
// complete when its first rows are taken.
__host__ __device__ constexpr int ms_mandatory(int pi) { return (pi == 0 || pi == 4 || pi == 5 || pi == 8 || pi == 9 || pi == 12 || pi == 13) ? 6 : 0; }
__host__ __device__ constexpr int ms_nold(int NBLK) { return NBLK >= 2 ? (NBLK - 1) * 4 * MS_LW : 0; }
__host__ __device__ constexpr int ms_budget(int NBLK) { return (ms_nold(NBLK) + 42 + 14) / 15; }
__host__ __device__ constexpr int ms_old_cnt(int NBLK, int pi)
{
    int used = 0;
    for (int q = 0; q <= pi; ++q) {
        int c = q == 15 ? 0 : ms_budget(NBLK) - ms_mandatory(q);
        if (c < 0) c = 0;
        if (used + c > ms_nold(NBLK)) c = ms_nold(NBLK) - used;
        if (q == pi) return c;
        used += c;
    }
    return 0;
}
__host__ __device__ constexpr int ms_old_start(int NBLK, int pi)
{
    int used = 0;
    for (int q = 0; q < pi; ++q) used += ms_old_cnt(NBLK, q);
    return used;
}
static_assert(ms_old_start(4, 15) + ms_old_cnt(4, 15) == ms_nold(4), "all products with older blocks are scheduled (K <= 64)");
static_assert(ms_old_start(2, 15) + ms_old_cnt(2, 15) == ms_nold(2), "all products with older blocks are scheduled (K <= 32)");

template <int NBLK, bool BWD>
__device__ __forceinline__ void mscan_body(const Params &p, double *lds, const int grp, const int warm, const int tier)
{
    constexpr int NLB = NBLK > 2 ? NBLK - 2 : 0;  // blocks of the window kept in LDS (the two newest are registers)
    constexpr int LW = MS_LW;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int r = lane >> 4, tk = lane & 15;
    const int K = p.K, C = p.C, KC = K * C, Delta = p.Delta, N = p.N;
    double *Wtab = lds;                                                   // [24][88]
    double *zb = Wtab + MS_CT * MS_WT_LEN;                                // [2][4 waves][6 groups][64]
    double *ysum = zb + 2 * 4 * 6 * 64;                                   // [4 waves][16]
    double *stage = ysum + 64;                                            // [4][LW][64]: one block, one wave at a time
    double *lwin = stage + 4 * LW * 64 + (size_t)w * NLB * 4 * LW * 64;   // this wave: [NLB][4][LW][64]

    // ---- task of this lane's column
    const int ntask = p.B * N;
    const int tsk = grp * MS_TASKS + tk;
    bool valid = tsk < ntask;
    const int b = valid ? tsk / N : 0, j = valid ? tsk % N : 0;
    const SeqHdr h = p.hdr[b];
    const int L = h.L, J = h.J, Jm = J - 1;
    if (tier > 0 && p.spec_ok[b * 2 + (BWD ? 1 : 0)]) valid = false;  // accepted with the shorter warm-up
    if (J < MS_JMIN) valid = false;                                    // left to the one-wave kernel
    const int lo = j * Delta;
    if (lo >= L) valid = false;
    if (!__any(valid)) return;  // the same for all four waves: they look at the same 16 tasks
    const int hin = lo + Delta, hi = hin < L ? hin : L;
    const int tbase = BWD ? hin + warm - 1 : lo - warm;
    const int s0 = BWD ? (tbase < L ? tbase : L) : (tbase > 0 ? tbase : 0);

    for (int i = threadIdx.x; i < MS_CT * MS_WT_LEN; i += 256) {
        const int lb = i / MS_WT_LEN, k = i % MS_WT_LEN - MS_WT_OFF;
        Wtab[i] = (lb < C && k >= 1 && k <= K) ? p.W[(size_t)(k - 1) * C + lb] : 0.0;
    }
    for (int i = lane; i < NLB * 4 * LW * 64; i += 64) lwin[i] = 0.0;

    // ---- labels: label-row layout (slot 0: 4w + row; slot 1: 16 + 2w + row, rows 0 and 1 only)
    int lab[2];
    bool lv[2];
    lab[0] = 4 * w + r;
    lab[1] = 16 + 2 * w + (r & 1);
    lv[0] = lab[0] < C;
    lv[1] = r < 2 && lab[1] < C;
    const int labc[2] = {lab[0] < C ? lab[0] : C - 1, lab[1] < C ? lab[1] : C - 1};
    double Wk[4][2];  // W[k, label of the lane], k = 1..4: what the chunk itself (and, for its first position, the
                      // previous chunk) adds by plain multiply-adds
#pragma unroll
    for (int k = 1; k <= 4; ++k)
#pragma unroll
        for (int s = 0; s < 2; ++s) Wk[k - 1][s] = (lv[s] && k <= K) ? p.W[(size_t)(k - 1) * C + lab[s]] : 0.0;
    // A operands of the partial transition product: A[m = destination 16*tile + lane%16][kk = lane/16 = source row of slot s]
    double EtA[2][2];
#pragma unroll
    for (int tile = 0; tile < 2; ++tile)
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int cout = 16 * tile + tk;
            const int cin = s == 0 ? 4 * w + r : 16 + 2 * w + r;
            const bool ok = cout < C && cin < C && (s == 0 || r < 2);
            EtA[tile][s] = ok ? (BWD ? p.Etr[(size_t)cout * C + cin] : p.Etr[(size_t)cin * C + cout]) : 0.0;
        }
    // position-row layout: register lbl holds label plab(lbl)
    const double *wt[LW];  // A operand of a window product with source-chunk offset delta: wt[lbl][delta]
#pragma unroll
    for (int lbl = 0; lbl < LW; ++lbl) {
        const int pl = lbl < 4 ? 4 * w + lbl : 16 + 2 * w + (lbl - 4);
        wt[lbl] = Wtab + pl * MS_WT_LEN + MS_WT_OFF + tk - r;
    }

    // Addresses are formed from the kernel arguments and 32-bit element indices at the point of use (the sizes
    // this kernel is launched for keep every index below 2^31), so that no 64-bit pointer is held per lane.
    const int row0C = b * (p.T + 1) * C;                      // first element of the sequence in the [B][T+1][C] arrays
    const unsigned eidx[2] = {(unsigned)(row0C + labc[0]), (unsigned)(row0C + labc[1])};
    const size_t ckstride = (size_t)KC + C;
    auto ck1 = [&]() { return (BWD ? p.ckB : p.ckA) + ((size_t)b * (N + 1) + (BWD ? j + 1 : j)) * ckstride; };
    auto ck2 = [&]() { return (BWD ? p.ckB2 : p.ckA2) + ((size_t)b * (N + 1) + (BWD ? j : j + 1)) * ckstride; };
    auto ckY1 = [&]() { return (BWD ? p.ckYB : p.ckYA) + (size_t)b * (N + 1) + (BWD ? j + 1 : j); };
    auto ckY2 = [&]() { return (BWD ? p.ckYB2 : p.ckYA2) + (size_t)b * (N + 1) + (BWD ? j : j + 1); };
    const bool rec1 = valid && (!BWD || (hi == hin && hi < L));  // the state at L is the known start of the backward scan
    const bool keep = valid && (BWD ? p.marg != 0 : p.fuse != 0);
    const int rowbase = (b * N + j) * Delta;                  // first row of the task's slot in the row arrays
    double2 *const rows = (double2 *)(BWD ? p.bloc : p.aloc);
    double *const rowsY = BWD ? p.blocY : p.alocY;
    double2 *const sink = (double2 *)p.sink;   // 10 KB nobody reads

    // ---- state
    double WR[2][4][LW];    // window, position rows: [1] the block being filled, [0] the one before it
    mfma_d4 accC[LW], accN[LW];  // what the window adds to the 16 positions of the current / the next block
    double X[4][2];         // label rows: accumulated part of x for the 4 positions of the chunk at hand
    double q[4][2], qprev[4][2];  // label rows: new messages of the chunk at hand / of the previous chunk
    double ylast[2] = {0.0, 0.0};
    double Y = 0.0, Yrec = 0.0;
#pragma unroll
    for (int d = 0; d < 2; ++d)
#pragma unroll
        for (int v = 0; v < 4; ++v)
#pragma unroll
            for (int lbl = 0; lbl < LW; ++lbl) WR[d][v][lbl] = 0.0;
#pragma unroll
    for (int lbl = 0; lbl < LW; ++lbl) {
        accC[lbl] = mfma_d4{0.0, 0.0, 0.0, 0.0};
        accN[lbl] = mfma_d4{0.0, 0.0, 0.0, 0.0};
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int s = 0; s < 2; ++s) X[i][s] = 0.0, q[i][s] = 0.0, qprev[i][s] = 0.0;
    int par = 0;
    lds_barrier();  // tables and the LDS part of the window are in place

    auto pos_of = [&](const int n) { return BWD ? tbase - n : tbase + n; };
    auto load_e = [&](double2 (&e)[MS_PFD][2], const int nfirst) {
#pragma unroll
        for (int i = 0; i < MS_PFD; ++i) {
            int t = pos_of(nfirst + i);
            t = t < 0 ? 0 : (t > L ? L : t);
#pragma unroll
            for (int s = 0; s < 2; ++s) e[i][s] = p.EI[eidx[s] + (unsigned)(t * C)];
        }
    };
    // exponent step of the lane's labels at the scaling-block boundary in front of the block that starts at step n
    auto boundary_at = [&](const int n) {
        const int tb = pos_of(n);
        return valid && (BWD ? (tb < s0 && ((tb + 1) & Jm) == 0 && tb >= 0) : (tb > s0 && (tb & Jm) == 0 && tb <= L));
    };
    auto load_dn = [&](int (&dn)[2], const int n) {
        const int tb = pos_of(n);
        const bool need = boundary_at(n);
        const int jn = need ? (BWD ? (tb + 1) / J : tb / J) : 1;
#pragma unroll
        for (int s = 0; s < 2; ++s)
            dn[s] = need ? p.nbase[eidx[s] + (unsigned)(jn * C)] - p.nbase[eidx[s] + (unsigned)((jn - 1) * C)] : 0;
    };
    auto lds_slot = [&](const int blk) { return NLB > 0 ? ((blk % NLB) + NLB) % NLB : 0; };
    auto lwin_at = [&](const int slot, const int v, const int lbl) -> double & {
        return lwin[(size_t)((slot * 4 + v) * LW + lbl) * 64 + lane];
    };
    auto window_mfma = [&](mfma_d4 &acc, const double bval, const int lbl, const int delta) {
        acc = __builtin_amdgcn_mfma_f64_16x16x4f64(wt[lbl][delta], bval, acc, 0, 0, 0);
    };
    // rows of an accumulator component (position rows) -> X (label rows)
    auto extract = [&](const mfma_d4 (&acc)[LW], auto ctag, const bool first_only) {
        constexpr int comp = decltype(ctag)::value;
#ifdef MS_NO_EXTRACT
        return;
#endif
        double a0 = acc[0][comp], a1 = acc[1][comp], a2 = acc[2][comp], a3 = acc[3][comp];
        transpose4(a0, a1, a2, a3);
        double b0 = acc[4][comp], b1 = acc[5][comp], b2 = 0.0, b3 = 0.0;
        transpose4(b0, b1, b2, b3);
        if (first_only) {
            X[0][0] = a0; X[0][1] = b0;
        } else {
            X[1][0] = a1; X[2][0] = a2; X[3][0] = a3;
            X[1][1] = b1; X[2][1] = b2; X[3][1] = b3;
        }
    };
    // Checkpoint record: the K-1 positions before position tnew (forward; tnew itself is patched in after it has
    // been processed) or the K positions from the newest one, tnew, on (backward).  blk = index of the block that
    // follows; the window still holds the NBLK blocks before it.  Records are rare (two per task), so this is
    // written for small code and few registers: a block in LDS is copied out by a loop over the lane's 24
    // entries, and the two blocks in registers go through a staging area in LDS first, one wave at a time.
    // All four waves call it at the same steps (the barriers inside are uniform).
    auto dump_block = [&](double *ck, const int tm, const int bd, const double *blkbase, const bool on) {
#pragma nounroll
        for (int e = 0; e < 4 * LW; ++e) {
            const int v = e / LW, lbl = e - v * LW;
            const int pl = lbl < 4 ? 4 * w + lbl : 16 + 2 * w + (lbl - 4);
            const int dist = BWD ? 16 * (bd - 1) + 4 * (3 - v) + (3 - r) : 16 * bd - 4 * v - r;
            int slot = BWD ? tm + dist : tm - dist;
            if (BWD) { if (slot >= K) slot -= K; } else { if (slot < 0) slot += K; }
            const double val = blkbase[(size_t)e * 64 + lane];
            if (on && dist <= K - 1 && pl < C) ck[(size_t)slot * C + pl] = val;
        }
    };
    auto dump = [&](double *ck, const int tnew, const int blk, const bool on) {
#ifdef MS_NO_DUMP
        return;
#endif
        const int tm = on ? tnew % K : 0;
#pragma unroll
        for (int bd = 3; bd <= NBLK; ++bd) dump_block(ck, tm, bd, lwin + (size_t)lds_slot(blk - bd) * 4 * LW * 64, on);
        lds_barrier();  // everybody is done with the exchange buffers of the last position
#pragma unroll
        for (int bd = 1; bd <= (NBLK < 2 ? NBLK : 2); ++bd) {
#pragma nounroll
            for (int turn = 0; turn < 4; ++turn) {
                if (w == turn) {
#pragma unroll
                    for (int v = 0; v < 4; ++v)
#pragma unroll
                        for (int lbl = 0; lbl < LW; ++lbl) stage[(size_t)(v * LW + lbl) * 64 + lane] = WR[2 - bd][v][lbl];
                    lds_wave_fence();
                    dump_block(ck, tm, bd, stage, on);
                }
                lds_barrier();
            }
        }
    };

    const int NB = (warm + Delta) / 16;
    const int brec = warm / 16;
    double2 ecur[MS_PFD][2];  // (ES, 1/ES) of the lane's labels at the next MS_PFD positions; a slot is reloaded once used
    load_e(ecur, 0);
    int dnx[2];
    load_dn(dnx, 16);

    // one position: chunk v, position i of the chunk, step n.  windows = false for the single position a forward
    // task runs after its last block.
    auto position = [&](auto vtag, auto itag, auto wtag, const int n, const int blk) {
        constexpr int v = decltype(vtag)::value, i = decltype(itag)::value;
        constexpr bool windows = decltype(wtag)::value != 0;
        const int t = pos_of(n);
        const bool inject = valid && t == s0;
        const bool started = valid && (BWD ? t <= s0 : (t >= s0 && t <= hi));
        double y[2], e1[2], e2[2];
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            double x = X[i][s];
            if constexpr (i == 0) {  // durations 4..1 from the previous chunk (later positions get them from a window product)
#pragma unroll
                for (int jp = 0; jp < 4; ++jp) x = fma(Wk[3 - jp][s], qprev[jp][s], x);
            }
#pragma unroll
            for (int jq = 0; jq < i; ++jq) x = fma(Wk[i - jq - 1][s], q[jq][s], x);
            const bool on = started && lv[s];
            constexpr int es = i % MS_PFD;
            e1[s] = on ? (BWD ? ecur[es][s].y : ecur[es][s].x) : 0.0;
            e2[s] = on ? (BWD ? ecur[es][s].x : ecur[es][s].y) : 0.0;
            {  // the same slot MS_PFD positions on
                int tn = pos_of(n + MS_PFD);
                tn = tn < 0 ? 0 : (tn > L ? L : tn);
#ifndef MS_NO_ELOAD
                ecur[es][s] = p.EI[eidx[s] + (unsigned)(tn * C)];
#endif
            }
            y[s] = x * e1[s];
            if (!BWD) y[s] = inject ? (lv[s] ? 1.0 : 0.0) : y[s];                   // alpha_{s0} = 0 for every label
            else y[s] = inject ? ((lv[s] && lab[s] == 0) ? 1.0 : 0.0) : y[s];       // scale reference 1 at the start
        }
        // partial transition product over this wave's source labels, all destinations
        mfma_d4 Z0 = {0.0, 0.0, 0.0, 0.0}, Z1 = {0.0, 0.0, 0.0, 0.0};
        Z0 = __builtin_amdgcn_mfma_f64_16x16x4f64(EtA[0][0], y[0], Z0, 0, 0, 0);
        Z1 = __builtin_amdgcn_mfma_f64_16x16x4f64(EtA[1][0], y[0], Z1, 0, 0, 0);
        Z0 = __builtin_amdgcn_mfma_f64_16x16x4f64(EtA[0][1], y[1], Z0, 0, 0, 0);
        Z1 = __builtin_amdgcn_mfma_f64_16x16x4f64(EtA[1][1], y[1], Z1, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        // exchange of the partials; the owner of a destination label adds them in wave order
        double *zw = zb + (size_t)((par * 4 + w) * 6) * 64 + lane;
        zw[0] = Z0[0]; zw[64] = Z0[1]; zw[128] = Z0[2]; zw[192] = Z0[3]; zw[256] = Z1[0]; zw[320] = Z1[1];
        __builtin_amdgcn_sched_barrier(0);
        // window products in the shadow of this position's exchange: the partials are on their way through LDS and
        // the other waves are arriving at the barrier meanwhile
#ifndef MS_NO_WINDOWS
        if constexpr (windows) {
            constexpr int pi = 4 * v + i;
            constexpr int vp = v > 0 ? v - 1 : 0;
            if constexpr (pi == 0) {  // the last chunk of the previous block -> this block (its first chunk took that by multiply-adds)
                ms_static_for<LW>([&](auto lt) {
                    constexpr int lbl = decltype(lt)::value;
                    window_mfma(accC[lbl], WR[0][3][lbl], lbl, 4);
                });
            }
            if constexpr (pi == 4 || pi == 8 || pi == 12) {  // chunk v-1 -> the rest of this block (positions 1..3 of chunk v on)
                ms_static_for<LW>([&](auto lt) {
                    constexpr int lbl = decltype(lt)::value;
                    window_mfma(accC[lbl], WR[1][vp][lbl], lbl, -4 * vp);
                });
            }
            if constexpr (pi == 5 || pi == 9 || pi == 13) {  // chunk v-1 -> the next block
                ms_static_for<LW>([&](auto lt) {
                    constexpr int lbl = decltype(lt)::value;
                    window_mfma(accN[lbl], WR[1][vp][lbl], lbl, 16 - 4 * vp);
                });
            }
            constexpr int m0 = ms_old_start(NBLK, pi), mc = ms_old_cnt(NBLK, pi);
            ms_static_for<mc>([&](auto mt) {
                constexpr int m = m0 + decltype(mt)::value;
                constexpr int cidx = m / LW, lbl = m % LW;            // chunk of an older block, oldest block first
                constexpr int drel = NBLK - cidx / 4, vs = cidx % 4;  // the block drel blocks before the next one
                double bval;
                if constexpr (drel == 2) bval = WR[0][vs][lbl];
                else bval = lwin_at(lds_slot(blk + 1 - drel), vs, lbl);
                window_mfma(accN[lbl], bval, lbl, 16 * drel - 4 * vs);
            });
        }
#endif
        __builtin_amdgcn_sched_barrier(0);
#ifndef MS_NO_POSBARRIER
        lds_barrier();
#endif
        const double *zr = zb + (size_t)(par * 4 * 6) * 64;
        const int lane1 = (((r & 1) + 2 * (w & 1)) << 4) + tk;
        double z[2];
        z[0] = ((zr[(0 * 6 + w) * 64 + lane] + zr[(1 * 6 + w) * 64 + lane]) + zr[(2 * 6 + w) * 64 + lane]) + zr[(3 * 6 + w) * 64 + lane];
        const int g1 = 4 + (w >> 1);
        z[1] = ((zr[(0 * 6 + g1) * 64 + lane1] + zr[(1 * 6 + g1) * 64 + lane1]) + zr[(2 * 6 + g1) * 64 + lane1]) + zr[(3 * 6 + g1) * 64 + lane1];
        par ^= 1;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            if (BWD) z[s] = inject ? 1.0 : z[s];  // beta_{s0} = 0
            q[i][s] = lv[s] ? z[s] * e2[s] : 0.0;
            if constexpr ((v == 0 && i == 0) || (v == 3 && i == 3)) ylast[s] = y[s];  // read by records and rescaling only
        }
        if (t == (BWD ? hi : lo)) Yrec = Y;
        if (!BWD && valid && t == hi) {  // the message vector and scale at the interval's far end (logZ of the last interval)
#pragma unroll
            for (int s = 0; s < 2; ++s)
                if (lv[s]) ck2()[KC + lab[s]] = y[s];
            if (w == 0 && r == 0) *ckY2() = Y;
        }
#ifndef MS_NO_ROWS
        // The rows of the interval proper (and, when nothing is to be kept, the same number of stores into a sink):
        // every position issues the same memory operations, so that the waits for the prefetched (ES, 1/ES) pairs
        // count exactly and never cover a younger request.
        {
            const bool st = keep && t >= lo && t < hi;
            const unsigned rix = (unsigned)((rowbase + t - lo) * C);
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                double2 *dst = (st && lv[s]) ? rows + (rix + (unsigned)lab[s]) : sink + (2 * threadIdx.x + s);
                *dst = make_double2(y[s], q[i][s]);
            }
            double *dsty = (st && w == 0 && r == 0) ? rowsY + (unsigned)(rowbase + t - lo) : (double *)(sink + 512) + threadIdx.x;
            *dsty = Y - Yrec;
        }
#endif
    };

    // Every stored value of the lane's labels times 2^shift (exact): window, accumulators of the next block and
    // the messages of the chunk just finished move into the frame of the scaling block that starts.
    auto rescale = [&](const int sl0, const int sl1) {
        int sp0[4], sp1[4];
        bcast_rows(sl0, sp0);
        bcast_rows(sl1, sp1);
        const int sp[LW] = {sp0[0], sp0[1], sp0[2], sp0[3], sp1[0], sp1[1]};
#pragma unroll
        for (int lbl = 0; lbl < LW; ++lbl) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                WR[0][v][lbl] = ms_scale(WR[0][v][lbl], sp[lbl]);
                WR[1][v][lbl] = ms_scale(WR[1][v][lbl], sp[lbl]);
                accN[lbl][v] = ms_scale(accN[lbl][v], sp[lbl]);
            }
            __builtin_amdgcn_sched_barrier(0);  // one label at a time
        }
        if (NLB > 0) {  // the blocks in LDS: a loop over the lane's entries (label = entry mod 6)
#pragma nounroll
            for (int e = 0; e < NLB * 4 * LW; ++e) {
                const int lbl = e % LW;
                const int sh = lbl == 0 ? sp[0] : (lbl == 1 ? sp[1] : (lbl == 2 ? sp[2] : (lbl == 3 ? sp[3] : (lbl == 4 ? sp[4] : sp[5]))));
                double *qp = lwin + (size_t)e * 64 + lane;
                *qp = ms_scale(*qp, sh);
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            qprev[i][0] = ms_scale(qprev[i][0], sl0);
            qprev[i][1] = ms_scale(qprev[i][1], sl1);
        }
    };

    for (int blk = 0;; ++blk) {
        const int n0 = blk * 16;
        if (blk > 0) {
            // -------- between two blocks: block blk-1 is complete (WR[1]), WR[0] is the one before it
            const int tb = pos_of(n0);
            if (BWD && (blk == brec || blk == NB)) {  // backward records sit on a block's last position
                const bool fin = blk == NB;
                const bool on = fin ? valid : rec1;
                double *const ck = fin ? ck2() : ck1();
                dump(ck, tb + 1, blk, on);
                if (on) {
#pragma unroll
                    for (int s = 0; s < 2; ++s)
                        if (lv[s]) ck[KC + lab[s]] = ylast[s];
                    if (w == 0 && r == 0) *(fin ? ckY2() : ckY1()) = Y;
                }
                if (fin) break;
            }
            const bool needb = boundary_at(n0);
            if (__any(needb)) {
                // scale reference: exponent of the sum of the last message vector, all labels (waves in order)
                double ps = ylast[0] + ylast[1];
                ps = add_across_32(ps);
                ps = add_across_16(ps);
                if (r == 0) ysum[w * 16 + tk] = ps;
                lds_barrier();
                const double tot = ((ysum[tk] + ysum[16 + tk]) + ysum[32 + tk]) + ysum[48 + tk];
                const int ex = needb ? safe_exponent(tot) : 0;
                Y += (double)ex;
                rescale(needb ? dnx[0] - ex : 0, needb ? dnx[1] - ex : 0);
            }
            load_dn(dnx, n0 + 16);
            if (!BWD && (blk == brec || blk == NB)) dump(blk == NB ? ck2() : ck1(), tb, blk, valid);
            // -------- the window moves on by one block
            if (NLB > 0) {
                const int sl = lds_slot(blk - 2);
#pragma unroll
                for (int v = 0; v < 4; ++v) {
#pragma unroll
                    for (int lbl = 0; lbl < LW; ++lbl) lwin_at(sl, v, lbl) = WR[0][v][lbl];
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
#pragma unroll
            for (int v = 0; v < 4; ++v)
#pragma unroll
                for (int lbl = 0; lbl < LW; ++lbl) WR[0][v][lbl] = WR[1][v][lbl];
#pragma unroll
            for (int lbl = 0; lbl < LW; ++lbl) {
                accC[lbl] = accN[lbl];
                accN[lbl] = mfma_d4{0.0, 0.0, 0.0, 0.0};
            }
            extract(accC, std::integral_constant<int, 0>{}, true);
        }
        if (blk == NB) {  // forward only: the interval's far end is the first position of the block after the last
            position(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, n0, blk);
            const int tm = valid ? (lo + Delta) % K : 0;
            if (valid) {
#pragma unroll
                for (int s = 0; s < 2; ++s)
                    if (lv[s]) ck2()[(size_t)tm * C + lab[s]] = q[0][s];
            }
            break;
        }
        ms_static_for<4>([&](auto vtag) {
            constexpr int v = decltype(vtag)::value;
            ms_static_for<4>([&](auto itag) {
                constexpr int i = decltype(itag)::value;
                position(vtag, itag, std::integral_constant<int, 1>{}, n0 + 4 * v + i, blk);
                // positions 1..3 of the chunk: their rows now hold what the previous chunk adds as well
                if constexpr (i == 0) extract(accC, vtag, false);
                if (!BWD && v == 0 && i == 0 && blk == brec && valid) {  // forward checkpoint: its newest position
                    const int tm = lo % K;
#pragma unroll
                    for (int s = 0; s < 2; ++s)
                        if (lv[s]) {
                            ck1()[(size_t)tm * C + lab[s]] = q[0][s];
                            ck1()[KC + lab[s]] = ylast[s];
                        }
                    if (w == 0 && r == 0) *ckY1() = Y;
                }
            });
            // the chunk's messages: label rows -> position rows of the window
            {
                double a0 = q[0][0], a1 = q[1][0], a2 = q[2][0], a3 = q[3][0];
                transpose4(a0, a1, a2, a3);
                WR[1][v][0] = a0; WR[1][v][1] = a1; WR[1][v][2] = a2; WR[1][v][3] = a3;
                double b0 = q[0][1], b1 = q[1][1], b2 = q[2][1], b3 = q[3][1];
                transpose4(b0, b1, b2, b3);
                WR[1][v][4] = b0; WR[1][v][5] = b1;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int s = 0; s < 2; ++s) qprev[i][s] = q[i][s];
            if constexpr (v < 3) extract(accC, std::integral_constant<int, (v < 3 ? v + 1 : 0)>{}, true);
        });
    }
}

template <int NBLK>
__global__ __launch_bounds__(256) void k_mscan(Params p, int both, int warm, int tier)
{
    extern __shared__ double lds_raw[];
    const int ngrp = (p.B * p.N + MS_TASKS - 1) / MS_TASKS;
    const int dir = (int)blockIdx.x / ngrp, grp = (int)blockIdx.x % ngrp;
    (void)both;
    if (dir == 0) mscan_body<NBLK, false>(p, lds_raw, grp, warm, tier);
    else mscan_body<NBLK, true>(p, lds_raw, grp, warm, tier);
}

}  // namespace

// The lock-step scan on the matrix cores applies to 17..24 labels, K <= 64 and checkpoint intervals
// that are multiples of 32 (scaling-block boundaries then fall on block starts in every task).
bool mscan_applies(int K, int C, int Delta)
{
    return C > 16 && C <= MS_CT && K <= 64 && Delta % 32 == 0;  // (the caller also bounds B*(T+1)*C: 32-bit indices)
}

namespace {

template <int NBLK>
int launch_mscan_k(const Params &p, hipStream_t st, bool both, int warm, int tier)
{
    const size_t lds = ms_lds_doubles(NBLK) * sizeof(double);
    if (hipFuncSetAttribute((const void *)k_mscan<NBLK>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) !=
        hipSuccess)
        return SEMICRF_ELAUNCH;
    const int ngrp = (p.B * p.N + MS_TASKS - 1) / MS_TASKS;
    hipLaunchKernelGGL((k_mscan<NBLK>), dim3(ngrp * (both ? 2 : 1)), dim3(256), lds, st, p, both ? 1 : 0, warm, tier);
    return SEMICRF_OK;
}

}  // namespace

int launch_mscan(const Params &p, hipStream_t st, bool both, int warm, int tier)
{
    const int wm = (warm + 31) / 32 * 32;  // whole blocks, scaling-block aligned
    if (p.K <= 16) return launch_mscan_k<1>(p, st, both, wm, tier);
    if (p.K <= 32) return launch_mscan_k<2>(p, st, both, wm, tier);
    return launch_mscan_k<4>(p, st, both, wm, tier);
}


}  // namespace semicrf_impl
