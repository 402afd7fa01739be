// Declarations shared by the translation units of libsemicrf: sizes, the kernel parameter block,
// small device helpers, and the launchers one unit offers to another.
#ifndef SEMICRF_COMMON_H
#define SEMICRF_COMMON_H

#include <hip/hip_runtime.h>
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <type_traits>
#include <utility>

#include "semicrf.h"
#include "geometry.h"
#include "plan.h"

namespace semicrf_impl {

constexpr double LN2 = 0.6931471805599453094;
constexpr double LOG2E = 1.4426950408889634074;
constexpr double RANGE_NATS = 300.0;  // growth allowed inside one scaling block (2x this < ln DBL_MAX)

struct SeqHdr {
    int L;          // clamped length
    int J;          // scaling block length (power of two <= JMAX)
    int flags;      // bit 0: scores exceed the supported per-position range
    int pad;
    double logZ;    // from the forward scan
    double logZb;   // from the backward scan (diagnostic: must equal logZ)
};
static_assert(sizeof(SeqHdr) == SEQ_HDR_BYTES, "the plan sizes the header array with SEQ_HDR_BYTES");

struct Params {
    // problem
    const void *emis;   // [B][T][C] float, or 2-byte IEEE half / bfloat16 (emis_type 1 / 2)
    int emis_type;
    const int32_t *lengths;
    const float *trans;
    const float *dur;
    const float *grad_logz;
    // optional boundary terms of Eq. 4 (any of them may be null)
    const float *proj_start;  // [B][T][C]  start score of a segment whose first token is t
    const float *proj_end;    // [B][T][C]  end score of a segment whose last token is t
    const float *pi_start;    // [C]        scalar boundary of the sequence's first segment
    const float *pi_end;      // [C]        scalar boundary of the sequence's last segment
    int B, T, K, C;
    int Delta, N;       // checkpoint interval and intervals per padded sequence
    int NCH;            // prefix-sum chunks per sequence (covers t = 0..T)
    int center;
    int want_grad;
    int nslot;
    // workspace
    SeqHdr *hdr;        // [B]
    double *nu;         // [B][C]
    double *chsum;      // [B][NCH][C] chunk sums, then exclusive chunk offsets
    double *chmax;      // [B][NCH]
    double *tabmax;     // [2]: max dur, max trans
    double *W;          // [K][C]
    double *Etr;        // [C][C]
    double2 *EI;        // [B][T+1][C]  .x = ES = exp(S - n ln2), .y = 1/ES
    int *nbase;         // [B][T+1][C] (row j = scaling block j)
    double *ckA;        // [B][N+1][K*C + C]
    double *ckB;        // [B][N+1][K*C + C]
    double *ckYA;       // [B][N+1]
    double *ckYB;       // [B][N+1]
    // chunk-parallel scan: states reached at the END of a chunk (compared with the next
    // chunk's warm-up state), their scales, per-boundary log2 scale ratios and mismatches
    double *ckA2;       // [B][N+1][K*C + C]
    double *ckB2;       // [B][N+1][K*C + C]
    double *ckYA2;      // [B][N+1]
    double *ckYB2;      // [B][N+1]
    double *spec_lr;    // [B][2][N+1]
    double *spec_err;   // [B][2][N+1]
    int *spec_ok;       // [B][2]  1: the chunk-parallel scan of (sequence, direction) was accepted
    int logpair;        // k_prefix stores the log-domain pair (S + end score, start score - S): Viterbi
    double2 *vr;        // [B][T+1][C] Viterbi: (V_t(c), r_t(c)) = best score arriving at / leaving position t
    int *vbest;         // [B] Viterbi: label of the last segment
    int *vbp;           // [B][T+1][C] Viterbi back-pointers: (duration << 8) | predecessor label
    int *vpar[2];       // [B][T+1][C] parent node (position * C + label) and its doublings (ping-pong)
    int *vexit;         // [B][T+1][C] second buffer of the interval-exit pointers (the first is vpar[1])
    unsigned char *vmark;  // [B][T+1][C] 1: the node lies on the best path
    float *vscore;      // Viterbi outputs
    int32_t *vlabels, *vstarts, *vnseg;
    int spec;           // chunk-parallel scan enabled for this call
    int mscan;          // its tasks may run sixteen at a time in lock step on the matrix cores
    double *sink;       // [1536] target of stores that must be issued but whose value nobody wants
    int spec2;          // chunk-parallel scan tasks with two waves each (tip + helper): 0 where it pays, 1 always, 2 never
    int lowmem;         // low-memory plan: interval at the spacing of Algorithm 1, a few row slots per sequence
    int warm0;          // first warm-up length of the chunk-parallel scans asked for by the caller (0 = default)
    int marg_route;     // 0 automatic, 1 marginals from the stored rows of both scans, 2 per-interval recurrence
    int vit_global;     // Viterbi trace-back by pointer doubling over all nodes (test of the fallback route)
    int fuse;           // its forward tasks also store the interval stage's forward rows (one slot per task)
    double *aloc;       // [nslot][Delta][2C]
    double *alocY;      // [nslot][Delta]
    double *bloc;       // [nslot][Delta][2C] backward rows (p_t, v_t) of the chunk-parallel backward tasks
    double *blocY;      // [nslot][Delta]     their scale relative to the interval's upper end
    int marg;           // marginals from the stored rows of both scans (no recurrence in the interval stage)
    int msplit;         // parts per interval of the one-wave stored-row marginals; a sequence they handle has its partial
                        // sums per part (index interval*msplit + part), any other per interval (index interval)
    int NP;             // N * msplit: partial sums of a sequence in partD, partTr, tot, sumR, carry
    double *partD;      // [B][NP][K][C]
    double *partTr;     // [B][NP][C][C]
    double *tot;        // [B][NP][C]
    double *sumR;       // [B][NP][C]
    double *carry;      // [B][NP][C]
    double *mean;       // [B][FIN_SLICES][C]  sums behind the per-label mean of the position marginals
    double *out0;       // [B][C]  mass of the segments that start at position 0, per label
    double *inL;        // [B][C]  mass of the segments that end at position L, per label
    // outputs
    double *cum;        // optional [B][T+1][C]
    float *logz;
    float *grad_emis;
    float *grad_trans;
    float *grad_dur;
    float *pos_marg;
    float *g_proj_start;  // optional [B][T][C]
    float *g_proj_end;    // optional [B][T][C]
    float *g_pi_start;    // optional [C]
    float *g_pi_end;      // optional [C]
    float *bdy_post;      // optional [B][T+1]
    // duration-dependent transitions (null / unused otherwise)
    const float *trans3;  // [K][C][C] trans3[k-1][c'][c] in place of trans[c'][c]
    double *G3;           // [K][C][C] exp(dur[k-1,c] + trans3[k-1,c',c])
    double *dtA;          // [B][T+1][C] forward messages a_t(c), scaled
    double *dtY;          // [B][T+1]    log2 scale of that row relative to its interval's first position
    double *dtV;          // [B][T+1][C] backward messages v_t(c) = b_t(c) ES_t(c), scaled
    double *dtD;          // [B][T+1][C] (mass of the segments that start at t) - (that end at t), scaled
    double *dtYb;         // [B][T+1]    log2 scale of those two rows relative to the interval's upper end
    double *partG;        // [dt_nwg][K][C][C] per-workgroup sums of the weighted segment marginals
    double *sumG;         // [K][C][C] their fixed-order total
    int dt_nwg;
    float *grad_trans3;   // output [K][C][C]
};

// emission i of the [B][T][C] array; ET = storage type (0 float, 1 IEEE half, 2 bfloat16)
template <int ET>
__device__ __forceinline__ double emis_at(const Params &p, size_t i)
{
    if (ET == 0) return (double)((const float *)p.emis)[i];
    if (ET == 1) return (double)(float)((const _Float16 *)p.emis)[i];
    return (double)__uint_as_float((uint32_t)((const uint16_t *)p.emis)[i] << 16);  // bfloat16: upper half of a float
}

__device__ __forceinline__ int seq_len(const Params &p, int b)
{
    int L = p.lengths ? p.lengths[b] : p.T;
    L = L < 0 ? 0 : L;
    return L > p.T ? p.T : L;
}

__device__ __forceinline__ int safe_exponent(double m)
{
    if (!(m > 0.0) || !(m < DBL_MAX)) return 0;
    int e;
    (void)frexp(m, &e);
    return e;
}

__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// The tip's end-of-step barrier: no s_waitcnt.  The only LDS write of the step that
// other waves read (the ring entry) is not read by them before the NEXT barrier.
__device__ __forceinline__ void tip_step_barrier()
{
    asm volatile("s_barrier" ::: "memory");
}

// orders LDS accesses of one wave (LDS executes a wave's instructions in order)
__device__ __forceinline__ void lds_wave_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
}

// v + (v of the lane 32 away), in every lane: rows 2,3 of one copy are swapped with
// rows 0,1 of the other (a row is 16 lanes), then the copies are added.
__device__ __forceinline__ double add_across_32(double v)
{
    const unsigned lo = (unsigned)__double2loint(v), hi = (unsigned)__double2hiint(v);
    const auto a = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
    const auto b = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
    return __hiloint2double((int)b[0], (int)a[0]) + __hiloint2double((int)b[1], (int)a[1]);
}

// A stored row (two doubles) that a later kernel reads once: written past the caches.
__device__ __forceinline__ void store_row(double2 *dst, const double a, const double b)
{
    typedef double d2_t __attribute__((ext_vector_type(2)));
    __builtin_nontemporal_store(d2_t{a, b}, (d2_t *)dst);
}

// The value lanes 0..31 hold (-> lo_half) and the one lanes 32..63 hold (-> hi_half), lane l paired with lane
// l + 32, both delivered to both lanes.
__device__ __forceinline__ void both_halves(const double v, double &lo_half, double &hi_half)
{
    const unsigned lo = (unsigned)__double2loint(v), hi = (unsigned)__double2hiint(v);
    const auto a = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
    const auto b = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
    lo_half = __hiloint2double((int)b[0], (int)a[0]);
    hi_half = __hiloint2double((int)b[1], (int)a[1]);
}

// v + (v of the lane 16 away): odd rows of one copy are swapped with even rows of the other
__device__ __forceinline__ double add_across_16(double v)
{
    const unsigned lo = (unsigned)__double2loint(v), hi = (unsigned)__double2hiint(v);
    const auto a = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
    const auto b = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
    return __hiloint2double((int)b[0], (int)a[0]) + __hiloint2double((int)b[1], (int)a[1]);
}

// v + (v of the lane 8 away inside a row of 16): DPP row rotate by 8
__device__ __forceinline__ double add_across_8(double v)
{
    const int lo = __double2loint(v), hi = __double2hiint(v);
    const int lo2 = __builtin_amdgcn_update_dpp(0, lo, 0x128, 0xf, 0xf, false);
    const int hi2 = __builtin_amdgcn_update_dpp(0, hi, 0x128, 0xf, 0xf, false);
    return v + __hiloint2double(hi2, lo2);
}

// sum over the 64/CTP lanes of a wave that share lane % CTP; every lane gets the total
template <int CTP>
__device__ __forceinline__ double group_sum(double v)
{
    if (CTP <= 8) v = add_across_8(v);
    if (CTP <= 16) v = add_across_16(v);
    if (CTP <= 32) v = add_across_32(v);
    return v;
}

// ---- the lock-step scan on the matrix cores (mscan.hip)
constexpr int MS_JMIN = 16;  // shortest scaling block that kernel handles; shorter ones are left to the one-wave scan
bool mscan_applies(int K, int C, int Delta);
// enqueues the kernel; SEMICRF_OK or SEMICRF_ELAUNCH
int launch_mscan(const Params &p, hipStream_t st, bool both, int warm, int tier);

}  // namespace semicrf_impl

#endif  // SEMICRF_COMMON_H
