// Sizes and LDS geometry of the kernels, as plain C++ (no HIP): what the kernels are instantiated with and what
// the host-side planning code computes workspace layouts and launch shapes from.  constexpr functions are usable
// on both sides of a HIP compilation.
#ifndef SEMICRF_GEOMETRY_H
#define SEMICRF_GEOMETRY_H

#include <stddef.h>

namespace semicrf_impl {

constexpr int NT = 256;          // threads per workgroup in the scan kernels
constexpr int PREP_CH = 256;     // positions per prefix-sum chunk (multiple of JMAX)
constexpr int JMAX = 32;         // largest scaling block
constexpr int NSLOT_MAX = 1024;  // resident tasks of the interval kernel (one wave per SIMD)
constexpr int LOWMEM_SLOTS_PER_SEQ = 8;  // row slots per sequence in the low-memory plan
constexpr int GRAD_CMAX = 64;    // most labels the gradient path holds transition accumulators for
constexpr size_t LDS_LIMIT = 160 * 1024;
constexpr size_t SEQ_HDR_BYTES = 32;  // sizeof(SeqHdr), the per-sequence header at the front of the workspace
constexpr int SINK_DOUBLES = 1536;    // target of stores that must be issued but whose value nobody wants

constexpr int MB = 4;      // positions per time block of the one-wave kernels
constexpr int MG_TG = 32;  // stored-row marginals: positions staged at a time
constexpr int MG_KS = 8;   // stored-row marginals: durations per thread of the duration kernel
constexpr int MG_TE = 64;  // stored-row marginals: positions per group of the transition/emission kernel
constexpr int FIN_SLICES = 4;    // workgroups per sequence of the carry / mean reduction (sums behind the mean per slice)
constexpr int MG_SIMDS = 1024;  // SIMDs of the chip (256 compute units of four)

// Tasks of the one-wave stored-row marginals a SIMD holds: two where the duration strip of a lane (NKW) and the
// transition tiles (CT) leave the kernel within half the register file, else one.
constexpr int mg_waves_per_simd(int CT, int NKW) { return (CT <= 32 && NKW <= 32) ? 2 : 1; }

constexpr size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

constexpr int pow2_ge8(int x)
{
    int r = 8;
    while (r < x) r <<= 1;
    return r;
}

// LDS doubles of the workgroup-per-sequence kernels (sequential scan, generic interval kernel):
//   ring[K*C]  Wl[K*C]  El[C*(C|1)]  red[G*C]  yv, zv, av, qv [C]  sc[C] (int)  and, interval kernel only, accD[K*C]
constexpr size_t lds_doubles(int K, int C, int G, bool interval)
{
    return 2 * (size_t)K * C + (size_t)C * (size_t)(C | 1) + (size_t)G * C + 5 * (size_t)C +
           (interval ? (size_t)K * C : 0);
}

// Label tile of the one-wave kernels for C labels (C <= 64).
constexpr int spec_ct_of(int C)
{
    return C <= 8 ? 8 : (C <= 16 ? 16 : (C <= 24 ? 24 : (C <= 32 ? 32 : 64)));
}

// Window entries per lane: NKW, plus one when a half-wave holds several lane groups, so
// that the groups' rows fall into different LDS banks.
constexpr int wave_nk(int CT, int NKW)
{
    return NKW + ((64 / pow2_ge8(CT)) > 2 ? 1 : 0);
}

// Rows of slack behind the sliding window: a quarter of the window (the window is moved back once
// per that many positions), an eighth for the deepest window, where the quarter would cost the
// fourth resident task of a compute unit its LDS.
constexpr int lin_slack(int KW)
{
    return KW / 4 < 8 ? 8 : (KW >= 512 ? ((KW / 8 + 3) & ~3) : ((KW / 4 + 3) & ~3));
}

constexpr size_t wave_lds_doubles(int CT, int NKW)
{
    const int CTP = pow2_ge8(CT);
    const int KW = wave_nk(CT, NKW) * (64 / CTP);
    const int YS = CTP < 16 ? 16 : CTP;
    return (size_t)(KW + lin_slack(KW)) * CT + (size_t)(CTP - CT) + (size_t)MB * YS;
}

// Single-wave tasks of one workgroup of the interval kernel.
constexpr int interval_waves(int CT, int NKW) { return CT == 64 ? 4 : (NKW == 64 ? 3 : 1); }

constexpr size_t interval_wtab_doubles(int CT, int NKW)
{
    return NKW == 64 ? (size_t)(wave_nk(CT, NKW) * (64 / pow2_ge8(CT)) + MB) * CT + (size_t)(pow2_ge8(CT) - CT) : 0;
}

constexpr size_t interval_lds_doubles(int CT, int NKW)
{
    return (CT == 64 ? 2 * (size_t)CT * CT : 0) + interval_wtab_doubles(CT, NKW) +
           (size_t)interval_waves(CT, NKW) * wave_lds_doubles(CT, NKW);
}

}  // namespace semicrf_impl
#endif
