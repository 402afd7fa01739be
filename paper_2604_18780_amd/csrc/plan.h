// Host-side planning of a call: argument checks, the checkpoint interval, and the layout of the caller's
// workspace.  Plain C++ (no HIP), so that it also builds for the host alone under the sanitizers.
#ifndef SEMICRF_PLAN_H
#define SEMICRF_PLAN_H

#include <stddef.h>

#include "geometry.h"
#include "semicrf.h"

namespace semicrf_impl {

struct Plan {
    int Delta, N, NCH, nslot, G;
    int rows;  // the backward scan tasks have row storage (stored-row marginals possible)
    int msplit;  // parts an interval is cut into by the one-wave stored-row marginals (per-part partial sums)
    size_t lds_mg_dur, lds_mg_te;
    size_t lds_scan, lds_interval;
    size_t total;
    size_t off[32];
    size_t size[32];  // bytes of each array before alignment (0 = not planned)
    int narrays;
};

// Indices of the workspace arrays in Plan::off.
enum PlanArray {
    PL_HDR = 0, PL_NU, PL_CHSUM, PL_CHMAX, PL_TABMAX, PL_W, PL_ETR, PL_EI, PL_SPEC, PL_NBASE, PL_CKA, PL_CKB,
    PL_CKYA, PL_CKYB, PL_ALOC, PL_ALOCY, PL_PARTD, PL_PARTTR, PL_TOT, PL_SUMR, PL_CARRY, PL_MEAN, PL_CKA2,
    PL_CKB2, PL_CKYA2, PL_CKYB2, PL_OUT0, PL_INL, PL_BLOC, PL_BLOCY, PL_SINK, PL_COUNT
};

// Kinds of plan (the want_grad argument of semicrf_workspace_bytes): 0 forward only, 1 gradients (with the row
// slots of the stored-row marginals where that route applies), 2 gradients of a caller that never takes the
// stored-row marginals, 3 the same plan as 1 (a caller that asks for that route by flag); plus PLAN_LOW_MEMORY.
constexpr int PLAN_LOW_MEMORY = 8;

// First warm-up length of the chunk-parallel sum scans: one and a half maximal segment lengths.
// The products of positive maps forget their start fast enough that the boundary mismatch is at the
// rounding floor there on all workloads (it reaches 1e-11 at 1.25 K; the acceptance bound is 1e-10).
inline int sum_warmup(int K) { return 3 * K / 2 < 32 ? 32 : (3 * K + 1) / 2; }

// Single-wave tasks a compute unit holds at once for these sizes (scan kernel, interval kernel); false when
// the one-wave kernels do not apply.
bool wave_tasks_per_cu(int K, int C, int *scan, int *interval);

// The chunk-parallel scan kernels cover these sizes.
bool spec_applies(int K, int C);

// Automatic checkpoint interval of the default plan (one task per SIMD where the sizes allow it).
int auto_interval(int B, int T, int K, int C);

// Checkpoint interval of the low-memory plan: the spacing of Algorithm 1, ceil(sqrt(T*K)), as a multiple of 8.
int low_memory_interval(int T, int K);

// SEMICRF_OK or the status an entry point returns for these sizes; fills *pl.
int make_plan(int B, int T, int K, int C, int ckpt_interval, int want_grad, Plan *pl);

// Flag combinations no entry point accepts.
int check_flags(unsigned flags);

}  // namespace semicrf_impl
#endif
