// Sweeps the host-side planning code (checkpoint interval, workspace layout, argument and flag checks) over
// small, typical and extreme sizes; built with -fsanitize=address,undefined by tests/test_sanitizers_cpu.py,
// which fails on any report.  Also checks the layout invariants the kernels rely on.
#include <stdio.h>

#include <initializer_list>

#include "plan.h"

using namespace semicrf_impl;

static int bad = 0;
#define CHECK(cond)                                                            \
    do {                                                                       \
        if (!(cond)) {                                                         \
            printf("FAILED %s:%d %s\n", __FILE__, __LINE__, #cond);          \
            bad = 1;                                                           \
        }                                                                      \
    } while (0)

static void one(int B, int T, int K, int C, int interval, int kind)
{
    Plan *pl = new Plan;  // on the heap: an overrun of off[] / size[] is a report
    const int rc = make_plan(B, T, K, C, interval, kind, pl);
    if (rc == SEMICRF_OK) {
        CHECK(pl->Delta >= 1 && pl->Delta <= T);
        CHECK(pl->N == (int)(((long long)T + pl->Delta - 1) / pl->Delta));
        CHECK(pl->nslot >= 1 && pl->nslot % 12 == 0 && pl->nslot <= NSLOT_MAX + 11);
        CHECK(pl->narrays == PL_COUNT && PL_COUNT <= 32);
        size_t end = 0;
        for (int j = 0; j < pl->narrays; ++j) {
            CHECK(pl->off[j] % 256 == 0);
            CHECK(pl->off[j] >= end);  // arrays do not overlap
            end = pl->off[j] + pl->size[j];
        }
        CHECK(pl->total >= end && pl->total % 256 == 0);
        if (interval > 0) CHECK(pl->Delta == (interval > T ? T : interval));
        if ((kind & 7) == 0) CHECK(pl->size[PL_ALOC] == 0 && pl->size[PL_CKB] == 0);
        if (kind & PLAN_LOW_MEMORY) CHECK(pl->rows == 0 && pl->nslot <= (LOWMEM_SLOTS_PER_SEQ * B + 11) / 12 * 12);
        CHECK(pl->lds_scan <= LDS_LIMIT);
    } else {
        CHECK(rc == SEMICRF_EINVAL || rc == SEMICRF_EUNSUPPORTED);
    }
    delete pl;
}

int main()
{
    const int Bs[] = {-1, 0, 1, 2, 4, 64, 1000, 100000};
    const int Ts[] = {-5, 0, 1, 7, 256, 2000, 100000, 400000, 1 << 30, (1 << 30) + 1, 2147483647};
    const int Ks[] = {-1, 0, 1, 2, 16, 64, 512, 1024, 100000, 2147483647};
    const int Cs[] = {-1, 0, 1, 3, 8, 24, 64, 65, 256, 257, 2147483647};
    const int Ds[] = {-1, 0, 1, 8, 1000, 2147483647};
    const int kinds[] = {-1, 0, 1, 2, 3, 4, 8, 9, 10, 11, 12, 16};
    long n = 0;
    for (int B : Bs)
        for (int T : Ts)
            for (int K : Ks)
                for (int C : Cs)
                    for (int D : Ds)
                        for (int kind : kinds) {
                            one(B, T, K, C, D, kind);
                            ++n;
                        }
    // the helpers on their own
    for (int T : {1, 5, 1000, 100000, 1 << 30})
        for (int K : {1, 64, 1024, 100000}) {
            const int d = low_memory_interval(T, K);
            CHECK(d >= 1 && d <= T);
            int a = 0, b = 0;
            if (wave_tasks_per_cu(K, 24, &a, &b)) CHECK(a >= 1 && b >= 1);
            const int e = auto_interval(4, T, K, 24);
            CHECK(e >= 1 && e <= T);
        }
    CHECK(check_flags(SEMICRF_CENTER) == SEMICRF_OK);
    CHECK(check_flags(SEMICRF_EMIS_F16 | SEMICRF_EMIS_BF16) == SEMICRF_EINVAL);
    CHECK(check_flags(SEMICRF_MARGINALS_ROWS | SEMICRF_MARGINALS_INTERVAL) == SEMICRF_EINVAL);
    CHECK(check_flags(SEMICRF_LOW_MEMORY | SEMICRF_MARGINALS_ROWS) == SEMICRF_EINVAL);
    CHECK(check_flags(SEMICRF_LOW_MEMORY | SEMICRF_MARGINALS_INTERVAL | SEMICRF_WARMUP(40)) == SEMICRF_OK);
    printf("%ld plans\n%s\n", n, bad ? "FAILED" : "ALL OK");
    return bad;
}
