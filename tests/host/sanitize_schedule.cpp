// Host-only driver for a sanitizer build (g++ -fsanitize=address,undefined) of the schedule planner
// (paper_2410_14312_amd/csrc/schedule.cpp): walks the planner's C ABI over a sweep of (W, N, mini-batches),
// the exact-capacity and too-small output arrays and the argument errors, and prints every plan as text
// (one line per case) so that the caller can compare it with an independent simulation.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>

#include <vector>

#include "../../include/tmps.h"

namespace tmps {
static char g_text[512];
int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_text, sizeof(g_text), fmt, ap);
    va_end(ap);
    return code;
}
}  // namespace tmps

static int expect(bool ok, const char* what) {
    if (!ok) fprintf(stderr, "FAILED: %s\n", what);
    return ok ? 0 : 1;
}

int main() {
    int bad = 0;
    for (int W = 1; W <= 9; ++W)
        for (int N = 1; N <= 8; ++N)
            for (int n : {1, 2, 5, 3 * W + 4}) {
                const int tasks = tmps_schedule_plan(W, N, n, nullptr, 0);
                bad += expect(tasks == W * (n * N + n), "task count");
                // an array of exactly the needed size: a write past it is what the sanitizer is here to see
                std::vector<int32_t> ops((size_t)tasks * 7);
                bad += expect(tmps_schedule_plan(W, N, n, ops.data(), (size_t)tasks) == tasks, "plan");
                if (tasks > 1) {
                    std::vector<int32_t> small((size_t)(tasks - 1) * 7);
                    bad += expect(tmps_schedule_plan(W, N, n, small.data(), (size_t)tasks - 1) == TMPS_ECAP, "capacity error");
                }
                if (n == 5) {
                    printf("plan %d %d %d", W, N, n);
                    for (int32_t v : ops) printf(" %d", v);
                    printf("\n");
                }
            }
    for (int W = 1; W <= 12; ++W)
        for (int N = 1; N <= 9; ++N) {
            printf("v %d %d %d", W, N, tmps_version_diff_simulated(W, N));
            for (int s = 0; s < W; ++s) printf(" %d:%d", tmps_schedule_stash_groups(W, N, s), tmps_schedule_shadow_versions(W, N, s));
            printf("\n");
            if (W >= 2 && N >= 2) bad += expect(tmps_version_diff_formula(W, N) == (W + N - 2) / N, "formula");
        }
    for (int W = 1; W <= 9; ++W)
        for (int n : {1, 2, W, 3 * W + 5}) {
            const int tasks = tmps_schedule_plan_1f1b(W, n, nullptr, 0);
            bad += expect(tasks == 2 * W * n, "1F1B task count");
            std::vector<int32_t> ops((size_t)tasks * 7);
            bad += expect(tmps_schedule_plan_1f1b(W, n, ops.data(), (size_t)tasks) == tasks, "1F1B plan");
            std::vector<int32_t> small((size_t)(tasks - 1) * 7);
            bad += expect(tmps_schedule_plan_1f1b(W, n, small.data(), (size_t)tasks - 1) == TMPS_ECAP, "1F1B capacity error");
            if (n == 3 * W + 5) {
                printf("plan1f1b %d %d", W, n);
                for (int32_t v : ops) printf(" %d", v);
                printf("\n");
            }
        }
    bad += expect(tmps_schedule_plan_1f1b(0, 3, nullptr, 0) == TMPS_EINVAL, "1F1B W = 0");
    bad += expect(tmps_schedule_plan(0, 4, 3, nullptr, 0) == TMPS_EINVAL, "W = 0");
    bad += expect(tmps_schedule_plan(4, 0, 3, nullptr, 0) == TMPS_EINVAL, "N = 0");
    bad += expect(tmps_schedule_plan(4, 4, 0, nullptr, 0) == TMPS_EINVAL, "no mini-batches");
    bad += expect(tmps_schedule_stash_groups(4, 4, 4) == TMPS_EINVAL, "stage out of range");
    bad += expect(tmps_schedule_stash_groups(4, 4, -1) == TMPS_EINVAL, "negative stage");
    bad += expect(tmps_schedule_shadow_versions(4, 4, 7) == TMPS_EINVAL, "stage out of range");
    bad += expect(tmps_version_diff_formula(1, 4) == TMPS_EINVAL, "formula outside its domain");
    bad += expect(tmps_version_diff_simulated(0, 1) == TMPS_EINVAL, "W = 0");
    return bad ? 1 : 0;
}
