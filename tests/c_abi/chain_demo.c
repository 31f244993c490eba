/*
 * The C ABI used from plain C (no Python, no torch): the hand-worked two-task chain of
 * tests/golden/p1_two_task_chain.json.  Prints one line per search; exit status 0 only if
 * every result equals the values worked out on paper.
 */
#include <stdio.h>
#include <string.h>

#include "jsv.h"

static int check(const char* what, int ok)
{
    printf("%-46s %s\n", what, ok ? "ok" : "MISMATCH");
    return ok ? 0 : 1;
}

int main(void)
{
    const uint32_t units[2] = {1, 2}, batch[2] = {1, 2};
    const uint32_t lat[2 * 8] = {10000, 16000, 6000, 10000, 20000, 32000, 12000, 20000,
                                 5000, 8000, 3000, 5000, 15000, 24000, 9000, 15000};
    const double acc[2 * 2] = {0.80, 0.90, 0.70, 0.95};
    const uint16_t src[1] = {0}, dst[1] = {1};
    const uint32_t mult[2] = {1000, 1000};
    int bad = 0;

    jsv_ctx* ctx = NULL;
    if (jsv_create(&ctx, 0, NULL) != JSV_OK) return 2;
    if (jsv_load_profile(ctx, 2, 2, 2, 2, units, batch, lat, NULL, acc) != JSV_OK) return 3;
    if (jsv_set_dag(ctx, 2, 1, src, dst, mult, 12, 2) != JSV_OK) return 4;

    const uint32_t sweep[5] = {100000, 200000, 260000, 400000, 800000};
    jsv_result res[5];
    jsv_summary sum;
    int rc = jsv_search(ctx, sweep, 5, 40000, 0.85, 0, res, &sum);
    if (rc != JSV_OK) { printf("jsv_search: %s (hip %d)\n", jsv_error_string(rc), jsv_last_hip_error(ctx)); return 5; }
    const int32_t want_cost[4] = {3, 6, 9, 12};
    for (int l = 0; l < 4; ++l)
        bad += check("sweep level: index 48, cost 3/6/9/12",
                     res[l].feasible && res[l].index == 48 && res[l].cost_units == want_cost[l] &&
                     res[l].choice[0] == 0 && res[l].choice[1] == 6 && res[l].latency_us == 38000);
    bad += check("800 rps does not fit 12 units", !res[4].feasible && res[4].index == UINT64_MAX);
    bad += check("max serviceable demand 400 rps at level 3", sum.best_level == 3 && sum.max_demand_mrps == 400000);

    if (jsv_set_objective(ctx, 1, 1.0, 0.035) != JSV_OK) return 6;
    if (jsv_set_dag(ctx, 2, 1, src, dst, mult, 0, 2) != JSV_OK) return 7;
    const uint32_t one[1] = {260000};
    rc = jsv_search(ctx, one, 1, 100000, 0.0, 0, res, NULL);
    if (rc != JSV_OK) return 8;
    bad += check("Eq. 14 objective: index 37, cost 9, 0.685",
                 res[0].feasible && res[0].index == 37 && res[0].cost_units == 9 && res[0].latency_us == 94000 &&
                 res[0].objective > 0.685 - 1e-12 && res[0].objective < 0.685 + 1e-12);

    /* error paths */
    const uint16_t cyc_src[2] = {0, 1}, cyc_dst[2] = {1, 0};
    bad += check("a cycle is reported", jsv_set_dag(ctx, 2, 2, cyc_src, cyc_dst, mult, 0, 2) == JSV_E_CYCLE);
    bad += check("null pointers are reported", jsv_search(ctx, NULL, 1, 1, 0.0, 0, res, NULL) == JSV_E_NULL);
    jsv_destroy(ctx);
    return bad ? 1 : 0;
}
