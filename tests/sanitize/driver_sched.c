/* Runs the native scheduling simulator (host code only) with exactly sized output arrays under
 * -fsanitize=address,undefined: every strategy, with and without pipeline, segments and a slot limit.  Exit code 0 = clean. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "mars_sched.h"

int main(void) {
    const int32_t one = 1 << 24;
    for (int strategy = 0; strategy < 3; ++strategy)
        for (int variant = 0; variant < 4; ++variant) {
            mars_sched_config_t c;
            memset(&c, 0, sizeof c);
            c.problems = 24; c.group_size = 8; c.n_select = 2; c.strategy = strategy;
            c.pipeline = variant & 1; c.segment = (variant & 2) ? 4096 : (1 << 20); c.capacity = (variant & 2) ? 37 : (1 << 20);
            c.seed = 2511u + 7u * (unsigned)variant; c.adv_eps = 1e-6;
            for (int r = 0; r < 5; ++r) {
                c.short_lo[r] = 500; c.short_hi[r] = 4000; c.long_hi[r] = 20000; c.p_long[r] = one / 8;
                c.p_correct[r] = one / 2; c.p_keep[r] = one * 9 / 10; c.p_flag_wrong[r] = one * 7 / 10; c.p_flag_right[r] = one / 5;
            }
            int64_t mi = 0, mg = 0;
            if (mars_sched_bounds(&c, &mi, &mg) != 0) { fprintf(stderr, "bounds failed\n"); return 1; }
            mars_sched_arrays_t a;
            int32_t **i32[] = {&a.item_problem, &a.item_role, &a.item_group, &a.item_member, &a.item_parent, &a.item_length,
                               &a.item_value, &a.item_reward};
            for (size_t k = 0; k < sizeof i32 / sizeof i32[0]; ++k) *i32[k] = (int32_t *)malloc(sizeof(int32_t) * (size_t)mi);
            a.item_t_done = (int64_t *)malloc(sizeof(int64_t) * (size_t)mi);
            int32_t **g32[] = {&a.group_problem, &a.group_role, &a.group_index, &a.group_parent};
            for (size_t k = 0; k < sizeof g32 / sizeof g32[0]; ++k) *g32[k] = (int32_t *)malloc(sizeof(int32_t) * (size_t)mg);
            int64_t **g64[] = {&a.group_t_submit, &a.group_t_group, &a.group_t_train};
            for (size_t k = 0; k < sizeof g64 / sizeof g64[0]; ++k) *g64[k] = (int64_t *)malloc(sizeof(int64_t) * (size_t)mg);
            a.group_adv = (double *)malloc(sizeof(double) * (size_t)mg * (size_t)c.group_size);
            mars_sched_summary_t s;
            if (mars_sched_simulate(&c, &s, &a, mi, mg) != 0) { fprintf(stderr, "simulate failed\n"); return 1; }
            if (s.n_items < c.problems * c.group_size || s.n_items > mi || s.n_groups > mg) { fprintf(stderr, "counts out of range\n"); return 1; }
            if (mars_sched_simulate(&c, &s, NULL, mi, mg) != 0) { fprintf(stderr, "summary-only run failed\n"); return 1; }
            for (size_t k = 0; k < sizeof i32 / sizeof i32[0]; ++k) free(*i32[k]);
            for (size_t k = 0; k < sizeof g32 / sizeof g32[0]; ++k) free(*g32[k]);
            for (size_t k = 0; k < sizeof g64 / sizeof g64[0]; ++k) free(*g64[k]);
            free(a.item_t_done); free(a.group_adv);
        }
    mars_sched_config_t bad;
    memset(&bad, 0, sizeof bad);
    int64_t x, y;
    if (mars_sched_bounds(&bad, &x, &y) == 0 || mars_sched_bounds(NULL, &x, &y) == 0) { fprintf(stderr, "bad configuration accepted\n"); return 1; }
    puts("scheduling simulator clean under the sanitizers");
    return 0;
}
