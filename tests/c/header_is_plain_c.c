/* The public headers must be usable from plain C: this file includes them in a C99 translation
 * unit, takes the address of every entry point with its declared type, and checks the layout
 * of the structures that cross the boundary.  Compiled (not run) by tests/test_host_library.py. */
#include "eager.h"
#include "eager_tuning.h"

#include <stddef.h>

typedef char static_check_plan[(sizeof(eager_plan) == 40 && offsetof(eager_plan, mask) == 16 &&
                                offsetof(eager_plan, flags) == 32) ? 1 : -1];
typedef char static_check_stats[(sizeof(eager_bucket_stats) == 32 &&
                                 offsetof(eager_bucket_stats, rate) == 24) ? 1 : -1];
typedef char static_check_opt[(offsetof(eager_opt, lr) == 2 * sizeof(void *)) ? 1 : -1];

int (*const p_create)(eager_ctx **, int, int, const int64_t *, const int64_t *, int, int) = eager_create;
int (*const p_destroy)(eager_ctx *) = eager_destroy;
const char *(*const p_last_error)(const eager_ctx *) = eager_last_error;
const char *(*const p_status_string)(int) = eager_status_string;
int (*const p_plan)(int, int, const double *, uint64_t, uint64_t, double, uint32_t, eager_plan *) =
    eager_plan_participation;
int (*const p_plan_quorum)(int, const double *, int, uint64_t, double, eager_plan *) = eager_plan_quorum;
int (*const p_designated)(uint64_t, uint64_t, int, int *) = eager_designated_initiator;
int (*const p_open_round)(int, int, uint64_t, int, int, uint64_t, uint64_t, int *, eager_plan *) =
    eager_plan_open_round;
int (*const p_solo)(eager_ctx *, const eager_plan *, int, int, const void *const *, float *const *,
                    float *, const eager_opt *, void *) = eager_partial_allreduce_solo;
int (*const p_majority)(eager_ctx *, const eager_plan *, int, int, const void *const *, float *const *,
                        float *, const eager_opt *, void *) = eager_partial_allreduce_majority;
int (*const p_quorum)(eager_ctx *, const eager_plan *, int, int, const void *const *, float *const *,
                      float *, const eager_opt *, void *) = eager_partial_allreduce_quorum;
int (*const p_lagging)(eager_ctx *, const eager_plan *, uint64_t, int, int, const void *const *,
                       float *const *, float *, const eager_opt *, void *) = eager_partial_allreduce_lagging;
int (*const p_exchange)(eager_ctx *, const eager_plan *, const void **, float **, float *, const eager_opt *,
                        void *) = eager_partial_allreduce_exchange;
int (*const p_stash)(eager_ctx *, int, int, int, const void *, float *, void *) = eager_stash;
int (*const p_flush)(eager_ctx *, int, int, float *const *, float *, const eager_opt *, void *) = eager_flush;
int (*const p_sgd)(eager_ctx *, int, int, const float *, const eager_opt *, void *) = eager_sgd_step;
int (*const p_lars)(eager_ctx *, int, int, const float *, const eager_opt *, float, float, void *) =
    eager_sgd_step_lars;
int (*const p_lars_static)(eager_ctx *, int, int, const float *, const eager_opt *, float, float,
                           eager_bucket_stats *, void *) = eager_sgd_step_lars_static;
const char *(*const p_source_hash)(void) = eager_source_hash;
int (*const p_views)(eager_ctx *, int, int, const float *, int, float *const *, float *const *, float,
                     float, void *) = eager_sgd_step_views;
int (*const p_average)(eager_ctx *, int, int, int, float *const *, void *) = eager_average_views;
int (*const p_rule)(eager_ctx *, float, int) = eager_set_update_rule;
int (*const p_stats_bytes)(const eager_ctx *, int64_t *) = eager_stats_workspace_bytes;
int (*const p_stats_attach)(eager_ctx *, eager_bucket_stats *, void *, int64_t, void *) = eager_stats_attach;
int (*const p_get_valid)(const eager_ctx *, int, uint64_t *) = eager_get_valid;
int (*const p_set_valid)(eager_ctx *, int, uint64_t) = eager_set_valid;
int (*const p_set_launch)(eager_ctx *, const char *, int) = eager_set_launch;
int (*const p_calib_copy)(void *, const void *, int64_t, void *) = eager_calib_copy;
int (*const p_calib_read)(const void *, int64_t, float *, void *) = eager_calib_read;
int (*const p_calib_mix)(const void *const *, int, uint64_t, void *const *, int, int64_t, int, float *,
                         void *) = eager_calib_mix;

/* host-only calls can run without a GPU: plan one round of each kind */
int main(void)
{
    const double arrival[4] = {3.0, 1.0, 2.0, 1.0};
    eager_plan plan;
    if (eager_plan_participation(EAGER_SOLO, 4, arrival, 1u, 0u, 0.0, 0u, &plan) != EAGER_OK) return 1;
    if (plan.initiator != 1 || plan.mask != 0xAu || plan.nap != 2) return 2;      /* tie: ranks 1 and 3 */
    if (eager_plan_quorum(4, arrival, 3, 0u, 0.0, &plan) != EAGER_OK) return 3;
    if (plan.initiator != 2 || plan.mask != 0xEu || plan.mode != EAGER_QUORUM) return 4;
    if (eager_plan_quorum(4, arrival, 5, 0u, 0.0, &plan) != EAGER_EINVAL) return 5;
    {
        int go = -1, rank = -1;
        if (eager_designated_initiator(0u, 0u, 64, &rank) != EAGER_OK || rank != 0x2F) return 6;
        if (eager_plan_open_round(EAGER_QUORUM, 4, 0x6u, 2, 3, 0u, 7u, &go, &plan) != EAGER_OK || go != 0) return 7;
        if (eager_plan_open_round(EAGER_QUORUM, 4, 0x7u, 0, 3, 0u, 7u, &go, &plan) != EAGER_OK || go != 1) return 8;
        if (plan.initiator != 0 || plan.mask != 0x7u || plan.nap != 3 || plan.step != 7u) return 9;
        if (eager_plan_open_round(EAGER_SOLO, 4, 0xCu, 3, 0, 0u, 1u, &go, &plan) != EAGER_OK || !go ||
            plan.initiator != 2) return 10;
        if (eager_plan_open_round(EAGER_SOLO, 4, 0x0u, 0, 0, 0u, 1u, &go, &plan) != EAGER_EINVAL) return 11;
    }
    return 0;
}
