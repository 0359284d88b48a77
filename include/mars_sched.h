/*
 * mars_sched.h - C ABI of a discrete-event simulator of MarsRL's agentic rollout scheduling (host code only; no GPU).
 *
 * It models what the paper describes around the policy's forward passes: the Verifier-Corrector pipeline unrolled
 * over five roles with at most five rollout iterations per problem (Section 3.1), agent-specific verifiable rewards
 * (Section 3.2), grouped agentic rollouts and agentic pipeline parallelism (Section 3.3), the Random / Balanced /
 * Adaptive sampling strategies (Section 3.4), group-normalised advantages (Section 2.2, Eq. 1) and segment rollout
 * (Section 2.3).  Output lengths and success rates are synthetic inputs; what the simulator answers is when each
 * group of outputs becomes available for training under a given schedule.
 *
 * Model
 *   roles 0..4 = Solver, Verifier1, Corrector1, Verifier2, Corrector2.  The Solver produces one group of group_size
 *   outputs per problem; when an agent's groups for a problem are all back, the next agent picks up to n_select of
 *   their outputs (a Corrector only bug reports that flag an error) and produces a group for each; no candidate ends
 *   the trajectory early, Corrector2 ends it always.
 *   value: Solver/Corrector output 1 = correct solution; Verifier output 1 = flags an error.  reward: value for
 *   Solver/Corrector; for a Verifier 1 exactly when it flags an incorrect solution or passes a correct one.
 *   strategies: 0 Random; 1 Balanced (n_select/2 of reward 1, the rest of reward 0, filled from what is left when a
 *   class runs out); 2 Adaptive (Verifiers take reward-0 outputs first, Correctors reward-1 outputs first).
 *   time: decoding advances in stages; in a stage every sequence holding one of `capacity` slots (0 = unlimited,
 *   first in first out) decodes min(segment, what it has left) tokens, the stage lasts as long as the longest of
 *   these, and finished sequences are handed back at its end.  A group's t_group is the end of the stage in which its
 *   last member finished; t_train = t_group with pipeline != 0, else the time its problem's trajectory ended.
 *   advantages: (r - mean) / (population std + adv_eps) inside each group.
 *   random draws: SplitMix64 of SplitMix64(seed) ^ key, key = ((((problem*8 + role)*4 + group)*64 + member)*8 +
 *   purpose), purposes 0 length class, 1 length, 2 outcome, 3 pick (group 3, member 8*list + position); a probability
 *   p (in units of 2^-24) holds when (draw >> 40) < p; a number in [0, n) is (draw >> 11) mod n; picks are a partial
 *   Fisher-Yates shuffle of the candidate list in creation order.  Lengths: with probability p_long uniform in
 *   [short_hi, long_hi], else uniform in [short_lo, short_hi].
 *
 * All pointers are HOST pointers, owned by the caller.  Nothing is kept between calls.
 */
#ifndef MARS_SCHED_H
#define MARS_SCHED_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t problems, group_size, n_select, segment, capacity, strategy, pipeline, reserved;
    uint64_t seed;
    double adv_eps;
    int32_t short_lo[5], short_hi[5], long_hi[5];                  /* tokens, per role */
    int32_t p_long[5], p_correct[5], p_keep[5], p_flag_wrong[5], p_flag_right[5];   /* 2^-24 units, per role */
} mars_sched_config_t;

typedef struct {
    int64_t makespan, tokens, sum_t_train, sum_wait;               /* sum_wait = sum over groups of t_train - t_submit */
    int32_t n_items, n_groups;
    int32_t early_stop[5];                                         /* trajectories that ended before role r ran */
} mars_sched_summary_t;

/* Outputs, each an array the caller sizes from mars_sched_bounds(); any pointer may be NULL (not written). */
typedef struct {
    int32_t *item_problem, *item_role, *item_group, *item_member, *item_parent, *item_length, *item_value, *item_reward;
    int64_t *item_t_done;
    int32_t *group_problem, *group_role, *group_index, *group_parent;
    int64_t *group_t_submit, *group_t_group, *group_t_train;
    double *group_adv;                                             /* [n_groups * group_size] */
} mars_sched_arrays_t;

/* 0 = ok, 1 = NULL argument, 2 = bad configuration (counts < 1, n_select > 8, group_size > 64, ranges not ordered,
 * strategy outside 0..2, probabilities outside [0, 2^24]), 3 = arrays too small. */
int mars_sched_bounds(const mars_sched_config_t *cfg, int64_t *max_items, int64_t *max_groups);
int mars_sched_simulate(const mars_sched_config_t *cfg, mars_sched_summary_t *summary, const mars_sched_arrays_t *out,
                        int64_t cap_items, int64_t cap_groups);

#ifdef __cplusplus
}
#endif
#endif /* MARS_SCHED_H */
