/*
 * grpo_loss.h - C ABI of the token log-probability and GRPO objective step for AMD gfx950 (MI355X), one GPU.
 *
 * This is the other half of "log-prob recompute": after the policy's forward pass has produced the logits of
 * every response token, the trainer needs log pi_theta(o_t) for the importance ratio (Section 2.2, Eq. 3) and
 * the clipped, KL-regularised surrogate built from it (Eq. 2) with group-normalised advantages (Eq. 1).
 *
 *   N response tokens (the G responses of one group, concatenated), V vocabulary entries, G responses.
 *   response i owns tokens [resp_offsets[i], resp_offsets[i+1]);  resp_offsets[0] = 0, resp_offsets[G] = N.
 *
 *   logp[t]   = logits[t, target[t]] - log( sum_v exp(logits[t, v]) )                       (log-softmax, gathered)
 *   A_i       = (r_i - mean(r)) / (std(r) + adv_eps),   std = population standard deviation  (Eq. 1)
 *   ratio_t   = exp(logp[t] - logp_old[t])                                                    (Eq. 3)
 *   kl_t      = exp(d) - d - 1,  d = logp_ref[t] - logp[t]     (the per-token estimator of D_KL(pi_theta || pi_ref)
 *               that GRPO uses; the paper writes the divergence without naming an estimator)
 *   term_t    = min(ratio_t * A_i, clip(ratio_t, 1-eps, 1+eps) * A_i) - beta * kl_t          (Eq. 2, inner bracket)
 *   mean_i    = (1/|o_i|) sum_{t in response i} term_t      (0 for a response without tokens)
 *   J         = (1/G) sum_i mean_i                                                            (Eq. 2)
 *
 * Conventions are those of moe_ffn.h: device pointers unless marked host, caller-owned buffers and stream,
 * nothing allocated, nothing synchronised, arguments validated on the host before any HIP call (N == 0 or
 * G == 0 is MOE_OK and enqueues nothing), 16-byte aligned pointers.  V must be a multiple of 8.  Arithmetic is
 * float; the log-sum-exp runs online (running maximum and rescaled sum) in one pass over the logits, which is
 * what bounds the step: N*V stored elements read once from HBM.  Results are deterministic (fixed reduction
 * trees, no atomics).
 */
#ifndef GRPO_LOSS_H
#define GRPO_LOSS_H

#include "moe_ffn.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t N;        /* response tokens (>= 0) */
    int32_t V;        /* vocabulary size, multiple of 8 */
    int32_t G;        /* responses in the group (>= 0) */
    int32_t dtype;    /* storage type of logits: MOE_BF16 or MOE_F32 */
    float clip_eps;   /* epsilon of the clipped surrogate */
    float beta;       /* weight of the KL term */
    float adv_eps;    /* added to the standard deviation in Eq. 1 */
} grpo_shape_t;

/* logp[t] for every token.  logits [N,V] dtype, target [N] int32 in [0,V) (clamped if outside), logp [N] float out. */
moe_status_t grpo_token_logprob(const grpo_shape_t *shape, const void *logits, const int32_t *target,
                                float *logp, void *stream);

/* Eq. 1-3 from token log-probabilities.
 *   logp, logp_old, logp_ref [N] float; rewards [G] float; resp_offsets [G+1] int32 (non-decreasing, as above)
 *   advantage [G] float out; token_term [N] float out; resp_mean [G] float out; objective [1] float out */
moe_status_t grpo_objective(const grpo_shape_t *shape, const float *logp, const float *logp_old,
                            const float *logp_ref, const float *rewards, const int32_t *resp_offsets,
                            float *advantage, float *token_term, float *resp_mean, float *objective,
                            void *stream);

/* Both steps in one call: logits -> logp -> objective.  logp [N] float is an output as well. */
moe_status_t grpo_logprob_objective(const grpo_shape_t *shape, const void *logits, const int32_t *target,
                                    const float *logp_old, const float *logp_ref, const float *rewards,
                                    const int32_t *resp_offsets, float *logp, float *advantage,
                                    float *token_term, float *resp_mean, float *objective, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* GRPO_LOSS_H */
