/*
 * mi355pg -- the policy-gradient loss arithmetic of the paper's reinforcement-learning trainer, for
 * AMD MI355X (gfx950), fp32.  Part of the same library as mi355conv.h.
 *
 * The paper's Appendix A (Sigmoid model, two actions) and Appendix B (Softmax model, any number of
 * actions) walk through one training step on a finished episode; the functions below are its
 * steps 3 and 8-11 for a whole batch of episodes stored back to back ("steps" = all time steps of
 * all episodes):
 *
 *   pg_sigmoid_sample_action  action = (random < Aprob) ? 0 : 1                    (Appendix A, step 3)
 *   pg_discount_rewards       R[t] = reward[t] + gamma R[t+1] inside each episode,
 *                             R past the episode's end = 0                          (step 9)
 *   pg_sigmoid_bottom_diff    Dlogps = (action == 0) ? 1 - Aprob : 0 - Aprob        (step 8)
 *                             bottom_diff = -Dlogps * R[t]                          (steps 10-11)
 *   pg_softmax_bottom_diff    probs = softmax(logits row); Dlogps = probs - onehot(action)
 *                             bottom_diff = Dlogps * R[t]                           (Appendix B, steps 8, 10-11)
 *
 * Sign of the Sigmoid bottom_diff: Figure 6 prints diff = -Dlogps together with
 * new weight = old weight - diff, which is the sign that reinforces the action taken when the
 * solver subtracts the diff; Figure 9 prints diff = softmax - target for the Softmax model.
 * gamma is a parameter (the paper gives none); the discounted rewards are not normalised.
 * discounted == NULL means a weight of 1 for every step (the figures' worked rows).
 *
 * Layouts: dense fp32 / int32 DEVICE memory, 16-byte aligned bases:
 *   aprob, random, reward, discounted, dlogps, sigmoid bottom_diff : [steps]      action : int32 [steps]
 *   logits, probs, softmax bottom_diff : [steps][actions]      episode_offsets : int32 [episodes + 1],
 *   episode e = steps [episode_offsets[e], episode_offsets[e+1]), first entry 0, last = steps.
 * An action outside its range is never used as an index: the Sigmoid model treats any non-zero
 * value as action 1, the Softmax model then has no target (Dlogps = probs).  Offsets are clamped
 * to [0, steps] inside the kernel.  Outputs must not overlap inputs.
 *
 * No workspace, no descriptor, no device allocation; enqueued on the caller's hipStream_t
 * (void*, NULL = default stream) without synchronising.  Returns a conv_status_t: CONV_EINVAL
 * for null pointers / negative sizes / actions < 1, CONV_ESHAPE when steps (or episodes) exceed
 * 2^31 - 65536 or steps * actions >= 2^31.
 * steps == 0 (or episodes == 0) is a no-op.  The first pg_softmax_bottom_diff call of a process
 * with exactly 32 actions performs a one-time, thread-safe kernel attribute set-up (66 KB of LDS)
 * and must be made outside HIP stream capture; every other call only enqueues kernels.
 */
#ifndef MI355PG_H
#define MI355PG_H

#include "mi355conv.h"

#ifdef __cplusplus
extern "C" {
#endif

int pg_sigmoid_sample_action(const float* aprob, const float* random, int32_t* action, int32_t steps,
                             void* hip_stream);
int pg_discount_rewards(const float* reward, const int32_t* episode_offsets, int32_t episodes, int32_t steps,
                        float gamma, float* discounted, void* hip_stream);
/* dlogps may be NULL (not wanted); discounted may be NULL (weight 1). */
int pg_sigmoid_bottom_diff(const float* aprob, const int32_t* action, const float* discounted, float* dlogps,
                           float* bottom_diff, int32_t steps, void* hip_stream);
/* probs may be NULL (not wanted); discounted may be NULL (weight 1). */
int pg_softmax_bottom_diff(const float* logits, const int32_t* action, const float* discounted, float* probs,
                           float* bottom_diff, int32_t steps, int32_t actions, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif
