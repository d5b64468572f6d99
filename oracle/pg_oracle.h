/*
 * CPU oracle for the policy-gradient loss arithmetic of the paper's reinforcement-learning
 * trainer (test infrastructure; shares nothing with the GPU library).
 *
 * Steps and notation follow the paper's two walk-throughs (Appendix A, Sigmoid model; Appendix B,
 * Softmax model), in its order, in double precision:
 *
 *   step 3   action = (random < Aprob) ? 0 : 1                        (Appendix A; random is an input)
 *   step 8   Sigmoid:  Dlogps = (action == 0) ? 1 - Aprob : 0 - Aprob (Appendix A, "Sigmoid Gradient Calculation")
 *            Softmax:  softmax from the action logits; Dlogps = softmax - target, target = one-hot(action)
 *                                                                      (Appendix B, "Softmax Gradient Calculation")
 *   step 9   discounted rewards, accumulated from the end of the episode backwards: R[t] = reward[t] + gamma * R[t+1]
 *            inside each episode, R past the episode's last step = 0
 *   step 10  modulated gradient = Dlogps * discounted reward of that step
 *   step 11  Bottom.diff of the layer feeding the loss
 *
 * Readings (the paper is silent or at odds with itself here):
 *   - gamma is not given: it is a parameter.  No normalisation of the discounted rewards is
 *     described, so none is applied.
 *   - Sign of the Sigmoid Bottom.diff: the formula line says Bottom.diff = Dlogps * discounted
 *     rewards, but Figure 6 prints diff = -Dlogps (Dlogps -0.1 -> diff 0.1) together with
 *     new weight = old weight - diff (1 -> 0.9) and "new result" 0.09; the solver subtracts the
 *     diff, so the table's sign is the one that reinforces the action taken.  The oracle follows
 *     the table: sigmoid bottom_diff = -Dlogps * R.  Figure 9 (Softmax) prints diff = softmax -
 *     target with the same weight rule, which agrees with its formula: bottom_diff = Dlogps * R.
 *   - discounted == NULL means "all ones" (the figures' worked rows use reward weight 1).
 *
 * Every function returns 0 on success, -1 on invalid arguments.
 * Parity pins: tests/test_pg_oracle_pins.py checks every function against the rows the paper
 * prints in Figure 6 and Figure 9 (tests/golden/pg_figure6.json, pg_figure9.json), closed forms
 * of the discount recurrence, brute force and planted mistakes.  Nothing is unpinned.
 */
#ifndef PG_ORACLE_H
#define PG_ORACLE_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

int oracle_pg_sigmoid_sample_action(const double* aprob, const double* random, int64_t steps, int64_t* action);
int oracle_pg_sigmoid_dlogps(const double* aprob, const int64_t* action, int64_t steps, double* dlogps);
/* probs (may be NULL) and dlogps are [steps][actions]. */
int oracle_pg_softmax_dlogps(const double* logits, const int64_t* action, int64_t steps, int64_t actions,
                             double* probs, double* dlogps);
/* episode e covers steps [offsets[e], offsets[e+1]); offsets[0] = 0, non-decreasing. */
int oracle_pg_discount_rewards(const double* reward, const int64_t* offsets, int64_t episodes, double gamma,
                               double* discounted);
/* bottom_diff[t][a] = sign * dlogps[t][a] * (discounted ? discounted[t] : 1), sign = -1 for the
 * Sigmoid model (actions must be 1), +1 for the Softmax model. */
int oracle_pg_bottom_diff(const double* dlogps, const double* discounted, int64_t steps, int64_t actions,
                          int sigmoid_model, double* bottom_diff);

#ifdef __cplusplus
}
#endif
#endif
