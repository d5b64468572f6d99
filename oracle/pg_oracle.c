/* CPU oracle for the policy-gradient loss arithmetic: see pg_oracle.h.  Test infrastructure. */
#include "pg_oracle.h"

#include <math.h>
#include <stddef.h>

int oracle_pg_sigmoid_sample_action(const double* aprob, const double* random, int64_t steps, int64_t* action) {
  if (steps < 0 || (steps > 0 && (!aprob || !random || !action))) return -1;
  for (int64_t t = 0; t < steps; ++t) action[t] = (random[t] < aprob[t]) ? 0 : 1;
  return 0;
}

int oracle_pg_sigmoid_dlogps(const double* aprob, const int64_t* action, int64_t steps, double* dlogps) {
  if (steps < 0 || (steps > 0 && (!aprob || !action || !dlogps))) return -1;
  for (int64_t t = 0; t < steps; ++t) {
    if (action[t] != 0 && action[t] != 1) return -1;
    dlogps[t] = (action[t] == 0) ? 1.0 - aprob[t] : 0.0 - aprob[t];
  }
  return 0;
}

int oracle_pg_softmax_dlogps(const double* logits, const int64_t* action, int64_t steps, int64_t actions,
                             double* probs, double* dlogps) {
  if (steps < 0 || actions < 1 || (steps > 0 && (!logits || !action || !dlogps))) return -1;
  for (int64_t t = 0; t < steps; ++t) {
    const double* l = logits + t * actions;
    if (action[t] < 0 || action[t] >= actions) return -1;
    double top = l[0];
    for (int64_t a = 1; a < actions; ++a)
      if (l[a] > top) top = l[a];
    double sum = 0.0;
    for (int64_t a = 0; a < actions; ++a) sum += exp(l[a] - top);
    for (int64_t a = 0; a < actions; ++a) {
      const double softmax = exp(l[a] - top) / sum;
      const double target = (a == action[t]) ? 1.0 : 0.0;
      if (probs) probs[t * actions + a] = softmax;
      dlogps[t * actions + a] = softmax - target;
    }
  }
  return 0;
}

int oracle_pg_discount_rewards(const double* reward, const int64_t* offsets, int64_t episodes, double gamma,
                               double* discounted) {
  if (episodes < 0 || !offsets || offsets[0] != 0) return -1;
  for (int64_t e = 0; e < episodes; ++e)
    if (offsets[e + 1] < offsets[e]) return -1;
  if (offsets[episodes] > 0 && (!reward || !discounted)) return -1;
  for (int64_t e = 0; e < episodes; ++e) {
    double running = 0.0; /* R past the end of the episode */
    for (int64_t t = offsets[e + 1] - 1; t >= offsets[e]; --t) {
      running = reward[t] + gamma * running;
      discounted[t] = running;
    }
  }
  return 0;
}

int oracle_pg_bottom_diff(const double* dlogps, const double* discounted, int64_t steps, int64_t actions,
                          int sigmoid_model, double* bottom_diff) {
  if (steps < 0 || actions < 1 || (steps > 0 && (!dlogps || !bottom_diff))) return -1;
  if (sigmoid_model && actions != 1) return -1;
  const double sign = sigmoid_model ? -1.0 : 1.0;
  for (int64_t t = 0; t < steps; ++t)
    for (int64_t a = 0; a < actions; ++a)
      bottom_diff[t * actions + a] = sign * dlogps[t * actions + a] * (discounted ? discounted[t] : 1.0);
  return 0;
}
