/* CPU oracle for the InnerProduct layer (+ optional ReLU): see ip_oracle.h.  Test infrastructure. */
#include "ip_oracle.h"

#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int valid(const oracle_ip_params* p) {
  return p && p->m >= 0 && p->k >= 1 && p->num_output >= 1 && (p->bias_term == 0 || p->bias_term == 1) &&
         (p->relu == 0 || p->relu == 1);
}

int oracle_ip_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

int oracle_ip_forward(const oracle_ip_params* p, const double* x, const double* w, const double* b, double* y) {
  if (!valid(p) || !x || !w || !y) return -1;
  if ((p->bias_term != 0) != (b != NULL)) return -1;
  const int64_t M = p->m, K = p->k, O = p->num_output;
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t n = 0; n < M; ++n)
    for (int64_t o = 0; o < O; ++o) {
      double z = p->bias_term ? b[o] : 0.0;
      for (int64_t k = 0; k < K; ++k) z += x[n * K + k] * w[o * K + k];
      y[n * O + o] = (p->relu && !(z > 0.0)) ? 0.0 : z;
    }
  return 0;
}

int oracle_ip_relu_backward(const oracle_ip_params* p, const double* y, const double* dy, double* dz) {
  if (!valid(p) || !dy || !dz) return -1;
  if (p->relu && !y) return -1;
  const int64_t cnt = p->m * p->num_output;
  for (int64_t i = 0; i < cnt; ++i) dz[i] = (!p->relu || y[i] > 0.0) ? dy[i] : 0.0;
  return 0;
}

int oracle_ip_backward_data(const oracle_ip_params* p, const double* w, const double* dz, double* dx) {
  if (!valid(p) || !w || !dz || !dx) return -1;
  const int64_t M = p->m, K = p->k, O = p->num_output;
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t n = 0; n < M; ++n)
    for (int64_t k = 0; k < K; ++k) {
      double s = 0.0;
      for (int64_t o = 0; o < O; ++o) s += dz[n * O + o] * w[o * K + k];
      dx[n * K + k] = s;
    }
  return 0;
}

int oracle_ip_backward_filter(const oracle_ip_params* p, const double* x, const double* dz, double* dw, double beta) {
  if (!valid(p) || !x || !dz || !dw) return -1;
  const int64_t M = p->m, K = p->k, O = p->num_output;
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t o = 0; o < O; ++o)
    for (int64_t k = 0; k < K; ++k) {
      double s = 0.0;
      for (int64_t n = 0; n < M; ++n) s += dz[n * O + o] * x[n * K + k];
      dw[o * K + k] = (beta == 0.0) ? s : beta * dw[o * K + k] + s;
    }
  return 0;
}

int oracle_ip_backward_bias(const oracle_ip_params* p, const double* dz, double* db, double beta) {
  if (!valid(p) || !dz || !db) return -1;
  if (!p->bias_term) return -1;
  const int64_t M = p->m, O = p->num_output;
  for (int64_t o = 0; o < O; ++o) {
    double s = 0.0;
    for (int64_t n = 0; n < M; ++n) s += dz[n * O + o];
    db[o] = (beta == 0.0) ? s : beta * db[o] + s;
  }
  return 0;
}
