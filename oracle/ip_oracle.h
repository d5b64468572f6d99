/*
 * CPU oracle for the Caffe-semantics InnerProduct layer with an optional ReLU on its output
 * (test infrastructure).
 *
 * This is a checker, not a product path: only tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it.  It shares no header, helper, table or constant with the GPU
 * library.
 *
 * What it computes.  The paper lists the layer families it carries over from C++ Caffe ("All
 * common layers", "All neuron layers", Table 1) and uses an InnerProduct layer as the one that
 * feeds the loss in both policy-gradient models (Appendix A, Appendix B); it prints no formula,
 * so the arithmetic is Caffe's plain definition, written as direct loops in double precision:
 *
 *   z[n][o]  = (bias_term ? b[o] : 0) + sum_k x[n][k] * w[o][k]          (weights [num_output][k])
 *   y[n][o]  = relu ? max(z[n][o], 0) : z[n][o]
 *   dz[n][o] = relu ? (y[n][o] > 0 ? dy[n][o] : 0) : dy[n][o]            (ReLU passes the gradient
 *                                                                          only where its input was > 0)
 *   dx[n][k] = sum_o dz[n][o] * w[o][k]                                   (overwrites)
 *   dw[o][k] = beta*dw[o][k] + sum_n dz[n][o] * x[n][k]
 *   db[o]    = beta*db[o]    + sum_n dz[n][o]
 *
 * The bottom blob [n][c][h][w] is read flattened from axis 1: k = c*h*w, row-major.
 * beta = 1 is Caffe's accumulate-into-diff convention (the policy-gradient trainer accumulates
 * gradients over a batch of episodes, Appendix A step 11), beta = 0 overwrites without reading.
 *
 * Every function returns 0 on success, -1 on invalid parameters.
 * Parity pins: tests/test_ip_oracle_pins.py (hand-worked fixture, brute force, the convolution
 * oracle with a full-size kernel, matmul, adjoint identities, finite differences through the
 * ReLU, mask edge cases).  Nothing is unpinned.
 */
#ifndef IP_ORACLE_H
#define IP_ORACLE_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
  int64_t m;           /* rows of the bottom blob = batch size n */
  int64_t k;           /* inputs per row = c*h*w */
  int64_t num_output;
  int64_t bias_term;
  int64_t relu;
} oracle_ip_params;

int oracle_ip_forward(const oracle_ip_params* p, const double* x, const double* w, const double* b, double* y);
int oracle_ip_relu_backward(const oracle_ip_params* p, const double* y, const double* dy, double* dz);
int oracle_ip_backward_data(const oracle_ip_params* p, const double* w, const double* dz, double* dx);
int oracle_ip_backward_filter(const oracle_ip_params* p, const double* x, const double* dz, double* dw, double beta);
int oracle_ip_backward_bias(const oracle_ip_params* p, const double* dz, double* db, double beta);
int oracle_ip_num_threads(void);

#ifdef __cplusplus
}
#endif
#endif
