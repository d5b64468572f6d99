/*
 * CPU oracle for the Caffe-semantics 2-D ConvolutionLayer (test infrastructure).
 *
 * This is a checker, not a product path: only tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it.  It is independent of the GPU
 * library: it shares no header, helper, table or constant with it.
 *
 * What it computes.  The paper only names the layer family ("All vision
 * layers", Table 1) and says the stack follows C++ Caffe (Abstract); the
 * arithmetic below is therefore the plain textbook definition of Caffe's
 * convolution (a cross-correlation, kernel not flipped) with num_output,
 * kernel, stride, pad, dilation, group and bias_term, over dense NCHW blobs,
 * written as direct nested loops in double precision: no lowering, no GEMM,
 * no blocking.  The paper's remark that the base type is either float or double (section after Table 1)
 * is why inputs are fp32 values widened to double by the caller.
 *
 * Layouts (all dense, last index fastest):
 *   x, dx : [n][c][h][w]              y, dy : [n][num_output][oh][ow]
 *   w, dw : [num_output][c/group][kernel_h][kernel_w]      b, db : [num_output]
 * Group g uses input channels [g*c/group, (g+1)*c/group) and output channels
 * [g*num_output/group, (g+1)*num_output/group).
 *
 * Every function returns 0 on success, -1 on invalid parameters.
 * Parity pins: every function here is pinned by tests/test_oracle_pins.py
 * (hand-worked fixtures, brute force from the definition, adjoint identities,
 * finite differences, reductions to library routines).  Nothing is unpinned.
 */
#ifndef CONV_ORACLE_H
#define CONV_ORACLE_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
  int64_t n, c, h, w;            /* bottom blob shape */
  int64_t num_output;
  int64_t kernel_h, kernel_w;
  int64_t stride_h, stride_w;
  int64_t pad_h, pad_w;
  int64_t dilation_h, dilation_w;
  int64_t group;
  int64_t bias_term;
} oracle_conv_params;

/* floor((in + 2*pad - dilation*(kernel-1) - 1) / stride) + 1; <= 0 means "no output". */
int64_t oracle_conv_out_size(int64_t in, int64_t kernel, int64_t stride, int64_t pad, int64_t dilation);
int oracle_conv_output_shape(const oracle_conv_params* p, int64_t* oh, int64_t* ow);

/* y = bias + correlation(x, w).  b may be NULL iff bias_term == 0. */
int oracle_conv_forward(const oracle_conv_params* p, const double* x, const double* w, const double* b, double* y);
/* dx = adjoint of the linear part applied to dy (overwrites dx). */
int oracle_conv_backward_data(const oracle_conv_params* p, const double* w, const double* dy, double* dx);
/* dw = beta*dw + sum over n,oh,ow of dy * shifted x. */
int oracle_conv_backward_filter(const oracle_conv_params* p, const double* x, const double* dy, double* dw, double beta);
/* db = beta*db + sum over n,oh,ow of dy. */
int oracle_conv_backward_bias(const oracle_conv_params* p, const double* dy, double* db, double beta);

/* One-by-one versions for full-size spot checks: out[s] = the element with flat index idx[s]. */
int oracle_conv_forward_at(const oracle_conv_params* p, const double* x, const double* w, const double* b,
                           const int64_t* idx, int64_t count, double* out);
int oracle_conv_backward_data_at(const oracle_conv_params* p, const double* w, const double* dy,
                                 const int64_t* idx, int64_t count, double* out);
/* beta-free: returns only the gradient sum for the sampled dw elements. */
int oracle_conv_backward_filter_at(const oracle_conv_params* p, const double* x, const double* dy,
                                   const int64_t* idx, int64_t count, double* out);

/* OpenMP threads the loops above run on (1 when built without OpenMP). */
int oracle_num_threads(void);

#ifdef __cplusplus
}
#endif
#endif
