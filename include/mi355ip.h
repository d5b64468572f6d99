/*
 * mi355ip -- Caffe-semantics InnerProduct layer with an optional fused ReLU, for AMD MI355X
 * (gfx950), fp32.  Part of the same library as mi355conv.h and built on the same kernels.
 *
 * The paper carries the layer over from C++ Caffe ("All common layers" and "All neuron layers"
 * in its Table 1) and makes it the layer that feeds the loss in both policy-gradient models of
 * its Appendix A and Appendix B; the boundary rules are those of its "General Architecture"
 * section (plain values and opaque handles in, data stays on the device).
 *
 * Semantics (x is the bottom blob [m][c][h][w] read flattened from axis 1, k = c*h*w):
 *   forward          z[n][o] = bias[o] + sum_i x[n][i] * w[o][i];   y = relu ? max(z, 0) : z
 *                    (bias add and ReLU are fused into the kernel that finishes the sums)
 *   relu backward    dz[n][o] = y[n][o] > 0 ? dy[n][o] : 0          (relu = 0: dz = dy)
 *   backward data    dx[n][i] = sum_o dz[n][o] * w[o][i]            (overwrites dx)
 *   backward filter  dw[o][i] = beta dw[o][i] + sum_n dz[n][o] * x[n][i]
 *   backward bias    db[o]    = beta db[o]    + sum_n dz[n][o]
 * beta is 0 (overwrite, never reads the old contents) or 1 (Caffe's accumulate-into-diff rule,
 * which the Appendix A/B training loops rely on).  The three gradient passes take dz, i.e. the
 * top gradient after ip_relu_backward when the descriptor has relu = 1.
 *
 * Layouts: dense row-major fp32 DEVICE memory, 16-byte aligned bases:
 *   x, dx : [m][k]      w, dw : [num_output][k]      y, dy, dz : [m][num_output]      bias, db : [num_output]
 * Outputs must not overlap inputs or the workspace, except that dz may be dy itself.
 *
 * Ownership, execution and errors are as in mi355conv.h: the caller owns all device memory
 * including the workspace, every pass is enqueued on the caller's hipStream_t (void*, NULL =
 * default stream) without synchronising, and every function returns a conv_status_t
 * (CONV_ESHAPE: a tensor of 2^30 or more elements).  m may be 0: forward, relu backward and
 * backward data are then no-ops and the two parameter gradients become beta times themselves.
 */
#ifndef MI355IP_H
#define MI355IP_H

#include "mi355conv.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
  int32_t m;          /* rows of the bottom blob (batch size), >= 0 */
  int32_t k;          /* inputs per row, >= 1 */
  int32_t num_output; /* >= 1 */
  int32_t bias_term;  /* 0 or 1 */
  int32_t relu;       /* 0 or 1: clamp the output at zero from below */
} ip_params_t;

typedef struct ip_desc ip_desc_t;

/* Validates p, picks kernels and sizes the workspace; touches no device.  *out is written only on success. */
int ip_desc_create(ip_desc_t** out, const ip_params_t* p);
int ip_desc_destroy(ip_desc_t* d);
/* Largest workspace any pass of this descriptor needs, in bytes. */
int ip_desc_workspace_bytes(const ip_desc_t* d, size_t* bytes);
/* "fwd=...;bwd_data=...;bwd_filter=...;bwd_bias=..." -- the kernel variants chosen; owned by d. */
const char* ip_desc_kernel_names(const ip_desc_t* d);

/* bias must be NULL exactly when bias_term == 0. */
int ip_forward(const ip_desc_t* d, const float* x, const float* w, const float* bias, float* y, void* ws,
               size_t ws_bytes, void* hip_stream);
/* y is the forward output; ignored (may be NULL) when relu == 0, where dz = dy is copied unless dz == dy. */
int ip_relu_backward(const ip_desc_t* d, const float* y, const float* dy, float* dz, void* hip_stream);
int ip_backward_data(const ip_desc_t* d, const float* w, const float* dz, float* dx, void* ws, size_t ws_bytes,
                     void* hip_stream);
int ip_backward_filter(const ip_desc_t* d, const float* x, const float* dz, float* dw, float beta, void* ws,
                       size_t ws_bytes, void* hip_stream);
/* CONV_EINVAL when bias_term == 0. */
int ip_backward_bias(const ip_desc_t* d, const float* dz, float* db, float beta, void* ws, size_t ws_bytes,
                     void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif
