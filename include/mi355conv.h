/*
 * mi355conv -- Caffe-semantics 2-D ConvolutionLayer for AMD MI355X (gfx950), fp32.
 *
 * The paper lists the convolution layer among the "vision layers" of its Table 1 and
 * states in its Abstract that the stack follows C++ Caffe; its "General Architecture"
 * section describes a low-level native library that owns the device work, is called
 * with plain values and opaque handles, and never moves data off the GPU.  This header
 * is that boundary for the convolution layer: plain C, opaque descriptor, device
 * pointers in, device pointers out, no host<->device copies, no device allocation.
 *
 * Semantics (Cg = c/group, Kg = num_output/group, xz = x extended by zero):
 *   OH = floor((h + 2 pad_h - dilation_h (kernel_h - 1) - 1) / stride_h) + 1, same for OW
 *   forward         y[n,k,oh,ow] = bias[k] + sum_{c',i,j} w[k,c',i,j] *
 *                     xz[n, (k / Kg) Cg + c', oh stride_h - pad_h + i dilation_h,
 *                                             ow stride_w - pad_w + j dilation_w]
 *                   (a cross-correlation: the kernel is not flipped)
 *   backward data   dx = the transpose of the linear map x -> y applied to dy (overwrites dx)
 *   backward filter dw[k,c',i,j] = beta dw[k,c',i,j] + sum_{n,oh,ow} dy[n,k,oh,ow] * xz[... same tap ...]
 *   backward bias   db[k] = beta db[k] + sum_{n,oh,ow} dy[n,k,oh,ow]
 * beta = 1 is Caffe's "parameter diffs accumulate until the solver applies them" rule
 * (the paper's Appendix A/B training loops rely on it); beta = 0 overwrites and never
 * reads the old contents (NaN-safe).
 *
 * Layouts: dense, last index fastest, fp32, DEVICE memory, 16-byte aligned bases:
 *   x, dx : [n][c][h][w]          y, dy : [n][num_output][OH][OW]
 *   w, dw : [num_output][c/group][kernel_h][kernel_w]        bias, db : [num_output]
 * An output buffer must not overlap any input buffer or the workspace.
 *
 * Ownership: the caller owns every device buffer including the workspace; the library
 * keeps no pointer after a call returns and allocates no device memory.  A conv_desc_t
 * is host memory owned by the library from conv_desc_create to conv_desc_destroy; it is
 * immutable and may be shared between threads.
 *
 * Execution: every pass is enqueued on the caller's HIP stream (`hip_stream` is a
 * hipStream_t passed as void*; NULL = the default stream) and returns without
 * synchronising.  Passes that use the workspace must not run concurrently on different
 * streams with the same workspace.  A pass is one to three kernel launches (helper kernels
 * pack the weights, clear or add partial results around the main kernel).  The first call
 * of a pass in a process may also perform a one-time, thread-safe kernel attribute set-up
 * (the opt-in to more than 64 KB of LDS), which is a host-side runtime call and not an
 * enqueue: make that first call outside HIP stream capture; every later call only enqueues
 * kernels and can be captured into a HIP graph.
 *
 * Errors: every function returns a conv_status_t (0 = success, negative = error); no
 * exception, abort or printing crosses this boundary.  Argument, shape and workspace
 * errors are detected before anything is enqueued.  CONV_EHIP means the HIP runtime
 * refused a launch: helper kernels of the same pass launched before it stay enqueued
 * and the output buffer's contents are then unspecified.
 */
#ifndef MI355CONV_H
#define MI355CONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  CONV_OK = 0,
  CONV_EINVAL = -1,     /* null pointer, non-positive size, divisibility, bias/bias_term mismatch, beta not 0/1 */
  CONV_ESHAPE = -2,     /* computed OH or OW < 1, or a tensor (or the workspace) of 2^30 or more elements:
                           the kernels address every buffer with unsigned 32-bit byte offsets */
  CONV_EWORKSPACE = -3, /* workspace null or smaller than conv_desc_workspace_bytes */
  CONV_EHIP = -4        /* the HIP runtime refused a launch; see conv_last_hip_error */
} conv_status_t;

/* Caffe's convolution parameters plus the bottom blob shape (2-D spatial, channel axis 1). */
typedef struct {
  int32_t n, c, h, w;             /* bottom blob shape; n may be 0 (every pass is then a no-op) */
  int32_t num_output;             /* K >= 1 */
  int32_t kernel_h, kernel_w;     /* >= 1 */
  int32_t stride_h, stride_w;     /* >= 1 */
  int32_t pad_h, pad_w;           /* >= 0 */
  int32_t dilation_h, dilation_w; /* >= 1 */
  int32_t group;                  /* >= 1; c % group == 0 and num_output % group == 0 */
  int32_t bias_term;              /* 0 or 1 */
} conv_params_t;

typedef struct conv_desc conv_desc_t;

/*
 * Validates `p`, computes OH/OW, picks the kernel variants and sizes the workspace.
 * Host-only: touches no device.  *out is set only on success.
 */
int conv_desc_create(conv_desc_t** out, const conv_params_t* p);
int conv_desc_destroy(conv_desc_t* d);
/* Any of n, k, oh, ow may be NULL. */
int conv_desc_output_shape(const conv_desc_t* d, int32_t* n, int32_t* k, int32_t* oh, int32_t* ow);
/* Bytes of device workspace sufficient for any of the four passes (may be 0). */
int conv_desc_workspace_bytes(const conv_desc_t* d, size_t* bytes);

/* y = bias + w (*) x.  `bias` must be NULL iff bias_term == 0.  The bias add is fused. */
int conv_forward(const conv_desc_t* d, const float* x, const float* w, const float* bias, float* y,
                 void* ws, size_t ws_bytes, void* hip_stream);

/* dx = transpose-of-forward applied to dy; every element of dx is written. */
int conv_backward_data(const conv_desc_t* d, const float* w, const float* dy, float* dx,
                       void* ws, size_t ws_bytes, void* hip_stream);

/* dw = beta*dw + filter gradient; beta must be exactly 0 or 1.  Deterministic (no float atomics). */
int conv_backward_filter(const conv_desc_t* d, const float* x, const float* dy, float* dw, float beta,
                         void* ws, size_t ws_bytes, void* hip_stream);

/*
 * Backward filter and backward bias of one layer in one pass: dw = beta*dw + filter gradient and
 * db = beta*db + sum of dy over n, oh, ow (the two parameter gradients a Caffe layer produces in its
 * backward step, with the same accumulate rule), from a single read of dy -- the filter-gradient kernel
 * adds up the dy tiles it stages for the matrix unit, so the separate pass over dy that
 * conv_backward_bias makes (as large as the top blob) is saved.  Results are bit-identical from run
 * to run; dw is bit-identical to conv_backward_filter's, db may differ from conv_backward_bias's in
 * the last bits (another summation order).  CONV_EINVAL on a bias_term == 0 descriptor; otherwise the
 * rules of conv_backward_filter; the workspace is covered by conv_desc_workspace_bytes.
 */
int conv_backward_filter_bias(const conv_desc_t* d, const float* x, const float* dy, float* dw, float* db, float beta,
                              void* ws, size_t ws_bytes, void* hip_stream);

/*
 * conv_backward_filter for callers that cannot allocate or pass device memory for a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * semantics, layouts and result (bit for bit) as conv_backward_filter, without `ws`: the split
 * partials go to a fixed 32 MiB device array that belongs to the library (every GPU the library
 * runs on holds its own copy until the process ends).  The call allocates and frees nothing.
 * CONV_EWORKSPACE when the layer's filter-gradient workspace exceeds conv_static_workspace_limit()
 * (conv_desc_create sizes the partials to at most 32 MiB, so only a weight blob larger than that
 * is refused); use conv_backward_filter with a workspace of your own then.  All calls on one GPU share
 * that GPU's array: calls that may overlap on one GPU (different streams or threads) race on it and
 * must be ordered by the caller; calls on one stream are ordered by the stream.  The array keeps the
 * last call's contents and nothing in it needs clearing between calls.  The first call on a device
 * looks up the array's address (a host-side runtime call, thread-safe): make it outside stream capture.
 */
int conv_backward_filter_static(const conv_desc_t* d, const float* x, const float* dy, float* dw, float beta,
                                void* hip_stream);
/* Size in bytes of the fixed array behind conv_backward_filter_static. */
size_t conv_static_workspace_limit(void);

/* db = beta*db + sum of dy over n, oh, ow; CONV_EINVAL on a bias_term == 0 descriptor. */
int conv_backward_bias(const conv_desc_t* d, const float* dy, float* db, float beta,
                       void* ws, size_t ws_bytes, void* hip_stream);

/*
 * Double base type (the paper builds every layer for either a float or a double base type, section after
 * Table 1).  The same descriptor, semantics, layouts, ownership, execution and error rules as the
 * fp32 passes above, with every blob in doubles; products and sums are fp64 (fp64 matrix
 * instructions).  The workspace size differs: use conv_desc_workspace_bytes_f64.  A descriptor
 * with a blob of 2^29 or more elements has no double path: these functions return CONV_ESHAPE.
 */
int conv_desc_workspace_bytes_f64(const conv_desc_t* d, size_t* bytes);
/* Kernel variants of the double path ("fwd=...;bwd_data=...;..."); "" when the descriptor has none. */
const char* conv_desc_kernel_names_f64(const conv_desc_t* d);
int conv_forward_f64(const conv_desc_t* d, const double* x, const double* w, const double* bias, double* y, void* ws,
                     size_t ws_bytes, void* hip_stream);
int conv_backward_data_f64(const conv_desc_t* d, const double* w, const double* dy, double* dx, void* ws,
                           size_t ws_bytes, void* hip_stream);
int conv_backward_filter_f64(const conv_desc_t* d, const double* x, const double* dy, double* dw, double beta,
                             void* ws, size_t ws_bytes, void* hip_stream);
int conv_backward_bias_f64(const conv_desc_t* d, const double* dy, double* db, double beta, void* ws, size_t ws_bytes,
                           void* hip_stream);

const char* conv_status_string(int status);
/* hipError_t value of the most recent CONV_EHIP on the calling thread (0 if none). */
int conv_last_hip_error(void);
/* Names of the kernel variants the descriptor selected, for logs and profiles ("fwd=...;bwd_data=...;..."). */
const char* conv_desc_kernel_names(const conv_desc_t* d);

#ifdef __cplusplus
}
#endif
#endif /* MI355CONV_H */
