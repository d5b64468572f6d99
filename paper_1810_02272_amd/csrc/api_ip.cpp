// Host side of the InnerProduct boundary.  The layer's three contractions are the convolution
// passes of one 1x1 "role-exchanged" problem -- a single image whose channels are the num_output
// rows of w, whose width is k, and whose output channels are the m rows of the batch:
//   forward          y[m][o]  = x w^T      = filter gradient  (dy' = x,  x' = w)      + bias/ReLU in its reduce
//   backward data    dx[m][k] = dz w       = forward          (w' = dz,  x' = w)
//   backward filter  dw[o][k] = dz^T x     = backward data    (w' = dz,  dy' = x)     + beta
// so every operand is read along its contiguous axis and no transposed copy is made.
#include <stdio.h>
#include <string.h>

#include <new>
#include <string>

#include "internal.h"
#include "mi355ip.h"

using namespace mi355conv;

struct ip_desc {
  ip_params_t p;
  conv_desc_t* inner;  // null when m == 0
  ColSumArgs cs;
  size_t cs_ws, ws_bytes;
  char names[320];
};

namespace {

constexpr int64_t kMaxElems = (int64_t)1 << 30;

std::string field(const char* names, const char* key) {
  const char* b = strstr(names, key);
  if (!b) return "?";
  b += strlen(key);
  const char* e = strchr(b, ';');
  return e ? std::string(b, e) : std::string(b);
}

}  // namespace

extern "C" {

int ip_desc_create(ip_desc_t** out, const ip_params_t* pp) {
  if (!out || !pp) return CONV_EINVAL;
  const ip_params_t p = *pp;
  if (p.m < 0 || p.k < 1 || p.num_output < 1) return CONV_EINVAL;
  if ((p.bias_term != 0 && p.bias_term != 1) || (p.relu != 0 && p.relu != 1)) return CONV_EINVAL;
  const int64_t M = p.m, K = p.k, O = p.num_output;
  if (M * K >= kMaxElems || O * K >= kMaxElems || M * O >= kMaxElems) return CONV_ESHAPE;
  ip_desc* d = new (std::nothrow) ip_desc;
  if (!d) return CONV_EINVAL;
  memset(d, 0, sizeof(*d));
  d->p = p;
  if (p.m > 0) {
    conv_params_t c = {};
    c.n = 1;
    c.c = p.num_output;
    c.h = 1;
    c.w = p.k;
    c.num_output = p.m;
    c.kernel_h = c.kernel_w = c.stride_h = c.stride_w = c.dilation_h = c.dilation_w = c.group = 1;
    c.bias_term = 0;
    const int rc = conv_desc_create(&d->inner, &c);
    if (rc != CONV_OK) {
      delete d;
      return rc;
    }
    conv_desc_workspace_bytes(d->inner, &d->ws_bytes);
  }
  // bias gradient: column sums of dz[m][num_output], the rows split so that the grid has a few
  // hundred workgroups
  ColSumArgs& cs = d->cs;
  cs.rows = p.m;
  cs.cols = p.num_output;
  const int64_t col_blocks = (O + 255) / 256;
  int64_t S = 512 / col_blocks;
  if (S > (M + 7) / 8) S = (M + 7) / 8;
  if (S < 1) S = 1;
  cs.rows_per_split = (int32_t)((M + S - 1) / S > 0 ? (M + S - 1) / S : 1);
  cs.S = (int32_t)(M > 0 ? (M + cs.rows_per_split - 1) / cs.rows_per_split : 1);
  d->cs_ws = p.bias_term ? (size_t)cs.S * O * 4 : 0;
  if (d->cs_ws > d->ws_bytes) d->ws_bytes = d->cs_ws;
  const char* in = d->inner ? conv_desc_kernel_names(d->inner) : "";
  const bool one_launch = M * O * 4 <= ((int64_t)4 << 20);  // see ip_backward_bias
  snprintf(d->names, sizeof(d->names), "fwd=%s;bwd_data=%s;bwd_filter=%s;bwd_bias=colsum(S=%d,L=%d)",
           field(in, "bwd_filter=").c_str(), field(in, "fwd=").c_str(), field(in, "bwd_data=").c_str(),
           one_launch ? 1 : cs.S, one_launch ? 1 : 2);
  *out = d;
  return CONV_OK;
}

int ip_desc_destroy(ip_desc_t* d) {
  if (!d) return CONV_EINVAL;
  if (d->inner) conv_desc_destroy(d->inner);
  delete d;
  return CONV_OK;
}

int ip_desc_workspace_bytes(const ip_desc_t* d, size_t* bytes) {
  if (!d || !bytes) return CONV_EINVAL;
  *bytes = d->ws_bytes;
  return CONV_OK;
}

const char* ip_desc_kernel_names(const ip_desc_t* d) { return d ? d->names : ""; }

int ip_forward(const ip_desc_t* d, const float* x, const float* w, const float* bias, float* y, void* ws,
               size_t ws_bytes, void* hip_stream) {
  if (!d || !w) return CONV_EINVAL;
  if ((d->p.bias_term != 0) != (bias != nullptr)) return CONV_EINVAL;
  if (d->p.m == 0) return CONV_OK;
  if (!x || !y) return CONV_EINVAL;
  ReduceExtras ex;
  ex.bias = bias;
  ex.chan_elems = 1;
  ex.channels = d->p.num_output;
  ex.relu = d->p.relu;
  return run_backward_filter(d->inner, /*x'=*/w, /*dy'=*/x, /*dw'=*/y, 0.f, ws, ws_bytes, hip_stream, ex);
}

int ip_relu_backward(const ip_desc_t* d, const float* y, const float* dy, float* dz, void* hip_stream) {
  if (!d) return CONV_EINVAL;
  if (d->p.m == 0) return CONV_OK;
  if (!dy || !dz) return CONV_EINVAL;
  if (d->p.relu && !y) return CONV_EINVAL;
  if (!d->p.relu && dz == dy) return CONV_OK;
  ReluBwdArgs a = {};
  a.y = d->p.relu ? y : nullptr;
  a.dy = dy;
  a.dz = dz;
  a.count = d->p.m * d->p.num_output;
  const int e = launch_relu_bwd(a, hip_stream);
  return e ? record_hip_error(e) : CONV_OK;
}

int ip_backward_data(const ip_desc_t* d, const float* w, const float* dz, float* dx, void* ws, size_t ws_bytes,
                     void* hip_stream) {
  if (!d || !w) return CONV_EINVAL;
  if (d->p.m == 0) return CONV_OK;
  if (!dz || !dx) return CONV_EINVAL;
  return run_forward(d->inner, /*x'=*/w, /*w'=*/dz, nullptr, /*y'=*/dx, ws, ws_bytes, hip_stream);
}

int ip_backward_filter(const ip_desc_t* d, const float* x, const float* dz, float* dw, float beta, void* ws,
                       size_t ws_bytes, void* hip_stream) {
  if (!d || !dw) return CONV_EINVAL;
  if (!(beta == 0.f || beta == 1.f)) return CONV_EINVAL;
  if (d->p.m == 0) {  // empty sum: dw = beta*dw
    ReduceArgs r = {};
    r.dst = dw;
    r.count = d->p.num_output * d->p.k;
    r.S = 0;
    r.beta = beta;
    r.chan_elems = r.channels = 1;
    r.mChanElems = r.mChannels = make_magic(1);
    const int e = launch_reduce(r, hip_stream);
    return e ? record_hip_error(e) : CONV_OK;
  }
  if (!x || !dz) return CONV_EINVAL;
  return run_backward_data(d->inner, /*w'=*/dz, /*dy'=*/x, /*dx'=*/dw, beta, ws, ws_bytes, hip_stream);
}

int ip_backward_bias(const ip_desc_t* d, const float* dz, float* db, float beta, void* ws, size_t ws_bytes,
                     void* hip_stream) {
  if (!d || !db) return CONV_EINVAL;
  if (!d->p.bias_term) return CONV_EINVAL;
  if (!(beta == 0.f || beta == 1.f)) return CONV_EINVAL;
  const bool empty = d->p.m == 0;
  if (!empty && !dz) return CONV_EINVAL;
  if (!empty && (!ws || ws_bytes < d->cs_ws)) return CONV_EWORKSPACE;
  ColSumArgs a = d->cs;
  a.src = dz;
  a.part = static_cast<float*>(ws);
  // up to 4 MiB of dz: one launch sums every column and finishes db (the second launch would cost
  // more than the lost parallelism)
  if (!empty && (int64_t)d->p.m * d->p.num_output * 4 <= ((int64_t)4 << 20)) {
    a.dst = db;
    a.beta = beta;
    const int e1 = launch_colsum(a, hip_stream);
    return e1 ? record_hip_error(e1) : CONV_OK;
  }
  int e = empty ? 0 : launch_colsum(a, hip_stream);
  if (e) return record_hip_error(e);
  ReduceArgs r = {};
  r.part = a.part;
  r.dst = db;
  r.count = d->p.num_output;
  r.S = empty ? 0 : a.S;
  r.beta = beta;
  r.chan_elems = r.channels = 1;
  r.mChanElems = r.mChannels = make_magic(1);
  e = launch_reduce(r, hip_stream);
  return e ? record_hip_error(e) : CONV_OK;
}

}  // extern "C"
