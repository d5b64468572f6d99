/*
 * CPU oracle for the Caffe-semantics 2-D ConvolutionLayer -- test infrastructure only.
 * See conv_oracle.h for the contract.  Plain C, double precision, direct nested loops
 * that follow the definition term by term; OpenMP only spreads independent output
 * elements over host threads (no atomics, no reordering inside one sum).
 *
 * Definition used (the paper names the layer family in Table 1 and defers to C++ Caffe
 * in its Abstract; this is that layer's standard mathematical statement):
 *   Cg = c/group, Kg = num_output/group, grp(k) = k div Kg, xz = x extended by zero.
 *   forward:   y[n,k,oh,ow] = b[k] + sum_{c',i,j} w[k,c',i,j] *
 *                             xz[n, grp(k)*Cg + c', oh*s_h - p_h + i*d_h, ow*s_w - p_w + j*d_w]
 *   bwd data:  dx = transpose of that linear map applied to dy
 *   bwd filter: dw[k,c',i,j] = beta*dw + sum_{n,oh,ow} dy[n,k,oh,ow] * xz[...same tap...]
 *   bwd bias:  db[k] = beta*db + sum_{n,oh,ow} dy[n,k,oh,ow]
 */
#include "conv_oracle.h"

#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int64_t floor_div(int64_t a, int64_t b) { /* b > 0 */
  int64_t q = a / b;
  if ((a % b != 0) && (a < 0)) --q;
  return q;
}

int64_t oracle_conv_out_size(int64_t in, int64_t kernel, int64_t stride, int64_t pad, int64_t dilation) {
  int64_t extent = dilation * (kernel - 1) + 1;
  return floor_div(in + 2 * pad - extent, stride) + 1;
}

static int params_ok(const oracle_conv_params* p) {
  if (!p) return 0;
  if (p->n < 0 || p->c < 1 || p->h < 1 || p->w < 1 || p->num_output < 1) return 0;
  if (p->kernel_h < 1 || p->kernel_w < 1 || p->stride_h < 1 || p->stride_w < 1) return 0;
  if (p->pad_h < 0 || p->pad_w < 0 || p->dilation_h < 1 || p->dilation_w < 1) return 0;
  if (p->group < 1 || p->c % p->group != 0 || p->num_output % p->group != 0) return 0;
  if (p->bias_term != 0 && p->bias_term != 1) return 0;
  if (oracle_conv_out_size(p->h, p->kernel_h, p->stride_h, p->pad_h, p->dilation_h) < 1) return 0;
  if (oracle_conv_out_size(p->w, p->kernel_w, p->stride_w, p->pad_w, p->dilation_w) < 1) return 0;
  return 1;
}

int oracle_conv_output_shape(const oracle_conv_params* p, int64_t* oh, int64_t* ow) {
  if (!params_ok(p) || !oh || !ow) return -1;
  *oh = oracle_conv_out_size(p->h, p->kernel_h, p->stride_h, p->pad_h, p->dilation_h);
  *ow = oracle_conv_out_size(p->w, p->kernel_w, p->stride_w, p->pad_w, p->dilation_w);
  return 0;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* flat offsets of the dense layouts */
#define X_AT(p, n_, c_, h_, w_) ((((n_) * (p)->c + (c_)) * (p)->h + (h_)) * (p)->w + (w_))
#define Y_AT(p, OH, OW, n_, k_, oh_, ow_) ((((n_) * (p)->num_output + (k_)) * (OH) + (oh_)) * (OW) + (ow_))
#define W_AT(p, Cg, k_, c_, i_, j_) ((((k_) * (Cg) + (c_)) * (p)->kernel_h + (i_)) * (p)->kernel_w + (j_))

/* one forward output element, straight from the definition */
static double forward_element(const oracle_conv_params* p, const double* x, const double* w, const double* b,
                              int64_t n, int64_t k, int64_t oh, int64_t ow) {
  const int64_t Cg = p->c / p->group, Kg = p->num_output / p->group;
  const int64_t g = k / Kg;
  double acc = (p->bias_term && b) ? b[k] : 0.0;
  for (int64_t cc = 0; cc < Cg; ++cc)
    for (int64_t i = 0; i < p->kernel_h; ++i)
      for (int64_t j = 0; j < p->kernel_w; ++j) {
        const int64_t ih = oh * p->stride_h - p->pad_h + i * p->dilation_h;
        const int64_t iw = ow * p->stride_w - p->pad_w + j * p->dilation_w;
        if (ih < 0 || ih >= p->h || iw < 0 || iw >= p->w) continue; /* zero extension */
        acc += w[W_AT(p, Cg, k, cc, i, j)] * x[X_AT(p, n, g * Cg + cc, ih, iw)];
      }
  return acc;
}

int oracle_conv_forward(const oracle_conv_params* p, const double* x, const double* w, const double* b, double* y) {
  int64_t OH, OW;
  if (oracle_conv_output_shape(p, &OH, &OW) || !x || !w || !y) return -1;
  if (p->bias_term && !b) return -1;
  if (!p->bias_term && b) return -1;
  const int64_t K = p->num_output;
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t n = 0; n < p->n; ++n)
    for (int64_t k = 0; k < K; ++k)
      for (int64_t oh = 0; oh < OH; ++oh)
        for (int64_t ow = 0; ow < OW; ++ow)
          y[Y_AT(p, OH, OW, n, k, oh, ow)] = forward_element(p, x, w, b, n, k, oh, ow);
  return 0;
}

int oracle_conv_forward_at(const oracle_conv_params* p, const double* x, const double* w, const double* b,
                           const int64_t* idx, int64_t count, double* out) {
  int64_t OH, OW;
  if (oracle_conv_output_shape(p, &OH, &OW) || !x || !w || !idx || !out) return -1;
  if (p->bias_term && !b) return -1;
  if (!p->bias_term && b) return -1;
  const int64_t total = p->n * p->num_output * OH * OW;
  for (int64_t s = 0; s < count; ++s)
    if (idx[s] < 0 || idx[s] >= total) return -1;
#pragma omp parallel for schedule(static)
  for (int64_t s = 0; s < count; ++s) {
    int64_t r = idx[s];
    const int64_t ow = r % OW; r /= OW;
    const int64_t oh = r % OH; r /= OH;
    const int64_t k = r % p->num_output; r /= p->num_output;
    out[s] = forward_element(p, x, w, b, r, k, oh, ow);
  }
  return 0;
}

/*
 * Backward data as the literal transpose of the forward loop nest: walk every
 * (output element, tap) pair of the forward sum and send w*dy to the input
 * element that tap read.  Images are independent, so they go to separate threads.
 */
int oracle_conv_backward_data(const oracle_conv_params* p, const double* w, const double* dy, double* dx) {
  int64_t OH, OW;
  if (oracle_conv_output_shape(p, &OH, &OW) || !w || !dy || !dx) return -1;
  const int64_t Cg = p->c / p->group, Kg = p->num_output / p->group;
#pragma omp parallel for schedule(static)
  for (int64_t n = 0; n < p->n; ++n) {
    for (int64_t e = 0; e < p->c * p->h * p->w; ++e) dx[n * p->c * p->h * p->w + e] = 0.0;
    for (int64_t k = 0; k < p->num_output; ++k) {
      const int64_t g = k / Kg;
      for (int64_t oh = 0; oh < OH; ++oh)
        for (int64_t ow = 0; ow < OW; ++ow) {
          const double gy = dy[Y_AT(p, OH, OW, n, k, oh, ow)];
          for (int64_t cc = 0; cc < Cg; ++cc)
            for (int64_t i = 0; i < p->kernel_h; ++i)
              for (int64_t j = 0; j < p->kernel_w; ++j) {
                const int64_t ih = oh * p->stride_h - p->pad_h + i * p->dilation_h;
                const int64_t iw = ow * p->stride_w - p->pad_w + j * p->dilation_w;
                if (ih < 0 || ih >= p->h || iw < 0 || iw >= p->w) continue;
                dx[X_AT(p, n, g * Cg + cc, ih, iw)] += w[W_AT(p, Cg, k, cc, i, j)] * gy;
              }
        }
    }
  }
  return 0;
}

/*
 * One dx element: sum over the output channels of the element's group and over
 * the taps (i,j) of w*dy at the output position that tap connects to, i.e. the
 * (oh,ow) solving oh*s_h - p_h + i*d_h = h and ow*s_w - p_w + j*d_w = w when such
 * integers exist inside the output.
 */
int oracle_conv_backward_data_at(const oracle_conv_params* p, const double* w, const double* dy,
                                 const int64_t* idx, int64_t count, double* out) {
  int64_t OH, OW;
  if (oracle_conv_output_shape(p, &OH, &OW) || !w || !dy || !idx || !out) return -1;
  const int64_t Cg = p->c / p->group, Kg = p->num_output / p->group;
  const int64_t total = p->n * p->c * p->h * p->w;
  for (int64_t s = 0; s < count; ++s)
    if (idx[s] < 0 || idx[s] >= total) return -1;
#pragma omp parallel for schedule(static)
  for (int64_t s = 0; s < count; ++s) {
    int64_t r = idx[s];
    const int64_t iw = r % p->w; r /= p->w;
    const int64_t ih = r % p->h; r /= p->h;
    const int64_t c = r % p->c; r /= p->c;
    const int64_t n = r;
    const int64_t g = c / Cg, cc = c % Cg;
    double acc = 0.0;
    for (int64_t k = g * Kg; k < (g + 1) * Kg; ++k)
      for (int64_t i = 0; i < p->kernel_h; ++i) {
        const int64_t th = ih + p->pad_h - i * p->dilation_h; /* must equal oh*s_h */
        if (th < 0 || th % p->stride_h != 0) continue;
        const int64_t oh = th / p->stride_h;
        if (oh >= OH) continue;
        for (int64_t j = 0; j < p->kernel_w; ++j) {
          const int64_t tw = iw + p->pad_w - j * p->dilation_w;
          if (tw < 0 || tw % p->stride_w != 0) continue;
          const int64_t ow = tw / p->stride_w;
          if (ow >= OW) continue;
          acc += w[W_AT(p, Cg, k, cc, i, j)] * dy[Y_AT(p, OH, OW, n, k, oh, ow)];
        }
      }
    out[s] = acc;
  }
  return 0;
}

/* gradient sum of one filter element, straight from the definition */
static double filter_grad_element(const oracle_conv_params* p, const double* x, const double* dy,
                                  int64_t OH, int64_t OW, int64_t k, int64_t cc, int64_t i, int64_t j) {
  const int64_t Cg = p->c / p->group, Kg = p->num_output / p->group;
  const int64_t g = k / Kg;
  double acc = 0.0;
  for (int64_t n = 0; n < p->n; ++n)
    for (int64_t oh = 0; oh < OH; ++oh) {
      const int64_t ih = oh * p->stride_h - p->pad_h + i * p->dilation_h;
      if (ih < 0 || ih >= p->h) continue;
      for (int64_t ow = 0; ow < OW; ++ow) {
        const int64_t iw = ow * p->stride_w - p->pad_w + j * p->dilation_w;
        if (iw < 0 || iw >= p->w) continue;
        acc += dy[Y_AT(p, OH, OW, n, k, oh, ow)] * x[X_AT(p, n, g * Cg + cc, ih, iw)];
      }
    }
  return acc;
}

int oracle_conv_backward_filter(const oracle_conv_params* p, const double* x, const double* dy, double* dw,
                                double beta) {
  int64_t OH, OW;
  if (oracle_conv_output_shape(p, &OH, &OW) || !x || !dy || !dw) return -1;
  const int64_t Cg = p->c / p->group;
  const int64_t per_k = Cg * p->kernel_h * p->kernel_w;
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t k = 0; k < p->num_output; ++k)
    for (int64_t e = 0; e < per_k; ++e) {
      const int64_t j = e % p->kernel_w;
      const int64_t i = (e / p->kernel_w) % p->kernel_h;
      const int64_t cc = e / (p->kernel_w * p->kernel_h);
      const double grad = filter_grad_element(p, x, dy, OH, OW, k, cc, i, j);
      const int64_t at = W_AT(p, Cg, k, cc, i, j);
      dw[at] = (beta == 0.0 ? 0.0 : beta * dw[at]) + grad;
    }
  return 0;
}

int oracle_conv_backward_filter_at(const oracle_conv_params* p, const double* x, const double* dy,
                                   const int64_t* idx, int64_t count, double* out) {
  int64_t OH, OW;
  if (oracle_conv_output_shape(p, &OH, &OW) || !x || !dy || !idx || !out) return -1;
  const int64_t Cg = p->c / p->group;
  const int64_t total = p->num_output * Cg * p->kernel_h * p->kernel_w;
  for (int64_t s = 0; s < count; ++s)
    if (idx[s] < 0 || idx[s] >= total) return -1;
#pragma omp parallel for schedule(dynamic)
  for (int64_t s = 0; s < count; ++s) {
    int64_t r = idx[s];
    const int64_t j = r % p->kernel_w; r /= p->kernel_w;
    const int64_t i = r % p->kernel_h; r /= p->kernel_h;
    const int64_t cc = r % Cg; r /= Cg;
    out[s] = filter_grad_element(p, x, dy, OH, OW, r, cc, i, j);
  }
  return 0;
}

int oracle_conv_backward_bias(const oracle_conv_params* p, const double* dy, double* db, double beta) {
  int64_t OH, OW;
  if (oracle_conv_output_shape(p, &OH, &OW) || !dy || !db) return -1;
  if (!p->bias_term) return -1;
#pragma omp parallel for schedule(static)
  for (int64_t k = 0; k < p->num_output; ++k) {
    double acc = 0.0;
    for (int64_t n = 0; n < p->n; ++n)
      for (int64_t oh = 0; oh < OH; ++oh)
        for (int64_t ow = 0; ow < OW; ++ow) acc += dy[Y_AT(p, OH, OW, n, k, oh, ow)];
    db[k] = (beta == 0.0 ? 0.0 : beta * db[k]) + acc;
  }
  return 0;
}
