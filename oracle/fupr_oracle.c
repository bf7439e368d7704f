/*
 * CPU oracle for the inference path of a residual network before operator
 * fusion and before filter removal.  TEST INFRASTRUCTURE ONLY: nothing in the
 * GPU library includes, links or calls this file.
 *
 * Every operator is the plain definition, evaluated in double precision on
 * NCHW tensors, one output element at a time:
 *   - convolution operator with weights k x c x r x s (Sec. III; Sec. IV-B-1),
 *     cross-correlation with zero padding;
 *   - batch normalisation in its literal form with gamma, beta, mean, var and
 *     eps (the quantities of Sec. IV-B-2, Eq. 3-5, before they are collapsed
 *     into omega and lambda);
 *   - ReLU and element-wise addition, the scalar operators of Sec. III;
 *   - the remaining operators of Table II (max-pool, global mean, fc).
 * Filter importance is the l1 or l2 norm over (c, r, s) of a filter
 * (Sec. IV-C, Eq. 6), summed sequentially in that index order.
 *
 * Loops are parallel over (image, filter) with OpenMP; within one output
 * element the summation order is c, then r, then s.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int orc_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

static int out_extent(int in, int k, int stride, int pad) { return (in + 2 * pad - k) / stride + 1; }

/* y[n,k,p,q] = sum_c sum_r sum_s x[n,c,p*stride+r-pad,q*stride+s-pad] * w[k,c,r,s]; 0 outside. */
void orc_conv2d(const double* x, const double* w, double* y, int N, int C, int H, int W, int K,
                int R, int S, int stride, int pad) {
  const int P = out_extent(H, R, stride, pad), Q = out_extent(W, S, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int k = 0; k < K; ++k) {
      double* yk = y + ((size_t)n * K + k) * P * Q;
      for (int i = 0; i < P * Q; ++i) yk[i] = 0.0;
      for (int c = 0; c < C; ++c) {
        const double* xc = x + ((size_t)n * C + c) * H * W;
        for (int r = 0; r < R; ++r)
          for (int s = 0; s < S; ++s) {
            const double wv = w[(((size_t)k * C + c) * R + r) * S + s];
            for (int p = 0; p < P; ++p) {
              const int ih = p * stride + r - pad;
              if (ih < 0 || ih >= H) continue;
              for (int q = 0; q < Q; ++q) {
                const int iw = q * stride + s - pad;
                if (iw < 0 || iw >= W) continue;
                yk[p * Q + q] += xc[ih * W + iw] * wv;
              }
            }
          }
      }
    }
}

/* y = gamma * (x - mean) / sqrt(var + eps) + beta, per channel. */
void orc_batchnorm(const double* x, double* y, const double* gamma, const double* beta,
                   const double* mean, const double* var, double eps, int N, int K, int HW) {
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int k = 0; k < K; ++k) {
      const double* xi = x + ((size_t)n * K + k) * HW;
      double* yi = y + ((size_t)n * K + k) * HW;
      const double d = sqrt(var[k] + eps);
      for (int i = 0; i < HW; ++i) yi[i] = gamma[k] * (xi[i] - mean[k]) / d + beta[k];
    }
}

void orc_relu(const double* x, double* y, size_t count) {
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < count; ++i) y[i] = x[i] > 0.0 ? x[i] : 0.0;
}

void orc_add(const double* a, const double* b, double* y, size_t count) {
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < count; ++i) y[i] = a[i] + b[i];
}

/* Parameter-free shortcut across a resolution change: spatial subsampling by
 * `stride`, channels c < C copied, channels C <= k < K zero. */
void orc_shortcut_subsample_pad(const double* x, double* y, int N, int C, int H, int W, int K,
                                int stride) {
  const int P = (H + stride - 1) / stride, Q = (W + stride - 1) / stride;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int k = 0; k < K; ++k) {
      double* yk = y + ((size_t)n * K + k) * P * Q;
      for (int p = 0; p < P; ++p)
        for (int q = 0; q < Q; ++q)
          yk[p * Q + q] = k < C ? x[(((size_t)n * C + k) * H + p * stride) * W + q * stride] : 0.0;
    }
}

/* Max over the taps of a k x k window that fall inside the image. */
void orc_maxpool(const double* x, double* y, int N, int C, int H, int W, int k, int stride,
                 int pad) {
  const int P = out_extent(H, k, stride, pad), Q = out_extent(W, k, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int c = 0; c < C; ++c) {
      const double* xc = x + ((size_t)n * C + c) * H * W;
      double* yc = y + ((size_t)n * C + c) * P * Q;
      for (int p = 0; p < P; ++p)
        for (int q = 0; q < Q; ++q) {
          double m = -INFINITY;
          for (int r = 0; r < k; ++r)
            for (int s = 0; s < k; ++s) {
              const int ih = p * stride + r - pad, iw = q * stride + s - pad;
              if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
              const double v = xc[ih * W + iw];
              if (v > m) m = v;
            }
          yc[p * Q + q] = m;
        }
    }
}

/* y[n,c] = mean over the H*W positions of x[n,c,:,:]. */
void orc_global_mean(const double* x, double* y, int N, int C, int HW) {
#pragma omp parallel for schedule(static)
  for (int i = 0; i < N * C; ++i) {
    double s = 0.0;
    for (int j = 0; j < HW; ++j) s += x[(size_t)i * HW + j];
    y[i] = s / HW;
  }
}

/* y[n,o] = b[o] + sum_i W[o,i] x[n,i]. */
void orc_fc(const double* x, const double* w, const double* b, double* y, int N, int In, int Out) {
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int o = 0; o < Out; ++o) {
      double s = 0.0;
      for (int i = 0; i < In; ++i) s += w[(size_t)o * In + i] * x[(size_t)n * In + i];
      y[(size_t)n * Out + o] = s + b[o];
    }
}

/* norms[k] = l1 (norm == 1) or l2 (norm == 2) norm of filter k over its c*r*s weights. */
void orc_filter_norms(const double* w, int K, int CRS, int norm, double* norms) {
  for (int k = 0; k < K; ++k) {
    double s = 0.0;
    for (int i = 0; i < CRS; ++i) {
      const double v = w[(size_t)k * CRS + i];
      s += norm == 1 ? fabs(v) : v * v;
    }
    norms[k] = norm == 1 ? s : sqrt(s);
  }
}
