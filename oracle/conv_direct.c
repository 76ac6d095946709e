/*
 * TEST INFRASTRUCTURE ONLY -- the CPU oracle's convolution, written out from the
 * textbook definition in float64.  Nothing of the product path may call this.
 *
 * The sub-ResNet's local SGD step (Algorithm 1, inner loop; Sec. 2.3) is an ordinary
 * training step of a ResNet that lacks some residual blocks, so its convolutions are
 * the plain definition:
 *
 *   y[n,k,p,q]  = sum_{c,r,s} x[n,c,p*st+r-pad,q*st+s-pad] * w[k,c,r,s]   (zero padding)
 *   dx[n,c,h,w] = sum_{k,r,s : h=p*st+r-pad, w=q*st+s-pad} dy[n,k,p,q] * w[k,c,r,s]
 *   dw[k,c,r,s] = sum_{n,p,q} dy[n,k,p,q] * x[n,c,p*st+r-pad,q*st+s-pad]
 *
 * Layouts: x [N,C,H,W], w [K,C,R,S], y [N,K,P,Q], all row-major float64.
 * No blocking, no im2col, no reordering beyond picking which loop runs in parallel.
 */
#include <stddef.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* number of threads the parallel loops below run on (1 without OpenMP): reported next to timings */
int oracle_num_threads(void) {
#ifdef _OPENMP
  int n = 1;
#pragma omp parallel
  {
#pragma omp single
    n = omp_get_num_threads();
  }
  return n;
#else
  return 1;
#endif
}

static int out_dim(int in, int k, int stride, int pad) { return (in + 2 * pad - k) / stride + 1; }

/* first / one-past-last output index q with 0 <= q*stride + s - pad < W */
static void valid_range(int Q, int W, int stride, int s, int pad, int *q0, int *q1) {
  int lo = pad - s;                       /* need q*stride >= lo */
  int a = lo <= 0 ? 0 : (lo + stride - 1) / stride;
  int hi = W - 1 + pad - s;               /* need q*stride <= hi */
  int b = hi < 0 ? 0 : hi / stride + 1;
  if (b > Q) b = Q;
  if (a > b) a = b;
  *q0 = a; *q1 = b;
}

void oracle_conv2d_fwd(const double *x, const double *w, double *y, int N, int C, int H, int W,
                       int K, int R, int S, int stride, int pad) {
  const int P = out_dim(H, R, stride, pad), Q = out_dim(W, S, stride, pad);
  /* threads only pay off on large layers; the arithmetic is the same either way */
  const int big = (double)N * K * P * Q * C * R * S > 2e5;
#pragma omp parallel for collapse(2) schedule(static) if (big)
  for (int n = 0; n < N; ++n)
    for (int k = 0; k < K; ++k) {
      double *yk = y + ((size_t)n * K + k) * P * Q;
      memset(yk, 0, sizeof(double) * (size_t)P * Q);
      for (int c = 0; c < C; ++c) {
        const double *xc = x + ((size_t)n * C + c) * H * W;
        for (int r = 0; r < R; ++r)
          for (int s = 0; s < S; ++s) {
            const double wv = w[(((size_t)k * C + c) * R + r) * S + s];
            int p0, p1, q0, q1;
            valid_range(P, H, stride, r, pad, &p0, &p1);
            valid_range(Q, W, stride, s, pad, &q0, &q1);
            for (int p = p0; p < p1; ++p) {
              const double *xr = xc + (size_t)(p * stride + r - pad) * W + (s - pad);
              double *yr = yk + (size_t)p * Q;
              for (int q = q0; q < q1; ++q) yr[q] += xr[q * stride] * wv;
            }
          }
      }
    }
}

void oracle_conv2d_dgrad(const double *dy, const double *w, double *dx, int N, int C, int H, int W,
                         int K, int R, int S, int stride, int pad) {
  const int P = out_dim(H, R, stride, pad), Q = out_dim(W, S, stride, pad);
  /* threads only pay off on large layers; the arithmetic is the same either way */
  const int big = (double)N * K * P * Q * C * R * S > 2e5;
#pragma omp parallel for collapse(2) schedule(static) if (big)
  for (int n = 0; n < N; ++n)
    for (int c = 0; c < C; ++c) {
      double *dxc = dx + ((size_t)n * C + c) * H * W;
      memset(dxc, 0, sizeof(double) * (size_t)H * W);
      for (int k = 0; k < K; ++k) {
        const double *dyk = dy + ((size_t)n * K + k) * P * Q;
        for (int r = 0; r < R; ++r)
          for (int s = 0; s < S; ++s) {
            const double wv = w[(((size_t)k * C + c) * R + r) * S + s];
            int p0, p1, q0, q1;
            valid_range(P, H, stride, r, pad, &p0, &p1);
            valid_range(Q, W, stride, s, pad, &q0, &q1);
            for (int p = p0; p < p1; ++p) {
              double *xr = dxc + (size_t)(p * stride + r - pad) * W + (s - pad);
              const double *yr = dyk + (size_t)p * Q;
              for (int q = q0; q < q1; ++q) xr[q * stride] += yr[q] * wv;
            }
          }
      }
    }
}

void oracle_conv2d_wgrad(const double *dy, const double *x, double *dw, int N, int C, int H, int W,
                         int K, int R, int S, int stride, int pad) {
  const int P = out_dim(H, R, stride, pad), Q = out_dim(W, S, stride, pad);
  /* threads only pay off on large layers; the arithmetic is the same either way */
  const int big = (double)N * K * P * Q * C * R * S > 2e5;
#pragma omp parallel for collapse(2) schedule(static) if (big)
  for (int k = 0; k < K; ++k)
    for (int c = 0; c < C; ++c)
      for (int r = 0; r < R; ++r)
        for (int s = 0; s < S; ++s) {
          int p0, p1, q0, q1;
          valid_range(P, H, stride, r, pad, &p0, &p1);
          valid_range(Q, W, stride, s, pad, &q0, &q1);
          double acc = 0.0;
          for (int n = 0; n < N; ++n) {
            const double *dyk = dy + ((size_t)n * K + k) * P * Q;
            const double *xc = x + ((size_t)n * C + c) * H * W;
            for (int p = p0; p < p1; ++p) {
              const double *xr = xc + (size_t)(p * stride + r - pad) * W + (s - pad);
              const double *yr = dyk + (size_t)p * Q;
              double row = 0.0;
#pragma omp simd reduction(+ : row)
              for (int q = q0; q < q1; ++q) row += yr[q] * xr[q * stride];
              acc += row;
            }
          }
          dw[(((size_t)k * C + c) * R + r) * S + s] = acc;
        }
}
