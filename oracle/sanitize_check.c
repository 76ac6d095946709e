/*
 * TEST INFRASTRUCTURE ONLY -- driver for the sanitizer build of the oracle's convolution
 * (oracle/build.py --sanitize: gcc -fsanitize=address,undefined, no -O3).  Runs the three loops of
 * conv_direct.c on small shapes that reach every border case (stride 1 and 2, padding 0..3, filter
 * sizes 1, 3, 5, 7, single pixels, outputs smaller than the filter) with each tensor in its own
 * exactly-sized heap block, so an index one past either end of any tensor is reported; and checks
 * the adjoint identities <conv(x,w), y> = <x, dgrad(y,w)> = <w, wgrad(y,x)> that tie the three loops
 * to one another.  Exit status 0 = clean.
 */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

void oracle_conv2d_fwd(const double *x, const double *w, double *y, int N, int C, int H, int W, int K, int R, int S,
                       int stride, int pad);
void oracle_conv2d_dgrad(const double *dy, const double *w, double *dx, int N, int C, int H, int W, int K, int R, int S,
                         int stride, int pad);
void oracle_conv2d_wgrad(const double *dy, const double *x, double *dw, int N, int C, int H, int W, int K, int R, int S,
                         int stride, int pad);

static unsigned long long state = 88172645463325252ULL;
static double rnd(void) { /* xorshift64, values in (-1, 1) */
  state ^= state << 13; state ^= state >> 7; state ^= state << 17;
  return (double)(state >> 11) / 9007199254740992.0 * 2.0 - 1.0;
}
static double *filled(size_t n) {
  double *p = (double *)malloc(sizeof(double) * (n ? n : 1));
  if (!p) { fprintf(stderr, "out of memory\n"); exit(2); }
  for (size_t i = 0; i < n; ++i) p[i] = rnd();
  return p;
}
static double dot(const double *a, const double *b, size_t n) {
  double s = 0;
  for (size_t i = 0; i < n; ++i) s += a[i] * b[i];
  return s;
}

int main(void) {
  /*                      N  C  H   W   K  R  st pad */
  static const int cases[][8] = {{2, 3, 5, 7, 4, 3, 1, 1}, {1, 2, 8, 6, 3, 3, 2, 1}, {2, 4, 4, 4, 5, 1, 1, 0}, {2, 4, 6, 6, 5, 1, 2, 0},
                                 {1, 1, 1, 1, 1, 1, 1, 0}, {1, 2, 3, 3, 2, 3, 1, 1}, {1, 2, 2, 2, 2, 3, 2, 1}, {2, 3, 9, 11, 2, 5, 1, 2},
                                 {1, 3, 10, 8, 2, 5, 2, 2}, {1, 3, 12, 12, 4, 7, 2, 3}, {1, 2, 7, 7, 2, 7, 1, 3}, {1, 1, 3, 5, 1, 7, 1, 3},
                                 {3, 2, 5, 5, 2, 3, 1, 0}, {1, 2, 6, 5, 3, 3, 2, 0}, {40, 8, 12, 12, 16, 3, 1, 1} /* large enough for the threaded path */};
  int bad = 0;
  for (size_t i = 0; i < sizeof(cases) / sizeof(cases[0]); ++i) {
    const int N = cases[i][0], C = cases[i][1], H = cases[i][2], W = cases[i][3], K = cases[i][4], R = cases[i][5],
              st = cases[i][6], pad = cases[i][7];
    const int P = (H + 2 * pad - R) / st + 1, Q = (W + 2 * pad - R) / st + 1;
    if (P < 1 || Q < 1) { fprintf(stderr, "case %zu has no output\n", i); return 2; }
    const size_t nx = (size_t)N * C * H * W, nw = (size_t)K * C * R * R, ny = (size_t)N * K * P * Q;
    double *x = filled(nx), *w = filled(nw), *g = filled(ny);
    double *y = filled(ny), *dx = filled(nx), *dw = filled(nw);
    oracle_conv2d_fwd(x, w, y, N, C, H, W, K, R, R, st, pad);
    oracle_conv2d_dgrad(g, w, dx, N, C, H, W, K, R, R, st, pad);
    oracle_conv2d_wgrad(g, x, dw, N, C, H, W, K, R, R, st, pad);
    const double a = dot(y, g, ny), b = dot(x, dx, nx), c = dot(w, dw, nw);
    const double tol = 1e-12 * (fabs(a) + 1.0) * sqrt((double)(C * R * R));
    if (fabs(a - b) > tol || fabs(a - c) > tol) {
      fprintf(stderr, "case %zu: adjoint identity broken: %.17g %.17g %.17g\n", i, a, b, c);
      bad = 1;
    }
    free(x); free(w); free(g); free(y); free(dx); free(dw);
  }
  if (!bad) printf("oracle convolution: %zu cases clean\n", sizeof(cases) / sizeof(cases[0]));
  return bad;
}
