// Pooling, the fully connected head and the loss of the sub-ResNet's training step (NHWC).
// Pooling reads and writes activations in their storage type (fp32 or bf16); pooled features,
// logits, loss and everything behind them are fp32.  These are small or bandwidth-bound kernels;
// every reduction runs in a fixed order.
#include "elem.h"
#include "internal.h"

namespace resist {

namespace {

// ---- max pool 3x3 stride 2 pad 1 -----------------------------------------------------------------
// argmax stores the window tap (r*3+s) of the first maximum in row-major window order.
// A thread owns V = 4 (fp32) or 8 (bf16) consecutive channels of one pixel.
template <typename T>
__global__ __launch_bounds__(256) void maxpool_fwd_kernel(const T *__restrict__ x, T *__restrict__ y,
                                                          uint8_t *__restrict__ arg, int N, int H, int W, int C, int P, int Q) {
  constexpr int V = Vec<T>::N;
  const long long total = (long long)N * P * Q * (C / V);
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int c = (int)(i % (C / V)) * V;
  long long pix = i / (C / V);
  const int q = (int)(pix % Q); pix /= Q;
  const int p = (int)(pix % P);
  const int n = (int)(pix / P);
  float best[V];
  int bi[V];
#pragma unroll
  for (int e = 0; e < V; ++e) { best[e] = -INFINITY; bi[e] = 0; }
  bool any = false;
  for (int r = 0; r < 3; ++r) {
    const int ih = p * 2 + r - 1;
    if (ih < 0 || ih >= H) continue;
    for (int s = 0; s < 3; ++s) {
      const int iw = q * 2 + s - 1;
      if (iw < 0 || iw >= W) continue;
      float v[V];
      Vec<T>::load(x + ((size_t)(n * H + ih) * W + iw) * C + c, v);
#pragma unroll
      for (int e = 0; e < V; ++e)
        if (!any || v[e] > best[e]) { best[e] = v[e]; bi[e] = r * 3 + s; }
      any = true;
    }
  }
  const size_t off = ((size_t)(n * P + p) * Q + q) * C + c;
  Vec<T>::store(y + off, best);
#pragma unroll
  for (int e = 0; e < V; e += 4)
    *reinterpret_cast<uchar4 *>(arg + off + e) = make_uchar4((uint8_t)bi[e], (uint8_t)bi[e + 1], (uint8_t)bi[e + 2], (uint8_t)bi[e + 3]);
}

// gather form: every input pixel looks at the (at most 2x2) windows that cover it
template <typename T>
__global__ __launch_bounds__(256) void maxpool_bwd_kernel(const T *__restrict__ dy, const uint8_t *__restrict__ arg,
                                                          T *__restrict__ dx, int N, int H, int W, int C, int P, int Q) {
  constexpr int V = Vec<T>::N;
  const long long total = (long long)N * H * W * (C / V);
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int c = (int)(i % (C / V)) * V;
  long long pix = i / (C / V);
  const int w = (int)(pix % W); pix /= W;
  const int h = (int)(pix % H);
  const int n = (int)(pix / H);
  float acc[V];
#pragma unroll
  for (int e = 0; e < V; ++e) acc[e] = 0.f;
  // windows p with 2p-1 <= h <= 2p+1
  for (int p = (h >> 1); p <= ((h + 1) >> 1); ++p) {
    if (p < 0 || p >= P) continue;
    const int r = h - (2 * p - 1);
    for (int q = (w >> 1); q <= ((w + 1) >> 1); ++q) {
      if (q < 0 || q >= Q) continue;
      const int s = w - (2 * q - 1);
      const size_t off = ((size_t)(n * P + p) * Q + q) * C + c;
      float g[V];
      Vec<T>::load(dy + off, g);
      const int tap = r * 3 + s;
#pragma unroll
      for (int e = 0; e < V; ++e)
        if (arg[off + e] == tap) acc[e] += g[e];
    }
  }
  Vec<T>::store(dx + ((size_t)(n * H + h) * W + w) * C + c, acc);
}

// ---- global mean pool ------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void avgpool_fwd_kernel(const T *__restrict__ x, float *__restrict__ y, int N, int HW, int C) {
  constexpr int V = Vec<T>::N;
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= N * (C / V)) return;
  const int c = (i % (C / V)) * V, n = i / (C / V);
  float acc[V];
#pragma unroll
  for (int e = 0; e < V; ++e) acc[e] = 0.f;
  for (int p = 0; p < HW; ++p) {
    float v[V];
    Vec<T>::load(x + ((size_t)n * HW + p) * C + c, v);
#pragma unroll
    for (int e = 0; e < V; ++e) acc[e] += v[e];
  }
  const float inv = 1.0f / (float)HW;
#pragma unroll
  for (int e = 0; e < V; ++e) y[(size_t)n * C + c + e] = acc[e] * inv;
}

template <typename T>
__global__ __launch_bounds__(256) void avgpool_bwd_kernel(const float *__restrict__ dy, const T *__restrict__ mask, T *__restrict__ dx,
                                                          int N, int HW, int C) {
  constexpr int V = Vec<T>::N;
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (long long)N * HW * (C / V)) return;
  const int c = (int)(i % (C / V)) * V;
  const int n = (int)(i / ((long long)HW * (C / V)));
  const float inv = 1.0f / (float)HW;
  float g[V];
#pragma unroll
  for (int e = 0; e < V; ++e) g[e] = dy[(size_t)n * C + c + e] * inv;
  if (mask) {   // the ReLU that produced the pooled tensor: the gradient passes where its output is positive
    float m[V];
    Vec<T>::load(mask + i * V, m);
#pragma unroll
    for (int e = 0; e < V; ++e) g[e] = m[e] > 0.f ? g[e] : 0.f;
  }
  Vec<T>::store(dx + i * V, g);
}

// ---- fully connected -------------------------------------------------------------------------------
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
  return v;
}

// The three small GEMMs of the classifier are register-tiled 4 x 4 (classes x samples, or classes x
// channel vectors) so that every 16-byte load feeds 16 multiply-adds; rows past N or J are handled by
// clamping the row index and discarding the result.  Every sum runs in a fixed order.

// z[n][j] = b[j] + sum_c x[n][c] * w[j][c].  A workgroup owns 4 classes and 16 samples, each of its waves
// 4 of the samples; the 64 lanes stride over the channels, then the 16 dot products are reduced over the lanes.
__global__ __launch_bounds__(256) void fc_fwd_kernel(const float *__restrict__ x, const float *__restrict__ w,
                                                     const float *__restrict__ b, float *__restrict__ z, int N, int C, int J) {
  const int j0 = blockIdx.x * 4, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float *wr[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) wr[k] = w + (size_t)min(j0 + k, J - 1) * C;
  for (int n0 = blockIdx.y * 16 + wave * 4; n0 < N && n0 < (int)blockIdx.y * 16 + 16; n0 += 16) {
    const float *xr[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) xr[s] = x + (size_t)min(n0 + s, N - 1) * C;
    float acc[4][4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
      for (int s = 0; s < 4; ++s) acc[k][s] = 0.f;
#pragma unroll 2
    for (int c = lane * 4; c < C; c += 256) {
      f32x4 xv[4], wv[4];
#pragma unroll
      for (int s = 0; s < 4; ++s) xv[s] = *reinterpret_cast<const f32x4 *>(xr[s] + c);
#pragma unroll
      for (int k = 0; k < 4; ++k) wv[k] = *reinterpret_cast<const f32x4 *>(wr[k] + c);
#pragma unroll
      for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int s = 0; s < 4; ++s)
          acc[k][s] += xv[s][0] * wv[k][0] + xv[s][1] * wv[k][1] + xv[s][2] * wv[k][2] + xv[s][3] * wv[k][3];
    }
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const float t = wave_sum(acc[k][s]);
        if (lane == 0 && j0 + k < J && n0 + s < N) z[(size_t)(n0 + s) * J + j0 + k] = t + b[j0 + k];
      }
  }
}

// dx[n][c] = sum_j dz[n][j] * w[j][c].  A workgroup owns 4 samples and 256 channels: 64 threads
// cover the channels (4 each), the 4 waves take every 4th class and their partial sums are added in
// wave order.  C is a multiple of 4; channels past C are skipped.
__global__ __launch_bounds__(256) void fc_bwd_dx_kernel(const float *__restrict__ dz, const float *__restrict__ w,
                                                        float *__restrict__ dx, int N, int C, int J) {
  __shared__ f32x4 red[4][4][64];
  const int n0 = blockIdx.y * 4, tx = threadIdx.x & 63, jg = threadIdx.x >> 6;
  const int c = blockIdx.x * 256 + tx * 4;
  f32x4 acc[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) acc[s] = f32x4{0.f, 0.f, 0.f, 0.f};
  if (c < C) {
    const float *dzr[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) dzr[s] = dz + (size_t)min(n0 + s, N - 1) * J;
#pragma unroll 4
    for (int j = jg; j < J; j += 4) {
      const f32x4 wv = *reinterpret_cast<const f32x4 *>(w + (size_t)j * C + c);
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const float d = dzr[s][j];
        acc[s][0] = fmaf(d, wv[0], acc[s][0]); acc[s][1] = fmaf(d, wv[1], acc[s][1]);
        acc[s][2] = fmaf(d, wv[2], acc[s][2]); acc[s][3] = fmaf(d, wv[3], acc[s][3]);
      }
    }
  }
#pragma unroll
  for (int s = 0; s < 4; ++s) red[jg][s][tx] = acc[s];
  __syncthreads();
  if (jg == 0 && c < C) {
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      if (n0 + s >= N) break;
      f32x4 t = acc[s];
      t += red[1][s][tx];
      t += red[2][s][tx];
      t += red[3][s][tx];
      *reinterpret_cast<f32x4 *>(dx + (size_t)(n0 + s) * C + c) = t;
    }
  }
}

// dw[j][c] = sum_n dz[n][j] * x[n][c].  A thread owns 4 classes x 4 consecutive channels and walks the
// samples in order; blockIdx.y selects the group of 4 classes.
__global__ __launch_bounds__(256) void fc_bwd_dw_kernel(const float *__restrict__ dz, const float *__restrict__ x,
                                                        float *__restrict__ dw, int N, int C, int J) {
  const int c = (blockIdx.x * blockDim.x + threadIdx.x) * 4;
  const int j0 = blockIdx.y * 4;
  if (c >= C) return;
  int jr[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) jr[k] = min(j0 + k, J - 1);
  f32x4 acc[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) acc[k] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 2
  for (int n = 0; n < N; ++n) {
    const f32x4 xv = *reinterpret_cast<const f32x4 *>(x + (size_t)n * C + c);
    const float *dzr = dz + (size_t)n * J;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float d = dzr[jr[k]];
      acc[k][0] = fmaf(d, xv[0], acc[k][0]); acc[k][1] = fmaf(d, xv[1], acc[k][1]);
      acc[k][2] = fmaf(d, xv[2], acc[k][2]); acc[k][3] = fmaf(d, xv[3], acc[k][3]);
    }
  }
#pragma unroll
  for (int k = 0; k < 4; ++k)
    if (j0 + k < J) *reinterpret_cast<f32x4 *>(dw + (size_t)(j0 + k) * C + c) = acc[k];
}

// db over the padded length (multiple of 4): entries past J are written as zero
__global__ __launch_bounds__(256) void fc_bwd_db_kernel(const float *__restrict__ dz, float *__restrict__ db, int N, int J, int Jpad) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= Jpad) return;
  float acc = 0.f;
  if (j < J)
    for (int n = 0; n < N; ++n) acc += dz[(size_t)n * J + j];
  db[j] = acc;
}

// ---- softmax cross-entropy ---------------------------------------------------------------------------
// one wave per sample: row_loss[n] = logsumexp(z_n) - z_n[label]; dz = (softmax - onehot)/N
__global__ __launch_bounds__(64) void softmax_ce_kernel(const float *__restrict__ z, const int32_t *__restrict__ labels,
                                                        float *__restrict__ row_loss, float *__restrict__ dz, int N, int J) {
  const int n = blockIdx.x, lane = threadIdx.x;
  const float *zr = z + (size_t)n * J;
  float mx = -INFINITY;
  for (int j = lane; j < J; j += 64) mx = fmaxf(mx, zr[j]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
  float se = 0.f;
  for (int j = lane; j < J; j += 64) se += expf(zr[j] - mx);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) se += __shfl_xor(se, o, 64);
  const int lab = labels[n];
  const float invN = 1.0f / (float)N;
  const float inv = 1.0f / se;
  for (int j = lane; j < J; j += 64) {
    const float p = expf(zr[j] - mx) * inv;
    dz[(size_t)n * J + j] = (p - (j == lab ? 1.f : 0.f)) * invN;
  }
  // a label outside [0,J) is a caller error: it must not turn into an out-of-bounds read
  if (lane == 0) row_loss[n] = (lab >= 0 && lab < J) ? (logf(se) + mx) - zr[lab] : NAN;
}

__global__ void mean_loss_kernel(const float *__restrict__ row_loss, float *__restrict__ loss, int N) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    double acc = 0;
    for (int n = 0; n < N; ++n) acc += (double)row_loss[n];
    *loss = (float)(acc / (double)N);
  }
}

unsigned blocks_for(long long n, int t = 256) { return (unsigned)((n + t - 1) / t); }

}  // namespace

int maxpool_fwd(int dt, const void *x, void *y, uint8_t *argmax, int N, int H, int W, int C, int P, int Q, hipStream_t st) {
  const int V = dt == DT_BF16 ? 8 : 4;
  if (C % V) return set_error(RESIST_ESHAPE, "max-pool: C=%d must be a multiple of %d", C, V);
  prof::Scope ps("maxpool_fwd", 0, (double)esize(dt) * N * C * ((double)H * W + (double)P * Q) + (double)N * P * Q * C, st);
  const dim3 grid(blocks_for((long long)N * P * Q * (C / V)));
  if (dt == DT_BF16) hipLaunchKernelGGL(maxpool_fwd_kernel<__bf16>, grid, dim3(256), 0, st, (const __bf16 *)x, (__bf16 *)y, argmax, N, H, W, C, P, Q);
  else hipLaunchKernelGGL(maxpool_fwd_kernel<float>, grid, dim3(256), 0, st, (const float *)x, (float *)y, argmax, N, H, W, C, P, Q);
  RESIST_CHECK_LAUNCH("maxpool_fwd");
  return RESIST_OK;
}
int maxpool_bwd(int dt, const void *dy, const uint8_t *argmax, void *dx, int N, int H, int W, int C, int P, int Q, hipStream_t st) {
  const int V = dt == DT_BF16 ? 8 : 4;
  if (C % V) return set_error(RESIST_ESHAPE, "max-pool: C=%d must be a multiple of %d", C, V);
  prof::Scope ps("maxpool_bwd", 0, (double)esize(dt) * N * C * ((double)H * W + (double)P * Q) + (double)N * P * Q * C, st);
  const dim3 grid(blocks_for((long long)N * H * W * (C / V)));
  if (dt == DT_BF16) hipLaunchKernelGGL(maxpool_bwd_kernel<__bf16>, grid, dim3(256), 0, st, (const __bf16 *)dy, argmax, (__bf16 *)dx, N, H, W, C, P, Q);
  else hipLaunchKernelGGL(maxpool_bwd_kernel<float>, grid, dim3(256), 0, st, (const float *)dy, argmax, (float *)dx, N, H, W, C, P, Q);
  RESIST_CHECK_LAUNCH("maxpool_bwd");
  return RESIST_OK;
}
int avgpool_fwd(int dt, const void *x, float *y, int N, int HW, int C, hipStream_t st) {
  const int V = dt == DT_BF16 ? 8 : 4;
  if (C % V) return set_error(RESIST_ESHAPE, "mean pool: C=%d must be a multiple of %d", C, V);
  prof::Scope ps("avgpool_fwd", 0, 0, st);
  const dim3 grid(blocks_for((long long)N * (C / V)));
  if (dt == DT_BF16) hipLaunchKernelGGL(avgpool_fwd_kernel<__bf16>, grid, dim3(256), 0, st, (const __bf16 *)x, y, N, HW, C);
  else hipLaunchKernelGGL(avgpool_fwd_kernel<float>, grid, dim3(256), 0, st, (const float *)x, y, N, HW, C);
  RESIST_CHECK_LAUNCH("avgpool_fwd");
  return RESIST_OK;
}
int avgpool_bwd(int dt, const float *dy, const void *relu_mask, void *dx, int N, int HW, int C, hipStream_t st) {
  const int V = dt == DT_BF16 ? 8 : 4;
  if (C % V) return set_error(RESIST_ESHAPE, "mean pool: C=%d must be a multiple of %d", C, V);
  prof::Scope ps("avgpool_bwd", 0, 0, st);
  const dim3 grid(blocks_for((long long)N * HW * (C / V)));
  if (dt == DT_BF16) hipLaunchKernelGGL(avgpool_bwd_kernel<__bf16>, grid, dim3(256), 0, st, dy, (const __bf16 *)relu_mask, (__bf16 *)dx, N, HW, C);
  else hipLaunchKernelGGL(avgpool_bwd_kernel<float>, grid, dim3(256), 0, st, dy, (const float *)relu_mask, (float *)dx, N, HW, C);
  RESIST_CHECK_LAUNCH("avgpool_bwd");
  return RESIST_OK;
}
int fc_fwd_f32(const float *x, const float *w, const float *b, float *z, int N, int C, int J, hipStream_t st) {
  prof::Scope ps("fc_fwd", 0, 0, st);
  if (C % 4 || N < 1 || J < 1) return set_error(RESIST_ESHAPE, "fully connected layer: N=%d C=%d J=%d (C must be a multiple of 4)", N, C, J);
  hipLaunchKernelGGL(fc_fwd_kernel, dim3((J + 3) / 4, (N + 15) / 16), dim3(256), 0, st, x, w, b, z, N, C, J);
  RESIST_CHECK_LAUNCH("fc_fwd");
  return RESIST_OK;
}
int fc_bwd_dx_f32(const float *dz, const float *w, float *dx, int N, int C, int J, hipStream_t st) {
  prof::Scope ps("fc_bwd_dx", 0, 0, st);
  if (C % 4) return set_error(RESIST_ESHAPE, "fully connected layer: C=%d must be a multiple of 4", C);
  hipLaunchKernelGGL(fc_bwd_dx_kernel, dim3((C + 255) / 256, (N + 3) / 4), dim3(256), 0, st, dz, w, dx, N, C, J);
  RESIST_CHECK_LAUNCH("fc_bwd_dx");
  return RESIST_OK;
}
int fc_bwd_params_f32(const float *dz, const float *x, float *dw, float *db, int N, int C, int J, hipStream_t st) {
  prof::Scope ps("fc_bwd_params", 0, 0, st);
  if (C % 4) return set_error(RESIST_ESHAPE, "fully connected layer: C=%d must be a multiple of 4", C);
  hipLaunchKernelGGL(fc_bwd_dw_kernel, dim3((C / 4 + 255) / 256, (J + 3) / 4), dim3(256), 0, st, dz, x, dw, N, C, J);
  RESIST_CHECK_LAUNCH("fc_bwd_dw");
  const int Jpad = (J + 3) & ~3;
  hipLaunchKernelGGL(fc_bwd_db_kernel, dim3(blocks_for(Jpad)), dim3(256), 0, st, dz, db, N, J, Jpad);
  RESIST_CHECK_LAUNCH("fc_bwd_db");
  return RESIST_OK;
}
int softmax_ce_f32(const float *z, const int32_t *labels, float *dz, float *row_loss, int N, int J, hipStream_t st) {
  prof::Scope ps("softmax_ce", 0, 0, st);
  hipLaunchKernelGGL(softmax_ce_kernel, dim3(N), dim3(64), 0, st, z, labels, row_loss, dz, N, J);
  RESIST_CHECK_LAUNCH("softmax_ce");
  return RESIST_OK;
}
int mean_loss_f32(const float *row_loss, float *loss, int N, hipStream_t st) {
  prof::Scope ps("mean_loss", 0, 0, st);
  hipLaunchKernelGGL(mean_loss_kernel, dim3(1), dim3(64), 0, st, row_loss, loss, N);
  RESIST_CHECK_LAUNCH("mean_loss");
  return RESIST_OK;
}

}  // namespace resist
