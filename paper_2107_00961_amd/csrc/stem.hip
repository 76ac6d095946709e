// Input preparation for the stem convolution.  The logical [N,C,H,W] fp32 batch (C = 3) is
// expanded into im2col rows [N*P*Q][kpad] with column (r*S + s)*C + c and zero columns up to kpad
// (a multiple of the GEMM K-chunk), so that the stem runs as a 1x1 convolution on the same MFMA
// kernels as every other layer, in both the forward pass and the weight gradient.
// The rows are written in the storage type of the activations (fp32, or bf16 rounded to nearest even).
#include "elem.h"
#include "internal.h"

namespace resist {
namespace {

// one thread writes V consecutive columns of one row (a 16-byte store); kpad is a multiple of 32
template <typename T>
__global__ __launch_bounds__(256) void stem_im2col_kernel(const float *__restrict__ x, T *__restrict__ col, int N, int C,
                                                          int H, int W, int R, int stride, int pad, int P, int Q, int kpad) {
  constexpr int V = Vec<T>::N;
  const int vpr = kpad / V;
  const long long total = (long long)N * P * Q * vpr;
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int j0 = (int)(i % vpr) * V;
  long long m = i / vpr;
  const int q = (int)(m % Q); m /= Q;
  const int p = (int)(m % P);
  const int n = (int)(m / P);
  float v[V];
#pragma unroll
  for (int e = 0; e < V; ++e) {
    const int j = j0 + e;
    float t = 0.f;
    if (j < R * R * C) {
      const int c = j % C, tap = j / C;
      const int r = tap / R, s = tap % R;
      const int ih = p * stride + r - pad, iw = q * stride + s - pad;
      if (ih >= 0 && ih < H && iw >= 0 && iw < W) t = x[((size_t)(n * C + c) * H + ih) * W + iw];
    }
    v[e] = t;
  }
  Vec<T>::store(col + i * V, v);
}

template <typename T>
__global__ __launch_bounds__(256) void repitch_rows_kernel(const float *__restrict__ src, T *__restrict__ dst, int rows,
                                                           int n, int src_pitch, int dst_pitch) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (long long)rows * dst_pitch) return;
  const int j = (int)(i % dst_pitch);
  const long long r = i / dst_pitch;
  Vec<T>::put(dst + i, j < n ? src[r * src_pitch + j] : 0.f);
}

}  // namespace

int stem_im2col(int dt, const float *x, void *col, int N, int C, int H, int W, int R, int stride, int pad, int P, int Q,
                int kpad, hipStream_t st) {
  const long long total = (long long)N * P * Q * kpad;
  if (total > 0x7fffffffLL * 256) return set_error(RESIST_ESHAPE, "im2col too large");
  prof::Scope ps("stem_im2col", 0, 4.0 * N * C * H * W + (double)esize(dt) * total, st);
  const int V = dt == DT_BF16 ? 8 : 4;
  if (kpad % 32) return set_error(RESIST_ESHAPE, "im2col row length %d is not a multiple of 32", kpad);
  const dim3 grid((unsigned)((total / V + 255) / 256));
  if (dt == DT_BF16)
    hipLaunchKernelGGL(stem_im2col_kernel<__bf16>, grid, dim3(256), 0, st, x, (__bf16 *)col, N, C, H, W, R, stride, pad, P, Q, kpad);
  else
    hipLaunchKernelGGL(stem_im2col_kernel<float>, grid, dim3(256), 0, st, x, (float *)col, N, C, H, W, R, stride, pad, P, Q, kpad);
  RESIST_CHECK_LAUNCH("stem_im2col");
  return RESIST_OK;
}

int pad_rows(int dt, const float *src, void *dst, int rows, int n, int npad, hipStream_t st) {
  const long long total = (long long)rows * npad;
  const dim3 grid((unsigned)((total + 255) / 256));
  if (dt == DT_BF16) hipLaunchKernelGGL(repitch_rows_kernel<__bf16>, grid, dim3(256), 0, st, src, (__bf16 *)dst, rows, n, n, npad);
  else hipLaunchKernelGGL(repitch_rows_kernel<float>, grid, dim3(256), 0, st, src, (float *)dst, rows, n, n, npad);
  RESIST_CHECK_LAUNCH("pad_rows");
  return RESIST_OK;
}

int unpad_rows_f32(const float *src, float *dst, int rows, int n, int npad, hipStream_t st) {
  const long long total = (long long)rows * n;
  hipLaunchKernelGGL(repitch_rows_kernel<float>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, src, dst, rows, n, npad, n);
  RESIST_CHECK_LAUNCH("unpad_rows");
  return RESIST_OK;
}

}  // namespace resist
