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

// The same expansion, one workgroup per output row (n, p): the R input rows of the C channels that
// this output row touches are staged in LDS with coalesced loads (rows outside the image as zeros),
// a small table maps every im2col column to its LDS offset, and the Q*kpad outputs are then assembled
// from LDS and written as 16-byte vectors.  The element-wise kernel above does one scattered global
// load and a handful of integer divisions per element; at ImageNet size it ran at 1.2 TB/s.
template <typename T>
__global__ __launch_bounds__(256) void stem_im2col_rows_kernel(const float *__restrict__ x, T *__restrict__ col, int C, int H,
                                                               int W, int R, int stride, int pad, int P, int Q, int kpad) {
  extern __shared__ float lds[];          // [R][C][W] input rows, then kpad table entries
  constexpr int V = Vec<T>::N;
  const int n = blockIdx.x / P, p = blockIdx.x - n * P;
  const int rows = R * C;
  int *base_of = reinterpret_cast<int *>(lds + rows * W);   // LDS offset of column j at q = 0 without the -pad shift; -1: zero column
  int *shift_of = base_of + kpad;                            // s - pad of column j
  for (int i = threadIdx.x; i < rows * W; i += 256) {
    const int rc = i / W, w = i - rc * W;
    const int r = rc / C, c = rc - r * C;
    const int ih = p * stride + r - pad;
    lds[i] = (ih >= 0 && ih < H) ? x[((size_t)(n * C + c) * H + ih) * W + w] : 0.f;
  }
  for (int j = threadIdx.x; j < kpad; j += 256) {
    int b = -1, sh = 0;
    if (j < R * R * C) {
      const int c = j % C, tap = j / C;
      const int r = tap / R, s2 = tap - r * R;
      b = (r * C + c) * W;
      sh = s2 - pad;
    }
    base_of[j] = b;
    shift_of[j] = sh;
  }
  __syncthreads();
  // thread (ql, jv): vector jv of the row, output pixels ql, ql + nq, ...; its V table entries stay in registers
  const int vpr = kpad / V;
  const int nq = 256 / vpr;
  const int ql = threadIdx.x / vpr, jv = threadIdx.x - ql * vpr;
  if (ql >= nq) return;
  int b[V], sh[V];
#pragma unroll
  for (int e = 0; e < V; ++e) { b[e] = base_of[jv * V + e]; sh[e] = shift_of[jv * V + e]; }
  T *out = col + (size_t)blockIdx.x * Q * kpad + jv * V;
  for (int q = ql; q < Q; q += nq) {
    const int w0 = q * stride;
    float v[V];
#pragma unroll
    for (int e = 0; e < V; ++e) {
      const int iw = w0 + sh[e];
      v[e] = (b[e] >= 0 && iw >= 0 && iw < W) ? lds[b[e] + iw] : 0.f;
    }
    Vec<T>::store(out + (size_t)q * kpad, v);
  }
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
  const size_t lds_bytes = ((size_t)R * C * W + 2 * (size_t)kpad) * 4;
  if (lds_bytes <= 48 * 1024 && (long long)N * P < 0x7fffffffLL && kpad / V <= 256) {
    // one workgroup per output row, input rows staged in LDS
    const dim3 rows_grid((unsigned)(N * P));
    if (dt == DT_BF16)
      hipLaunchKernelGGL(stem_im2col_rows_kernel<__bf16>, rows_grid, dim3(256), lds_bytes, st, x, (__bf16 *)col, C, H, W, R, stride, pad, P, Q, kpad);
    else
      hipLaunchKernelGGL(stem_im2col_rows_kernel<float>, rows_grid, dim3(256), lds_bytes, st, x, (float *)col, C, H, W, R, stride, pad, P, Q, kpad);
    RESIST_CHECK_LAUNCH("stem_im2col");
    return RESIST_OK;
  }
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
