// Training-mode batch normalisation on NHWC activations viewed as a matrix [M = N*H*W][C], fused
// with ReLU and the residual add of a block (forward), and with the ReLU mask (backward).
//   forward   mean_c, var_c (biased) over the M rows; a = [relu](gamma*(y-mean)*invstd + beta [+ res])
//   backward  gm = g*[mask>0]; dbeta = sum gm; dgamma = sum gm*xhat;
//             dy = gamma*invstd*(gm - dbeta/M - xhat*dgamma/M)
// These kernels are bound by HBM bandwidth.  Per-channel sums are accumulated in float64 (the
// vector fp64 rate is far above what the memory stream needs), in a fixed order, so results are
// bit-stable from run to run and free of the cancellation a float32 sum-of-squares would suffer.
// Activations are stored as fp32 or bf16; a thread owns V = 4 (fp32) or 8 (bf16) consecutive channels
// (one 16-byte access) and all arithmetic is fp32 / fp64.
#include "elem.h"
#include "internal.h"

namespace resist {

namespace {

constexpr int kThreads = 256;
constexpr int kMaxParts = 512;  // row-slices per channel tile

struct ColMap {
  int tpr;       // threads per row (each owns V consecutive channels)
  int rpp;       // rows per pass of one workgroup
  int ctiles;    // channel tiles of tpr*V channels
};
inline ColMap col_map(int C, int V) {
  ColMap m;
  const int cv = C / V;   // C is a multiple of 16, so cv >= 2
  // tpr must divide 256: the largest power of two that divides cv
  int t = 1;
  while (t * 2 <= cv && (cv % (t * 2)) == 0 && t * 2 <= kThreads) t *= 2;
  m.tpr = t;
  m.rpp = kThreads / m.tpr;
  m.ctiles = cv / m.tpr;
  return m;
}
inline int num_parts(int64_t M, const ColMap &m) {
  // aim at ~2048 workgroups in total, at least 8 passes of rows each
  int64_t want = 2048 / m.ctiles;
  if (want < 1) want = 1;
  int64_t maxp = (M + (int64_t)m.rpp * 8 - 1) / ((int64_t)m.rpp * 8);
  int64_t p = want < maxp ? want : maxp;
  if (p < 1) p = 1;
  if (p > kMaxParts) p = kMaxParts;
  return (int)p;
}

// ---- forward statistics --------------------------------------------------------------------------
// grid (parts, ctiles); scratch layout [2][parts][C] doubles: sum, sum of squares
template <typename T>
__global__ __launch_bounds__(kThreads) void bn_stats_partial_kernel(const T *__restrict__ y, long long M, int C,
                                                                    int tpr, int rpp, double *__restrict__ scratch) {
  constexpr int V = Vec<T>::N;
  __shared__ double red[2][kThreads][V];
  const int tid = threadIdx.x;
  const int tc = tid % tpr, tr = tid / tpr;
  const int c = (blockIdx.y * tpr + tc) * V;
  const int parts = gridDim.x;
  const long long rows_per_part = (M + parts - 1) / parts;
  const long long r0 = blockIdx.x * rows_per_part;
  long long r1 = r0 + rows_per_part;
  if (r1 > M) r1 = M;
  double s[V], q[V];
#pragma unroll
  for (int e = 0; e < V; ++e) { s[e] = 0; q[e] = 0; }
  for (long long r = r0 + tr; r < r1; r += rpp) {
    float v[V];
    Vec<T>::load(y + r * C + c, v);
#pragma unroll
    for (int e = 0; e < V; ++e) {
      const double d = (double)v[e];
      s[e] += d;
      q[e] = fma(d, d, q[e]);
    }
  }
#pragma unroll
  for (int e = 0; e < V; ++e) { red[0][tid][e] = s[e]; red[1][tid][e] = q[e]; }
  __syncthreads();
  if (tr == 0) {
    for (int j = 1; j < rpp; ++j)
#pragma unroll
      for (int e = 0; e < V; ++e) { s[e] += red[0][j * tpr + tc][e]; q[e] += red[1][j * tpr + tc][e]; }
    double *ps = scratch + (size_t)blockIdx.x * C + c;
    double *pq = scratch + (size_t)(parts + blockIdx.x) * C + c;
#pragma unroll
    for (int e = 0; e < V; ++e) { ps[e] = s[e]; pq[e] = q[e]; }
  }
}

// Final reduction over the row-slices: a workgroup owns 16 channels; 16 thread rows each sum every
// 16th slice in index order, then thread row 0 adds the 16 partial sums in order.
__device__ inline void reduce_parts(const double *__restrict__ scratch, int parts, int C, int c, int pl,
                                    double (*red)[16][16], double *out0, double *out1) {
  double s = 0, q = 0;
  for (int p = pl; p < parts; p += 16) {
    s += scratch[(size_t)p * C + c];
    q += scratch[(size_t)(parts + p) * C + c];
  }
  const int cl = c & 15;
  red[0][pl][cl] = s;
  red[1][pl][cl] = q;
  __syncthreads();
  if (pl == 0) {
    for (int j = 1; j < 16; ++j) { s += red[0][j][cl]; q += red[1][j][cl]; }
  }
  *out0 = s;
  *out1 = q;
}

__global__ __launch_bounds__(kThreads) void bn_stats_final_kernel(const double *__restrict__ scratch, int parts, int C,
                                                                  long long M, float eps, float momentum,
                                                                  float *__restrict__ mean, float *__restrict__ invstd,
                                                                  float *__restrict__ rmean, float *__restrict__ rvar) {
  __shared__ double red[2][16][16];
  const int c = blockIdx.x * 16 + (threadIdx.x & 15), pl = threadIdx.x >> 4;
  double s, q;
  reduce_parts(scratch, parts, C, c, pl, red, &s, &q);
  if (pl != 0) return;
  const double m = s / (double)M;
  double var = q / (double)M - m * m;
  if (var < 0) var = 0;
  mean[c] = (float)m;
  invstd[c] = (float)(1.0 / sqrt(var + (double)eps));
  if (rmean) {
    const double unb = M > 1 ? var * ((double)M / (double)(M - 1)) : var;
    rmean[c] = (float)((1.0 - momentum) * (double)rmean[c] + (double)momentum * m);
    rvar[c] = (float)((1.0 - momentum) * (double)rvar[c] + (double)momentum * unb);
  }
}

// ---- forward apply -------------------------------------------------------------------------------
struct ApplyArgs {
  const void *y; const float *gamma; const float *beta; const float *mean; const float *invstd;
  const void *res;                                        // raw residual or second pre-BN tensor
  const float *rgamma; const float *rbeta; const float *rmean; const float *rinvstd;  // BN of res
  void *a;
  long long M; int C; int tpr, rpp; int relu;
};

template <typename T>
__global__ __launch_bounds__(kThreads) void bn_apply_kernel(ApplyArgs p) {
  constexpr int V = Vec<T>::N;
  const int tid = threadIdx.x;
  const int tc = tid % p.tpr, tr = tid / p.tpr;
  const int c = (blockIdx.y * p.tpr + tc) * V;
  const T *y = static_cast<const T *>(p.y), *res = static_cast<const T *>(p.res);
  T *a = static_cast<T *>(p.a);
  float sc[V], sh[V], rsc[V], rsh[V];
#pragma unroll
  for (int e = 0; e < V; ++e) {
    sc[e] = p.gamma[c + e] * p.invstd[c + e];
    sh[e] = p.beta[c + e] - p.mean[c + e] * sc[e];
    if (p.rgamma) {
      rsc[e] = p.rgamma[c + e] * p.rinvstd[c + e];
      rsh[e] = p.rbeta[c + e] - p.rmean[c + e] * rsc[e];
    } else {
      rsc[e] = 1.f; rsh[e] = 0.f;
    }
  }
  const long long stride = (long long)gridDim.x * p.rpp;
  for (long long r = (long long)blockIdx.x * p.rpp + tr; r < p.M; r += stride) {
    const size_t off = (size_t)r * p.C + c;
    float v[V], o[V];
    Vec<T>::load(y + off, v);
#pragma unroll
    for (int e = 0; e < V; ++e) o[e] = fmaf(v[e], sc[e], sh[e]);
    if (res) {
      float rv[V];
      Vec<T>::load(res + off, rv);
#pragma unroll
      for (int e = 0; e < V; ++e) o[e] += fmaf(rv[e], rsc[e], rsh[e]);
    }
    if (p.relu) {
#pragma unroll
      for (int e = 0; e < V; ++e) o[e] = o[e] > 0.f ? o[e] : 0.f;
    }
    Vec<T>::store(a + off, o);
  }
}

// ---- backward ------------------------------------------------------------------------------------
// pass 1: per-channel sums of gm and gm*xhat; scratch [2][parts][C]
template <typename T>
__global__ __launch_bounds__(kThreads) void bn_bwd_partial_kernel(const T *__restrict__ g, const T *__restrict__ mask,
                                                                  const T *__restrict__ y, long long M, int C, int tpr,
                                                                  int rpp, const float *__restrict__ mean,
                                                                  const float *__restrict__ invstd,
                                                                  double *__restrict__ scratch) {
  constexpr int V = Vec<T>::N;
  __shared__ double red[2][kThreads][V];
  const int tid = threadIdx.x;
  const int tc = tid % tpr, tr = tid / tpr;
  const int c = (blockIdx.y * tpr + tc) * V;
  const int parts = gridDim.x;
  const long long rows_per_part = (M + parts - 1) / parts;
  const long long r0 = blockIdx.x * rows_per_part;
  long long r1 = r0 + rows_per_part;
  if (r1 > M) r1 = M;
  float mu[V], is[V];
  double sb[V], sg[V];
#pragma unroll
  for (int e = 0; e < V; ++e) { mu[e] = mean[c + e]; is[e] = invstd[c + e]; sb[e] = 0; sg[e] = 0; }
  for (long long r = r0 + tr; r < r1; r += rpp) {
    const size_t off = (size_t)r * C + c;
    float gv[V], yv[V];
    Vec<T>::load(g + off, gv);
    Vec<T>::load(y + off, yv);
    if (mask) {
      float mv[V];
      Vec<T>::load(mask + off, mv);
#pragma unroll
      for (int e = 0; e < V; ++e) gv[e] = mv[e] > 0.f ? gv[e] : 0.f;
    }
#pragma unroll
    for (int e = 0; e < V; ++e) {
      const float xh = (yv[e] - mu[e]) * is[e];
      sb[e] += (double)gv[e];
      sg[e] = fma((double)gv[e], (double)xh, sg[e]);
    }
  }
#pragma unroll
  for (int e = 0; e < V; ++e) { red[0][tid][e] = sb[e]; red[1][tid][e] = sg[e]; }
  __syncthreads();
  if (tr == 0) {
    for (int j = 1; j < rpp; ++j)
#pragma unroll
      for (int e = 0; e < V; ++e) { sb[e] += red[0][j * tpr + tc][e]; sg[e] += red[1][j * tpr + tc][e]; }
    double *pb = scratch + (size_t)blockIdx.x * C + c;
    double *pg = scratch + (size_t)(parts + blockIdx.x) * C + c;
#pragma unroll
    for (int e = 0; e < V; ++e) { pb[e] = sb[e]; pg[e] = sg[e]; }
  }
}

__global__ __launch_bounds__(kThreads) void bn_bwd_final_kernel(const double *__restrict__ scratch, int parts, int C,
                                                                float *__restrict__ dgamma, float *__restrict__ dbeta) {
  __shared__ double red[2][16][16];
  const int c = blockIdx.x * 16 + (threadIdx.x & 15), pl = threadIdx.x >> 4;
  double b, g;
  reduce_parts(scratch, parts, C, c, pl, red, &b, &g);
  if (pl != 0) return;
  dbeta[c] = (float)b;
  dgamma[c] = (float)g;
}

struct BwdApplyArgs {
  const void *g; const void *mask; const void *y;
  const float *gamma; const float *mean; const float *invstd; const float *dgamma; const float *dbeta;
  void *dy; void *gm_out;
  long long M; int C; int tpr, rpp;
};

template <typename T>
__global__ __launch_bounds__(kThreads) void bn_bwd_apply_kernel(BwdApplyArgs p) {
  constexpr int V = Vec<T>::N;
  const int tid = threadIdx.x;
  const int tc = tid % p.tpr, tr = tid / p.tpr;
  const int c = (blockIdx.y * p.tpr + tc) * V;
  const T *g = static_cast<const T *>(p.g), *mask = static_cast<const T *>(p.mask), *y = static_cast<const T *>(p.y);
  T *dy = static_cast<T *>(p.dy), *gm_out = static_cast<T *>(p.gm_out);
  const float invM = 1.0f / (float)p.M;
  float mu[V], is[V], k0[V], k1[V], k2[V];
#pragma unroll
  for (int e = 0; e < V; ++e) {
    mu[e] = p.mean[c + e]; is[e] = p.invstd[c + e];
    k0[e] = p.gamma[c + e] * is[e];          // scale
    k1[e] = p.dbeta[c + e] * invM;           // mean of gm
    k2[e] = p.dgamma[c + e] * invM;          // mean of gm*xhat
  }
  const long long stride = (long long)gridDim.x * p.rpp;
  for (long long r = (long long)blockIdx.x * p.rpp + tr; r < p.M; r += stride) {
    const size_t off = (size_t)r * p.C + c;
    float gv[V], yv[V], o[V];
    Vec<T>::load(g + off, gv);
    Vec<T>::load(y + off, yv);
    if (mask) {
      float mv[V];
      Vec<T>::load(mask + off, mv);
#pragma unroll
      for (int e = 0; e < V; ++e) gv[e] = mv[e] > 0.f ? gv[e] : 0.f;
    }
#pragma unroll
    for (int e = 0; e < V; ++e) {
      const float xh = (yv[e] - mu[e]) * is[e];
      o[e] = k0[e] * (gv[e] - k1[e] - xh * k2[e]);
    }
    Vec<T>::store(dy + off, o);
    if (gm_out) Vec<T>::store(gm_out + off, gv);   // exact: gm is g or zero
  }
}

int check_bn(int dt, int64_t M, int C) {
  if (dt != DT_F32 && dt != DT_BF16) return set_error(RESIST_EINVAL, "dtype %d", dt);
  if (M < 1 || C < 16 || (C % 16)) return set_error(RESIST_ESHAPE, "BN on [%lld][%d]: C must be a positive multiple of 16", (long long)M, C);
  return RESIST_OK;
}

unsigned apply_grid_x(int64_t M, const ColMap &m) {
  int64_t want = 4096 / m.ctiles;
  if (want < 1) want = 1;
  const int64_t maxb = (M + m.rpp - 1) / m.rpp;
  return (unsigned)(want < maxb ? want : maxb);
}

inline int vec_of(int dt) { return dt == DT_BF16 ? 8 : 4; }

}  // namespace

int64_t bn_scratch_doubles(int C) { return (int64_t)2 * kMaxParts * C; }

int bn_stats(int dt, const void *y, int64_t M, int C, const BnBufs &b, float eps, float momentum, double *scratch,
             hipStream_t st) {
  RESIST_TRY(check_bn(dt, M, C));
  const ColMap m = col_map(C, vec_of(dt));
  const int parts = num_parts(M, m);
  prof::Scope ps("bn_stats", 0, (double)esize(dt) * M * C, st);
  if (dt == DT_BF16)
    hipLaunchKernelGGL(bn_stats_partial_kernel<__bf16>, dim3(parts, m.ctiles), dim3(kThreads), 0, st, (const __bf16 *)y, (long long)M, C, m.tpr, m.rpp, scratch);
  else
    hipLaunchKernelGGL(bn_stats_partial_kernel<float>, dim3(parts, m.ctiles), dim3(kThreads), 0, st, (const float *)y, (long long)M, C, m.tpr, m.rpp, scratch);
  RESIST_CHECK_LAUNCH("bn_stats_partial");
  hipLaunchKernelGGL(bn_stats_final_kernel, dim3(C / 16), dim3(kThreads), 0, st, scratch, parts, C,
                     (long long)M, eps, momentum, b.mean, b.invstd, b.rmean, b.rvar);
  RESIST_CHECK_LAUNCH("bn_stats_final");
  return RESIST_OK;
}

int bn_apply(int dt, const void *y, int64_t M, int C, const BnBufs &b, const void *res, const BnBufs *res_bn, bool relu,
             void *a, hipStream_t st) {
  RESIST_TRY(check_bn(dt, M, C));
  const ColMap m = col_map(C, vec_of(dt));
  ApplyArgs p{};
  p.y = y; p.gamma = b.gamma; p.beta = b.beta; p.mean = b.mean; p.invstd = b.invstd;
  p.res = res;
  if (res_bn) { p.rgamma = res_bn->gamma; p.rbeta = res_bn->beta; p.rmean = res_bn->mean; p.rinvstd = res_bn->invstd; }
  p.a = a; p.M = M; p.C = C; p.tpr = m.tpr; p.rpp = m.rpp; p.relu = relu ? 1 : 0;
  prof::Scope ps("bn_apply", 0, (double)esize(dt) * M * C * (res ? 3 : 2), st);
  if (dt == DT_BF16) hipLaunchKernelGGL(bn_apply_kernel<__bf16>, dim3(apply_grid_x(M, m), m.ctiles), dim3(kThreads), 0, st, p);
  else hipLaunchKernelGGL(bn_apply_kernel<float>, dim3(apply_grid_x(M, m), m.ctiles), dim3(kThreads), 0, st, p);
  RESIST_CHECK_LAUNCH("bn_apply");
  return RESIST_OK;
}

int bn_backward(int dt, const void *g, const void *mask, const void *y, int64_t M, int C, const BnBufs &b, void *dy,
                void *gm_out, double *scratch, hipStream_t st) {
  RESIST_TRY(check_bn(dt, M, C));
  const ColMap m = col_map(C, vec_of(dt));
  const int parts = num_parts(M, m);
  prof::Scope ps("bn_backward", 0, (double)esize(dt) * M * C * ((mask ? 3 : 2) + (mask ? 4 : 3) + (gm_out ? 1 : 0)), st);
  if (dt == DT_BF16)
    hipLaunchKernelGGL(bn_bwd_partial_kernel<__bf16>, dim3(parts, m.ctiles), dim3(kThreads), 0, st, (const __bf16 *)g,
                       (const __bf16 *)mask, (const __bf16 *)y, (long long)M, C, m.tpr, m.rpp, b.mean, b.invstd, scratch);
  else
    hipLaunchKernelGGL(bn_bwd_partial_kernel<float>, dim3(parts, m.ctiles), dim3(kThreads), 0, st, (const float *)g,
                       (const float *)mask, (const float *)y, (long long)M, C, m.tpr, m.rpp, b.mean, b.invstd, scratch);
  RESIST_CHECK_LAUNCH("bn_bwd_partial");
  hipLaunchKernelGGL(bn_bwd_final_kernel, dim3(C / 16), dim3(kThreads), 0, st, scratch, parts, C,
                     b.dgamma, b.dbeta);
  RESIST_CHECK_LAUNCH("bn_bwd_final");
  BwdApplyArgs p{};
  p.g = g; p.mask = mask; p.y = y; p.gamma = b.gamma; p.mean = b.mean; p.invstd = b.invstd;
  p.dgamma = b.dgamma; p.dbeta = b.dbeta; p.dy = dy; p.gm_out = gm_out;
  p.M = M; p.C = C; p.tpr = m.tpr; p.rpp = m.rpp;
  if (dt == DT_BF16) hipLaunchKernelGGL(bn_bwd_apply_kernel<__bf16>, dim3(apply_grid_x(M, m), m.ctiles), dim3(kThreads), 0, st, p);
  else hipLaunchKernelGGL(bn_bwd_apply_kernel<float>, dim3(apply_grid_x(M, m), m.ctiles), dim3(kThreads), 0, st, p);
  RESIST_CHECK_LAUNCH("bn_bwd_apply");
  return RESIST_OK;
}

}  // namespace resist
