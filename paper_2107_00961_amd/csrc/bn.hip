// Training-mode batch normalisation on NHWC activations viewed as a matrix [M = N*H*W][C], fused
// with ReLU and the residual add of a block (forward), and with this BN's own ReLU decision (backward).
//   forward   mean_c, var_c (biased) over the M rows; a = [relu](gamma*(y-mean)*invstd + beta [+ res])
//   backward  gm = g, or g where this BN's own ReLU passed; dbeta = sum gm; dgamma = sum gm*xhat;
//             dy = gamma*invstd*(gm - dbeta/M - xhat*dgamma/M)
// These kernels are bound by HBM bandwidth.  The forward statistics arrive as per-row-tile fp32
// shifted column sums written by the convolution that produced y (at most 128 rows each) and are
// merged in float64; the backward sums are accumulated in float64 throughout (the vector fp64 rate is far
// above what the memory stream needs).  Every reduction has a fixed order, so results are bit-stable
// from run to run.
// Activations are stored as fp32 or bf16; a thread owns V = 4 (fp32) or 8 (bf16) consecutive channels
// (one 16-byte access) and all arithmetic is fp32 / fp64.
#include "elem.h"
#include "internal.h"

namespace resist {

namespace {

constexpr int kThreads = 256;
constexpr int kMaxParts = 512;  // most row-slices per channel tile (scratch capacity)

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

// per-channel fp32 parameters of the V channels a thread owns (16-byte aligned by construction)
template <int V>
__device__ inline void load_params(const float *__restrict__ p, float (&v)[V]) {
#pragma unroll
  for (int e = 0; e < V; e += 4) {
    const f32x4 t = *reinterpret_cast<const f32x4 *>(p + e);
    v[e] = t[0]; v[e + 1] = t[1]; v[e + 2] = t[2]; v[e + 3] = t[3];
  }
}

// ---- forward statistics --------------------------------------------------------------------------
// A convolution leaves, per row tile p (n_p rows) and channel, a shift k_p and the sums
// s1_p = sum(y - k_p), s2_p = sum((y - k_p)^2) over the tile's rows.  Tiles are merged by moving each to
// the shift k of the first one: with d = k_p - k,
//     sum(y - k) = s1_p + n_p*d,      sum((y - k)^2) = s2_p + d*(2*s1_p + n_p*d),
// so mean = k + S1/M and var = S2/M - (S1/M)^2 with S1/M of the order of the standard deviation
// whatever the mean is: no cancellation between large numbers.  All merging is float64.
//
// Reduction over `parts` triples per channel, layout [3][parts][C]: a workgroup owns 16 channels;
// R thread rows (R = 16 in a workgroup of 256 threads, 64 in one of 1024) each merge every R-th part
// in index order, then thread row 0 adds the R partial sums in order.  Part p holds
// min(rows, M - p*rows) rows.
template <typename S, int R>
__device__ inline void merge_parts(const S *__restrict__ st, int p0, int p1, int parts, int C, int c, int pl, long long M,
                                   long long rows, double (*red)[R][16], double *k_out, double *s1_out, double *s2_out) {
  const double k = (double)st[(size_t)p0 * C + c];
  double s = 0, q = 0;
  int p = p0 + pl;
  auto merge = [&](int pp, S kp, S a1, S a2) {
    long long n = M - (long long)pp * rows;
    n = n < rows ? n : rows;
    const double d = (double)kp - k, n_d = (double)n * d;
    s += (double)a1 + n_d;
    q += (double)a2 + d * (2.0 * (double)a1 + n_d);
  };
  // four loads of each array in flight per thread; the additions keep their order
  for (; p + 3 * R < p1; p += 4 * R) {
    S vk[4], v1[4], v2[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      vk[u] = st[(size_t)(p + R * u) * C + c];
      v1[u] = st[(size_t)(parts + p + R * u) * C + c];
      v2[u] = st[(size_t)(2 * parts + p + R * u) * C + c];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) merge(p + R * u, vk[u], v1[u], v2[u]);
  }
  for (; p < p1; p += R) merge(p, st[(size_t)p * C + c], st[(size_t)(parts + p) * C + c], st[(size_t)(2 * parts + p) * C + c]);
  const int cl = c & 15;
  red[0][pl][cl] = s;
  red[1][pl][cl] = q;
  __syncthreads();
  if (pl == 0) {
    for (int j = 1; j < R; ++j) { s += red[0][j][cl]; q += red[1][j][cl]; }
  }
  *k_out = k;
  *s1_out = s;
  *s2_out = q;
}

// first level for long lists of parts: workgroup (x, z) merges parts [z*kSlice, (z+1)*kSlice) of 16
// channels; output [3][Z][C] float64 triples (slice z then holds kSlice*rows rows, the last one fewer)
constexpr int kSlice = 64;
__global__ __launch_bounds__(kThreads) void bn_stats_reduce_kernel(const float *__restrict__ stats, int parts, int C,
                                                                   long long M, long long rows, double *__restrict__ out) {
  __shared__ double red[2][16][16];
  const int c = blockIdx.x * 16 + (threadIdx.x & 15), pl = threadIdx.x >> 4;
  const int z = blockIdx.y, Z = gridDim.y;
  const int p0 = z * kSlice, p1 = min(parts, p0 + kSlice);
  double k, s, q;
  merge_parts<float, 16>(stats, p0, p1, parts, C, c, pl, M, rows, red, &k, &s, &q);
  if (pl != 0) return;
  out[(size_t)z * C + c] = k;
  out[(size_t)(Z + z) * C + c] = s;
  out[(size_t)(2 * Z + z) * C + c] = q;
}

template <typename S, int R>
__global__ __launch_bounds__(16 * R) void bn_finalize_kernel(const S *__restrict__ stats, int parts, long long rows, int C,
                                                               long long M, float eps, float momentum,
                                                               const float *__restrict__ gamma, const float *__restrict__ beta,
                                                               float *__restrict__ mean, float *__restrict__ invstd,
                                                               float *__restrict__ scale, float *__restrict__ shift,
                                                               float *__restrict__ rmean, float *__restrict__ rvar) {
  __shared__ double red[2][R][16];
  const int c = blockIdx.x * 16 + (threadIdx.x & 15), pl = threadIdx.x >> 4;
  double k, s, q;
  merge_parts<S, R>(stats, 0, parts, parts, C, c, pl, M, rows, red, &k, &s, &q);
  if (pl != 0) return;
  const double off = s / (double)M;       // mean - k
  const double m = k + off;
  double var = q / (double)M - off * off;
  if (var < 0) var = 0;
  const float mf = (float)m, isf = (float)(1.0 / sqrt(var + (double)eps));
  mean[c] = mf;
  invstd[c] = isf;
  const float sc = gamma[c] * isf;
  scale[c] = sc;
  shift[c] = beta[c] - mf * sc;
  if (rmean) {
    const double unb = M > 1 ? var * ((double)M / (double)(M - 1)) : var;
    rmean[c] = (float)((1.0 - momentum) * (double)rmean[c] + (double)momentum * m);
    rvar[c] = (float)((1.0 - momentum) * (double)rvar[c] + (double)momentum * unb);
  }
}

// evaluation mode: the affine map from the running statistics, times a scalar `s` (the test-time
// scaling of a residual branch): scale = s*gamma/sqrt(rvar+eps), shift = s*(beta - rmean*gamma/sqrt(rvar+eps))
__global__ __launch_bounds__(kThreads) void bn_eval_affine_kernel(const float *__restrict__ gamma, const float *__restrict__ beta,
                                                                  const float *__restrict__ rmean, const float *__restrict__ rvar,
                                                                  float eps, float s, float *__restrict__ scale,
                                                                  float *__restrict__ shift, int C) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= C) return;
  const double k = (double)gamma[c] / sqrt((double)rvar[c] + (double)eps);
  scale[c] = (float)((double)s * k);
  shift[c] = (float)((double)s * ((double)beta[c] - (double)rmean[c] * k));
}

// ---- forward apply -------------------------------------------------------------------------------
struct ApplyArgs {
  const void *y; const float *scale; const float *shift;
  const void *res;                                        // raw residual or second pre-BN tensor
  const float *rscale; const float *rshift;               // BN of res (NULL: res is added as it is)
  void *a;
  long long M; int C; int tpr, rpp; int relu;
};

constexpr int kUnroll = 4;   // rows in flight per thread

template <typename T>
__global__ __launch_bounds__(kThreads) void bn_apply_kernel(ApplyArgs p) {
  constexpr int V = Vec<T>::N;
  const int tid = threadIdx.x;
  const int tc = tid % p.tpr, tr = tid / p.tpr;
  const int c = (blockIdx.y * p.tpr + tc) * V;
  const T *y = static_cast<const T *>(p.y), *res = static_cast<const T *>(p.res);
  T *a = static_cast<T *>(p.a);
  float sc[V], sh[V], rsc[V], rsh[V];
  load_params<V>(p.scale + c, sc);
  load_params<V>(p.shift + c, sh);
  if (p.rscale) {
    load_params<V>(p.rscale + c, rsc);
    load_params<V>(p.rshift + c, rsh);
  } else {
#pragma unroll
    for (int e = 0; e < V; ++e) { rsc[e] = 1.f; rsh[e] = 0.f; }
  }
  const long long stride = (long long)gridDim.x * p.rpp;
  for (long long r0 = (long long)blockIdx.x * p.rpp + tr; r0 < p.M; r0 += stride * kUnroll) {
    float v[kUnroll][V], rv[kUnroll][V];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const long long r = r0 + u * stride;
      if (r < p.M) {
        Vec<T>::load(y + (size_t)r * p.C + c, v[u]);
        if (res) Vec<T>::load(res + (size_t)r * p.C + c, rv[u]);
      }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const long long r = r0 + u * stride;
      if (r < p.M) {
        float o[V];
#pragma unroll
        for (int e = 0; e < V; ++e) o[e] = fmaf(v[u][e], sc[e], sh[e]);
        if (res) {
#pragma unroll
          for (int e = 0; e < V; ++e) o[e] += fmaf(rv[u][e], rsc[e], rsh[e]);
        }
        if (p.relu) {
#pragma unroll
          for (int e = 0; e < V; ++e) o[e] = o[e] > 0.f ? o[e] : 0.f;
        }
        Vec<T>::store(a + (size_t)r * p.C + c, o);
      }
    }
  }
}

// ---- backward ------------------------------------------------------------------------------------
// mask modes: the gradient passes where ...
constexpr int kMaskNone = 0;     // everywhere (a ReLU behind this BN's output was applied by whoever produced g)
constexpr int kMaskSelf = 2;     // this BN's own output scale*y + shift is positive (its ReLU decision)

// pass 1: per-channel sums of gm and gm*xhat; scratch [2][parts][C]
template <typename T, int MASK>
__global__ __launch_bounds__(kThreads) void bn_bwd_partial_kernel(const T *__restrict__ g,
                                                                  const T *__restrict__ y, long long M, int C, int tpr,
                                                                  int rpp, const float *__restrict__ mean,
                                                                  const float *__restrict__ invstd,
                                                                  const float *__restrict__ scale,
                                                                  const float *__restrict__ shift,
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
  float mu[V], is[V], sc[V], sh[V];
  load_params<V>(mean + c, mu);
  load_params<V>(invstd + c, is);
  if (MASK == kMaskSelf) { load_params<V>(scale + c, sc); load_params<V>(shift + c, sh); }
  double sb[V], sg[V];
#pragma unroll
  for (int e = 0; e < V; ++e) { sb[e] = 0; sg[e] = 0; }
  for (long long rr = r0 + tr; rr < r1; rr += 2 * rpp) {
    float gv[2][V], yv[2][V];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const long long r = rr + u * rpp;
      if (r < r1) {
        const size_t off = (size_t)r * C + c;
        Vec<T>::load(g + off, gv[u]);
        Vec<T>::load(y + off, yv[u]);
      }
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const long long r = rr + u * rpp;
      if (r < r1) {
#pragma unroll
        for (int e = 0; e < V; ++e) {
          float gm = gv[u][e];
          if (MASK == kMaskSelf) gm = fmaf(yv[u][e], sc[e], sh[e]) > 0.f ? gm : 0.f;
          const float xh = (yv[u][e] - mu[e]) * is[e];
          sb[e] += (double)gm;
          sg[e] = fma((double)gm, (double)xh, sg[e]);
        }
      }
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

// plain fixed-order reduction of two sums per channel, layout [2][parts][C] (the backward pass)
template <int R, typename S>
__device__ inline void reduce_parts(const S *__restrict__ scratch, int parts, int C, int c, int pl,
                                    double (*red)[R][16], double *out0, double *out1) {
  double s = 0, q = 0;
  int p = pl;
  // eight loads of each sum in flight per thread; the additions keep their order
  for (; p + 7 * R < parts; p += 8 * R) {
    S vs[8], vq[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      vs[u] = scratch[(size_t)(p + R * u) * C + c];
      vq[u] = scratch[(size_t)(parts + p + R * u) * C + c];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) { s += vs[u]; q += vq[u]; }
  }
  for (; p < parts; p += R) {
    s += scratch[(size_t)p * C + c];
    q += scratch[(size_t)(parts + p) * C + c];
  }
  const int cl = c & 15;
  red[0][pl][cl] = s;
  red[1][pl][cl] = q;
  __syncthreads();
  if (pl == 0) {
    for (int j = 1; j < R; ++j) { s += red[0][j][cl]; q += red[1][j][cl]; }
  }
  *out0 = s;
  *out1 = q;
}

// S = double: partial sums of bn_bwd_partial_kernel; S = float: per-row-tile sums left by a data gradient
template <typename S>
__global__ __launch_bounds__(kThreads) void bn_bwd_final_kernel(const S *__restrict__ scratch, int parts, int C,
                                                                float *__restrict__ dgamma, float *__restrict__ dbeta) {
  __shared__ double red[2][16][16];
  const int c = blockIdx.x * 16 + (threadIdx.x & 15), pl = threadIdx.x >> 4;
  double b, g;
  reduce_parts<16, S>(scratch, parts, C, c, pl, red, &b, &g);
  if (pl != 0) return;
  dbeta[c] = (float)b;
  dgamma[c] = (float)g;
}

struct BwdApplyArgs {
  const void *g; const void *y;
  const void *addend;   // optional: added to dy in fp32 before it is stored
  const float *mean; const float *invstd; const float *scale; const float *shift;
  const float *dgamma; const float *dbeta;
  void *dy;
  long long M; int C; int tpr, rpp;
};

template <typename T, int MASK>
__global__ __launch_bounds__(kThreads) void bn_bwd_apply_kernel(BwdApplyArgs p) {
  constexpr int V = Vec<T>::N;
  const int tid = threadIdx.x;
  const int tc = tid % p.tpr, tr = tid / p.tpr;
  const int c = (blockIdx.y * p.tpr + tc) * V;
  const T *g = static_cast<const T *>(p.g), *y = static_cast<const T *>(p.y);
  T *dy = static_cast<T *>(p.dy);
  const T *addend = static_cast<const T *>(p.addend);
  const float invM = 1.0f / (float)p.M;
  float mu[V], is[V], k0[V], sh[V], k1[V], k2[V];
  load_params<V>(p.mean + c, mu);
  load_params<V>(p.invstd + c, is);
  load_params<V>(p.scale + c, k0);          // gamma * invstd
  load_params<V>(p.shift + c, sh);
  load_params<V>(p.dbeta + c, k1);
  load_params<V>(p.dgamma + c, k2);
#pragma unroll
  for (int e = 0; e < V; ++e) { k1[e] *= invM; k2[e] *= invM; }   // means of gm and of gm*xhat
  const long long stride = (long long)gridDim.x * p.rpp;
  for (long long r0 = (long long)blockIdx.x * p.rpp + tr; r0 < p.M; r0 += stride * 2) {
    float gv[2][V], yv[2][V], mv[2][V];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const long long r = r0 + u * stride;
      if (r < p.M) {
        const size_t off = (size_t)r * p.C + c;
        Vec<T>::load(g + off, gv[u]);
        Vec<T>::load(y + off, yv[u]);
      }
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const long long r = r0 + u * stride;
      if (r < p.M) {
        const size_t off = (size_t)r * p.C + c;
        float o[V];
#pragma unroll
        for (int e = 0; e < V; ++e) {
          float gm = gv[u][e];
          if (MASK == kMaskSelf) gm = fmaf(yv[u][e], k0[e], sh[e]) > 0.f ? gm : 0.f;
          gv[u][e] = gm;
          const float xh = (yv[u][e] - mu[e]) * is[e];
          o[e] = k0[e] * (gm - k1[e] - xh * k2[e]);
        }
        if (addend) {
          float ad[V];
          Vec<T>::load(addend + off, ad);
#pragma unroll
          for (int e = 0; e < V; ++e) o[e] += ad[e];
        }
        Vec<T>::store(dy + off, o);
      }
    }
  }
}

int check_bn(int dt, int64_t M, int C) {
  if (dt != DT_F32 && dt != DT_BF16) return set_error(RESIST_EINVAL, "dtype %d", dt);
  if (M < 1 || C < 16 || (C % 16)) return set_error(RESIST_ESHAPE, "BN on [%lld][%d]: C must be a positive multiple of 16", (long long)M, C);
  return RESIST_OK;
}

// workgroups along the rows for the streaming kernels: every thread gets about `rows_per_thread`
// rows, at most 4096 workgroups in total
unsigned apply_grid_x(int64_t M, const ColMap &m, int rows_per_thread) {
  int64_t want = (M + (int64_t)m.rpp * rows_per_thread - 1) / ((int64_t)m.rpp * rows_per_thread);
  const int64_t cap = 4096 / m.ctiles > 0 ? 4096 / m.ctiles : 1;
  if (want > cap) want = cap;
  if (want < 1) want = 1;
  return (unsigned)want;
}

inline int vec_of(int dt) { return dt == DT_BF16 ? 8 : 4; }

template <typename T>
void launch_bwd(int mode, dim3 gp, dim3 ga, hipStream_t st, const void *g, const void *y, int64_t M, int C,
                const ColMap &m, const BnBufs &b, double *scratch, const BwdApplyArgs &p, int parts, const float *pre_sums) {
  const T *gg = (const T *)g, *yy = (const T *)y;
#define RESIST_BN_BWD(MODE)                                                                                              \
  if (pre_sums) {                                                                                                        \
    hipLaunchKernelGGL(bn_bwd_final_kernel<float>, dim3(C / 16), dim3(kThreads), 0, st, pre_sums, parts, C, b.dgamma, b.dbeta); \
  } else {                                                                                                               \
    hipLaunchKernelGGL((bn_bwd_partial_kernel<T, MODE>), gp, dim3(kThreads), 0, st, gg, yy, (long long)M, C, m.tpr, m.rpp, \
                       b.mean, b.invstd, b.scale, b.shift, scratch);                                                    \
    hipLaunchKernelGGL(bn_bwd_final_kernel<double>, dim3(C / 16), dim3(kThreads), 0, st, (const double *)scratch, parts, C, b.dgamma, b.dbeta); \
  }                                                                                                                      \
  hipLaunchKernelGGL((bn_bwd_apply_kernel<T, MODE>), ga, dim3(kThreads), 0, st, p);
  if (mode == kMaskSelf) { RESIST_BN_BWD(kMaskSelf) }
  else { RESIST_BN_BWD(kMaskNone) }
#undef RESIST_BN_BWD
}

}  // namespace

int64_t bn_scratch_doubles(int C) { return (int64_t)3 * kMaxParts * C; }

int bn_finalize(const float *stats, StatParts sp, int64_t M, int C, const BnBufs &b, float eps, float momentum, double *scratch,
                hipStream_t st) {
  RESIST_TRY(check_bn(DT_F32, M, C));
  const int parts = sp.parts;
  const long long rows = sp.rows;
  if (parts < 1 || rows < 1 || !stats || (long long)parts * rows < M || (long long)(parts - 1) * rows >= M)
    return set_error(RESIST_EINVAL, "bn_finalize: %d partial sums of %lld rows for %lld rows", parts, rows, (long long)M);
  prof::Scope ps("bn_finalize", 0, 12.0 * parts * C, st);
  if (parts > 4096) {
    // very long lists of row tiles: a first level over slices of kSlice parts, in its own launch
    const int Z = (parts + kSlice - 1) / kSlice;
    if (Z > kMaxParts || !scratch) return set_error(RESIST_ESHAPE, "bn_finalize: %d partial sums", parts);
    hipLaunchKernelGGL(bn_stats_reduce_kernel, dim3(C / 16, Z), dim3(kThreads), 0, st, stats, parts, C, (long long)M, rows, scratch);
    RESIST_CHECK_LAUNCH("bn_stats_reduce");
    hipLaunchKernelGGL((bn_finalize_kernel<double, 16>), dim3(C / 16), dim3(kThreads), 0, st, (const double *)scratch, Z,
                       rows * kSlice, C, (long long)M, eps, momentum, b.gamma, b.beta, b.mean, b.invstd, b.scale, b.shift, b.rmean,
                       b.rvar);
  } else if (parts > 2 * kSlice) {
    // one launch: 1024 threads per 16 channels, 64 thread rows share the parts
    hipLaunchKernelGGL((bn_finalize_kernel<float, 64>), dim3(C / 16), dim3(1024), 0, st, stats, parts, rows, C, (long long)M, eps,
                       momentum, b.gamma, b.beta, b.mean, b.invstd, b.scale, b.shift, b.rmean, b.rvar);
  } else {
    hipLaunchKernelGGL((bn_finalize_kernel<float, 16>), dim3(C / 16), dim3(kThreads), 0, st, stats, parts, rows, C, (long long)M,
                       eps, momentum, b.gamma, b.beta, b.mean, b.invstd, b.scale, b.shift, b.rmean, b.rvar);
  }
  RESIST_CHECK_LAUNCH("bn_finalize");
  return RESIST_OK;
}

int bn_eval_affine(int C, const BnBufs &b, float eps, float s, hipStream_t st) {
  if (C < 1) return set_error(RESIST_ESHAPE, "bn_eval_affine: C=%d", C);
  prof::Scope ps("bn_eval_affine", 0, 24.0 * C, st);
  hipLaunchKernelGGL(bn_eval_affine_kernel, dim3((C + kThreads - 1) / kThreads), dim3(kThreads), 0, st, b.gamma, b.beta, b.rmean,
                     b.rvar, eps, s, b.scale, b.shift, C);
  RESIST_CHECK_LAUNCH("bn_eval_affine");
  return RESIST_OK;
}

int bn_apply(int dt, const void *y, int64_t M, int C, const BnBufs &b, const void *res, const BnBufs *res_bn, bool relu,
             void *a, hipStream_t st) {
  RESIST_TRY(check_bn(dt, M, C));
  const ColMap m = col_map(C, vec_of(dt));
  ApplyArgs p{};
  p.y = y; p.scale = b.scale; p.shift = b.shift;
  p.res = res;
  if (res_bn) { p.rscale = res_bn->scale; p.rshift = res_bn->shift; }
  p.a = a; p.M = M; p.C = C; p.tpr = m.tpr; p.rpp = m.rpp; p.relu = relu ? 1 : 0;
  prof::Scope ps("bn_apply", 0, (double)esize(dt) * M * C * (res ? 3 : 2), st);
  const dim3 grid(apply_grid_x(M, m, 2 * kUnroll), m.ctiles);
  if (dt == DT_BF16) hipLaunchKernelGGL(bn_apply_kernel<__bf16>, grid, dim3(kThreads), 0, st, p);
  else hipLaunchKernelGGL(bn_apply_kernel<float>, grid, dim3(kThreads), 0, st, p);
  RESIST_CHECK_LAUNCH("bn_apply");
  return RESIST_OK;
}

int bn_backward(int dt, const void *g, bool relu_of_self, const void *y, int64_t M, int C, const BnBufs &b, void *dy,
                const void *addend, double *scratch, hipStream_t st, const float *pre_sums, StatParts pre) {
  RESIST_TRY(check_bn(dt, M, C));
  const ColMap m = col_map(C, vec_of(dt));
  if (pre_sums && (pre.parts < 1 || pre.rows < 1 || (long long)pre.parts * pre.rows < M ||
                   (long long)(pre.parts - 1) * pre.rows >= M))
    return set_error(RESIST_EINVAL, "bn_backward: %d pre-computed partial sums of %d rows for %lld rows", pre.parts, pre.rows, (long long)M);
  const int parts = pre_sums ? pre.parts : num_parts(M, m);
  const int mode = relu_of_self ? kMaskSelf : kMaskNone;
  const int reads = 2;
  prof::Scope ps("bn_backward", 0, (double)esize(dt) * M * C * ((pre_sums ? 1 : 2) * reads + 1 + (addend ? 1 : 0)), st);
  BwdApplyArgs p{};
  p.g = g; p.y = y; p.addend = addend; p.mean = b.mean; p.invstd = b.invstd; p.scale = b.scale; p.shift = b.shift;
  p.dgamma = b.dgamma; p.dbeta = b.dbeta; p.dy = dy;
  p.M = M; p.C = C; p.tpr = m.tpr; p.rpp = m.rpp;
  const dim3 gp(parts, m.ctiles), ga(apply_grid_x(M, m, 4), m.ctiles);
  if (dt == DT_BF16) launch_bwd<__bf16>(mode, gp, ga, st, g, y, M, C, m, b, scratch, p, parts, pre_sums);
  else launch_bwd<float>(mode, gp, ga, st, g, y, M, C, m, b, scratch, p, parts, pre_sums);
  RESIST_CHECK_LAUNCH("bn_backward");
  return RESIST_OK;
}

}  // namespace resist
