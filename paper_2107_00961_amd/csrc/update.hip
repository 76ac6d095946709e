// SGD-with-momentum update of every trainable parameter of a sub-ResNet (Algorithm 1's inner
// update, with the momentum and weight decay of the paper's experimental setup), and the
// reassembly kernel that averages the copies of a block held by several sub-ResNets (Sec. 2.3;
// Appendix B: W = sum_v W_v M_v / sum_v M_v).  Both are pure streaming kernels bound by HBM
// bandwidth: 16-byte accesses, one pass, segment tables passed by value in the kernel arguments.
#include "internal.h"

namespace resist {

typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kChunk = 4096;  // floats per workgroup (256 threads x 4 float4)
constexpr int kSgdSegs = 48;
constexpr int kAggSrc = 16;   // most sub-ResNets that may hold one block

struct SgdTable {
  float *w[kSgdSegs];
  float *v[kSgdSegs];
  const float *g[kSgdSegs];
  long long n[kSgdSegs];
  int first_wg[kSgdSegs + 1];
  int nseg;
  float lr, mu, wd;
};

// Segment of this workgroup: first_wg is ascending, so the segment index is the number of segment
// starts at or below blockIdx.x.  One lane per candidate and a ballot: a single round trip to the
// kernel arguments instead of a chain of dependent loads.  nseg <= 64.
__device__ inline int find_seg(const int *first_wg, int nseg) {
  const int lane = threadIdx.x & 63;
  const bool past = lane + 1 < nseg && (int)blockIdx.x >= first_wg[lane + 1];
  return __popcll(__ballot(past));
}

__global__ __launch_bounds__(256) void sgd_kernel(SgdTable t) {
  const int seg = find_seg(t.first_wg, t.nseg);
  const long long base = (long long)(blockIdx.x - t.first_wg[seg]) * kChunk;
  float *w = t.w[seg];
  float *v = t.v[seg];
  const float *g = t.g[seg];
  const long long n = t.n[seg];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const long long i = base + (u * 256 + threadIdx.x) * 4;
    if (i + 3 < n) {
      const f32x4 wv = *reinterpret_cast<const f32x4 *>(w + i);
      const f32x4 gv = *reinterpret_cast<const f32x4 *>(g + i);
      const f32x4 vv = *reinterpret_cast<const f32x4 *>(v + i);
      f32x4 nv, nw;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float gg = fmaf(t.wd, wv[e], gv[e]);
        nv[e] = fmaf(t.mu, vv[e], gg);
        nw[e] = fmaf(-t.lr, nv[e], wv[e]);
      }
      *reinterpret_cast<f32x4 *>(v + i) = nv;
      *reinterpret_cast<f32x4 *>(w + i) = nw;
    } else {
      for (long long k = i; k < n; ++k) {
        const float gg = fmaf(t.wd, w[k], g[k]);
        const float nv = fmaf(t.mu, v[k], gg);
        v[k] = nv;
        w[k] = fmaf(-t.lr, nv, w[k]);
      }
    }
  }
}

// The segment table travels in the kernel arguments (4 KB at most), so the number of segments one
// launch covers depends on how many sources a segment may have: 56 / 36 / 20 for up to 4 / 8 / 16.
template <int NSRC> struct AggTable {
  static constexpr int kSegs = NSRC <= 4 ? 56 : (NSRC <= 8 ? 36 : 20);
  float *dst[kSegs];
  const float *src[kSegs][NSRC];
  long long n[kSegs];
  int count[kSegs];
  int first_wg[kSegs + 1];
  int nseg;
};

template <int NSRC>
__global__ __launch_bounds__(256) void aggregate_kernel(AggTable<NSRC> t) {
  // the segment index is the same in every lane; telling the compiler so keeps the table lookups scalar
  const int seg = __builtin_amdgcn_readfirstlane(find_seg(t.first_wg, t.nseg));
  const long long base = (long long)(blockIdx.x - t.first_wg[seg]) * kChunk;
  float *dst = t.dst[seg];
  const long long n = t.n[seg];
  const int count = t.count[seg];
  const float fc = (float)count;
  if (base + kChunk <= n) {
    // whole chunk: every load of the workgroup is issued before the first sum; the only branches are
    // the uniform "source s present" ones
    constexpr int UB = NSRC <= 4 ? 4 : (NSRC <= 8 ? 2 : 1);   // vectors in flight per thread and source
#pragma unroll
    for (int u0 = 0; u0 < 4; u0 += UB) {
      f32x4 v[UB][NSRC];
#pragma unroll
      for (int s = 0; s < NSRC; ++s)
        if (s < count) {
          const float *src = t.src[seg][s];
#pragma unroll
          for (int u = 0; u < UB; ++u) v[u][s] = *reinterpret_cast<const f32x4 *>(src + base + ((u0 + u) * 256 + threadIdx.x) * 4);
        }
#pragma unroll
      for (int u = 0; u < UB; ++u) {
        f32x4 acc = v[u][0];
#pragma unroll
        for (int s = 1; s < NSRC; ++s)
          if (s < count) acc += v[u][s];      // ascending sub-ResNet order
        if (count > 1) {
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[e] = acc[e] / fc;
        }
        // the global model is next read by the partition's copies, long after this kernel: a nontemporal store
        // keeps it from displacing the source lines still to be read (measured 5.0 -> 6.3 TB/s at 419 MB)
        __builtin_nontemporal_store(acc, reinterpret_cast<f32x4 *>(dst + base + ((u0 + u) * 256 + threadIdx.x) * 4));
      }
    }
    return;
  }
  // ragged last chunk of a buffer
  for (int u = 0; u < 4; ++u) {
    const long long i = base + (u * 256 + threadIdx.x) * 4;
    for (long long k = i; k < i + 4 && k < n; ++k) {
      float acc = t.src[seg][0][k];
      if (count > 1) {
        for (int s = 1; s < count; ++s) acc += t.src[seg][s][k];
        acc = acc / fc;
      }
      dst[k] = acc;
    }
  }
}

__global__ __launch_bounds__(256) void fill_zero_kernel(float *p, long long n) {
  const long long stride = (long long)gridDim.x * blockDim.x;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = 0.f;
}

}  // namespace

int sgd_momentum_f32(const std::vector<SgdSeg> &segs, float lr, float mu, float wd, hipStream_t st) {
  size_t i = 0;
  while (i < segs.size()) {
    SgdTable t{};
    t.lr = lr; t.mu = mu; t.wd = wd;
    int wg = 0;
    while (i < segs.size() && t.nseg < kSgdSegs) {
      const SgdSeg &s = segs[i++];
      if (s.n <= 0) continue;
      t.w[t.nseg] = s.w; t.v[t.nseg] = s.v; t.g[t.nseg] = s.g; t.n[t.nseg] = s.n;
      t.first_wg[t.nseg] = wg;
      wg += (int)((s.n + kChunk - 1) / kChunk);
      ++t.nseg;
    }
    t.first_wg[t.nseg] = wg;
    if (wg == 0) continue;
    double nb = 0;
    for (int k = 0; k < t.nseg; ++k) nb += 20.0 * t.n[k];
    prof::Scope ps("sgd_momentum", 0, nb, st);
    hipLaunchKernelGGL(sgd_kernel, dim3(wg), dim3(256), 0, st, t);
    RESIST_CHECK_LAUNCH("sgd");
  }
  return RESIST_OK;
}

namespace {
template <int NSRC>
int aggregate_launch(const std::vector<AggSeg> &segs, hipStream_t st) {
  size_t i = 0;
  while (i < segs.size()) {
    AggTable<NSRC> t{};
    static_assert(sizeof(t) <= 4096, "kernel argument limit");
    int wg = 0;
    while (i < segs.size() && t.nseg < AggTable<NSRC>::kSegs) {
      const AggSeg &s = segs[i++];
      if (s.n <= 0 || s.count <= 0) continue;
      t.dst[t.nseg] = s.dst;
      for (int k = 0; k < s.count; ++k) t.src[t.nseg][k] = s.src[k];
      t.n[t.nseg] = s.n; t.count[t.nseg] = s.count;
      t.first_wg[t.nseg] = wg;
      wg += (int)((s.n + kChunk - 1) / kChunk);
      ++t.nseg;
    }
    t.first_wg[t.nseg] = wg;
    if (wg == 0) continue;
    double nb = 0;
    for (int k = 0; k < t.nseg; ++k) nb += 4.0 * t.n[k] * (t.count[k] + 1);
    prof::Scope ps("aggregate", 0, nb, st);
    hipLaunchKernelGGL(aggregate_kernel<NSRC>, dim3(wg), dim3(256), 0, st, t);
    RESIST_CHECK_LAUNCH("aggregate");
  }
  return RESIST_OK;
}
}  // namespace

int aggregate_f32(const std::vector<AggSeg> &segs, hipStream_t st) {
  int most = 0;
  for (const AggSeg &s : segs) most = s.count > most ? s.count : most;
  if (most > kAggSrc) return set_error(RESIST_EUNSUPPORTED, "a block is held by %d sub-ResNets; at most %d supported", most, kAggSrc);
  if (most <= 4) return aggregate_launch<4>(segs, st);
  if (most <= 8) return aggregate_launch<8>(segs, st);
  return aggregate_launch<16>(segs, st);
}

int fill_zero_f32(float *p, int64_t n, hipStream_t st) {
  if (n <= 0) return RESIST_OK;
  long long wg = (n + 1023) / 1024;
  if (wg > 4096) wg = 4096;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)wg), dim3(256), 0, st, p, (long long)n);
  RESIST_CHECK_LAUNCH("fill_zero");
  return RESIST_OK;
}

}  // namespace resist
