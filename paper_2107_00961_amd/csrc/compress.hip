// b-bit compression of the parameters a worker sends back, and reassembly of the global model
// straight from the compressed copies (appendix on quantised communication, Table 9; reassembly:
// Sec. 2.3).  The paper names no quantiser; this is the uniform min-max one, per tensor of a block:
//   lo = min w, hi = max w, delta = (hi - lo) / (2^b - 1), code = rint((w - lo) / delta),
//   decoded value lo + code * delta, all in fp32.
// A compressed block is a header of one record {lo, delta, begin, end} per tensor plus one code per
// float of the block buffer (a byte each for b > 4, a nibble each for b <= 4).  All kernels stream
// through HBM once; the reassembly kernel reads b-bit codes instead of fp32 copies and decodes them
// on the fly, so its traffic per parameter drops from 4*(count+1) to count*(1 or 1/2) + 4 bytes.
#include "internal.h"

namespace resist {

typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kChunk = 4096;  // floats per workgroup (256 threads x 4 vectors of 4)
constexpr int kMaxT = 24;     // most tensors in one block buffer (bottleneck block with shortcut: 20)
constexpr int kQSegs = 16;    // blocks per launch of the compression kernels
constexpr int kSub = 8;       // chunks one workgroup of the min/max kernel walks

struct QRange { float lo, delta; int begin, end; };
static_assert(sizeof(QRange) == sizeof(resist_qrange), "header record layout");

// order-preserving map float -> int, so that integer atomic min / max order floats
__device__ inline int f2ord(float f) {
  const int b = __float_as_int(f);
  return b >= 0 ? b : b ^ 0x7fffffff;
}
__device__ inline float ord2f(int o) { return __int_as_float(o >= 0 ? o : o ^ 0x7fffffff); }

struct QuantTable {
  const float *src[kQSegs];
  unsigned char *codes[kQSegs];
  QRange *ranges[kQSegs];
  int n[kQSegs];
  int nt[kQSegs];
  int begin[kQSegs][kMaxT];
  int end[kQSegs][kMaxT];
  int first_wg[kQSegs + 1];      // encode kernel: one workgroup per chunk
  int first_wg_mm[kQSegs + 1];   // min/max kernel: one workgroup per kSub chunks
  int nseg;
  int levels;   // 2^b - 1
  int nibble;   // two codes per byte
};
static_assert(sizeof(QuantTable) <= 4096, "kernel argument limit");

// Segment of this workgroup: first_wg is ascending, so the segment index is the number of segment
// starts at or below blockIdx.x.  One lane per candidate and a ballot: a single round trip to the
// kernel arguments instead of a chain of dependent loads.  nseg <= 64.
__device__ inline int find_seg(const int *first_wg, int nseg) {
  const int lane = threadIdx.x & 63;
  const bool past = lane + 1 < nseg && (int)blockIdx.x >= first_wg[lane + 1];
  return __popcll(__ballot(past));
}

// header records with the running minimum / maximum in their order-preserving integer form
__global__ __launch_bounds__(64) void quant_init_kernel(QuantTable t) {
  const int seg = blockIdx.x, j = threadIdx.x;
  if (j >= t.nt[seg]) return;
  int *rec = reinterpret_cast<int *>(t.ranges[seg] + j);
  rec[0] = f2ord(__int_as_float(0x7f800000));   // +inf
  rec[1] = f2ord(__int_as_float(0xff800000));   // -inf
  rec[2] = t.begin[seg][j];
  rec[3] = t.end[seg][j];
}

// Minimum and maximum of every tensor.  A workgroup walks kSub consecutive chunks and keeps
// per-thread running values as long as the chunks lie inside one tensor, so that a large tensor
// receives one pair of atomics per kSub chunks: device-wide atomics on one address execute one after
// the other at the memory side, and a pair per chunk made them the bottleneck of this kernel.

__global__ __launch_bounds__(256) void quant_minmax_kernel(QuantTable t) {
  __shared__ float red[2][4];
  const int seg = find_seg(t.first_wg_mm, t.nseg);
  const int wg_base = (blockIdx.x - t.first_wg_mm[seg]) * (kChunk * kSub);
  const float *src = t.src[seg];
  const int n = t.n[seg];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nt = t.nt[seg];
  int my_b = 0, my_e = 0;   // lane j holds the bounds of tensor j
  if (lane < nt) { my_b = t.begin[seg][lane]; my_e = t.end[seg][lane]; }
  const float inf = __int_as_float(0x7f800000);

  // workgroup reduction of (mn, mx) and one pair of atomics on the record of tensor tt
  auto publish = [&](int tt, float mn, float mx) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      mn = fminf(mn, __shfl_xor(mn, o));
      mx = fmaxf(mx, __shfl_xor(mx, o));
    }
    if (lane == 0) { red[0][wave] = mn; red[1][wave] = mx; }
    __syncthreads();
    if (threadIdx.x == 0) {
      mn = fminf(fminf(red[0][0], red[0][1]), fminf(red[0][2], red[0][3]));
      mx = fmaxf(fmaxf(red[1][0], red[1][1]), fmaxf(red[1][2], red[1][3]));
      int *rec = reinterpret_cast<int *>(t.ranges[seg] + tt);
      atomicMin(rec + 0, f2ord(mn));
      atomicMax(rec + 1, f2ord(mx));
    }
    __syncthreads();
  };
  auto load_chunk = [&](int base, float (&v)[4][4]) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = base + (u * 256 + threadIdx.x) * 4;
      if (i + 3 < n) {
        const f32x4 x = *reinterpret_cast<const f32x4 *>(src + i);
        v[u][0] = x[0]; v[u][1] = x[1]; v[u][2] = x[2]; v[u][3] = x[3];
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[u][e] = (i + e < n) ? src[i + e] : 0.f;
      }
    }
  };

  int cur = -1;              // tensor the running values belong to (the same in every thread)
  float run_mn = inf, run_mx = -inf;
  float v[4][4], vn[4][4];
  load_chunk(wg_base, v);
  for (int c = 0; c < kSub; ++c) {
    const int base = wg_base + c * kChunk;
    if (base >= n) break;
    if (c + 1 < kSub && base + kChunk < n) load_chunk(base + kChunk, vn);   // next chunk in flight meanwhile
    unsigned long long todo = __ballot(lane < nt && my_e > base && my_b < base + kChunk);
    const int first = __ffsll((long long)todo) - 1;
    const bool whole = first >= 0 && (todo & (todo - 1)) == 0 && __shfl(my_b, first) <= base &&
                       __shfl(my_e, first) >= base + kChunk;
    if (whole) {               // the usual case: the chunk lies inside one tensor
      if (first != cur) {
        if (cur >= 0) publish(cur, run_mn, run_mx);
        cur = first; run_mn = inf; run_mx = -inf;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e) { run_mn = fminf(run_mn, v[u][e]); run_mx = fmaxf(run_mx, v[u][e]); }
    } else {
      if (cur >= 0) { publish(cur, run_mn, run_mx); cur = -1; }
      while (todo) {
        const int tt = __ffsll((long long)todo) - 1;
        todo &= todo - 1;
        const int b = __shfl(my_b, tt), en = __shfl(my_e, tt);
        float mn = inf, mx = -inf;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int i = base + (u * 256 + threadIdx.x) * 4;
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (i + e >= b && i + e < en) { mn = fminf(mn, v[u][e]); mx = fmaxf(mx, v[u][e]); }
        }
        publish(tt, mn, mx);
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int e = 0; e < 4; ++e) v[u][e] = vn[u][e];
  }
  if (cur >= 0) publish(cur, run_mn, run_mx);
}

__global__ __launch_bounds__(256) void quant_encode_kernel(QuantTable t) {
  __shared__ float s_lo[kMaxT], s_delta[kMaxT];
  __shared__ int s_begin[kMaxT], s_end[kMaxT];
  const int seg = find_seg(t.first_wg, t.nseg);
  const int base = (blockIdx.x - t.first_wg[seg]) * kChunk;
  const float *src = t.src[seg];
  unsigned char *codes = t.codes[seg];
  const int n = t.n[seg], nt = t.nt[seg];
  const float levels = (float)t.levels;
  if ((int)threadIdx.x < nt) {
    const int *rec = reinterpret_cast<const int *>(t.ranges[seg] + threadIdx.x);
    const float lo = ord2f(rec[0]), hi = ord2f(rec[1]);
    s_lo[threadIdx.x] = lo;
    s_delta[threadIdx.x] = (hi - lo) / levels;
    s_begin[threadIdx.x] = rec[2];
    s_end[threadIdx.x] = rec[3];
  }
  __syncthreads();
  int tt = 0;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int i = base + (u * 256 + threadIdx.x) * 4;
    if (i >= n) break;
    float x[4];
    if (i + 3 < n) {
      const f32x4 xv = *reinterpret_cast<const f32x4 *>(src + i);
      x[0] = xv[0]; x[1] = xv[1]; x[2] = xv[2]; x[3] = xv[3];
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) x[e] = (i + e < n) ? src[i + e] : 0.f;
    }
    // tensors start at multiples of 4 floats: the vector lies in one tensor or in the padding behind it
    while (tt + 1 < nt && i >= s_begin[tt + 1]) ++tt;
    const int live = min(s_end[tt], n) - i;
    const float lo = s_lo[tt], d = s_delta[tt];
    unsigned c[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      c[e] = 0;
      if (e < live && d != 0.f) {
        float q = rintf((x[e] - lo) / d);
        q = fminf(fmaxf(q, 0.f), levels);
        c[e] = (unsigned)q;
      }
    }
    if (t.nibble) {
      if (i + 3 < n) {
        *reinterpret_cast<unsigned short *>(codes + (i >> 1)) = (unsigned short)(c[0] | (c[1] << 4) | (c[2] << 8) | (c[3] << 12));
      } else {
        codes[i >> 1] = (unsigned char)(c[0] | (c[1] << 4));   // elements past n were given code 0
        if (i + 2 < n) codes[(i >> 1) + 1] = (unsigned char)(c[2] | (c[3] << 4));
      }
    } else {
      if (i + 3 < n) {
        *reinterpret_cast<unsigned *>(codes + i) = c[0] | (c[1] << 8) | (c[2] << 16) | (c[3] << 24);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (i + e < n) codes[i + e] = (unsigned char)c[e];
      }
    }
  }
}

// header records into their final form {lo, delta, begin, end}
__global__ __launch_bounds__(64) void quant_finish_kernel(QuantTable t) {
  const int seg = blockIdx.x, j = threadIdx.x;
  if (j >= t.nt[seg]) return;
  int *rec = reinterpret_cast<int *>(t.ranges[seg] + j);
  const float lo = ord2f(rec[0]), hi = ord2f(rec[1]);
  reinterpret_cast<float *>(rec)[0] = lo;
  reinterpret_cast<float *>(rec)[1] = (hi - lo) / (float)t.levels;
}

// ---- reassembly from compressed copies ------------------------------------------------------
template <int NSRC> struct QAggTable {
  static constexpr int kSegs = NSRC <= 4 ? 40 : (NSRC <= 8 ? 24 : 12);
  float *dst[kSegs];
  const unsigned char *codes[kSegs][NSRC];
  const QRange *ranges[kSegs][NSRC];
  int n[kSegs];
  int nt[kSegs];
  int count[kSegs];
  int first_wg[kSegs + 1];
  int nseg;
  int nibble;
};

// One chunk of kChunk floats.  FULL: the chunk ends at or before n, so every access is a whole
// vector and the only branches left are uniform ones (source s present or not): all loads of the
// workgroup are issued back to back.  The ragged last chunk of a buffer takes the general path.
template <int NSRC, bool FULL, bool NIB>
__device__ __forceinline__ void aggregate_compressed_chunk(const QAggTable<NSRC> &t, int seg, int base, int n, int nt,
                                                           int count, float2 (*s_par)[kMaxT], int *s_begin, int *s_end) {
  float *dst = t.dst[seg];
  constexpr bool nib = NIB;
  const int j = threadIdx.x;
  // header records (thread j < nt: record j of every source) and code words are requested together:
  // the words do not depend on the header, so one memory round trip covers both
  QRange rec[NSRC];
#pragma unroll
  for (int s = 0; s < NSRC; ++s)
    if (s < count && j < nt) rec[s] = t.ranges[seg][s][j];
  unsigned w[4][NSRC];
#pragma unroll
  for (int s = 0; s < NSRC; ++s) {
    if (s < count) {
      const unsigned char *cp = t.codes[seg][s];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = base + (u * 256 + j) * 4;
        if (FULL) {
          w[u][s] = nib ? (unsigned)*reinterpret_cast<const unsigned short *>(cp + (i >> 1))
                        : *reinterpret_cast<const unsigned *>(cp + i);
        } else {
          w[u][s] = 0;
          if (i + 3 < n) {
            w[u][s] = nib ? (unsigned)*reinterpret_cast<const unsigned short *>(cp + (i >> 1))
                          : *reinterpret_cast<const unsigned *>(cp + i);
          } else if (i < n) {
            if (nib) {
              w[u][s] = cp[i >> 1] | (i + 2 < n ? (unsigned)cp[(i >> 1) + 1] << 8 : 0u);
            } else {
              for (int e = 0; e < 4; ++e)
                if (i + e < n) w[u][s] |= (unsigned)cp[i + e] << (8 * e);
            }
          }
        }
      }
    }
  }
#pragma unroll
  for (int s = 0; s < NSRC; ++s)
    if (s < count && j < nt) {
      s_par[s][j] = make_float2(rec[s].lo, rec[s].delta);
      if (s == 0) { s_begin[j] = rec[0].begin; s_end[j] = rec[0].end; }
    }
  __syncthreads();
  const float inv = 1.f / (float)count;
  int tt = 0;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int i = base + (u * 256 + j) * 4;
    if (FULL || i < n) {
      // tensors start at multiples of 4 floats: the vector lies in one tensor or in the padding behind it
      while (tt + 1 < nt && i >= s_begin[tt + 1]) ++tt;
      const int live = min(s_end[tt], n) - i;
      float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < NSRC; ++s) {
        if (s < count) {
          const float2 par = s_par[s][tt];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const unsigned c = nib ? (w[u][s] >> (4 * e)) & 15u : (w[u][s] >> (8 * e)) & 255u;
            const float d = fmaf((float)c, par.y, par.x);
            acc[e] = s == 0 ? d : acc[e] + d;
          }
        }
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if (count > 1) acc[e] = acc[e] * inv;
        if (e >= live) acc[e] = 0.f;   // alignment padding between tensors
      }
      if (FULL || i + 3 < n) {
        f32x4 o = {acc[0], acc[1], acc[2], acc[3]};
        __builtin_nontemporal_store(o, reinterpret_cast<f32x4 *>(dst + i));   // as in aggregate_kernel: 5.15 -> 5.4 TB/s
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (i + e < n) dst[i + e] = acc[e];
      }
    }
  }
}

template <int NSRC>
__global__ __launch_bounds__(256) void aggregate_compressed_kernel(QAggTable<NSRC> t) {
  __shared__ float2 s_par[NSRC][kMaxT];   // (lo, delta)
  __shared__ int s_begin[kMaxT], s_end[kMaxT];
  // the segment index is the same in every lane; telling the compiler so keeps the table lookups scalar
  const int seg = __builtin_amdgcn_readfirstlane(find_seg(t.first_wg, t.nseg));
  const int base = (blockIdx.x - t.first_wg[seg]) * kChunk;
  const int n = t.n[seg], nt = t.nt[seg], count = t.count[seg];
  if (t.nibble) {
    if (base + kChunk <= n) aggregate_compressed_chunk<NSRC, true, true>(t, seg, base, n, nt, count, s_par, s_begin, s_end);
    else aggregate_compressed_chunk<NSRC, false, true>(t, seg, base, n, nt, count, s_par, s_begin, s_end);
  } else {
    if (base + kChunk <= n) aggregate_compressed_chunk<NSRC, true, false>(t, seg, base, n, nt, count, s_par, s_begin, s_end);
    else aggregate_compressed_chunk<NSRC, false, false>(t, seg, base, n, nt, count, s_par, s_begin, s_end);
  }
}

struct QAggSeg {
  float *dst;
  const unsigned char *codes[16];
  const QRange *ranges[16];
  int count, nt;
  int64_t n;
};

template <int NSRC>
int aggregate_compressed_launch(const std::vector<QAggSeg> &segs, int nibble, hipStream_t st) {
  size_t i = 0;
  while (i < segs.size()) {
    QAggTable<NSRC> t{};
    static_assert(sizeof(t) <= 4096, "kernel argument limit");
    t.nibble = nibble;
    int wg = 0;
    double nb = 0;
    while (i < segs.size() && t.nseg < QAggTable<NSRC>::kSegs) {
      const QAggSeg &s = segs[i++];
      if (s.n <= 0 || s.count <= 0) continue;
      t.dst[t.nseg] = s.dst;
      for (int k = 0; k < s.count; ++k) { t.codes[t.nseg][k] = s.codes[k]; t.ranges[t.nseg][k] = s.ranges[k]; }
      t.n[t.nseg] = (int)s.n; t.nt[t.nseg] = s.nt; t.count[t.nseg] = s.count;
      t.first_wg[t.nseg] = wg;
      wg += (int)((s.n + kChunk - 1) / kChunk);
      nb += (double)s.n * (4.0 + s.count * (nibble ? 0.5 : 1.0)) + 16.0 * s.nt * s.count;
      ++t.nseg;
    }
    t.first_wg[t.nseg] = wg;
    if (wg == 0) continue;
    prof::Scope ps("aggregate_compressed", 0, nb, st);
    hipLaunchKernelGGL(aggregate_compressed_kernel<NSRC>, dim3(wg), dim3(256), 0, st, t);
    RESIST_CHECK_LAUNCH("aggregate_compressed");
  }
  return RESIST_OK;
}

int check_bits(int bits) {
  if (bits < 2 || bits > 8) return set_error(RESIST_EINVAL, "bits=%d: 2..8 supported", bits);
  return RESIST_OK;
}

// tensor ranges of a block buffer, in floats
int tensor_ranges(const Net &net, int key, std::vector<int> *begin, std::vector<int> *end, int64_t *n_total) {
  BlockLayout L;
  RESIST_TRY(block_layout(net, key, &L));
  if ((int)L.slots.size() > kMaxT) return set_error(RESIST_EUNSUPPORTED, "block %d has %d tensors; at most %d", key, (int)L.slots.size(), kMaxT);
  if (L.n_total >= (1LL << 31)) return set_error(RESIST_EUNSUPPORTED, "block %d has 2^31 or more parameters", key);
  begin->clear(); end->clear();
  for (const TensorSlot &s : L.slots) {
    if (s.offset % 4) return set_error(RESIST_EUNSUPPORTED, "block %d: a tensor does not start at a multiple of 4 floats", key);
    begin->push_back((int)s.offset);
    end->push_back((int)(s.offset + s.count));
  }
  *n_total = L.n_total;
  return RESIST_OK;
}

}  // namespace

extern "C" int resist_compressed_block_size(const resist_model_desc *desc, int32_t block, int32_t bits,
                                            int64_t *code_bytes, int32_t *n_tensors) {
  Net net;
  RESIST_TRY(build_net(desc, &net));
  RESIST_TRY(check_bits(bits));
  std::vector<int> b, e;
  int64_t n = 0;
  RESIST_TRY(tensor_ranges(net, block, &b, &e, &n));
  if (code_bytes) *code_bytes = bits <= 4 ? (n + 1) / 2 : n;
  if (n_tensors) *n_tensors = (int32_t)b.size();
  return RESIST_OK;
}

extern "C" int resist_compress_blocks(const resist_model_desc *desc, int32_t nkeys, const int32_t *keys, int32_t bits,
                                      void *const *params, void *const *codes, void *const *ranges, void *hip_stream) {
  Net net;
  RESIST_TRY(build_net(desc, &net));
  RESIST_TRY(check_bits(bits));
  if (nkeys < 0 || (nkeys > 0 && (!keys || !params || !codes || !ranges))) return set_error(RESIST_EINVAL, "NULL argument or nkeys < 0");
  hipStream_t st = (hipStream_t)hip_stream;
  for (int i = 0; i < nkeys; ++i) {
    if (!params[i] || !codes[i] || !ranges[i]) return set_error(RESIST_EINVAL, "entry %d: NULL buffer", i);
    if (((uintptr_t)params[i] | (uintptr_t)ranges[i]) % 16 || (uintptr_t)codes[i] % 4)
      return set_error(RESIST_EINVAL, "entry %d: params and ranges must be 16-byte aligned, codes 4-byte aligned", i);
  }
  int i = 0;
  while (i < nkeys) {
    QuantTable t{};
    t.levels = (1 << bits) - 1;
    t.nibble = bits <= 4;
    int wg = 0, wg_mm = 0;
    double nb = 0;
    for (; i < nkeys && t.nseg < kQSegs; ++i) {
      std::vector<int> b, e;
      int64_t n = 0;
      RESIST_TRY(tensor_ranges(net, keys[i], &b, &e, &n));
      const int k = t.nseg++;
      t.src[k] = (const float *)params[i];
      t.codes[k] = (unsigned char *)codes[i];
      t.ranges[k] = (QRange *)ranges[i];
      t.n[k] = (int)n;
      t.nt[k] = (int)b.size();
      for (size_t j = 0; j < b.size(); ++j) { t.begin[k][j] = b[j]; t.end[k][j] = e[j]; }
      t.first_wg[k] = wg;
      wg += (int)((n + kChunk - 1) / kChunk);
      t.first_wg_mm[k] = wg_mm;
      wg_mm += (int)((n + kChunk * kSub - 1) / (kChunk * kSub));
      nb += (double)n;
    }
    t.first_wg[t.nseg] = wg;
    t.first_wg_mm[t.nseg] = wg_mm;
    if (wg == 0) continue;
    {
      prof::Scope ps("compress_header", 0, 32.0 * kMaxT * t.nseg, st);
      hipLaunchKernelGGL(quant_init_kernel, dim3(t.nseg), dim3(64), 0, st, t);
      RESIST_CHECK_LAUNCH("quant_init");
    }
    {
      prof::Scope ps("compress_minmax", 0, 4.0 * nb, st);
      hipLaunchKernelGGL(quant_minmax_kernel, dim3(wg_mm), dim3(256), 0, st, t);
      RESIST_CHECK_LAUNCH("quant_minmax");
    }
    {
      prof::Scope ps("compress_encode", 0, (4.0 + (t.nibble ? 0.5 : 1.0)) * nb, st);
      hipLaunchKernelGGL(quant_encode_kernel, dim3(wg), dim3(256), 0, st, t);
      RESIST_CHECK_LAUNCH("quant_encode");
    }
    {
      prof::Scope ps("compress_header", 0, 32.0 * kMaxT * t.nseg, st);
      hipLaunchKernelGGL(quant_finish_kernel, dim3(t.nseg), dim3(64), 0, st, t);
      RESIST_CHECK_LAUNCH("quant_finish");
    }
  }
  return RESIST_OK;
}

extern "C" int resist_decompress_blocks(const resist_model_desc *desc, int32_t nkeys, const int32_t *keys, int32_t bits,
                                        void *const *codes, void *const *ranges, void *const *params, void *hip_stream) {
  Net net;
  RESIST_TRY(build_net(desc, &net));
  RESIST_TRY(check_bits(bits));
  if (nkeys < 0 || (nkeys > 0 && (!keys || !params || !codes || !ranges))) return set_error(RESIST_EINVAL, "NULL argument or nkeys < 0");
  std::vector<QAggSeg> segs((size_t)nkeys);
  for (int i = 0; i < nkeys; ++i) {
    if (!params[i] || !codes[i] || !ranges[i]) return set_error(RESIST_EINVAL, "entry %d: NULL buffer", i);
    if (((uintptr_t)params[i] | (uintptr_t)ranges[i]) % 16 || (uintptr_t)codes[i] % 4)
      return set_error(RESIST_EINVAL, "entry %d: params and ranges must be 16-byte aligned, codes 4-byte aligned", i);
    std::vector<int> b, e;
    int64_t n = 0;
    RESIST_TRY(tensor_ranges(net, keys[i], &b, &e, &n));
    QAggSeg &g = segs[i];
    g.dst = (float *)params[i];
    g.codes[0] = (const unsigned char *)codes[i];
    g.ranges[0] = (const QRange *)ranges[i];
    g.count = 1;
    g.nt = (int)b.size();
    g.n = n;
  }
  return aggregate_compressed_launch<4>(segs, bits <= 4, (hipStream_t)hip_stream);   // one source per block: a plain decode
}

extern "C" int resist_aggregate_compressed(const resist_model_desc *desc, int32_t S, const int32_t *sub_offsets,
                                           const int32_t *sub_blocks, int32_t bits, void *const *const *sub_codes,
                                           void *const *const *sub_ranges, void *const *global_block_params,
                                           void *hip_stream) {
  Net net;
  RESIST_TRY(build_net(desc, &net));
  RESIST_TRY(check_bits(bits));
  const int B = (int)net.blocks.size();
  if (S < 1 || !sub_offsets || !sub_blocks || !sub_codes || !sub_ranges || !global_block_params)
    return set_error(RESIST_EINVAL, "NULL argument or S < 1");
  if (S > 16) return set_error(RESIST_EUNSUPPORTED, "S=%d: at most 16 sub-ResNets supported", S);
  std::vector<QAggSeg> segs(B + 2);
  for (int key = -1; key <= B; ++key) {
    std::vector<int> b, e;
    int64_t n = 0;
    RESIST_TRY(tensor_ranges(net, key, &b, &e, &n));
    QAggSeg &g = segs[key + 1];
    g.dst = (float *)global_block_params[key + 1];
    g.count = 0;
    g.n = n;
    g.nt = (int)b.size();
    if (!g.dst) return set_error(RESIST_EINVAL, "global buffer %d is NULL", key + 1);
    if ((uintptr_t)g.dst % 16) return set_error(RESIST_EINVAL, "global buffer %d is not 16-byte aligned", key + 1);
  }
  for (int s = 0; s < S; ++s) {
    const int n_s = sub_offsets[s + 1] - sub_offsets[s];
    if (n_s < 0) return set_error(RESIST_EINVAL, "sub_offsets not ascending");
    if (!sub_codes[s] || !sub_ranges[s]) return set_error(RESIST_EINVAL, "sub_codes[%d] or sub_ranges[%d] is NULL", s, s);
    auto add = [&](int key, const void *c, const void *r) -> int {
      if (!c || !r) return set_error(RESIST_EINVAL, "sub-ResNet %d: compressed buffer for block %d is NULL", s, key);
      if ((uintptr_t)c % 4 || (uintptr_t)r % 16) return set_error(RESIST_EINVAL, "sub-ResNet %d, block %d: codes must be 4-byte and ranges 16-byte aligned", s, key);
      QAggSeg &g = segs[key + 1];
      g.codes[g.count] = (const unsigned char *)c;
      g.ranges[g.count] = (const QRange *)r;
      ++g.count;
      return RESIST_OK;
    };
    RESIST_TRY(add(-1, sub_codes[s][0], sub_ranges[s][0]));
    for (int i = 0; i < n_s; ++i) {
      const int b = sub_blocks[sub_offsets[s] + i];
      if (b < 0 || b >= B) return set_error(RESIST_EINVAL, "sub-ResNet %d holds block %d outside [0,%d)", s, b, B);
      if (i > 0 && b <= sub_blocks[sub_offsets[s] + i - 1]) return set_error(RESIST_EINVAL, "sub-ResNet %d: blocks not ascending", s);
      RESIST_TRY(add(b, sub_codes[s][1 + i], sub_ranges[s][1 + i]));
    }
    RESIST_TRY(add(B, sub_codes[s][1 + n_s], sub_ranges[s][1 + n_s]));
  }
  int most = 0;
  for (const QAggSeg &g : segs) most = g.count > most ? g.count : most;
  hipStream_t st = (hipStream_t)hip_stream;
  const int nibble = bits <= 4;
  if (most <= 4) return aggregate_compressed_launch<4>(segs, nibble, st);
  if (most <= 8) return aggregate_compressed_launch<8>(segs, nibble, st);
  return aggregate_compressed_launch<16>(segs, nibble, st);
}

}  // namespace resist
