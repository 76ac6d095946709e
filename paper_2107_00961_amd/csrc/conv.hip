// Implicit-GEMM convolutions on the CDNA4 matrix cores: fp32 (v_mfma_f32_32x32x2_f32) and
// bf16 operands with fp32 accumulation (v_mfma_f32_32x32x16_bf16).
//
// The convolutions of a residual block (the paper's local update, Algorithm 1 inner loop, is an
// ordinary SGD step of the blocks a worker keeps) are computed as GEMMs whose A operand is
// gathered on the fly from the NHWC activation tensor:
//   forward  Y[m=(n,p,q)][k]  = sum_{r,s,c} X[n, p*st+r-pad, q*st+s-pad, c] * W[k][r][s][c]
//   dgrad    dX[m=(n,h,w)][c] = sum_{r,s,k} dY[n, (h+pad-r)/st, (w+pad-s)/st, k] * WT[c][r][s][k]
//            (terms with a non-integer or out-of-range source pixel vanish; for stride 2 the output
//             pixels are processed one parity class at a time so that no such term is ever issued)
//   wgrad    dW[k][r][s][c]   = sum_{m=(n,p,q)} dY[m][k] * X[n, p*st+r-pad, q*st+s-pad, c]
// Tiles are staged through LDS (double buffered, one barrier per K-chunk); every wave owns a
// grid of 32x32 accumulator tiles held in registers.
#include <mutex>
#include <type_traits>

#include "elem.h"
#include "internal.h"

namespace resist {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

namespace {

constexpr int kThreads = 256;
#ifndef RESIST_BF16_GLOBAL_DEPTH
#define RESIST_BF16_GLOBAL_DEPTH 2   // chunks an eight-wave bf16 workgroup requests ahead of their use (1..3)
#endif
#ifndef RESIST_BF16_FRAG_DEPTH
#define RESIST_BF16_FRAG_DEPTH 1   // k-steps a bf16 fragment is fetched ahead of its MFMAs (1..3)
#endif
constexpr int kStages = 2;     // LDS double buffering in the implicit-GEMM kernels

// Element traits: a 16-byte vector holds VEC elements; one pair of 16-byte fragments (A, B) feeds
// the matrix core with 2*VEC values of the GEMM-K axis (lane group l/32 owns VEC consecutive ones).
template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int VEC = 4;
  __device__ static inline void mma(f32x16 &acc, const f32x4 &a, const f32x4 &b) {
#pragma unroll
    for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[e], b[e], acc, 0, 0, 0);
  }
  __device__ static inline float from_f32(float v) { return v; }
  __device__ static inline float to_f32(float v) { return v; }
};
template <> struct Elem<__bf16> {
  static constexpr int VEC = 8;
  __device__ static inline void mma(f32x16 &acc, const f32x4 &a, const f32x4 &b) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
  }
  __device__ static inline __bf16 from_f32(float v) { return (__bf16)v; }   // round to nearest even
  __device__ static inline float to_f32(__bf16 v) { return (float)v; }
};

// division by a runtime constant: q = (n * mul) >> sh, exact for 0 <= n < 2^31
struct FastDiv { unsigned mul; int sh; };
inline FastDiv make_fastdiv(unsigned d) {
  int L = 0;
  while ((1ull << L) < d) ++L;
  FastDiv f;
  f.sh = 31 + L;
  f.mul = (unsigned)((1ull << f.sh) / d + 1);
  return f;
}
__device__ inline int fdiv(int n, FastDiv f) { return (int)(((unsigned long long)(unsigned)n * f.mul) >> f.sh); }

struct IgemmArgs {
  const void *in;      // [N][IH][IW][IC]
  const void *wt;      // [OC][R][S][IC]
  void *out;           // [N][OH][OW][OC]
  const void *addend;  // optional, indexed like out
  const void *relu_mask;   // optional, indexed like out: out is zeroed where this is not positive (after the addend)
  float *stats;        // optional [3][tiles_m][OC]: per row tile and column a shift k, sum(out - k), sum((out - k)^2)
  // optional (data gradient, cls == 1): first pass of the backward of the BN whose output this
  // convolution read.  out is that BN's output gradient g; with its input bn_y (indexed like out) and
  // xhat = (bn_y - mean) * invstd the kernel leaves, per row tile and column, sum(gm) and sum(gm * xhat) in
  // bn_sums [2][tiles_m][OC], where gm = g, or g where scale * bn_y + shift > 0 and 0 elsewhere (bn_self)
  const void *bn_y;
  const float *bn_mean, *bn_invstd, *bn_scale, *bn_shift;
  float *bn_sums;
  int bn_self;
  int N, IH, IW, IC;
  int OH, OW, OC;
  int R, S, stride, pad;
  int cls;              // 1, or 2 when output pixels are split into 2x2 parity classes
  int OHc, OWc;         // OH/cls, OW/cls
  int Mrows;            // N*OHc*OWc: GEMM rows per class
  int tiles_m, tiles_n;
  FastDiv div_plane, div_w, div_tn, div_tm;   // by OHc*OWc, OWc, tiles_n, tiles_m: a tile's prologue is a chain of divisions
};

// A-gather modes
constexpr int kFwd = 0;  // source pixel = out*stride + tap - pad
constexpr int kBwd = 1;  // source pixel = (out + pad - tap) / stride

// Workgroups are handed to the 8 XCDs round-robin by their linear id, and each XCD has its own L2.
// This maps the hardware id to a logical tile index such that every XCD works on one contiguous
// range of logical tiles, so tiles that share operand rows meet in the same L2.
__device__ inline int xcd_contiguous(int hw_id, int total) {
  const int xcd = hw_id & 7, slot = hw_id >> 3;
  const int base = total >> 3, rem = total & 7;
  return xcd * base + (xcd < rem ? xcd : rem) + slot;
}

// Raw buffer descriptor over a tensor: loads whose byte offset is >= `bytes` return zero without
// touching memory, which is how padding pixels, ragged tile rows and channel tails are filled.
__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void *p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}
constexpr unsigned kOOB = 0x80000000u;   // every tensor is smaller than 2 GiB (checked on the host)

__device__ inline f32x4 buffer_load_16B(__amdgpu_buffer_rsrc_t r, unsigned voff) {
  return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, 0, 0));
}

// BK: K-chunk (elements) staged per step; LDS rows are padded by 16 bytes (conflict-free b128 reads).
//
// The K loop runs over (filter tap, channel chunk).  Its body is one straight-line block: the
// source pixel of every tile row is (hc + dh, wc + dw) with per-row (hc, wc) fixed for the whole
// kernel and per-tap scalars (dh, dw) kept in scalar registers, loads are hardware-bounds-checked
// buffer loads (an invalid element is requested at an out-of-range offset and comes back as zero),
// and the tap counters are advanced with selects.  With no branch in the loop the scheduler is free
// to place the address arithmetic, the LDS traffic and the global loads in the shadow of the MFMAs.
template <typename T, int BM, int BN, int BK, int WGM, int WGN, int MODE>
__global__ __launch_bounds__(WGM * WGN * 64) void igemm_kernel(IgemmArgs a) {
  using E = Elem<T>;
  constexpr int NT = WGM * WGN * 64;             // threads: one wave per wave tile, 4 or 8 waves
  constexpr int VEC = E::VEC;
  constexpr int ES = (int)sizeof(T);
  constexpr int LDK = BK + VEC;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;  // wave tile
  constexpr int TM = WTM / 32, TN = WTN / 32;    // 32x32 MFMA tiles per wave
  constexpr int KV = BK / VEC;                   // lanes per tile row (16 bytes each)
  constexpr int RPP = NT / KV;             // tile rows per load pass
  constexpr int PA = BM / RPP, PB = BN / RPP;    // load passes
  constexpr int NK = BK / (2 * VEC);             // k-steps per chunk
  static_assert((WGM * WGN == 4 || WGM * WGN == 8) && TM >= 1 && TN >= 1 && PA >= 1 && PB >= 1 && NK >= 2, "tile shape");
  // one LDS block: the operand stages during the K loop, the fp32 output tile afterwards
  constexpr int LDC = BN + 8;   // output tile pitch (floats): lanes l and l+32 (4 rows apart) hit disjoint banks
  constexpr size_t kOperandBytes = sizeof(T) * kStages * (BM + BN) * LDK;
  constexpr size_t kTileBytes = sizeof(float) * BM * LDC;
  static_assert(kTileBytes <= kOperandBytes, "output tile must fit in the operand stages");
  __shared__ __attribute__((aligned(16))) char lds_raw[kOperandBytes];
  T (*As)[BM][LDK] = reinterpret_cast<T (*)[BM][LDK]>(lds_raw);
  T (*Bs)[BN][LDK] = reinterpret_cast<T (*)[BN][LDK]>(lds_raw + sizeof(T) * kStages * BM * LDK);
  float (*Cs)[LDC] = reinterpret_cast<float (*)[LDC]>(lds_raw);
  __shared__ int row_off[BM];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;

  // Logical tile order: N-tiles fastest, so tiles sharing input rows are neighbours; each XCD gets a
  // contiguous range of them.  The stride-2 data gradient (4 parity classes of unequal work, class
  // slowest) keeps the hardware round-robin order, which measured faster for its short K loops.
  int bid = a.cls == 1 ? xcd_contiguous(blockIdx.x, gridDim.x) : (int)blockIdx.x;
  const int bq = fdiv(bid, a.div_tn);
  const int tn = bid - bq * a.tiles_n;
  const int cidx = fdiv(bq, a.div_tm);   // parity class
  const int tm = bq - cidx * a.tiles_m;
  const int ph = a.cls == 2 ? cidx >> 1 : 0, pw = a.cls == 2 ? cidx & 1 : 0;   // cls is 1 or 2
  const int m0 = tm * BM, n0 = tn * BN;

  // filter taps that contribute: r = r0, r0+tstep, ... < R (all taps unless MODE==kBwd, stride 2)
  int r0 = 0, s0 = 0, tstep = 1;
  if (MODE == kBwd && a.stride == 2) { r0 = (ph + a.pad) & 1; s0 = (pw + a.pad) & 1; tstep = 2; }
  const int nr = r0 < a.R ? (tstep == 2 ? (a.R - r0 + 1) >> 1 : a.R - r0) : 0;
  const int ns = s0 < a.S ? (tstep == 2 ? (a.S - s0 + 1) >> 1 : a.S - s0) : 0;
  const int cchunks = (a.IC + BK - 1) / BK;
  const int nchunks = nr * ns * cchunks;

  // per-thread tile rows: centre pixel (hc, wc) and byte offset of its first channel of interest
  const int lrow = tid / KV, kvec = (tid % KV) * VEC;
  int hc[PA], wc[PA], aoff[PA], boff[PB];
#pragma unroll
  for (int i = 0; i < PA; ++i) {
    const int m = m0 + i * RPP + lrow;
    if (m < a.Mrows) {
      const int n = fdiv(m, a.div_plane);
      const int rem = m - n * (a.OHc * a.OWc);
      const int ohc = fdiv(rem, a.div_w), owc = rem - ohc * a.OWc;
      if (MODE == kFwd) { hc[i] = ohc * a.stride - a.pad; wc[i] = owc * a.stride - a.pad; }
      else if (a.stride == 1) { hc[i] = ohc + a.pad; wc[i] = owc + a.pad; }
      else { hc[i] = ohc; wc[i] = owc; }
      aoff[i] = (((n * a.IH + hc[i]) * a.IW + wc[i]) * a.IC + kvec) * ES;
    } else {
      hc[i] = -(1 << 24); wc[i] = -(1 << 24); aoff[i] = 0;   // never in range
    }
  }
#pragma unroll
  for (int i = 0; i < PB; ++i) {
    const int oc = n0 + i * RPP + lrow;
    boff[i] = oc < a.OC ? (oc * a.R * a.S * a.IC + kvec) * ES : (int)kOOB;
  }
  for (int r = tid; r < BM; r += NT) {
    const int m = m0 + r;
    int off = -1;
    if (m < a.Mrows) {
      const int n = fdiv(m, a.div_plane);
      const int rem = m - n * (a.OHc * a.OWc);
      const int orow = fdiv(rem, a.div_w);
      const int oh = orow * a.cls + ph, ow = (rem - orow * a.OWc) * a.cls + pw;
      off = (n * a.OH + oh) * a.OW + ow;
    }
    row_off[r] = off;
  }

  const __amdgpu_buffer_rsrc_t rin = make_rsrc(a.in, (unsigned)a.N * a.IH * a.IW * a.IC * ES);
  const __amdgpu_buffer_rsrc_t rwt = make_rsrc(a.wt, (unsigned)a.OC * a.R * a.S * a.IC * ES);

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // loop state of the chunk that will be requested next (uniform across the workgroup)
  int tr = r0, ts = s0, tc = 0, issued = 0;
  // GD = how many chunks ahead of its use an operand chunk is requested from global memory (GD
  // register sets in a ring).  An eight-wave workgroup is alone on its CU, so no other workgroup
  // covers the latency of its loads, and a bf16 chunk is multiplied in less time than a load takes.
  constexpr int GD = (ES == 2 && NT == 512) ? RESIST_BF16_GLOBAL_DEPTH : 1;
  f32x4 ra[GD][PA], rb[GD][PB];
  // scalars of the chunk being requested (set by begin_chunk, used by request)
  int q_dh = 0, q_dw = 0, q_adelta = 0, q_bdelta = 0;
  bool q_kok = false;
  auto begin_chunk = [&]() {
    // tap scalars: source pixel displacement and the byte deltas of activation and filter
    if (MODE == kFwd) { q_dh = tr; q_dw = ts; }
    else if (a.stride == 1) { q_dh = -tr; q_dw = -ts; }
    else { q_dh = (ph + a.pad - tr) >> 1; q_dw = (pw + a.pad - ts) >> 1; }   // even by construction
    const bool live = issued < nchunks;
    const int c0 = tc * BK;
    q_adelta = ((q_dh * a.IW + q_dw) * a.IC + c0) * ES;
    q_bdelta = ((tr * a.S + ts) * a.IC + c0) * ES;
    q_kok = live && (c0 + kvec) < a.IC;
    // advance (tap, channel chunk) without branches
    ++issued;
    const bool cwrap = (tc + 1 == cchunks);
    tc = cwrap ? 0 : tc + 1;
    const bool swrap = cwrap && (ts + tstep >= a.S);
    ts = cwrap ? (swrap ? s0 : ts + tstep) : ts;
    tr = swrap ? tr + tstep : tr;
  };
  // register `part` (0..PA-1: activation rows, PA..PA+PB-1: filter rows) of the chunk begun last
  auto request = [&](int set, int part) {
    if (part < PA) {
      const int i = part;
      const bool ok = q_kok && (unsigned)(hc[i] + q_dh) < (unsigned)a.IH && (unsigned)(wc[i] + q_dw) < (unsigned)a.IW;
      ra[set][i] = buffer_load_16B(rin, ok ? (unsigned)(aoff[i] + q_adelta) : kOOB);
    } else {
      const int i = part - PA;
      rb[set][i] = buffer_load_16B(rwt, q_kok ? (unsigned)(boff[i] + q_bdelta) : kOOB);
    }
  };
  auto store_part = [&](int set, int stage, int part) {
    if (part < PA) *reinterpret_cast<f32x4 *>(&As[stage][part * RPP + lrow][kvec]) = ra[set][part];
    else *reinterpret_cast<f32x4 *>(&Bs[stage][(part - PA) * RPP + lrow][kvec]) = rb[set][part - PA];
  };
  auto load_global = [&](int set) {
    begin_chunk();
#pragma unroll
    for (int p = 0; p < PA + PB; ++p) request(set, p);
  };
  auto store_lds = [&](int set, int stage) {
#pragma unroll
    for (int p = 0; p < PA + PB; ++p) store_part(set, stage, p);
  };

  // Pipeline.  Chunk `it` is multiplied out of LDS stage it&1, one k-step (2*VEC values of K) at a
  // time; the fragments of a k-step are fetched from LDS during the MFMAs of the k-step before it,
  // also across the chunk boundary.  The registers holding chunk it+1 (requested from global memory
  // one chunk of MFMA time earlier) go to the other stage, and chunk it+2 is requested into them,
  // a few registers per k-step over k-steps 0 .. NK-FD-1, so that neither the LDS nor the memory
  // pipeline sees a burst.  The one barrier per chunk sits at the start of the first k-step whose
  // fetch reaches into the next chunk: by then every wave has all fragments of this stage in
  // registers and has written its share of the next stage, so after it the first fragments of chunk
  // it+1 can be fetched while the last MFMAs run.
  // FD = how many k-steps ahead of its MFMAs a fragment is fetched; NB fragment buffers in a ring.
  // The bf16 matrix instruction runs 32 cycles and every MFMA of a 32x32 wave tile depends on the one
  // before it, so one k-step ahead leaves a wave waiting on the LDS for most of each step.
  constexpr int FD = (ES == 2 && NK % 4 == 0) ? RESIST_BF16_FRAG_DEPTH : 1;
  constexpr int NB = FD == 1 ? 2 : 4;
  static_assert(NK % NB == 0 && FD >= 1 && FD < NB && FD < NK, "fragment ring");
  const int lr = lane & 31, lk = (lane >> 5) * VEC;
  f32x4 fa[NB][TM], fb[NB][TN];
  auto load_frags = [&](int buf, int stage, int ks) {
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[buf][i] = *reinterpret_cast<const f32x4 *>(&As[stage][wm * WTM + i * 32 + lr][ks * 2 * VEC + lk]);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[buf][j] = *reinterpret_cast<const f32x4 *>(&Bs[stage][wn * WTN + j * 32 + lr][ks * 2 * VEC + lk]);
  };
  auto lds_barrier = [&]() {
    __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0): this wave's LDS writes and reads are done
    __builtin_amdgcn_s_barrier();
  };

  load_global(0);
  store_lds(0, 0);
#pragma unroll
  for (int c = 1; c <= GD; ++c) load_global(c % GD);   // chunk c waits in register set c % GD
  lds_barrier();
#pragma unroll
  for (int d = 0; d < FD; ++d) load_frags(d, 0, d);
  __builtin_amdgcn_sched_barrier(0);

  // chunk `it`: multiplied out of its stage while chunk it+1 moves from register set `set` to the other
  // stage and chunk it+1+GD is requested into that set
  auto chunk_body = [&](int set, int stage) {
#pragma unroll
    for (int ks = 0; ks < NK; ++ks) {
      const int kn = ks + FD;              // the k-step whose fragments are fetched now
      if (kn < NK) {
        load_frags(kn % NB, stage, kn);
      } else {
        if (kn == NK) lds_barrier();       // once per chunk, at the start of k-step NK-FD
        load_frags(kn % NB, stage ^ 1, kn - NK);   // past the last chunk: zeros nobody uses
      }
      __builtin_amdgcn_sched_barrier(0);   // keep the fetches ahead of this k-step's MFMAs
      if (ks == 0) begin_chunk();
#pragma unroll
      for (int p = 0; p < PA + PB; ++p)
        if ((p * (NK - FD)) / (PA + PB) == ks) {   // parts spread evenly over k-steps 0 .. NK-FD-1
          store_part(set, stage ^ 1, p);
          request(set, p);
        }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) E::mma(acc[i][j], fa[ks % NB][i], fb[ks % NB][j]);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  for (int it = 0; it < nchunks; it += GD) {
#pragma unroll
    for (int j = 0; j < GD; ++j) {
      if (j > 0 && it + j >= nchunks) break;   // uniform across the workgroup
      chunk_body((j + 1) % GD, (it + j) & 1);
    }
  }

  // epilogue.  A lane holds column (lane%32) and rows 8*(e/4) + 4*(lane/32) + e%4 of each 32x32
  // tile.  The tile goes through LDS (the operand stages are free after the last barrier: every
  // fragment a wave uses was fetched before it) so that global memory sees 16-byte accesses along
  // the channel axis; the optional addend is added in fp32 before the one rounding to T.
  T *out = static_cast<T *>(a.out);
  const T *addend = static_cast<const T *>(a.addend);
  constexpr int CV = BN / VEC;            // 16-byte pieces per tile row
  constexpr int RPS = NT / CV;      // rows per pass
  constexpr int NP = BM / RPS;      // passes over the tile
  constexpr int PG = NP < 8 ? NP : 8;   // passes whose side inputs are in flight together
  static_assert(BM % RPS == 0 && CV <= 32 && NP % PG == 0, "output tile rows per pass");
  const int cv = (tid % CV) * VEC, row0 = tid / CV;
  const bool col_ok = n0 + cv < a.OC;     // OC is a multiple of VEC
  const bool bn_bwd = MODE == kBwd && a.bn_sums != nullptr;
  // The side inputs of the epilogue (addend, ReLU mask, BN input: up to three 16-byte loads per thread
  // and pass) are requested for up to eight passes at once, the first group here, before the
  // accumulators even go to LDS: taken one pass at a time, every pass would wait out a memory round
  // trip of its own (a store to `out` may alias the addend, so the compiler cannot move the loads
  // itself).  A thread reads only elements it writes later.
  const T *maskp = static_cast<const T *>(a.relu_mask), *bnyp = static_cast<const T *>(a.bn_y);
  const bool has_mask = MODE == kBwd && a.relu_mask != nullptr;
  typename Vec<T>::Raw q_ad[PG], q_mk[PG], q_y[PG];
  size_t offs[PG];
  bool live[PG];
  auto request_side = [&](int p0) {
#pragma unroll
    for (int g = 0; g < PG; ++g) {
      const int ro = row_off[row0 + (p0 + g) * RPS];
      live[g] = ro >= 0 && col_ok;
      offs[g] = live[g] ? (size_t)ro * a.OC + n0 + cv : 0;
      q_ad[g] = q_mk[g] = q_y[g] = typename Vec<T>::Raw{};
      if (live[g]) {
        if (addend) q_ad[g] = Vec<T>::load_raw(addend + offs[g]);
        if (has_mask) q_mk[g] = Vec<T>::load_raw(maskp + offs[g]);
        if (bn_bwd) q_y[g] = Vec<T>::load_raw(bnyp + offs[g]);
      }
    }
  };
  request_side(0);
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int cl = wn * WTN + j * 32 + lr;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int row = wm * WTM + i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
        Cs[row][cl] = acc[i][j][e];
      }
    }
  __syncthreads();
  // batch-norm statistics of this row tile: column sums of (v - k) and (v - k)^2 of the values v as
  // stored, with the shift k = the tile's first accumulated row of the column.  Any k within a few
  // standard deviations of the column keeps the sum of squares free of the cancellation that
  // sum(v^2) - (sum v)^2/n suffers when |mean| >> std.
  float s1[VEC], s2[VEC], kshift[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) { s1[e] = 0.f; s2[e] = 0.f; kshift[e] = 0.f; }
  float bmu[VEC], bis[VEC], bsc[VEC], bsh[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) { bmu[e] = 0.f; bis[e] = 0.f; bsc[e] = 0.f; bsh[e] = 0.f; }
  if (bn_bwd && col_ok) {
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      const int c = n0 + cv + e;
      bmu[e] = a.bn_mean[c]; bis[e] = a.bn_invstd[c]; bsc[e] = a.bn_scale[c]; bsh[e] = a.bn_shift[c];
    }
  }
  if (MODE == kFwd && a.stats) {
#pragma unroll
    for (int e = 0; e < VEC; e += 4) {
      const f32x4 t = *reinterpret_cast<const f32x4 *>(&Cs[0][cv + e]);
      kshift[e] = t[0]; kshift[e + 1] = t[1]; kshift[e + 2] = t[2]; kshift[e + 3] = t[3];
    }
  }
#pragma unroll
  for (int p0 = 0; p0 < NP; p0 += PG) {
    if (p0 > 0) request_side(p0);
#pragma unroll
    for (int g = 0; g < PG; ++g) {
      if (!live[g]) continue;
      const int r = row0 + (p0 + g) * RPS;
      const size_t off = offs[g];
      float v[VEC];
#pragma unroll
      for (int e = 0; e < VEC; e += 4) {
        const f32x4 t = *reinterpret_cast<const f32x4 *>(&Cs[r][cv + e]);
        v[e] = t[0]; v[e + 1] = t[1]; v[e + 2] = t[2]; v[e + 3] = t[3];
      }
      if (addend) {
        float ad[VEC];
        Vec<T>::unpack(q_ad[g], ad);
#pragma unroll
        for (int e = 0; e < VEC; ++e) v[e] += ad[e];
      }
      if (has_mask) {
        float mk[VEC];
        Vec<T>::unpack(q_mk[g], mk);
#pragma unroll
        for (int e = 0; e < VEC; ++e) v[e] = mk[e] > 0.f ? v[e] : 0.f;
      }
      Vec<T>::store(out + off, v);
      if (bn_bwd) {
        // the same arithmetic as the stand-alone first pass (bn_bwd_partial_kernel) on the values as stored
        float yv[VEC];
        Vec<T>::unpack(q_y[g], yv);
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          float gm = E::to_f32(E::from_f32(v[e]));
          if (a.bn_self) gm = fmaf(yv[e], bsc[e], bsh[e]) > 0.f ? gm : 0.f;
          const float xh = (yv[e] - bmu[e]) * bis[e];
          s1[e] += gm;
          s2[e] = fmaf(gm, xh, s2[e]);
        }
      }
      if (MODE == kFwd) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          const float sv = E::to_f32(E::from_f32(v[e])) - kshift[e];
          s1[e] += sv;
          s2[e] = fmaf(sv, sv, s2[e]);
        }
      }
    }
  }
  if ((MODE == kFwd && a.stats) || bn_bwd) {
    // A wave holds 64/CV rows of every column piece: butterfly over those lanes, then the waves add
    // up in wave order.  Every step has a fixed order, so the sums are bit-stable from run to run.
    constexpr int NW = WGM * WGN;
    __shared__ float red[2][NW][BN];
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
#pragma unroll
      for (int o = CV; o < 64; o <<= 1) {
        s1[e] += __shfl_xor(s1[e], o, 64);
        s2[e] += __shfl_xor(s2[e], o, 64);
      }
    }
    if (lane < CV) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) { red[0][wave][cv + e] = s1[e]; red[1][wave][cv + e] = s2[e]; }
    }
    __syncthreads();
    for (int c = tid; c < BN; c += NT) {
      if (n0 + c < a.OC) {
        float t1 = red[0][0][c], t2 = red[1][0][c];
#pragma unroll
        for (int w = 1; w < NW; ++w) { t1 += red[0][w][c]; t2 += red[1][w][c]; }
        if (MODE == kFwd) {
          a.stats[(size_t)tm * a.OC + n0 + c] = Cs[0][c];
          a.stats[((size_t)a.tiles_m + tm) * a.OC + n0 + c] = t1;
          a.stats[((size_t)2 * a.tiles_m + tm) * a.OC + n0 + c] = t2;
        } else {
          a.bn_sums[(size_t)tm * a.OC + n0 + c] = t1;
          a.bn_sums[((size_t)a.tiles_m + tm) * a.OC + n0 + c] = t2;
        }
      }
    }
  }
}

template <typename T, int BM, int BN, int BK, int WGM, int WGN, int MODE>
int launch_igemm(IgemmArgs a, hipStream_t st, StatParts *tiles_m_out) {
  a.tiles_m = (a.Mrows + BM - 1) / BM;
  if (tiles_m_out) { tiles_m_out->parts = a.tiles_m; tiles_m_out->rows = BM; }
  a.tiles_n = (a.OC + BN - 1) / BN;
  a.div_plane = make_fastdiv((unsigned)(a.OHc * a.OWc)); a.div_w = make_fastdiv((unsigned)a.OWc);
  a.div_tn = make_fastdiv((unsigned)a.tiles_n); a.div_tm = make_fastdiv((unsigned)a.tiles_m);
  const long long grid = (long long)a.tiles_m * a.tiles_n * a.cls * a.cls;
  if (grid <= 0 || grid > 0x7fffffffLL) return set_error(RESIST_ESHAPE, "igemm grid %lld", grid);
  {
    static const std::string label = std::string("igemm_") + (sizeof(T) == 4 ? "f32_" : "bf16_") + (MODE == kFwd ? "fwd_" : "bwd_") +
                                     std::to_string(BM) + "x" + std::to_string(BN) + "x" + std::to_string(BK) +
                                     (WGM * WGN == 8 ? "_w8" : "");
    // algorithmic work of the convolution this launch computes (forward or data gradient)
    const double flops = 2.0 * a.N * (MODE == kFwd ? (double)a.OH * a.OW : (double)a.IH * a.IW) * a.OC * a.IC * a.R * a.S;
    const double bytes = sizeof(T) * ((double)a.N * a.IH * a.IW * a.IC + (double)a.N * a.OH * a.OW * a.OC * (1 + (a.addend ? 1 : 0) + (a.relu_mask ? 1 : 0) + (MODE == kBwd && a.bn_sums ? 1 : 0)) +
                                      (double)a.OC * a.R * a.S * a.IC);
    prof::Scope ps(label.c_str(), flops, bytes, st);
    hipLaunchKernelGGL((igemm_kernel<T, BM, BN, BK, WGM, WGN, MODE>), dim3((unsigned)grid), dim3(WGM * WGN * 64), 0, st, a);
  }
  RESIST_CHECK_LAUNCH("igemm");
  return RESIST_OK;
}

template <typename T, int MODE>
int dispatch_igemm(const IgemmArgs &a, hipStream_t st, StatParts *tiles_m_out = nullptr) {
  // pick the largest tile that still yields enough workgroups to cover the 256 compute units
  constexpr int V = Elem<T>::VEC;   // K-chunks of 8*V and 16*V elements: 128 and 256 bytes per tile row
  const long long classes = (long long)a.cls * a.cls;
  auto tiles = [&](int bm, int bn) {
    return (long long)((a.Mrows + bm - 1) / bm) * ((a.OC + bn - 1) / bn) * classes;
  };
  constexpr long long kMin = 512;   // measured (fp32): 256 or fewer workgroups of a larger 4-wave tile are slower on every layer shape
  constexpr bool lp = sizeof(T) == 2;
  // Eight-wave workgroups on 128-wide tiles (bf16): when a layer has only about one such tile per compute unit,
  // a four-wave workgroup leaves the CU with four waves and nothing to overlap its barriers and load latency
  // with, while 64x64 tiles double the operand bytes every CU pulls through its L1.  Measured (layer_bench.py):
  // 128 -> 128 channels at 16x16, batch 128: 19.0 -> 15.9 us; 256 -> 256 at 14x14, batch 64: 29.0 -> 24.1 us;
  // 256 -> 256 at 8x8, batch 128: 20.0 -> 18.5 us; the full CIFAR-shaped model: 6.64 -> 6.36 ms per step.
  // (In fp32 the same tiles measured no faster inside a step; the fp32 kernels are bound by MFMA issue, not by L1.)
  if (lp && a.cls == 1 && a.OC >= 128) {
    const long long t128 = tiles(128, 128);
    if (t128 >= 192 && t128 < 320) return launch_igemm<T, 128, 128, 8 * V, 4, 2, MODE>(a, st, tiles_m_out);
    if (t128 < 192 && tiles(128, 64) >= 256 && a.IC % (16 * V) == 0)
      return launch_igemm<T, 128, 64, 16 * V, 4, 2, MODE>(a, st, tiles_m_out);
  }
  // bf16 kernels are bound by operand traffic rather than by the matrix cores, and the 128x128 tile
  // moves half the operand bytes per FLOP: measured faster down to ~190 workgroups (ImageNet-shaped
  // stage 2-4 layers: 17-30 us instead of 20-38), slower at 100-130
  constexpr long long kMin128 = lp ? 192 : kMin;
  if (a.OC > 64 && tiles(128, 128) >= kMin128) return launch_igemm<T, 128, 128, 8 * V, 2, 2, MODE>(a, st, tiles_m_out);
  if (lp && a.cls == 1 && a.OC <= 64 && tiles(128, 64) >= kMin) return launch_igemm<T, 128, 64, 8 * V, 4, 2, MODE>(a, st, tiles_m_out);
  if (tiles(128, 64) >= kMin) return launch_igemm<T, 128, 64, 8 * V, 2, 2, MODE>(a, st, tiles_m_out);
  if (a.IC % (16 * V) == 0) return launch_igemm<T, 64, 64, 16 * V, 2, 2, MODE>(a, st, tiles_m_out);
  return launch_igemm<T, 64, 64, 8 * V, 2, 2, MODE>(a, st, tiles_m_out);
}

int check_geom(const ConvGeom &g, int dt) {
  const int v = dt == DT_BF16 ? 8 : 4;
  if (dt != DT_F32 && dt != DT_BF16) return set_error(RESIST_EINVAL, "dtype %d", dt);
  if (g.N < 1 || g.H < 1 || g.W < 1 || g.C < v || g.K < v || (g.C % v) || (g.K % v))
    return set_error(RESIST_ESHAPE, "conv shape N%d H%d W%d C%d K%d (C, K must be multiples of %d)", g.N, g.H, g.W, g.C, g.K, v);
  if (g.R != g.S || (g.R != 1 && g.R != 3 && g.R != 5 && g.R != 7))
    return set_error(RESIST_ESHAPE, "filter %dx%d unsupported", g.R, g.S);
  if (g.stride < 1 || g.stride > 2 || g.pad < 0 || g.pad >= g.R)
    return set_error(RESIST_ESHAPE, "stride %d pad %d unsupported", g.stride, g.pad);
  if (g.P < 1 || g.Q < 1) return set_error(RESIST_ESHAPE, "empty convolution output");
  const long long lim = 0x7fffffffLL / (dt == DT_BF16 ? 2 : 4);   // byte offsets stay below the out-of-range marker
  if ((long long)g.N * g.H * g.W * g.C > lim || (long long)g.N * g.P * g.Q * g.K > lim ||
      (long long)g.K * g.R * g.S * g.C > lim)
    return set_error(RESIST_ESHAPE, "tensor exceeds 2 GiB");
  return RESIST_OK;
}

}  // namespace

int conv_check(const ConvGeom &g, int dt) { return check_geom(g, dt); }

int64_t conv_stats_floats(const ConvGeom &g) {
  // the smallest row tile any forward kernel uses is 64
  return (int64_t)3 * (((int64_t)g.N * g.P * g.Q + 63) / 64) * g.K;
}

int conv_fwd(const ConvGeom &g, int dt, const void *x, const void *w, void *y, const void *addend, float *stats, StatParts *stat_parts,
             hipStream_t st) {
  RESIST_TRY(check_geom(g, dt));
  if (stats && !stat_parts) return set_error(RESIST_EINVAL, "conv_fwd: stats without stat_parts");
  IgemmArgs a{};
  a.in = x; a.wt = w; a.out = y; a.addend = addend; a.stats = stats;
  a.N = g.N; a.IH = g.H; a.IW = g.W; a.IC = g.C;
  a.OH = g.P; a.OW = g.Q; a.OC = g.K;
  a.R = g.R; a.S = g.S; a.stride = g.stride; a.pad = g.pad;
  a.cls = 1; a.OHc = g.P; a.OWc = g.Q;
  a.Mrows = g.N * g.P * g.Q;
  return dt == DT_BF16 ? dispatch_igemm<__bf16, kFwd>(a, st, stat_parts) : dispatch_igemm<float, kFwd>(a, st, stat_parts);
}

int conv_dgrad(const ConvGeom &g, int dt, const void *dy, const void *wT, void *dx, const void *addend, const void *relu_mask,
               hipStream_t st, const BnBwdFuse *bn) {
  RESIST_TRY(check_geom(g, dt));
  if (g.stride == 2 && ((g.H & 1) || (g.W & 1)))
    return set_error(RESIST_ESHAPE, "stride-2 dgrad needs even input size, got %dx%d", g.H, g.W);
  IgemmArgs a{};
  a.in = dy; a.wt = wT; a.out = dx; a.addend = addend; a.relu_mask = relu_mask;
  a.N = g.N; a.IH = g.P; a.IW = g.Q; a.IC = g.K;
  a.OH = g.H; a.OW = g.W; a.OC = g.C;
  a.R = g.R; a.S = g.S; a.stride = g.stride; a.pad = g.pad;
  a.cls = g.stride; a.OHc = g.H / g.stride; a.OWc = g.W / g.stride;
  a.Mrows = g.N * a.OHc * a.OWc;
  StatParts parts;
  if (bn) {
    if (a.cls != 1 || !bn->y || !bn->sums || !bn->parts) return set_error(RESIST_EINVAL, "fused BN sums need a stride-1 data gradient");
    a.bn_y = bn->y; a.bn_mean = bn->b.mean; a.bn_invstd = bn->b.invstd; a.bn_scale = bn->b.scale; a.bn_shift = bn->b.shift;
    a.bn_sums = bn->sums; a.bn_self = bn->relu_of_self ? 1 : 0;
  }
  RESIST_TRY(dt == DT_BF16 ? (dispatch_igemm<__bf16, kBwd>(a, st, &parts)) : (dispatch_igemm<float, kBwd>(a, st, &parts)));
  if (bn) *bn->parts = parts;
  return RESIST_OK;
}

int64_t conv_dgrad_bn_sums_floats(const ConvGeom &g) {
  // the smallest row tile any data-gradient kernel uses is 64
  return (int64_t)2 * (((int64_t)g.N * g.H * g.W + 63) / 64) * g.C;
}

// ---- filter preparation: wT[c][r][s][k] = w[k][r][s][c] (and a low-precision copy of w) ------------
namespace {
template <typename S, typename T>
__global__ __launch_bounds__(256) void prepare_filter_kernel(const S *__restrict__ w, T *__restrict__ wlp, T *__restrict__ wT,
                                                             int K, int RS, int C) {
  // 32x32 tiles of the [K][C] matrix at a fixed tap, through LDS so both sides stay coalesced
  __shared__ float tile[32][33];
  const int tap = blockIdx.z;
  const int k0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
  for (int i = ty; i < 32; i += 8) {
    const int k = k0 + i, c = c0 + tx;
    float v = 0.f;
    if (k < K && c < C) {
      v = Elem<S>::to_f32(w[((size_t)k * RS + tap) * C + c]);
      if (wlp) wlp[((size_t)k * RS + tap) * C + c] = Elem<T>::from_f32(v);
    }
    tile[i][tx] = v;
  }
  __syncthreads();
  if (wT)
    for (int i = ty; i < 32; i += 8) {
      const int c = c0 + i, k = k0 + tx;
      if (k < K && c < C) wT[((size_t)c * RS + tap) * K + k] = Elem<T>::from_f32(tile[tx][i]);
    }
}
}  // namespace

// All filters of a step in one launch (or a few: the table travels in the kernel arguments).
namespace {
constexpr int kPrepSegs = 48;
struct PrepTable {
  const float *w[kPrepSegs];
  void *wlp[kPrepSegs];
  void *wT[kPrepSegs];
  int K[kPrepSegs], RS[kPrepSegs], C[kPrepSegs];
  float scale[kPrepSegs];
  int first_wg[kPrepSegs + 1];
  int nseg;
};
// four consecutive elements of T from four floats
__device__ inline void store4(float *p, float a, float b, float c, float d) {
  *reinterpret_cast<f32x4 *>(p) = f32x4{a, b, c, d};
}
__device__ inline void store4(__bf16 *p, float a, float b, float c, float d) {
  *reinterpret_cast<u32x2 *>(p) = u32x2{pack_bf16x2(a, b), pack_bf16x2(c, d)};
}

// One 64x64 tile of the [K][C] matrix of one tap per workgroup, through LDS so that both sides move whole
// vectors: 256-byte runs of the fp32 master in, 4-element vectors of the copy and of the transpose out.
template <typename T>
__global__ __launch_bounds__(256) void prepare_filters_kernel(PrepTable t) {
  constexpr int TS = 64;
  __shared__ float tile[TS][TS + 1];
  int seg = 0;
  while (seg + 1 < t.nseg && (int)blockIdx.x >= t.first_wg[seg + 1]) ++seg;
  const int K = t.K[seg], RS = t.RS[seg], C = t.C[seg];
  const int ct = (C + TS - 1) / TS, kt = (K + TS - 1) / TS;
  int id = blockIdx.x - t.first_wg[seg];
  const int c0 = (id % ct) * TS;
  id /= ct;
  const int k0 = (id % kt) * TS, tap = id / kt;
  const float *__restrict__ w = t.w[seg];
  const float sc = t.scale[seg];
  T *__restrict__ wlp = static_cast<T *>(t.wlp[seg]);
  T *__restrict__ wT = static_cast<T *>(t.wT[seg]);
  const int row = threadIdx.x >> 4, col = (threadIdx.x & 15) * 4;   // 16 rows x 16 vectors per pass
  // K and C are multiples of four (checked on the host)
  f32x4 v[TS / 16];
#pragma unroll
  for (int p = 0; p < TS / 16; ++p) {
    const int k = k0 + row + 16 * p, c = c0 + col;
    v[p] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (k < K && c < C) v[p] = *reinterpret_cast<const f32x4 *>(w + ((size_t)k * RS + tap) * C + c);
  }
#pragma unroll
  for (int p = 0; p < TS / 16; ++p) {
    const int k = k0 + row + 16 * p, c = c0 + col;
    v[p] *= sc;
    if (wlp && k < K && c < C) store4(wlp + ((size_t)k * RS + tap) * C + c, v[p][0], v[p][1], v[p][2], v[p][3]);
#pragma unroll
    for (int e = 0; e < 4; ++e) tile[row + 16 * p][col + e] = v[p][e];
  }
  __syncthreads();
  if (wT) {
#pragma unroll
    for (int p = 0; p < TS / 16; ++p) {
      const int c = c0 + row + 16 * p, k = k0 + col;
      if (c < C && k < K)
        store4(wT + ((size_t)c * RS + tap) * K + k, tile[col][row + 16 * p], tile[col + 1][row + 16 * p],
               tile[col + 2][row + 16 * p], tile[col + 3][row + 16 * p]);
    }
  }
}
}  // namespace

int prepare_filters(const std::vector<FilterPrep> &items, int dt, hipStream_t st) {
  size_t i = 0;
  while (i < items.size()) {
    PrepTable t{};
    int wg = 0;
    double bytes = 0;
    while (i < items.size() && t.nseg < kPrepSegs) {
      const FilterPrep &f = items[i++];
      if ((f.g.K & 3) || (f.g.C & 3)) return set_error(RESIST_ESHAPE, "filter %dx%d: channel counts must be multiples of 4", f.g.K, f.g.C);
      const int n = t.nseg++;
      t.w[n] = f.w; t.wlp[n] = f.w_lp; t.wT[n] = f.wT;
      t.K[n] = f.g.K; t.RS[n] = f.g.R * f.g.S; t.C[n] = f.g.C;
      t.scale[n] = f.scale;
      t.first_wg[n] = wg;
      wg += ((f.g.C + 63) / 64) * ((f.g.K + 63) / 64) * f.g.R * f.g.S;
      bytes += (4.0 + (f.w_lp ? esize(dt) : 0) + (f.wT ? esize(dt) : 0)) * f.g.K * f.g.R * f.g.S * f.g.C;
    }
    t.first_wg[t.nseg] = wg;
    if (wg == 0) continue;
    prof::Scope ps("prepare_filters", 0, bytes, st);
    if (dt == DT_BF16) hipLaunchKernelGGL(prepare_filters_kernel<__bf16>, dim3(wg), dim3(256), 0, st, t);
    else hipLaunchKernelGGL(prepare_filters_kernel<float>, dim3(wg), dim3(256), 0, st, t);
    RESIST_CHECK_LAUNCH("prepare_filters");
  }
  return RESIST_OK;
}

int prepare_filter(const ConvGeom &g, int src_dt, int dt, const void *w, void *w_lp, void *wT, hipStream_t st) {
  if (src_dt == DT_BF16 && dt != DT_BF16) return set_error(RESIST_EINVAL, "prepare_filter: bf16 source needs a bf16 target");
  dim3 grid((g.C + 31) / 32, (g.K + 31) / 32, g.R * g.S);
  prof::Scope ps("prepare_filter", 0, ((double)esize(src_dt) + (w_lp ? esize(dt) : 0) + (wT ? esize(dt) : 0)) * g.K * g.R * g.S * g.C, st);
  if (src_dt == DT_BF16)
    hipLaunchKernelGGL((prepare_filter_kernel<__bf16, __bf16>), grid, dim3(256), 0, st, (const __bf16 *)w, (__bf16 *)w_lp, (__bf16 *)wT, g.K, g.R * g.S, g.C);
  else if (dt == DT_BF16)
    hipLaunchKernelGGL((prepare_filter_kernel<float, __bf16>), grid, dim3(256), 0, st, (const float *)w, (__bf16 *)w_lp, (__bf16 *)wT, g.K, g.R * g.S, g.C);
  else
    hipLaunchKernelGGL((prepare_filter_kernel<float, float>), grid, dim3(256), 0, st, (const float *)w, (float *)w_lp, (float *)wT, g.K, g.R * g.S, g.C);
  RESIST_CHECK_LAUNCH("prepare_filter");
  return RESIST_OK;
}

// ---- wgrad --------------------------------------------------------------------------------------
namespace {

constexpr int kWBK = 32;  // reduction rows staged per step

struct WgradArgs {
  const void *dy;   // [M][K]
  const void *x;    // [N][H][W][C]
  float *out;       // [splits][K][R][S][C]
  int N, H, W, C, K, R, S, stride, pad, P, Q;
  int M;            // N*P*Q
  int rows_per_split;
  int tiles_k, tiles_c;
  FastDiv div_pq, div_q;
};

// Weight gradient: rows of the GEMM are output channels, columns are input channels of one filter
// tap, the reduction runs over output pixels m (split across workgroups).  Both operand tiles arrive
// "reduction-major" ([m][channel]) straight from the NHWC tensors.  Same pipeline as the forward
// kernel: straight-line loop body, bounds-checked buffer loads, LDS refill in the middle of the
// MFMAs, fragments fetched one k-step ahead.  This is the fp32 kernel: the matrix instruction takes
// one reduction index per lane, so fragments are single LDS words and no transpose is needed.
template <int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(kThreads) void wgrad_kernel(WgradArgs a) {
  constexpr int VEC = 4;
  constexpr int ES = 4;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int LDA = BM + 32, LDB = BN + 32;     // rows kk and kk+1 land on different bank halves
  constexpr int TPRA = BM / VEC, TPRB = BN / VEC; // threads per 32-row-chunk row
  constexpr int RPA = kThreads / TPRA, RPB = kThreads / TPRB;  // rows per pass
  constexpr int PA = (kWBK + RPA - 1) / RPA, PB = (kWBK + RPB - 1) / RPB;
  constexpr int NK = kWBK / 2;
  __shared__ float As[2][kWBK][LDA];
  __shared__ float Bs[2][kWBK][LDB];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  // order: tile fastest, then filter tap, then reduction split; every XCD gets one contiguous range
  // of that order, i.e. a range of reduction rows, so each L2 fetches only its share of dy and x
  // (with the hardware's round-robin order every XCD read both tensors in full: 8x the traffic, same speed)
  int bid = xcd_contiguous(blockIdx.x, gridDim.x);
  const int tile = bid % (a.tiles_k * a.tiles_c);
  bid /= a.tiles_k * a.tiles_c;
  const int tap = bid % (a.R * a.S), split = bid / (a.R * a.S);
  const int tk = tile / a.tiles_c, tc = tile % a.tiles_c;
  const int r = tap / a.S, s = tap - r * a.S;
  const int k0 = tk * BM, c0 = tc * BN;
  const int mbeg = split * a.rows_per_split;
  const int mend = min(a.M, mbeg + a.rows_per_split);
  const int nchunks = (mend - mbeg + kWBK - 1) / kWBK;

  const int arow = tid / TPRA, acol = (tid % TPRA) * VEC;
  const int brow = tid / TPRB, bcol = (tid % TPRB) * VEC;
  const unsigned acolb = (k0 + acol) < a.K ? (unsigned)(k0 + acol) * ES : kOOB;
  const unsigned bcolb = (c0 + bcol) < a.C ? (unsigned)(c0 + bcol) * ES : kOOB;
  const __amdgpu_buffer_rsrc_t rdy = make_rsrc(a.dy, (unsigned)a.M * a.K * ES);
  const __amdgpu_buffer_rsrc_t rx = make_rsrc(a.x, (unsigned)a.N * a.H * a.W * a.C * ES);

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  f32x4 ra[PA], rb[PB];
  int mc = mbeg;   // first reduction row of the chunk being requested
  // register `part` (0..PA-1: rows of dy, PA..PA+PB-1: rows of x) of the chunk starting at row mc
  auto request = [&](int part) {
    if (part < PA) {
      const int row = part * RPA + arow;
      const int m = mc + row;
      ra[part] = buffer_load_16B(rdy, (m < mend && row < kWBK) ? (unsigned)m * (unsigned)a.K * ES + acolb : kOOB);
    } else {
      const int i = part - PA;
      const int row = i * RPB + brow;
      const int m = mc + row;
      const int n = fdiv(m, a.div_pq);
      const int rem = m - n * (a.P * a.Q);
      const int p = fdiv(rem, a.div_q), q = rem - p * a.Q;
      const int ih = p * a.stride + r - a.pad, iw = q * a.stride + s - a.pad;
      const bool ok = m < mend && row < kWBK && (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W;
      rb[i] = buffer_load_16B(rx, ok ? (unsigned)((n * a.H + ih) * a.W + iw) * (unsigned)a.C * ES + bcolb : kOOB);
    }
  };
  auto store_part = [&](int stage, int part) {
    if (part < PA) {
      if (part * RPA + arow < kWBK) *reinterpret_cast<f32x4 *>(&As[stage][part * RPA + arow][acol]) = ra[part];
    } else {
      const int i = part - PA;
      if (i * RPB + brow < kWBK) *reinterpret_cast<f32x4 *>(&Bs[stage][i * RPB + brow][bcol]) = rb[i];
    }
  };
  auto load_global = [&]() {
#pragma unroll
    for (int p = 0; p < PA + PB; ++p) request(p);
    mc += kWBK;
  };
  auto store_lds = [&](int stage) {
#pragma unroll
    for (int p = 0; p < PA + PB; ++p) store_part(stage, p);
  };

  // same pipeline as the forward kernel: fragments one k-step ahead (also across chunks), refill of
  // the other stage spread over k-steps 0 .. NK-2, one barrier per chunk at the start of the last k-step
  static_assert(NK % 2 == 0, "fragment double buffer parity");
  const int lr = lane & 31, lh = lane >> 5;
  float fa[2][TM], fb[2][TN];
  auto load_frags = [&](int buf, int stage, int ks) {
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[buf][i] = As[stage][ks * 2 + lh][wm * WTM + i * 32 + lr];
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[buf][j] = Bs[stage][ks * 2 + lh][wn * WTN + j * 32 + lr];
  };
  auto lds_barrier = [&]() {
    __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
  };
  load_global();
  store_lds(0);
  load_global();
  lds_barrier();
  load_frags(0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  for (int it = 0; it < nchunks; ++it) {
    const int stage = it & 1;
#pragma unroll
    for (int ks = 0; ks < NK; ++ks) {
      if (ks + 1 < NK) {
        load_frags((ks + 1) & 1, stage, ks + 1);
      } else {
        lds_barrier();
        load_frags(0, stage ^ 1, 0);   // rows past mend were loaded as zeros
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int p = 0; p < PA + PB; ++p)
        if ((p * (NK - 1)) / (PA + PB) == ks) {   // refill spread evenly over k-steps 0 .. NK-2
          store_part(stage ^ 1, p);
          request(p);
        }
      if (ks == NK - 2) mc += kWBK;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[ks & 1][i], fb[ks & 1][j], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  float *out = a.out + (size_t)split * a.K * a.R * a.S * a.C;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int c = c0 + wn * WTN + j * 32 + lr;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int k = k0 + wm * WTM + i * 32 + (e >> 2) * 8 + lh * 4 + (e & 3);
        if (k < a.K && c < a.C) out[((size_t)k * a.R * a.S + tap) * a.C + c] = acc[i][j][e];
      }
    }
}

// LDS transpose read (ds_read_b64_tr_b16).  Within each block of 16 lanes, lane s supplies the
// address of 4 consecutive 16-bit values; lane j receives, as element e, the value number j%4 of
// the four that lane 4*e + j/4 pointed at.  When lane s points at row s/4, columns 4*(s%4)..+3 of a
// row-major tile, lane j therefore ends up with rows 0..3 of column j: a 4x16 -> 16x4 transpose.
typedef short s16x4 __attribute__((ext_vector_type(4)));
__device__ inline s16x4 lds_read_tr(const __bf16 *p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(p));
}

// Weight gradient with bf16 operands on v_mfma_f32_32x32x16_bf16.  The matrix instruction wants 8
// consecutive values of the reduction index (output pixels m) per lane, while both operands arrive
// from memory with the channel index contiguous ([m][channel]); the tiles are therefore stored in LDS
// as they arrive and read back through the LDS transpose read, two 4-deep reads per fragment.
// WBK: pixels staged per chunk (a multiple of 32); otherwise the same pipeline as the fp32 kernel.
template <int BM, int BN, int WBK>
__global__ __launch_bounds__(kThreads) void wgrad_bf16_kernel(WgradArgs a) {
  constexpr int WGM = 2, WGN = 2;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int LDA = BM + 32, LDB = BN + 32;     // row pitch = tile width + 64 bytes: 4 consecutive rows fall on disjoint banks
  constexpr int TPRA = BM / 8, TPRB = BN / 8;     // threads per tile row (16 bytes each)
  constexpr int RPA = kThreads / TPRA, RPB = kThreads / TPRB;
  constexpr int PA = WBK / RPA, PB = WBK / RPB;
  constexpr int NK = WBK / 16;
  static_assert(WBK % RPA == 0 && WBK % RPB == 0 && NK % 2 == 0 && TM >= 1 && TN >= 1, "tile shape");
  __shared__ __bf16 As[2][WBK][LDA];
  __shared__ __bf16 Bs[2][WBK][LDB];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  // every XCD gets a contiguous range of (tile, tap, split) ids, so the workgroups that read the same
  // pixels (all tiles and taps of one split) share an L2: this kernel is bound by memory traffic
  int bid = xcd_contiguous(blockIdx.x, gridDim.x);
  const int tile = bid % (a.tiles_k * a.tiles_c);
  bid /= a.tiles_k * a.tiles_c;
  const int tap = bid % (a.R * a.S), split = bid / (a.R * a.S);
  const int tk = tile / a.tiles_c, tc = tile % a.tiles_c;
  const int r = tap / a.S, s = tap - r * a.S;
  const int k0 = tk * BM, c0 = tc * BN;
  const int mbeg = split * a.rows_per_split;
  const int mend = min(a.M, mbeg + a.rows_per_split);
  const int nchunks = (mend - mbeg + WBK - 1) / WBK;

  const int arow = tid / TPRA, acol = (tid % TPRA) * 8;
  const int brow = tid / TPRB, bcol = (tid % TPRB) * 8;
  const unsigned acolb = (k0 + acol) < a.K ? (unsigned)(k0 + acol) * 2u : kOOB;
  const unsigned bcolb = (c0 + bcol) < a.C ? (unsigned)(c0 + bcol) * 2u : kOOB;
  const __amdgpu_buffer_rsrc_t rdy = make_rsrc(a.dy, (unsigned)a.M * a.K * 2u);
  const __amdgpu_buffer_rsrc_t rx = make_rsrc(a.x, (unsigned)a.N * a.H * a.W * a.C * 2u);

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  f32x4 ra[PA], rb[PB];
  int mc = mbeg;   // first reduction row of the chunk being requested
  auto request = [&](int part) {
    if (part < PA) {
      const int m = mc + part * RPA + arow;
      ra[part] = buffer_load_16B(rdy, m < mend ? (unsigned)m * (unsigned)a.K * 2u + acolb : kOOB);
    } else {
      const int i = part - PA;
      const int m = mc + i * RPB + brow;
      const int n = fdiv(m, a.div_pq);
      const int rem = m - n * (a.P * a.Q);
      const int p = fdiv(rem, a.div_q), q = rem - p * a.Q;
      const int ih = p * a.stride + r - a.pad, iw = q * a.stride + s - a.pad;
      const bool ok = m < mend && (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W;
      rb[i] = buffer_load_16B(rx, ok ? (unsigned)((n * a.H + ih) * a.W + iw) * (unsigned)a.C * 2u + bcolb : kOOB);
    }
  };
  auto store_part = [&](int stage, int part) {
    if (part < PA) *reinterpret_cast<f32x4 *>(&As[stage][part * RPA + arow][acol]) = ra[part];
    else *reinterpret_cast<f32x4 *>(&Bs[stage][(part - PA) * RPB + brow][bcol]) = rb[part - PA];
  };
  auto load_global = [&]() {
#pragma unroll
    for (int p = 0; p < PA + PB; ++p) request(p);
    mc += WBK;
  };
  auto store_lds = [&](int stage) {
#pragma unroll
    for (int p = 0; p < PA + PB; ++p) store_part(stage, p);
  };

  // fragment addressing of the transpose read: lane l supplies row 8*(l/32) + (l%16)/4 of a 16-row
  // k-step and columns 16*((l/16)%2) + 4*(l%4) .. +3 of a 32-column tile; it receives column l%32,
  // rows 8*(l/32) .. +3 (and +4 .. +7 from the second read)
  const int frow = (lane >> 5) * 8 + ((lane & 15) >> 2);
  const int fcol = ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
  bf16x8 fa[2][TM], fb[2][TN];
  auto load_frags = [&](int buf, int stage, int ks) {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const s16x4 lo = lds_read_tr(&As[stage][ks * 16 + frow][wm * WTM + i * 32 + fcol]);
      const s16x4 hi = lds_read_tr(&As[stage][ks * 16 + frow + 4][wm * WTM + i * 32 + fcol]);
      typedef short s16x8 __attribute__((ext_vector_type(8)));
      const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      fa[buf][i] = __builtin_bit_cast(bf16x8, v);
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const s16x4 lo = lds_read_tr(&Bs[stage][ks * 16 + frow][wn * WTN + j * 32 + fcol]);
      const s16x4 hi = lds_read_tr(&Bs[stage][ks * 16 + frow + 4][wn * WTN + j * 32 + fcol]);
      typedef short s16x8 __attribute__((ext_vector_type(8)));
      const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      fb[buf][j] = __builtin_bit_cast(bf16x8, v);
    }
  };
  auto lds_barrier = [&]() {
    __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
  };
  load_global();
  store_lds(0);
  load_global();
  lds_barrier();
  load_frags(0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  for (int it = 0; it < nchunks; ++it) {
    const int stage = it & 1;
#pragma unroll
    for (int ks = 0; ks < NK; ++ks) {
      if (ks + 1 < NK) {
        load_frags((ks + 1) & 1, stage, ks + 1);
      } else {
        lds_barrier();
        load_frags(0, stage ^ 1, 0);   // rows past mend were loaded as zeros
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int p = 0; p < PA + PB; ++p)
        if ((p * (NK - 1)) / (PA + PB) == ks) {   // refill spread evenly over k-steps 0 .. NK-2
          store_part(stage ^ 1, p);
          request(p);
        }
      if (ks == NK - 2) mc += WBK;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks & 1][i], fb[ks & 1][j], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  const int lr = lane & 31, lh = lane >> 5;
  float *out = a.out + (size_t)split * a.K * a.R * a.S * a.C;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int c = c0 + wn * WTN + j * 32 + lr;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int k = k0 + wm * WTM + i * 32 + (e >> 2) * 8 + lh * 4 + (e & 3);
        if (k < a.K && c < a.C) out[((size_t)k * a.R * a.S + tap) * a.C + c] = acc[i][j][e];
      }
    }
}

// Sum of the split partial results, in a fixed order (bit-stable from run to run): thread (x, g)
// adds splits g, g+G, g+2G, ... of output vector x in ascending order, then the G partial sums are
// added in ascending g.  G threads share one output vector so that many loads are in flight even
// when the output is small and the number of splits large.
template <int G>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *__restrict__ part, float *__restrict__ out,
                                                            long long n4, int splits) {
  constexpr int X = 256 / G;
  __shared__ f32x4 red[G][X];
  const int x = threadIdx.x % X, g = threadIdx.x / X;
  const long long i = (long long)blockIdx.x * X + x;
  const f32x4 *p = reinterpret_cast<const f32x4 *>(part);
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  if (i < n4)
    for (int z = g; z < splits; z += G) acc += p[i + (long long)z * n4];
  if (G > 1) {
    red[g][x] = acc;
    __syncthreads();
    if (g == 0) {
#pragma unroll
      for (int h = 1; h < G; ++h) acc += red[h][x];
    }
  }
  if (g == 0 && i < n4) reinterpret_cast<f32x4 *>(out)[i] = acc;
}

struct WgradPlan { int bm, bn, splits, rows_per_split; };

WgradPlan plan_wgrad(const ConvGeom &g) {
  WgradPlan p;
  p.bm = (g.K >= 128 && g.C >= 128 && (long long)g.K * g.C * g.R * g.S >= 128LL * 128 * 9 * 16) ? 128 : 64;
  p.bn = p.bm;
  const long long tiles = (long long)((g.K + p.bm - 1) / p.bm) * ((g.C + p.bn - 1) / p.bn) * g.R * g.S;
  const long long M = (long long)g.N * g.P * g.Q;
  long long splits = 768 / tiles;   // at most three workgroups per CU: all resident at once (measured best)
  const long long max_splits = (M + 255) / 256;  // at least 256 reduction rows per split
  if (splits > max_splits) splits = max_splits;
  if (splits < 1) splits = 1;
  if (splits > 256) splits = 256;
  long long rps = (M + splits - 1) / splits;
  rps = (rps + kWBK - 1) / kWBK * kWBK;
  p.rows_per_split = (int)rps;
  p.splits = (int)((M + rps - 1) / rps);
  return p;
}

}  // namespace

int64_t wgrad_scratch_floats(const ConvGeom &g) {
  const WgradPlan p = plan_wgrad(g);
  return p.splits > 1 ? (int64_t)p.splits * g.K * g.R * g.S * g.C : 0;
}

int conv_wgrad(const ConvGeom &g, int dt, const void *dy, const void *x, float *dw, float *partial, hipStream_t st) {
  RESIST_TRY(check_geom(g, dt));
  const WgradPlan p = plan_wgrad(g);
  if (p.splits > 1 && !partial) return set_error(RESIST_EWORKSPACE, "wgrad needs split scratch");
  WgradArgs a{};
  a.dy = dy; a.x = x; a.out = p.splits > 1 ? partial : dw;
  a.N = g.N; a.H = g.H; a.W = g.W; a.C = g.C; a.K = g.K; a.R = g.R; a.S = g.S;
  a.stride = g.stride; a.pad = g.pad; a.P = g.P; a.Q = g.Q;
  a.M = g.N * g.P * g.Q;
  a.rows_per_split = p.rows_per_split;
  a.tiles_k = (g.K + p.bm - 1) / p.bm;
  a.tiles_c = (g.C + p.bn - 1) / p.bn;
  a.div_pq = make_fastdiv((unsigned)(g.P * g.Q));
  a.div_q = make_fastdiv((unsigned)g.Q);
  dim3 grid((unsigned)(a.tiles_k * a.tiles_c * g.R * g.S * p.splits));
  {
    const double flops = 2.0 * a.M * g.K * g.C * g.R * g.S;
    const double bytes = esize(dt) * ((double)a.M * g.K + (double)g.N * g.H * g.W * g.C) + 4.0 * g.K * g.R * g.S * g.C;
    const char *label = dt == DT_BF16 ? (p.bm == 128 ? "wgrad_bf16_128x128" : "wgrad_bf16_64x64")
                                      : (p.bm == 128 ? "wgrad_f32_128x128" : "wgrad_f32_64x64");
    prof::Scope ps(label, flops, bytes, st);
    if (dt == DT_BF16) {
      if (p.bm == 128) hipLaunchKernelGGL((wgrad_bf16_kernel<128, 128, 32>), grid, dim3(kThreads), 0, st, a);
      else hipLaunchKernelGGL((wgrad_bf16_kernel<64, 64, 64>), grid, dim3(kThreads), 0, st, a);
    } else {
      if (p.bm == 128) hipLaunchKernelGGL((wgrad_kernel<128, 128, 2, 2>), grid, dim3(kThreads), 0, st, a);
      else hipLaunchKernelGGL((wgrad_kernel<64, 64, 2, 2>), grid, dim3(kThreads), 0, st, a);
    }
  }
  RESIST_CHECK_LAUNCH("wgrad");
  if (p.splits > 1) return splitk_reduce(partial, dw, (long long)g.K * g.R * g.S * g.C / 4, p.splits, st);
  return RESIST_OK;
}

int splitk_reduce(const float *partial, float *out, long long n4, int splits, hipStream_t st) {
  prof::Scope ps("splitk_reduce", 0, 16.0 * n4 * (splits + 1), st);
  // enough threads per output vector that the launch has at least ~64k loads in flight
  if (n4 * 4 >= 65536 || splits < 8)
    hipLaunchKernelGGL(splitk_reduce_kernel<4>, dim3((unsigned)((n4 + 63) / 64)), dim3(256), 0, st, partial, out, n4, splits);
  else
    hipLaunchKernelGGL(splitk_reduce_kernel<16>, dim3((unsigned)((n4 + 15) / 16)), dim3(256), 0, st, partial, out, n4, splits);
  RESIST_CHECK_LAUNCH("splitk_reduce");
  return RESIST_OK;
}

// ---- weight gradient with its split partial sums in library-owned static device memory ------------
// For callers that cannot allocate (HIP graph capture, serving loops): the split-reduction scratch of
// conv_wgrad lives in a file-scope device array instead of a caller-provided workspace.  Host code
// never uses the array's name as an address: its device address is looked up once per device.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kScratchDevices = 16;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kScratchDevices] = {};

// device address of `scratch` on the current device (each GPU holds its own copy at its own address)
int static_scratch(void **out) {
  int dev = 0;
  RESIST_CHECK_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kScratchDevices) return set_error(RESIST_EUNSUPPORTED, "device %d: at most %d devices", dev, kScratchDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    RESIST_CHECK_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return set_error(RESIST_EHIP, "hipGetSymbolAddress returned NULL");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return RESIST_OK;
}
}  // namespace

int64_t wgrad_static_scratch_bytes() { return (int64_t)kStaticScratchBytes; }

int conv_wgrad_static(const ConvGeom &g, int dt, const void *dy, const void *x, float *dw, hipStream_t st) {
  RESIST_TRY(check_geom(g, dt));
  const int64_t need = wgrad_scratch_floats(g) * 4;
  if (need > (int64_t)kStaticScratchBytes)
    return set_error(RESIST_EWORKSPACE, "split partial sums need %lld bytes, the static scratch holds %lld",
                     (long long)need, (long long)kStaticScratchBytes);
  void *ptr = nullptr;
  RESIST_TRY(static_scratch(&ptr));
  // every split writes its whole [K][R][S][C] slice before the reduction reads it: nothing to clear
  return conv_wgrad(g, dt, dy, x, dw, need > 0 ? static_cast<float *>(ptr) : nullptr, st);
}

}  // namespace resist
