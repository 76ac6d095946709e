// The stem convolution (3x3 stride 1, or 7x7 stride 2) straight from the logical [N,C,H,W] fp32 batch
// (C = 3): forward and weight gradient as implicit GEMMs on the matrix cores whose im2col operand is
// assembled from an image patch staged in LDS and never written to memory.  GEMM K runs over the filter
// positions j = (r*S + s)*C + c, padded with zero columns to kpad (a multiple of 32); the filter is
// handed over as [K][kpad] in the compute type (pad_rows below) and the weight gradient comes back in
// the same padded shape (unpad_rows_f32).
#include <type_traits>

#include "elem.h"
#include "internal.h"

namespace resist {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

// ---- the stem convolution as an implicit GEMM on the NCHW fp32 image ------------------------------------
// A workgroup owns a tile of RB output rows x QB output columns of one image (RB*QB <= 128 pixels, RB | P,
// QB | Q, so all tiles are alike).  The patch of the image those pixels touch -- C x PH x PW values,
// PH = (RB-1)*stride + R, PW = (QB-1)*stride + R, zeros outside the image -- is staged once in LDS as fp32.
// GEMM row = pixel, GEMM K = filter position j = (r*S + s)*C + c (padded with zero columns to kpad), and
// the element (pixel, j) of the never-materialised im2col matrix is  patch[tab[j] + pixoff[pixel]]  with
// tab[j] = (c*PH + r)*PW + s and pixoff = (row*stride)*PW + col*stride; padding columns point into a
// block of zeros.  MFMA fragments are assembled from those LDS words (rounded to bf16 in bf16 mode: the
// image is a bf16 operand there).
struct StemArgs {
  const float *x;      // [N][C][H][W]
  const void *wpad;    // forward: filter [K][kpad] in the compute type (zero columns past taps)
  void *y;             // forward: output [N][P][Q][K]
  float *stats;        // forward: [3][parts][K] shift, sum(y - shift), sum((y - shift)^2) per tile
  const void *dy;      // weight gradient: [N][P][Q][K]
  float *partial;      // weight gradient: [workgroups][K][kpad] partial sums
  int N, C, H, W, K, R, stride, pad, P, Q;
  int taps, kpad;
  int QB, RB, PH, PW;  // tile and patch shape
  int PWp;             // words between patch rows: PW, or in vector mode a multiple of 4 with room for up to 3 leading columns
  int vec;             // vector mode: W is a multiple of 4 and x is 16-byte aligned, so patch rows are staged as 16-byte pieces
  int tiles_q, tiles_p, tiles;   // tiles along Q and P of one image; N * tiles_p * tiles_q
  int zn;              // words of the zero block (largest pixel offset, lead included, + 1)
  int y0;              // weight gradient: first 64-channel group of this launch
  int parts;           // forward: tiles; weight gradient: workgroups
};

struct StemLds {       // offsets in bytes into dynamic LDS
  int patch, zero, tab, pixoff, op, total;
};
template <typename T>
__host__ __device__ inline StemLds stem_lds(const StemArgs &a, bool wgrad) {
  constexpr int VEC = 16 / (int)sizeof(T);
  StemLds L;
  int off = 0;
  auto take = [&](int bytes) { const int o = off; off += (bytes + 15) & ~15; return o; };
  L.patch = take(a.C * a.PH * a.PWp * 4);
  L.zero = take(a.zn * 4);
  L.tab = take(a.kpad * 4);
  L.pixoff = take(128 * 4);
  const int k32 = (a.K + 31) / 32 * 32;
  // forward: the filter [k32][kpad + VEC]; weight gradient: the output-gradient tile [128][k32 + 32 or 4]
  L.op = take(wgrad ? 128 * (k32 + (sizeof(T) == 2 ? 32 : 4)) * (int)sizeof(T) : k32 * (a.kpad + VEC) * (int)sizeof(T));
  // after the multiplications the whole block is reused: forward for the fp32 output tile [128][k32 + 4],
  // weight gradient for the fp32 sum of the waves' partial results [k32][kpad]
  const int reuse = wgrad ? k32 * a.kpad * 4 : 128 * (k32 + 4) * 4;
  L.total = off > reuse ? off : reuse;
  return L;
}

// stages patch, zero block and the two tables for tile `tile`; returns image index, first output pixel, and
// `lead`: the number of columns the patch starts left of the tile's first input column (to be added to every
// pixel offset).  Vector mode: the patch starts at the multiple of four at or below that column, so every
// 16-byte piece of a patch row is aligned in memory and lies wholly inside or wholly outside the image row.
template <typename T>
__device__ inline void stem_stage(const StemArgs &a, const StemLds &L, char *lds, int tile, int *n_out, int *p0_out, int *q0_out,
                                  int *lead_out) {
  float *patch = reinterpret_cast<float *>(lds + L.patch);
  float *zero = reinterpret_cast<float *>(lds + L.zero);
  int *tab = reinterpret_cast<int *>(lds + L.tab);
  int *pixoff = reinterpret_cast<int *>(lds + L.pixoff);
  const int tq = tile % a.tiles_q;
  const int tp = (tile / a.tiles_q) % a.tiles_p;
  const int n = tile / (a.tiles_q * a.tiles_p);
  const int p0 = tp * a.RB, q0 = tq * a.QB;
  const int h0 = p0 * a.stride - a.pad, w0 = q0 * a.stride - a.pad;
  for (int i = threadIdx.x; i < a.zn; i += 256) zero[i] = 0.f;
  const int zbase = (L.zero - L.patch) / 4;
  for (int j = threadIdx.x; j < a.kpad; j += 256) {
    int t = zbase;
    if (j < a.taps) {
      const int c = j % a.C, tap = j / a.C;
      const int r = tap / a.R, s2 = tap - r * a.R;
      t = (c * a.PH + r) * a.PWp + s2;
    }
    tab[j] = t;
  }
  for (int i = threadIdx.x; i < 128; i += 256) {
    int o = 0;
    if (i < a.RB * a.QB) {
      const int pr = i / a.QB, qc = i - pr * a.QB;
      o = pr * a.stride * a.PWp + qc * a.stride;
    }
    pixoff[i] = o;
  }
  const float *img = a.x + (size_t)n * a.C * a.H * a.W;
  if (a.vec) {
    // piece i = rc * V + pc of the patch (V pieces of 4 words per row); same walk as below
    const int lead = w0 & 3, w0a = w0 - lead;     // w0 may be negative: & 3 is the non-negative remainder
    const int V = a.PWp >> 2, total = a.C * a.PH * V;
    const int dq = 256 / V, dr = 256 - dq * V;
    int rc = (int)threadIdx.x / V, pc = (int)threadIdx.x - rc * V;
    constexpr int kBatch = 6;
    for (int base = threadIdx.x; base < total; base += 256 * kBatch) {
      f32x4 v[kBatch];
      int dst[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const int c = (rc >= a.PH) + (rc >= 2 * a.PH) + (rc >= 3 * a.PH);     // C <= 4
        const int ih = h0 + rc - c * a.PH, iw = w0a + 4 * pc;
        const bool ok = base + u * 256 < total && ih >= 0 && ih < a.H && iw >= 0 && iw < a.W;
        v[u] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (ok) v[u] = *reinterpret_cast<const f32x4 *>(img + ((size_t)c * a.H + ih) * a.W + iw);
        dst[u] = rc * a.PWp + 4 * pc;
        pc += dr; rc += dq;
        if (pc >= V) { pc -= V; ++rc; }
      }
#pragma unroll
      for (int u = 0; u < kBatch; ++u)
        if (base + u * 256 < total) *reinterpret_cast<f32x4 *>(patch + dst[u]) = v[u];
    }
    *n_out = n; *p0_out = p0; *q0_out = q0; *lead_out = lead;
    return;
  }
  // element i = rc * PW + pc of the patch; a thread takes i = tid, tid + 256, ...: a batch of loads is in flight
  // before the first LDS write, and (rc, pc) advance by (256 / PW, 256 % PW) without further divisions
  const int total = a.C * a.PH * a.PW;
  const int dq = 256 / a.PW, dr = 256 - dq * a.PW;
  int rc = (int)threadIdx.x / a.PW, pc = (int)threadIdx.x - rc * a.PW;
  auto stage = [&](auto batch_tag) {
    constexpr int kBatch = decltype(batch_tag)::value;
    for (int base = threadIdx.x; base < total; base += 256 * kBatch) {
      float v[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const int c = (rc >= a.PH) + (rc >= 2 * a.PH) + (rc >= 3 * a.PH);     // C <= 4
        const int ih = h0 + rc - c * a.PH, iw = w0 + pc;
        const bool ok = base + u * 256 < total && ih >= 0 && ih < a.H && iw >= 0 && iw < a.W;
        v[u] = ok ? img[((size_t)c * a.H + ih) * a.W + iw] : 0.f;
        pc += dr; rc += dq;
        if (pc >= a.PW) { pc -= a.PW; ++rc; }
      }
#pragma unroll
      for (int u = 0; u < kBatch; ++u)
        if (base + u * 256 < total) patch[base + u * 256] = v[u];
    }
  };
  // the ImageNet-shaped patch (3 x 7 x 229 words) arrives in one round trip of 24 loads per thread; small patches take 4
  if (total > 256 * 4) stage(std::integral_constant<int, 24>{});
  else stage(std::integral_constant<int, 4>{});
  *n_out = n; *p0_out = p0; *q0_out = q0; *lead_out = 0;
}

// the value a float has once it is stored in the activations' type
template <typename T> __device__ inline float as_stored(float v);
template <> __device__ inline float as_stored<float>(float v) { return v; }
template <> __device__ inline float as_stored<__bf16>(float v) { return (float)(__bf16)v; }

template <typename T> struct StemMma;
template <> struct StemMma<float> {
  static constexpr int KS = 2;     // reduction indices per matrix instruction
  typedef float Frag;
};
template <> struct StemMma<__bf16> {
  static constexpr int KS = 16;
  typedef bf16x8 Frag;
};

// y = conv(x, w) for one tile; wave w owns pixels 32w .. 32w+31 and all output channels.
// NTILES: 32-channel tiles of the output (a compile-time count keeps the accumulators in place and the
// multiplication loop free of branches).
template <typename T, int NTILES>
__global__ __launch_bounds__(256) void stem_fwd_kernel(StemArgs a) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  constexpr int VEC = 16 / (int)sizeof(T);
  constexpr int KS = StemMma<T>::KS;
  const StemLds L = stem_lds<T>(a, false);
  const float *patch = reinterpret_cast<const float *>(lds + L.patch);
  const int *tab = reinterpret_cast<const int *>(lds + L.tab);
  const int *pixoff = reinterpret_cast<const int *>(lds + L.pixoff);
  T *Ws = reinterpret_cast<T *>(lds + L.op);
  const int k32 = (a.K + 31) / 32 * 32;
  const int ldw = a.kpad + VEC;
  // filter rows (zero rows up to a multiple of 32 output channels): the first eight 16-byte loads of a thread are
  // issued before the patch is staged, so both arrive in one round trip
  const T *w = static_cast<const T *>(a.wpad);
  const int vpr = a.kpad / VEC, wtotal = k32 * vpr;
  const int wdq = 256 / vpr, wdr = 256 - wdq * vpr;
  int wk = (int)threadIdx.x / vpr, wv = (int)threadIdx.x - wk * vpr;
  f32x4 wt[8];
  int wdst[8];
  auto w_issue = [&](int base) {
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      wt[u] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (base + u * 256 < wtotal && wk < a.K) wt[u] = *reinterpret_cast<const f32x4 *>(w + (size_t)wk * a.kpad + wv * VEC);
      wdst[u] = wk * ldw + wv * VEC;
      wv += wdr; wk += wdq;
      if (wv >= vpr) { wv -= vpr; ++wk; }
    }
  };
  auto w_commit = [&](int base) {
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (base + u * 256 < wtotal) *reinterpret_cast<f32x4 *>(Ws + wdst[u]) = wt[u];
  };
  w_issue(threadIdx.x);
  int n, p0, q0, lead;
  stem_stage<T>(a, L, lds, blockIdx.x, &n, &p0, &q0, &lead);
  w_commit(threadIdx.x);
  for (int base = threadIdx.x + 256 * 8; base < wtotal; base += 256 * 8) {
    w_issue(base);
    w_commit(base);
  }
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lr = lane & 31, kg = lane >> 5;
  const int po = pixoff[wave * 32 + lr] + lead;
  const int nsteps = a.kpad / KS;
  float *Cs = reinterpret_cast<float *>(lds);
  const int ldc = k32 + 4;
  f32x16 acc[NTILES];                        // k32 == 32 * NTILES (the host picks the instance)
#pragma unroll
  for (int t = 0; t < NTILES; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
#pragma unroll 2
  for (int ks = 0; ks < nsteps; ++ks) {
    if constexpr (sizeof(T) == 2) {
      const int j0 = ks * 16 + kg * 8;
      bf16x8 fb[NTILES];
#pragma unroll
      for (int t = 0; t < NTILES; ++t) fb[t] = *reinterpret_cast<const bf16x8 *>(Ws + (t * 32 + lr) * ldw + j0);
      bf16x8 fa;
#pragma unroll
      for (int e = 0; e < 8; ++e) fa[e] = (__bf16)patch[tab[j0 + e] + po];
#pragma unroll
      for (int t = 0; t < NTILES; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb[t], acc[t], 0, 0, 0);
    } else {
      const int j = ks * 2 + kg;
      const float fa = patch[tab[j] + po];
      float fb[NTILES];
#pragma unroll
      for (int t = 0; t < NTILES; ++t) fb[t] = Ws[(t * 32 + lr) * ldw + j];
#pragma unroll
      for (int t = 0; t < NTILES; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa, fb[t], acc[t], 0, 0, 0);
    }
  }
  __syncthreads();   // every wave is done with patch and filter before the block is reused for the output tile
  // a lane holds column lane%32 and rows 8*(e/4) + 4*(lane/32) + e%4 of each 32x32 tile
#pragma unroll
  for (int t = 0; t < NTILES; ++t) {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int row = wave * 32 + (e >> 2) * 8 + kg * 4 + (e & 3);
      Cs[row * ldc + t * 32 + lr] = acc[t][e];
    }
  }
  __syncthreads();
  // output rows as 16-byte vectors along the channels
  T *y = static_cast<T *>(a.y);
  const int cvn = a.K / VEC;                 // vectors per pixel
  const int rps = 256 / cvn;                 // pixels per pass
  const int cv = (threadIdx.x % cvn) * VEC, r0 = threadIdx.x / cvn;
  const int valid = a.RB * a.QB;
  if (r0 < rps)
    for (int r = r0; r < valid; r += rps) {
      const int pr = r / a.QB, qc = r - pr * a.QB;
      const size_t pix = ((size_t)n * a.P + p0 + pr) * a.Q + q0 + qc;
      float v[VEC];
#pragma unroll
      for (int e = 0; e < VEC; ++e) v[e] = Cs[r * ldc + cv + e];
      Vec<T>::store(y + pix * a.K + cv, v);
    }
  if (!a.stats) return;
  // BN statistics of the tile: per channel a shift k (the tile's first pixel) and the sums of (y - k), (y - k)^2
  // of the values as stored; G thread rows share the pixels, added in thread-row order
  __shared__ float red[2][256];
  const int G = 256 / a.K;                   // K <= 256 is checked on the host
  const int c = threadIdx.x % a.K, g = threadIdx.x / a.K;
  float s1 = 0.f, s2 = 0.f, kshift = 0.f;
  if (g < G) {
    kshift = Cs[c];
    int r = g;
    for (; r + 3 * G < valid; r += 4 * G) {      // four LDS reads in flight; the sums keep their order
      float t[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) t[u] = Cs[(r + u * G) * ldc + c];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const float sv = as_stored<T>(t[u]) - kshift;
        s1 += sv;
        s2 = fmaf(sv, sv, s2);
      }
    }
    for (; r < valid; r += G) {
      const float sv = as_stored<T>(Cs[r * ldc + c]) - kshift;
      s1 += sv;
      s2 = fmaf(sv, sv, s2);
    }
    red[0][threadIdx.x] = s1;
    red[1][threadIdx.x] = s2;
  }
  __syncthreads();
  if (g == 0) {
    for (int h = 1; h < G; ++h) { s1 += red[0][h * a.K + c]; s2 += red[1][h * a.K + c]; }
    const size_t part = blockIdx.x;
    a.stats[part * a.K + c] = kshift;
    a.stats[((size_t)a.parts + part) * a.K + c] = s1;
    a.stats[((size_t)2 * a.parts + part) * a.K + c] = s2;
  }
}

// dw[k][j] = sum over pixels of dy[pixel][k] * im2col[pixel][j]: GEMM rows = output channels (64 per
// workgroup: blockIdx.y), columns = filter positions, reduction over the pixels.  A workgroup walks a
// contiguous range of tiles; per tile it stages the patch (as the forward kernel) and the output-gradient
// tile [128 pixels][channels] (zero rows past the tile's pixels), and wave w multiplies the pixels
// 32w .. 32w+31 into its own accumulators.  At the end the four waves' accumulators are added in wave
// order and written as this workgroup's partial result.
// MT: 32-channel tiles of this workgroup (1 or 2); NT: 32-column tiles of filter positions (kpad / 32, up to 5)
template <typename T, int MT, int NT>
__global__ __launch_bounds__(256, 2) void stem_wgrad_kernel(StemArgs a) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  constexpr int VEC = 16 / (int)sizeof(T);
  const StemLds L = stem_lds<T>(a, true);
  const float *patch = reinterpret_cast<const float *>(lds + L.patch);
  const int *tab = reinterpret_cast<const int *>(lds + L.tab);
  const int *pixoff = reinterpret_cast<const int *>(lds + L.pixoff);
  T *dyS = reinterpret_cast<T *>(lds + L.op);
  const int k32 = (a.K + 31) / 32 * 32;
  const int ldd = k32 + (sizeof(T) == 2 ? 32 : 4);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lr = lane & 31, kg = lane >> 5;
  const int k0 = (blockIdx.y + a.y0) * 64;   // this workgroup's output channels k0 .. k0 + 32*MT - 1
  const int t0 = (int)((long long)blockIdx.x * a.tiles / gridDim.x);
  const int t1 = (int)((long long)(blockIdx.x + 1) * a.tiles / gridDim.x);
  const int valid = a.RB * a.QB;
  f32x16 acc[MT][NT];
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[m][t][e] = 0.f;
  // transpose read of the output-gradient tile (bf16): lane l supplies row 8*(l/32) + (l%16)/4 of a 16-pixel
  // step and columns 16*((l/16)%2) + 4*(l%4) .. +3 of a 32-channel tile; it receives channel l%32, pixels
  // 8*(l/32) .. +3 (and +4 .. +7 from the second read)
  const int frow = (lane >> 5) * 8 + ((lane & 15) >> 2);
  const int fcol = ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
  for (int tile = t0; tile < t1; ++tile) {
    int n, p0, q0, lead;
    stem_stage<T>(a, L, lds, tile, &n, &p0, &q0, &lead);
    {  // output-gradient tile, eight 16-byte loads in flight per thread
      const T *dy = static_cast<const T *>(a.dy);
      const int vpr = k32 / VEC, total = 128 * vpr;
      const int dq = 256 / vpr, dr = 256 - dq * vpr;
      int r = (int)threadIdx.x / vpr, cv = (int)threadIdx.x - r * vpr;
      for (int base = threadIdx.x; base < total; base += 256 * 8) {
        f32x4 t[8];
        int dst[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          t[u] = f32x4{0.f, 0.f, 0.f, 0.f};
          const int c = cv * VEC;
          if (base + u * 256 < total && r < valid && c < a.K) {
            const int pr = r / a.QB, qc = r - pr * a.QB;
            const size_t pix = ((size_t)n * a.P + p0 + pr) * a.Q + q0 + qc;
            t[u] = *reinterpret_cast<const f32x4 *>(dy + pix * a.K + c);
          }
          dst[u] = r * ldd + c;
          cv += dr; r += dq;
          if (cv >= vpr) { cv -= vpr; ++r; }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
          if (base + u * 256 < total) *reinterpret_cast<f32x4 *>(dyS + dst[u]) = t[u];
      }
    }
    __syncthreads();
    if constexpr (sizeof(T) == 2) {
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {       // this wave's two 16-pixel steps
        const int px = wave * 32 + s2 * 16;
        bf16x8 fa[MT];
#pragma unroll
        for (int m = 0; m < MT; ++m) {
          {
            const __bf16 *base = reinterpret_cast<const __bf16 *>(dyS) + (px + frow) * ldd + k0 + m * 32 + fcol;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(base));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(base + 4 * ldd));
            const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            fa[m] = __builtin_bit_cast(bf16x8, v);
          }
        }
        int po[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) po[e] = pixoff[px + kg * 8 + e] + lead;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          const int tj = tab[t * 32 + lr];
          bf16x8 fb;
#pragma unroll
          for (int e = 0; e < 8; ++e) fb[e] = (__bf16)patch[tj + po[e]];
#pragma unroll
          for (int m = 0; m < MT; ++m) acc[m][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[m], fb, acc[m][t], 0, 0, 0);
        }
      }
    } else {
      const float *dyf = reinterpret_cast<const float *>(dyS);
      for (int s2 = 0; s2 < 16; ++s2) {      // this wave's sixteen 2-pixel steps
        const int px = wave * 32 + s2 * 2 + kg;
        float fa[MT];
#pragma unroll
        for (int m = 0; m < MT; ++m) fa[m] = dyf[px * ldd + k0 + m * 32 + lr];
        const int po = pixoff[px] + lead;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          const float fb = patch[tab[t * 32 + lr] + po];
#pragma unroll
          for (int m = 0; m < MT; ++m) acc[m][t] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[m], fb, acc[m][t], 0, 0, 0);
        }
      }
    }
    __syncthreads();   // before the next tile overwrites patch and gradient tile
  }
  // sum of the four waves' accumulators, in wave order, through LDS (the staging block is free now)
  float *Ds = reinterpret_cast<float *>(lds);          // [64][kpad]
  for (int w = 0; w < 4; ++w) {
    if (wave == w) {
#pragma unroll
      for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int t = 0; t < NT; ++t) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
              const int row = m * 32 + (e >> 2) * 8 + kg * 4 + (e & 3);
              float *d = Ds + row * a.kpad + t * 32 + lr;
              *d = (w == 0 ? 0.f : *d) + acc[m][t][e];
            }
          }
    }
    __syncthreads();
  }
  float *out = a.partial + (size_t)blockIdx.x * a.K * a.kpad;
  const int rows = min(32 * MT, a.K - k0);
  for (int i = threadIdx.x; i < rows * a.kpad / 4; i += 256)
    reinterpret_cast<f32x4 *>(out + (size_t)k0 * a.kpad)[i] = reinterpret_cast<const f32x4 *>(Ds)[i];
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

namespace {
int stem_args(int N, int C, int H, int W, int K, int R, int stride, int pad, int P, int Q, int kpad, StemArgs *out) {
  StemArgs a{};
  a.N = N; a.C = C; a.H = H; a.W = W; a.K = K; a.R = R; a.stride = stride; a.pad = pad; a.P = P; a.Q = Q;
  a.taps = R * R * C; a.kpad = kpad;
  if (N < 1 || C < 1 || C > 4 || K < 16 || K % 16 || K > 128 || kpad % 32 || kpad < a.taps || kpad > 160 || P < 1 || Q < 1)
    return set_error(RESIST_ESHAPE, "stem convolution: C=%d K=%d filter %dx%d (1 <= C <= 4, K a multiple of 16 up to 128, "
                                    "at most 160 filter positions)", C, K, R, R);
  // tile: QB output columns x RB output rows, QB | Q, RB | P, RB * QB <= 128
  int qb = 1, rb = 1;
  for (int d = 1; d <= Q && d <= 128; ++d)
    if (Q % d == 0) qb = d;
  for (int d = 1; d <= P && d * qb <= 128; ++d)
    if (P % d == 0) rb = d;
  a.QB = qb; a.RB = rb;
  a.PH = (rb - 1) * stride + R; a.PW = (qb - 1) * stride + R;
  a.PWp = a.PW; a.vec = 0;
  a.tiles_q = Q / qb; a.tiles_p = P / rb;
  const long long tiles = (long long)N * a.tiles_q * a.tiles_p;
  if (tiles > 0x7fffffffLL) return set_error(RESIST_ESHAPE, "stem convolution: %lld tiles", tiles);
  a.tiles = (int)tiles;
  a.zn = (rb - 1) * stride * a.PW + (qb - 1) * stride + 1;
  *out = a;
  return RESIST_OK;
}
// once the image pointer is known: vector mode where the rows allow it
inline void stem_set_mode(StemArgs &a, bool allow_vec = true) {
  a.vec = allow_vec && (a.W % 4 == 0) && (((uintptr_t)a.x & 15) == 0) ? 1 : 0;
  a.PWp = a.vec ? (a.PW + 3 + 3) / 4 * 4 : a.PW;
  a.zn = (a.RB - 1) * a.stride * a.PWp + (a.QB - 1) * a.stride + 1 + (a.vec ? 3 : 0);
}
constexpr int kStemLdsLimit = 64 * 1024;   // dynamic LDS a kernel gets without asking for more
inline int stem_wgrad_groups(const StemArgs &a) { return a.tiles < 512 ? a.tiles : 512; }
}  // namespace

StatParts stem_stat_parts(int N, int C, int H, int W, int K, int R, int stride, int pad, int P, int Q, int kpad) {
  StemArgs a;
  StatParts sp;
  if (stem_args(N, C, H, W, K, R, stride, pad, P, Q, kpad, &a) == RESIST_OK) { sp.parts = a.tiles; sp.rows = a.RB * a.QB; }
  return sp;
}

int64_t stem_wgrad_scratch_floats(int N, int C, int H, int W, int K, int R, int stride, int pad, int P, int Q, int kpad) {
  StemArgs a;
  if (stem_args(N, C, H, W, K, R, stride, pad, P, Q, kpad, &a) != RESIST_OK) return 0;
  return (int64_t)stem_wgrad_groups(a) * K * kpad;
}

int stem_conv_fwd(int dt, const float *x, const void *wpad, void *y, float *stats, StatParts *stat_parts, int N, int C, int H,
                  int W, int K, int R, int stride, int pad, int P, int Q, int kpad, hipStream_t st) {
  StemArgs a;
  RESIST_TRY(stem_args(N, C, H, W, K, R, stride, pad, P, Q, kpad, &a));
  if (stats && !stat_parts) return set_error(RESIST_EINVAL, "stem_conv_fwd: stats without stat_parts");
  a.x = x; a.wpad = wpad; a.y = y; a.stats = stats; a.parts = a.tiles;
  stem_set_mode(a);
  if (stat_parts) { stat_parts->parts = a.tiles; stat_parts->rows = a.RB * a.QB; }
  int lds = dt == DT_BF16 ? stem_lds<__bf16>(a, false).total : stem_lds<float>(a, false).total;
  if (lds > kStemLdsLimit && a.vec) {   // the wider patch rows of vector mode do not fit: one word at a time
    stem_set_mode(a, false);
    lds = dt == DT_BF16 ? stem_lds<__bf16>(a, false).total : stem_lds<float>(a, false).total;
  }
  if (lds > kStemLdsLimit) return set_error(RESIST_ESHAPE, "stem convolution: tile needs %d bytes of LDS", lds);
  const double flops = 2.0 * N * P * Q * K * a.taps;
  prof::Scope ps(dt == DT_BF16 ? "stem_conv_bf16_fwd" : "stem_conv_f32_fwd", flops,
                 4.0 * N * C * H * W + (double)esize(dt) * ((double)N * P * Q * K + (double)K * kpad), st);
  const int ntiles = (a.K + 31) / 32;        // 1..4: K <= 128 was checked above
#define RESIST_STEM_FWD(NTILES)                                                                                  \
  do {                                                                                                           \
    if (dt == DT_BF16) hipLaunchKernelGGL((stem_fwd_kernel<__bf16, NTILES>), dim3(a.tiles), dim3(256), lds, st, a); \
    else hipLaunchKernelGGL((stem_fwd_kernel<float, NTILES>), dim3(a.tiles), dim3(256), lds, st, a);             \
  } while (0)
  if (ntiles == 1) RESIST_STEM_FWD(1);
  else if (ntiles == 2) RESIST_STEM_FWD(2);
  else if (ntiles == 3) RESIST_STEM_FWD(3);
  else RESIST_STEM_FWD(4);
#undef RESIST_STEM_FWD
  RESIST_CHECK_LAUNCH("stem_conv_fwd");
  return RESIST_OK;
}

namespace {
template <int MT>
int launch_stem_wgrad(int dt, StemArgs a, dim3 grid, int lds, int y0, hipStream_t st) {
  a.y0 = y0;
#define RESIST_STEM_WGRAD(NT)                                                                                  \
  case NT:                                                                                                     \
    if (dt == DT_BF16) hipLaunchKernelGGL((stem_wgrad_kernel<__bf16, MT, NT>), grid, dim3(256), lds, st, a);   \
    else hipLaunchKernelGGL((stem_wgrad_kernel<float, MT, NT>), grid, dim3(256), lds, st, a);                  \
    break;
  switch (a.kpad / 32) {
    RESIST_STEM_WGRAD(1) RESIST_STEM_WGRAD(2) RESIST_STEM_WGRAD(3) RESIST_STEM_WGRAD(4) RESIST_STEM_WGRAD(5)
    default: return set_error(RESIST_ESHAPE, "stem weight gradient: %d filter positions", a.kpad);
  }
#undef RESIST_STEM_WGRAD
  RESIST_CHECK_LAUNCH("stem_conv_wgrad");
  return RESIST_OK;
}
}  // namespace

int stem_conv_wgrad(int dt, const void *dy, const float *x, float *dwpad, float *partial, int N, int C, int H, int W, int K,
                    int R, int stride, int pad, int P, int Q, int kpad, hipStream_t st) {
  StemArgs a;
  RESIST_TRY(stem_args(N, C, H, W, K, R, stride, pad, P, Q, kpad, &a));
  if (!partial) return set_error(RESIST_EWORKSPACE, "stem weight gradient needs its partial-sum scratch");
  a.x = x; a.dy = dy; a.partial = partial;
  stem_set_mode(a);
  const int groups = stem_wgrad_groups(a);
  a.parts = groups;
  int lds = dt == DT_BF16 ? stem_lds<__bf16>(a, true).total : stem_lds<float>(a, true).total;
  if (lds > kStemLdsLimit && a.vec) {
    stem_set_mode(a, false);
    lds = dt == DT_BF16 ? stem_lds<__bf16>(a, true).total : stem_lds<float>(a, true).total;
  }
  if (lds > kStemLdsLimit) return set_error(RESIST_ESHAPE, "stem weight gradient: tile needs %d bytes of LDS", lds);
  {
    const double flops = 2.0 * N * P * Q * K * a.taps;
    prof::Scope ps(dt == DT_BF16 ? "stem_wgrad_bf16" : "stem_wgrad_f32", flops,
                   4.0 * N * C * H * W + (double)esize(dt) * N * P * Q * K + 4.0 * K * kpad, st);
    // workgroups along y own 64 output channels each (two 32-channel tiles); a last group of 32 channels
    // (K = 32, 96) gets its own launch with one tile
    const int k32 = (K + 31) / 32 * 32;
    const int pairs = k32 / 64, odd = (k32 / 32) & 1;
    if (pairs > 0) RESIST_TRY(launch_stem_wgrad<2>(dt, a, dim3(groups, pairs), lds, 0, st));
    if (odd) RESIST_TRY(launch_stem_wgrad<1>(dt, a, dim3(groups, 1), lds, pairs, st));
  }
  return splitk_reduce(partial, dwpad, (long long)K * kpad / 4, groups, st);
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
