// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "resist.h"
#include "resist_ops.h"

namespace resist {

int set_error(int code, const char *fmt, ...);
#define RESIST_CHECK_HIP(expr)                                                          \
  do {                                                                                  \
    hipError_t e__ = (expr);                                                            \
    if (e__ != hipSuccess)                                                              \
      return ::resist::set_error(RESIST_EHIP, "%s: %s", #expr, hipGetErrorString(e__)); \
  } while (0)
#define RESIST_CHECK_LAUNCH(name)                                                        \
  do {                                                                                   \
    hipError_t e__ = hipGetLastError();                                                  \
    if (e__ != hipSuccess)                                                               \
      return ::resist::set_error(RESIST_EHIP, "launch %s: %s", name, hipGetErrorString(e__)); \
  } while (0)
#define RESIST_TRY(expr)      \
  do {                        \
    int rc__ = (expr);        \
    if (rc__ != 0) return rc__; \
  } while (0)

// ---- optional per-kernel event timing (prof.cpp) ----------------------------------------------
namespace prof {
bool enabled();
struct Scope {   // brackets the launches made during its lifetime with two events on `st`
  Scope(const char *label, double flops, double bytes, hipStream_t st);
  ~Scope();
  hipStream_t st_;
  int idx_;
};
}  // namespace prof

// ---- side stream for work off a step's critical path (overlap.cpp) -----------------------------
int overlap_mode();   // resist_set_overlap(): 0 off, 1 for steps with enough work (default), 2 always
int bn_fusion_mode(); // resist_set_bn_fusion(): 0 never, 1 in bf16 steps (default), 2 always
class SideStream {
 public:
  SideStream(hipStream_t main, bool enable);   // enable == false, or no stream to be had: every call below is a no-op
  bool on() const { return side_ != nullptr; }
  hipStream_t stream() const { return side_ ? side_ : main_; }   // where the off-path work goes
  hipStream_t main() const { return main_; }
  int fork();                     // the side stream waits for everything enqueued on the main stream so far
  int mark(hipEvent_t *ev);       // *ev: completes when everything enqueued on the side stream so far has
  int main_wait(hipEvent_t ev);   // the main stream waits for ev (NULL: nothing to wait for)
  int join();                     // the main stream waits for everything enqueued on the side stream

 private:
  hipEvent_t take();
  hipStream_t main_, side_;
  int dev_;
};

// ---- static description of the global network -------------------------------------------------
struct BlockShape {
  int stage, index;         // position
  int c_in, width, c_out;   // channels
  int stride;               // 1 or 2 (on the 3x3 convolution)
  bool has_ds;              // conv1x1(stride)+BN shortcut
  int h_in, w_in, h_out, w_out;
};

struct TensorSlot {  // one tensor inside a block buffer
  int kind, layer;
  int64_t offset, count;
  int dims[4];
};

struct BlockLayout {
  std::vector<TensorSlot> slots;
  int64_t n_total = 0, n_trainable = 0;
  // find offset of (kind, layer); -1 if absent
  int64_t off(int kind, int layer) const {
    for (const auto &s : slots)
      if (s.kind == kind && s.layer == layer) return s.offset;
    return -1;
  }
};

struct Net {
  resist_model_desc d;
  std::vector<BlockShape> blocks;   // B entries
  std::vector<int> stage_first;     // first block index of each stage
  int stem_rs, stem_stride, stem_pad;
  int stem_h, stem_w;               // stem conv output spatial size
  int body_h, body_w;               // after optional max-pool
  int head_c;                       // channels entering the head
  int expansion;
  bool preact;       // BN-ReLU before every convolution, no ReLU after the add (block_kind 2, 3)
  bool bottleneck;   // 1x1-3x3-1x1 blocks with expansion 4 (block_kind 1, 3)
};

int build_net(const resist_model_desc *desc, Net *net);          // validates
int block_layout(const Net &net, int block, BlockLayout *out);   // block in [-1, B]

enum { T_CONVW = 0, T_GAMMA = 1, T_BETA = 2, T_RMEAN = 3, T_RVAR = 4, T_FCW = 5, T_FCB = 6 };

// ---- kernels (launchers return a resist_status) -----------------------------------------------
struct ConvGeom {
  int N, H, W, C;   // input activation (NHWC)
  int K, R, S;      // filter
  int stride, pad;
  int P, Q;         // output spatial
};
inline ConvGeom make_geom(int N, int H, int W, int C, int K, int R, int stride, int pad) {
  ConvGeom g{N, H, W, C, K, R, R, stride, pad, 0, 0};
  g.P = (H + 2 * pad - R) / stride + 1;
  g.Q = (W + 2 * pad - R) / stride + 1;
  return g;
}

// Element types of activations / filters inside the library
enum { DT_F32 = 0, DT_BF16 = 1 };
inline int esize(int dt) { return dt == DT_BF16 ? 2 : 4; }

// implicit-GEMM convolution family (conv.hip); dt selects fp32 or bf16 tensors (fp32 accumulation)
// shape limits of the convolution kernels (channel multiples, filter sizes, tensors below 2 GiB); host only
int conv_check(const ConvGeom &g, int dt);
// y = conv(x, w) [+ addend].  stats (optional): per row tile (stat_parts->rows rows each, the last one
// ragged) and column a shift k, sum(y - k) and sum((y - k)^2) of y as stored, [3][stat_parts->parts][K]
// floats (capacity conv_stats_floats(g)); input of bn_finalize
struct StatParts { int parts = 0; int rows = 0; };
int64_t conv_stats_floats(const ConvGeom &g);
int conv_fwd(const ConvGeom &g, int dt, const void *x, const void *w, void *y, const void *addend, float *stats,
             StatParts *stat_parts, hipStream_t st);
// dx = dgrad(dy, wT) [+ addend]; wT is the [C][R][S][K] transpose made by prepare_filter.  relu_mask
// (optional, indexed like dx): the output of the ReLU that produced the convolution's input; dx is set
// to zero where it is not positive, i.e. the gradient leaves this kernel already taken through that ReLU
// bn (optional, stride 1 only): the convolution's input was the output of a BN (+ReLU); the kernel also
// leaves the first pass of that BN's backward, per row tile: sum(gm) and sum(gm * xhat) of the dx it stores
// against the BN's input y, in bn->sums [2][parts][C] (gm = dx, or dx where the BN's own ReLU passed),
// and says in bn->parts how many row tiles of how many rows it used.  bn_backward takes them as pre_sums.
struct BnBwdFuse;
int conv_dgrad(const ConvGeom &g, int dt, const void *dy, const void *wT, void *dx, const void *addend,
               const void *relu_mask, hipStream_t st, const BnBwdFuse *bn = nullptr);
int64_t conv_dgrad_bn_sums_floats(const ConvGeom &g);
// from a filter stored in src_dt: optional copy in dt (w_lp) and optional transpose in dt (wT)
int prepare_filter(const ConvGeom &g, int src_dt, int dt, const void *w, void *w_lp, void *wT, hipStream_t st);
// the same for many filters at once (fp32 masters -> copies and transposes in dt, times `scale`)
struct FilterPrep { ConvGeom g; const float *w; void *w_lp; void *wT; float scale = 1.f; };
int prepare_filters(const std::vector<FilterPrep> &items, int dt, hipStream_t st);
// dw (fp32) = wgrad(dy, x); partial: split-reduction scratch of wgrad_scratch_floats(g) floats
int64_t wgrad_scratch_floats(const ConvGeom &g);
int conv_wgrad(const ConvGeom &g, int dt, const void *dy, const void *x, float *dw, float *partial,
               hipStream_t st);
// the same with the split partial sums in the library's static device array (no allocation anywhere);
// RESIST_EWORKSPACE when wgrad_scratch_floats(g) * 4 exceeds wgrad_static_scratch_bytes()
int64_t wgrad_static_scratch_bytes();
int conv_wgrad_static(const ConvGeom &g, int dt, const void *dy, const void *x, float *dw, hipStream_t st);

// stem convolution as an implicit GEMM on the NCHW fp32 image (stem.hip).  wpad: filter [K][kpad] in dt with
// zero columns past R*R*C (pad_rows); y: [N][P][Q][K] in dt; stats as for conv_fwd (one part per tile of
// the kernel: stem_stat_parts).  Weight gradient: dwpad [K][kpad] fp32 (then unpad_rows_f32), partial:
// scratch of stem_wgrad_scratch_floats floats.  Limits: C <= 4, K a multiple of 16 up to 128, kpad <= 160.
StatParts stem_stat_parts(int N, int C, int H, int W, int K, int R, int stride, int pad, int P, int Q, int kpad);
int64_t stem_wgrad_scratch_floats(int N, int C, int H, int W, int K, int R, int stride, int pad, int P, int Q, int kpad);
int stem_conv_fwd(int dt, const float *x_nchw, const void *wpad, void *y, float *stats, StatParts *stat_parts, int N, int C,
                  int H, int W, int K, int R, int stride, int pad, int P, int Q, int kpad, hipStream_t st);
int stem_conv_wgrad(int dt, const void *dy, const float *x_nchw, float *dwpad, float *partial, int N, int C, int H, int W,
                    int K, int R, int stride, int pad, int P, int Q, int kpad, hipStream_t st);
// out[i] = sum over z < splits of part[z*n4 + i] (float4 elements), fixed order (conv.hip)
int splitk_reduce(const float *part, float *out, long long n4, int splits, hipStream_t st);
int pad_rows(int dt, const float *src, void *dst, int rows, int n, int npad, hipStream_t st);   // fp32 [rows][n] -> dt [rows][npad]
int unpad_rows_f32(const float *src, float *dst, int rows, int n, int npad, hipStream_t st);    // [rows][npad] -> [rows][n]

// BatchNorm on [M][C] activations in dt, fp32 arithmetic (bn.hip)
struct BnBufs {
  const float *gamma, *beta;
  float *rmean, *rvar;       // running statistics (updated by bn_finalize)
  float *mean, *invstd;      // [C] saved batch statistics
  float *scale, *shift;      // [C] gamma*invstd and beta - mean*gamma*invstd (written by bn_finalize)
  float *dgamma, *dbeta;     // [C] gradient outputs
};
int64_t bn_scratch_doubles(int C);   // partial-sum scratch for one bn_finalize or bn_backward call
// batch statistics from the per-tile sums a convolution left behind: mean, 1/sqrt(var+eps), the
// affine map of bn_apply, and the running statistics
int bn_finalize(const float *stats, StatParts parts, int64_t M, int C, const BnBufs &b, float eps, float momentum,
                double *scratch, hipStream_t st);
// evaluation mode: scale/shift from the running statistics, both multiplied by s
int bn_eval_affine(int C, const BnBufs &b, float eps, float s, hipStream_t st);
// a = [relu]( scale*y + shift [+ res] )            res: raw tensor, or BN(res_y) if res_bn given
int bn_apply(int dt, const void *y, int64_t M, int C, const BnBufs &b, const void *res,
             const BnBufs *res_bn, bool relu, void *a, hipStream_t st);
// gm = g, or (relu_of_self) g where this BN's own output scale*y + shift is positive -- the forward ReLU
// decision recomputed with the same arithmetic -- and 0 elsewhere; dbeta = sum gm; dgamma = sum gm*xhat(y);
// dy = gamma*invstd*(gm - dbeta/M - xhat*dgamma/M) [+ addend].  (A ReLU behind a block's last BN is
// applied by whoever produces g: see conv_dgrad's relu_mask and avgpool_bwd.)
// pre_sums (optional): the first pass already done by the data gradient that produced g
// ([2][pre.parts][C] floats, see conv_dgrad); then only the per-channel totals and the second pass run.
int bn_backward(int dt, const void *g, bool relu_of_self, const void *y, int64_t M, int C, const BnBufs &b, void *dy,
                const void *addend, double *scratch, hipStream_t st, const float *pre_sums = nullptr,
                StatParts pre = StatParts{});
struct BnBwdFuse {
  const void *y;        // the BN's input, [M][C] in the compute type
  BnBufs b;             // mean, invstd, scale, shift are read
  bool relu_of_self;    // the BN's output went through its own ReLU
  float *sums;          // [2][parts][C]
  StatParts *parts;     // out
};

// pooling / head / loss (head.hip); pooled features, logits and the loss stay fp32
int maxpool_fwd(int dt, const void *x, void *y, uint8_t *argmax, int N, int H, int W, int C, int P,
                int Q, hipStream_t st);
int maxpool_bwd(int dt, const void *dy, const uint8_t *argmax, void *dx, int N, int H, int W, int C,
                int P, int Q, hipStream_t st);
int avgpool_fwd(int dt, const void *x, float *y, int N, int HW, int C, hipStream_t st);
// dx = dy / HW broadcast over the positions; relu_mask (optional, indexed like dx): zero where it is not positive
int avgpool_bwd(int dt, const float *dy, const void *relu_mask, void *dx, int N, int HW, int C, hipStream_t st);
int fc_fwd_f32(const float *x, const float *w, const float *b, float *z, int N, int C, int J,
               hipStream_t st);
// backward of the fully connected layer in two parts: the gradient the chain continues with, and the parameter
// gradients, which only the update reads
int fc_bwd_dx_f32(const float *dz, const float *w, float *dx, int N, int C, int J, hipStream_t st);
int fc_bwd_params_f32(const float *dz, const float *x, float *dw, float *db, int N, int C, int J, hipStream_t st);
// per-sample losses and dz = (softmax - onehot) / N; the mean of the per-sample losses on its own
int softmax_ce_f32(const float *z, const int32_t *labels, float *dz, float *row_loss, int N, int J, hipStream_t st);
int mean_loss_f32(const float *row_loss, float *loss, int N, hipStream_t st);

// update / reassembly (update.hip)
struct SgdSeg { float *w; float *v; const float *g; int64_t n; };
int sgd_momentum_f32(const std::vector<SgdSeg> &segs, float lr, float mu, float wd, hipStream_t st);
struct AggSeg { float *dst; const float *src[16]; int count; int64_t n; };
int aggregate_f32(const std::vector<AggSeg> &segs, hipStream_t st);
int fill_zero_f32(float *p, int64_t n, hipStream_t st);

}  // namespace resist
