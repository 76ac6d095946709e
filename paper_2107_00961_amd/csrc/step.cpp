// resist_local_step: one SGD iteration of one sub-ResNet (the paper's Algorithm 1, inner loop),
// resist_workspace_bytes, and resist_aggregate (Sec. 2.3).  Host-side orchestration only: this file
// lays out the workspace, walks the kept blocks forward and backward, and enqueues the kernels.
// A block that is not in the list is simply not launched -- the residual stream passes through
// (Appendix B, forward recursion with mask 0).
#include <algorithm>
#include <cstdlib>

#include "internal.h"

namespace resist {
namespace {

inline double geom_flops(const ConvGeom &g) { return 2.0 * g.N * g.P * g.Q * g.K * g.C * g.R * g.S; }

// Weight gradients feed only the update at the end of a step; they run on a side stream next to the
// chain data gradient -> BN backward -> next layer, whose short kernels then overlap with them.  A
// weight gradient starts once its output gradient is complete (fork), and a buffer it reads is not
// overwritten before it has finished (before_write).
struct WgradSide {
  SideStream side;
  int dt;
  float *splitk;
  std::vector<std::pair<const void *, hipEvent_t>> readers;   // buffer -> its last reader on the side stream
  // `flops`: convolution work of the step.  Below ~20 GFLOP a step is bound by launch latency and the
  // event calls of the second stream cost more than the overlap returns: everything stays on `main`.
  WgradSide(hipStream_t main, int dt_, float *splitk_, double flops)
      : side(main, overlap_mode() == 2 || (overlap_mode() == 1 && flops >= 2e10)), dt(dt_), splitk(splitk_) {}
  hipStream_t stream() const { return side.stream(); }
  int launch(const ConvGeom &g, const void *dyb, const void *xin, float *dw) {
    RESIST_TRY(side.fork());
    RESIST_TRY(conv_wgrad(g, dt, dyb, xin, dw, splitk, side.stream()));
    hipEvent_t e = nullptr;
    RESIST_TRY(side.mark(&e));
    for (auto &r : readers)
      if (r.first == dyb) { r.second = e; return RESIST_OK; }
    readers.emplace_back(dyb, e);
    return RESIST_OK;
  }
  // the stem's weight gradient (implicit GEMM on the input image), same ordering rules
  int launch_stem(const Net &net, int N, int kpad, const void *dyb, const float *x, float *dwpad) {
    RESIST_TRY(side.fork());
    RESIST_TRY(stem_conv_wgrad(dt, dyb, x, dwpad, splitk, N, net.d.in_c, net.d.in_h, net.d.in_w, net.d.width[0], net.stem_rs,
                               net.stem_stride, net.stem_pad, net.stem_h, net.stem_w, kpad, side.stream()));
    hipEvent_t e = nullptr;
    RESIST_TRY(side.mark(&e));
    for (auto &r : readers)
      if (r.first == dyb) { r.second = e; return RESIST_OK; }
    readers.emplace_back(dyb, e);
    return RESIST_OK;
  }
  int before_write(const void *buf) {
    for (auto &r : readers)
      if (r.first == buf && r.second) { RESIST_TRY(side.main_wait(r.second)); r.second = nullptr; }
    return RESIST_OK;
  }
  // Filter copies and transposes.  In fp32 mode the forward pass multiplies the master filters, so the
  // transposes are first needed by the backward pass: made on the side stream while the forward runs.
  hipEvent_t prepared = nullptr;
  int prepare(const std::vector<FilterPrep> &prep) {
    if (dt != DT_F32 || !side.on()) return prepare_filters(prep, dt, side.main());
    RESIST_TRY(side.fork());
    RESIST_TRY(prepare_filters(prep, dt, side.stream()));
    return side.mark(&prepared);
  }
  int filters_ready() {   // before the first data gradient
    RESIST_TRY(side.main_wait(prepared));
    prepared = nullptr;
    return RESIST_OK;
  }
  // work that only the update or the caller reads (parameter gradients of the head, the mean loss), enqueued by
  // f(stream): off the chain like the weight gradients; what it reads must stay untouched until the join
  template <typename F> int off_chain(F &&f) {
    RESIST_TRY(side.fork());
    return f(side.stream());
  }
  bool joined = false;
  int join() {
    joined = true;
    return side.join();
  }
  // an error return in mid-step still leaves the caller's stream ordered after the side stream's work
  ~WgradSide() {
    if (!joined) (void)side.join();
  }
};

struct Arena {
  char *base;
  int64_t off = 0;
  explicit Arena(void *b) : base((char *)b) {}
  template <typename T>
  T *take(int64_t count) {
    off = (off + 255) & ~(int64_t)255;
    T *p = (T *)(base + off);   // with base == NULL this is only an offset; never dereferenced
    off += count * (int64_t)sizeof(T);
    return p;
  }
  // `count` activation elements of `es` bytes each
  void *take_act(int64_t count, int es) { return take<char>(count * es); }
};

struct ConvLayer {
  ConvGeom g;
  int64_t w_off, gamma_off, beta_off, rmean_off, rvar_off;  // offsets inside the block buffer
  const void *in = nullptr;  // activations are stored in the model's compute type (fp32 or bf16)
  void *y = nullptr;         // pre-BN output
  void *a = nullptr;         // post-BN(+ReLU) output; NULL for the layer that ends a block
  float *mean = nullptr, *invstd = nullptr, *scale = nullptr, *shift = nullptr;   // [K] each
  void *wlp = nullptr;       // the filter in the compute type (bf16 mode; fp32 mode multiplies the master)
  void *wT = nullptr;        // [C][R][S][K] transpose in the compute type, for the data gradient
  int64_t M() const { return (int64_t)g.N * g.P * g.Q; }
};

struct BlockPlan {
  int slot;                 // index into block_params (1 + position in `blocks`)
  std::vector<ConvLayer> convs;
  bool has_ds = false;
  ConvLayer ds;
  const void *in = nullptr;
  void *out = nullptr;
  int64_t out_elems = 0;
};

struct StepPlan {
  Net net;
  int batch = 0;
  std::vector<BlockLayout> layouts;   // per slot: stem, blocks..., head
  // stem
  int kpad = 0;
  ConvLayer stem;                     // the stem as a GEMM over kpad filter positions (geometry for sizes only)
  void *wpad = nullptr;               // the filter [K][kpad] in the compute type
  float *dwpad = nullptr;
  void *stem_pool = nullptr;
  uint8_t *stem_argmax = nullptr;
  std::vector<BlockPlan> blocks;
  // head
  float *pooled = nullptr, *z = nullptr, *dz = nullptr, *row_loss = nullptr, *dpooled = nullptr;
  const void *feat = nullptr;
  int feat_hw = 0;
  // shared scratch
  void *gbuf[2] = {nullptr, nullptr}, *gm = nullptr, *dy0 = nullptr, *dy1 = nullptr, *da = nullptr;
  float *splitk = nullptr;
  float *stats = nullptr;             // per-tile column sums left by a forward convolution
  double *bn_scratch = nullptr;
  float *stats_ds = nullptr;          // the same two for a shortcut convolution, whose forward pass runs next to
  double *bn_scratch_ds = nullptr;    // its block's residual branch
  std::vector<float *> own_grads;     // per slot, when the caller passes no gradient buffers
  int64_t bytes = 0;
};

// split-reduction scratch and statistics capacity the stem convolution needs
int64_t stem_scratch_floats(const Net &net, int N, int kpad) {
  return stem_wgrad_scratch_floats(N, net.d.in_c, net.d.in_h, net.d.in_w, net.d.width[0], net.stem_rs, net.stem_stride,
                                   net.stem_pad, net.stem_h, net.stem_w, kpad);
}
int64_t stem_stats_floats(const Net &net, int N, int kpad) {
  const StatParts sp = stem_stat_parts(N, net.d.in_c, net.d.in_h, net.d.in_w, net.d.width[0], net.stem_rs, net.stem_stride,
                                       net.stem_pad, net.stem_h, net.stem_w, kpad);
  return (int64_t)3 * sp.parts * net.d.width[0];
}
int stem_forward(const Net &net, int dt, int N, int kpad, const float *x, const void *wpad, void *y, float *stats,
                 StatParts *parts, hipStream_t st) {
  return stem_conv_fwd(dt, x, wpad, y, stats, parts, N, net.d.in_c, net.d.in_h, net.d.in_w, net.d.width[0], net.stem_rs,
                       net.stem_stride, net.stem_pad, net.stem_h, net.stem_w, kpad, st);
}

ConvLayer make_conv(const BlockLayout &L, int layer, int N, int H, int W, int C, int K, int R, int stride, int pad) {
  ConvLayer c;
  c.g = make_geom(N, H, W, C, K, R, stride, pad);
  c.w_off = L.off(T_CONVW, layer);
  c.gamma_off = L.off(T_GAMMA, layer);
  c.beta_off = L.off(T_BETA, layer);
  c.rmean_off = L.off(T_RMEAN, layer);
  c.rvar_off = L.off(T_RVAR, layer);
  return c;
}

int check_block_list(const Net &net, const int32_t *blocks, int32_t nblocks, int32_t batch) {
  const int B = (int)net.blocks.size();
  if (batch < 1) return set_error(RESIST_EINVAL, "batch=%d", batch);
  if (nblocks < 0 || (nblocks > 0 && !blocks)) return set_error(RESIST_EINVAL, "blocks/nblocks");
  for (int i = 0; i < nblocks; ++i) {
    if (blocks[i] < 0 || blocks[i] >= B) return set_error(RESIST_EINVAL, "blocks[%d]=%d outside [0,%d)", i, blocks[i], B);
    if (i > 0 && blocks[i] <= blocks[i - 1]) return set_error(RESIST_EINVAL, "blocks must be strictly ascending");
  }
  for (int f : net.stage_first)
    if (!std::binary_search(blocks, blocks + nblocks, f))
      return set_error(RESIST_ESHAPE, "first block %d of a stage is missing: the residual stream would change shape", f);
  return RESIST_OK;
}

int build_plan(const resist_model_desc *desc, const int32_t *blocks, int32_t nblocks, int32_t batch, void *ws,
               StepPlan *P) {
  RESIST_TRY(build_net(desc, &P->net));
  const Net &net = P->net;
  RESIST_TRY(check_block_list(net, blocks, nblocks, batch));
  const int B = (int)net.blocks.size();
  P->batch = batch;
  const int N = batch;
  const int es = esize(net.d.compute_dtype);
  Arena A(ws);

  P->layouts.resize(nblocks + 2);
  RESIST_TRY(block_layout(net, -1, &P->layouts[0]));
  for (int i = 0; i < nblocks; ++i) RESIST_TRY(block_layout(net, blocks[i], &P->layouts[i + 1]));
  RESIST_TRY(block_layout(net, B, &P->layouts[nblocks + 1]));

  int64_t max_act = 0, max_splitk = 0, max_stats = 0, max_stats_ds = 0;
  auto take_filters = [&](ConvLayer &c) {
    const int64_t n = (int64_t)c.g.K * c.g.R * c.g.S * c.g.C;
    c.wT = A.take_act(n, es);
    if (net.d.compute_dtype == DT_BF16) c.wlp = A.take_act(n, es);
  };
  auto take_bn = [&](ConvLayer &c) {
    float *p = A.take<float>((int64_t)4 * c.g.K);
    c.mean = p; c.invstd = p + c.g.K; c.scale = p + 2 * c.g.K; c.shift = p + 3 * c.g.K;
    max_stats = std::max<int64_t>(max_stats, conv_stats_floats(c.g));
  };
  int max_c = 16;
  int shape_rc = RESIST_OK;   // every convolution is checked here, before anything is launched
  auto track = [&](const ConvLayer &c, bool needs_dgrad) {
    if (shape_rc == RESIST_OK) shape_rc = conv_check(c.g, net.d.compute_dtype);
    max_act = std::max<int64_t>(max_act, c.M() * c.g.K);
    max_act = std::max<int64_t>(max_act, (int64_t)c.g.N * c.g.H * c.g.W * c.g.C);
    (void)needs_dgrad;
    max_splitk = std::max<int64_t>(max_splitk, wgrad_scratch_floats(c.g));
    max_c = std::max(max_c, c.g.K);
  };

  // ---- stem: implicit GEMM on the input image, kpad filter positions
  {
    const int taps = net.stem_rs * net.stem_rs * net.d.in_c;
    P->kpad = (taps + 31) / 32 * 32;
    const int K0 = net.d.width[0];
    ConvLayer &s = P->stem;
    s = make_conv(P->layouts[0], 0, N, net.stem_h, net.stem_w, P->kpad, K0, 1, 1, 0);
    P->wpad = A.take_act((int64_t)K0 * P->kpad, es);
    P->dwpad = A.take<float>((int64_t)K0 * P->kpad);
    s.y = A.take_act(s.M() * K0, es);
    s.a = A.take_act(s.M() * K0, es);
    take_bn(s);
    if (stem_scratch_floats(net, N, P->kpad) == 0) return RESIST_ESHAPE;   // message set by the stem's shape check
    max_act = std::max<int64_t>(max_act, s.M() * K0);
    max_splitk = std::max<int64_t>(max_splitk, stem_scratch_floats(net, N, P->kpad));
    max_stats = std::max<int64_t>(max_stats, stem_stats_floats(net, N, P->kpad));
    max_c = std::max(max_c, K0);
    if (net.d.stem_kind == 1) {
      const int64_t n = (int64_t)N * net.body_h * net.body_w * K0;
      P->stem_pool = A.take_act(n, es);
      P->stem_argmax = A.take<uint8_t>(n);
    }
  }
  const void *cur = net.d.stem_kind == 1 ? P->stem_pool : P->stem.a;

  // ---- residual blocks the sub-ResNet keeps
  P->blocks.resize(nblocks);
  for (int i = 0; i < nblocks; ++i) {
    const BlockShape &bs = net.blocks[blocks[i]];
    const BlockLayout &L = P->layouts[i + 1];
    BlockPlan &bp = P->blocks[i];
    bp.slot = i + 1;
    bp.in = cur;
    if (!net.bottleneck) {
      bp.convs.push_back(make_conv(L, 0, N, bs.h_in, bs.w_in, bs.c_in, bs.width, 3, bs.stride, 1));
      bp.convs.push_back(make_conv(L, 1, N, bs.h_out, bs.w_out, bs.width, bs.c_out, 3, 1, 1));
    } else {
      bp.convs.push_back(make_conv(L, 0, N, bs.h_in, bs.w_in, bs.c_in, bs.width, 1, 1, 0));
      bp.convs.push_back(make_conv(L, 1, N, bs.h_in, bs.w_in, bs.width, bs.width, 3, bs.stride, 1));
      bp.convs.push_back(make_conv(L, 2, N, bs.h_out, bs.w_out, bs.width, bs.c_out, 1, 1, 0));
    }
    const void *x = bp.in;
    for (size_t j = 0; j < bp.convs.size(); ++j) {
      ConvLayer &c = bp.convs[j];
      c.in = x;
      c.y = A.take_act(c.M() * c.g.K, es);
      take_bn(c);
      take_filters(c);
      if (j + 1 < bp.convs.size()) {
        c.a = A.take_act(c.M() * c.g.K, es);
        x = c.a;
      }
      track(c, true);
    }
    bp.has_ds = bs.has_ds;
    if (bs.has_ds) {
      ConvLayer &d = bp.ds;
      d = make_conv(L, 3, N, bs.h_in, bs.w_in, bs.c_in, bs.c_out, 1, bs.stride, 0);
      d.in = bp.in;
      d.y = A.take_act(d.M() * d.g.K, es);
      take_bn(d);
      take_filters(d);
      track(d, true);
      max_stats_ds = std::max<int64_t>(max_stats_ds, conv_stats_floats(d.g));
    }
    bp.out_elems = (int64_t)N * bs.h_out * bs.w_out * bs.c_out;
    bp.out = A.take_act(bp.out_elems, es);
    cur = bp.out;
  }

  RESIST_TRY(shape_rc);
  // ---- head
  {
    const BlockShape &last = net.blocks[blocks[nblocks - 1]];
    P->feat = cur;
    P->feat_hw = last.h_out * last.w_out;
    const int J = net.d.num_classes;
    P->pooled = A.take<float>((int64_t)N * net.head_c);
    P->dpooled = A.take<float>((int64_t)N * net.head_c);
    P->z = A.take<float>((int64_t)N * J);
    P->dz = A.take<float>((int64_t)N * J);
    P->row_loss = A.take<float>(N);
  }

  // ---- backward scratch shared by all layers (kernels are stream-ordered)
  P->gbuf[0] = A.take_act(max_act, es);
  P->gbuf[1] = A.take_act(max_act, es);
  P->gm = A.take_act(max_act, es);
  P->dy0 = A.take_act(max_act, es);
  P->dy1 = A.take_act(max_act, es);
  P->da = A.take_act(max_act, es);
  P->splitk = A.take<float>(max_splitk);
  P->stats = A.take<float>(max_stats);
  P->bn_scratch = A.take<double>(bn_scratch_doubles(max_c));
  if (max_stats_ds > 0) {
    P->stats_ds = A.take<float>(max_stats_ds);
    P->bn_scratch_ds = A.take<double>(bn_scratch_doubles(max_c));
  }
  P->own_grads.resize(nblocks + 2);
  for (int i = 0; i < nblocks + 2; ++i) P->own_grads[i] = A.take<float>(P->layouts[i].n_trainable);
  P->bytes = (A.off + 255) & ~(int64_t)255;
  return RESIST_OK;
}

// ---- test-time forward: nothing is kept, so every convolution output goes to one shared buffer and
// the activations alternate between two
struct ForwardPlan {
  Net net;
  std::vector<BlockLayout> layouts;
  int kpad = 0;
  ConvLayer stem;
  void *wpad = nullptr, *stem_pool = nullptr;
  uint8_t *stem_argmax = nullptr;
  std::vector<BlockPlan> blocks;
  float *affine[2] = {nullptr, nullptr};   // scale/shift scratch of the branch BN and the shortcut BN: [2][max_c] each
  float *pooled = nullptr, *dz = nullptr, *row_loss = nullptr;
  const void *feat = nullptr;
  int feat_hw = 0;
  int64_t bytes = 0;
};

int build_forward_plan(const resist_model_desc *desc, const int32_t *blocks, int32_t nblocks, int32_t batch, void *ws,
                       ForwardPlan *P) {
  RESIST_TRY(build_net(desc, &P->net));
  const Net &net = P->net;
  RESIST_TRY(check_block_list(net, blocks, nblocks, batch));
  const int B = (int)net.blocks.size();
  const int N = batch, es = esize(net.d.compute_dtype);
  Arena A(ws);
  P->layouts.resize(nblocks + 2);
  RESIST_TRY(block_layout(net, -1, &P->layouts[0]));
  for (int i = 0; i < nblocks; ++i) RESIST_TRY(block_layout(net, blocks[i], &P->layouts[i + 1]));
  RESIST_TRY(block_layout(net, B, &P->layouts[nblocks + 1]));

  // geometry first (to size the shared buffers), pointers afterwards
  const int taps = net.stem_rs * net.stem_rs * net.d.in_c;
  P->kpad = (taps + 31) / 32 * 32;
  const int K0 = net.d.width[0];
  P->stem = make_conv(P->layouts[0], 0, N, net.stem_h, net.stem_w, P->kpad, K0, 1, 1, 0);
  if (stem_scratch_floats(net, N, P->kpad) == 0) return RESIST_ESHAPE;
  int64_t max_act = P->stem.M() * K0;
  int max_c = K0;
  P->blocks.resize(nblocks);
  for (int i = 0; i < nblocks; ++i) {
    const BlockShape &bs = net.blocks[blocks[i]];
    const BlockLayout &L = P->layouts[i + 1];
    BlockPlan &bp = P->blocks[i];
    bp.slot = i + 1;
    if (!net.bottleneck) {
      bp.convs.push_back(make_conv(L, 0, N, bs.h_in, bs.w_in, bs.c_in, bs.width, 3, bs.stride, 1));
      bp.convs.push_back(make_conv(L, 1, N, bs.h_out, bs.w_out, bs.width, bs.c_out, 3, 1, 1));
    } else {
      bp.convs.push_back(make_conv(L, 0, N, bs.h_in, bs.w_in, bs.c_in, bs.width, 1, 1, 0));
      bp.convs.push_back(make_conv(L, 1, N, bs.h_in, bs.w_in, bs.width, bs.width, 3, bs.stride, 1));
      bp.convs.push_back(make_conv(L, 2, N, bs.h_out, bs.w_out, bs.width, bs.c_out, 1, 1, 0));
    }
    bp.has_ds = bs.has_ds;
    if (bs.has_ds) bp.ds = make_conv(L, 3, N, bs.h_in, bs.w_in, bs.c_in, bs.c_out, 1, bs.stride, 0);
    for (const ConvLayer &c : bp.convs) {
      RESIST_TRY(conv_check(c.g, net.d.compute_dtype));
      max_act = std::max<int64_t>(max_act, c.M() * c.g.K);
      max_c = std::max(max_c, c.g.K);
    }
    if (bs.has_ds) RESIST_TRY(conv_check(bp.ds.g, net.d.compute_dtype));
    bp.out_elems = (int64_t)N * bs.h_out * bs.w_out * bs.c_out;
  }
  P->wpad = A.take_act((int64_t)K0 * P->kpad, es);
  void *ybuf = A.take_act(max_act, es), *ydsbuf = A.take_act(max_act, es);
  void *abuf[2] = {A.take_act(max_act, es), A.take_act(max_act, es)};
  void *obuf[2] = {A.take_act(max_act, es), A.take_act(max_act, es)};
  P->stem.y = ybuf;
  P->stem.a = obuf[0];
  const void *cur = obuf[0];
  int oi = 1;
  if (net.d.stem_kind == 1) {
    const int64_t n = (int64_t)N * net.body_h * net.body_w * K0;
    P->stem_pool = obuf[1];
    P->stem_argmax = A.take<uint8_t>(n);
    cur = obuf[1];
    oi = 0;
  }
  for (BlockPlan &bp : P->blocks) {
    bp.in = cur;
    const void *x = cur;
    for (size_t j = 0; j < bp.convs.size(); ++j) {
      ConvLayer &c = bp.convs[j];
      c.in = x;
      c.y = ybuf;
      if (net.d.compute_dtype == DT_BF16) c.wlp = A.take_act((int64_t)c.g.K * c.g.R * c.g.S * c.g.C, es);
      if (j + 1 < bp.convs.size()) { c.a = abuf[j & 1]; x = c.a; }
    }
    if (bp.has_ds) {
      bp.ds.in = bp.in;
      bp.ds.y = ydsbuf;
      if (net.d.compute_dtype == DT_BF16) bp.ds.wlp = A.take_act((int64_t)bp.ds.g.K * bp.ds.g.C, es);
    }
    bp.out = obuf[oi];
    cur = bp.out;
    oi ^= 1;
  }
  P->feat = cur;
  const BlockShape &last = net.blocks[blocks[nblocks - 1]];
  P->feat_hw = last.h_out * last.w_out;
  P->affine[0] = A.take<float>((int64_t)2 * max_c);
  P->affine[1] = A.take<float>((int64_t)2 * max_c);
  P->pooled = A.take<float>((int64_t)N * net.head_c);
  P->dz = A.take<float>((int64_t)N * net.d.num_classes);
  P->row_loss = A.take<float>(N);
  P->bytes = (A.off + 255) & ~(int64_t)255;
  return RESIST_OK;
}

// running statistics and affine parameters of a BN inside a block buffer, scale/shift in `affine`
BnBufs bn_eval_bufs(const ConvLayer &c, float *params, float *affine) {
  BnBufs b{};
  b.gamma = params + c.gamma_off;
  b.beta = params + c.beta_off;
  b.rmean = params + c.rmean_off;
  b.rvar = params + c.rvar_off;
  b.scale = affine;
  b.shift = affine + c.g.K;
  return b;
}

// ---- pre-activation networks (block_kind 2, 3) -------------------------------------------------------
// A block is a chain of units  a_j = ReLU(BN_j(u_j)), h_j = conv_j(a_j)  with u_1 = the block input and
// u_j = h_{j-1};  out = h_n + shortcut, shortcut = input or conv1x1(stride)(a_1).  The statistics of a
// tensor are taken by the convolution that writes it (the stem convolution, or a block's last
// convolution after the shortcut has been added), so every BN starts from per-tile sums.
struct PreUnit {
  ConvGeom g;
  int64_t w_off, gamma_off, beta_off, rmean_off, rvar_off;
  const void *u = nullptr;   // BN input
  void *a = nullptr;         // ReLU(BN(u)): the convolution's input, kept for the backward pass
  void *h = nullptr;         // convolution output (the block output for the last unit)
  float *mean = nullptr, *invstd = nullptr, *scale = nullptr, *shift = nullptr;   // [g.C] each
  void *wlp = nullptr, *wT = nullptr;
  int64_t rows() const { return (int64_t)g.N * g.H * g.W; }   // rows of the BN input
};

struct PreBlock {
  int slot;
  const void *x = nullptr;
  std::vector<PreUnit> units;
  bool has_ds = false;
  ConvGeom dsg;
  int64_t ds_w_off = 0;
  void *ds_wlp = nullptr, *ds_wT = nullptr;
  void *out = nullptr;
};

struct PrePlan {
  Net net;
  std::vector<BlockLayout> layouts;
  int kpad = 0;
  ConvGeom stem;
  int64_t stem_w_off = 0;
  void *wpad = nullptr, *x0 = nullptr;
  float *dwpad = nullptr;
  std::vector<PreBlock> blocks;
  // head: BN-ReLU, mean pool, FC
  int64_t head_rows = 0;
  float *hmean = nullptr, *hinvstd = nullptr, *hscale = nullptr, *hshift = nullptr;
  float *pooled = nullptr, *z = nullptr, *dz = nullptr, *row_loss = nullptr, *dpooled = nullptr;
  const void *feat_in = nullptr;
  int feat_hw = 0;
  void *gbuf[2] = {nullptr, nullptr}, *sc = nullptr, *dsgrad = nullptr, *dy0 = nullptr, *dy1 = nullptr, *da = nullptr;
  float *splitk = nullptr, *stats = nullptr;
  double *bn_scratch = nullptr;
  std::vector<float *> own_grads;
  int64_t bytes = 0;
};

int build_preact_plan(const resist_model_desc *desc, const int32_t *blocks, int32_t nblocks, int32_t batch, void *ws, PrePlan *P) {
  RESIST_TRY(build_net(desc, &P->net));
  const Net &net = P->net;
  RESIST_TRY(check_block_list(net, blocks, nblocks, batch));
  const int B = (int)net.blocks.size();
  const int N = batch, es = esize(net.d.compute_dtype);
  const bool lp = net.d.compute_dtype == DT_BF16;
  Arena A(ws);
  P->layouts.resize(nblocks + 2);
  RESIST_TRY(block_layout(net, -1, &P->layouts[0]));
  for (int i = 0; i < nblocks; ++i) RESIST_TRY(block_layout(net, blocks[i], &P->layouts[i + 1]));
  RESIST_TRY(block_layout(net, B, &P->layouts[nblocks + 1]));
  int64_t max_act = 0, max_splitk = 0, max_stats = 0;
  int max_c = 16;
  int shape_rc = RESIST_OK;   // every convolution is checked here, before anything is launched
  auto track = [&](const ConvGeom &g, bool stats) {
    if (shape_rc == RESIST_OK) shape_rc = conv_check(g, net.d.compute_dtype);
    max_act = std::max<int64_t>(max_act, (int64_t)g.N * g.P * g.Q * g.K);
    max_act = std::max<int64_t>(max_act, (int64_t)g.N * g.H * g.W * g.C);
    max_splitk = std::max<int64_t>(max_splitk, wgrad_scratch_floats(g));
    if (stats) max_stats = std::max<int64_t>(max_stats, conv_stats_floats(g));
    max_c = std::max(max_c, std::max(g.K, g.C));
  };
  const int taps = net.stem_rs * net.stem_rs * net.d.in_c;
  P->kpad = (taps + 31) / 32 * 32;
  const int K0 = net.d.width[0];
  P->stem = make_geom(N, net.stem_h, net.stem_w, P->kpad, K0, 1, 1, 0);
  P->stem_w_off = P->layouts[0].off(T_CONVW, 0);
  const int64_t M0 = (int64_t)N * net.stem_h * net.stem_w;
  P->wpad = A.take_act((int64_t)K0 * P->kpad, es);
  P->dwpad = A.take<float>((int64_t)K0 * P->kpad);
  P->x0 = A.take_act(M0 * K0, es);
  if (stem_scratch_floats(net, N, P->kpad) == 0) return RESIST_ESHAPE;
  max_act = std::max<int64_t>(max_act, M0 * K0);
  max_splitk = std::max<int64_t>(max_splitk, stem_scratch_floats(net, N, P->kpad));
  max_stats = std::max<int64_t>(max_stats, stem_stats_floats(net, N, P->kpad));
  max_c = std::max(max_c, K0);
  const void *cur = P->x0;
  P->blocks.resize(nblocks);
  for (int i = 0; i < nblocks; ++i) {
    const BlockShape &bs = net.blocks[blocks[i]];
    const BlockLayout &L = P->layouts[i + 1];
    PreBlock &pb = P->blocks[i];
    pb.slot = i + 1;
    pb.x = cur;
    std::vector<ConvGeom> gs;
    if (!net.bottleneck) {
      gs.push_back(make_geom(N, bs.h_in, bs.w_in, bs.c_in, bs.width, 3, bs.stride, 1));
      gs.push_back(make_geom(N, bs.h_out, bs.w_out, bs.width, bs.c_out, 3, 1, 1));
    } else {
      gs.push_back(make_geom(N, bs.h_in, bs.w_in, bs.c_in, bs.width, 1, 1, 0));
      gs.push_back(make_geom(N, bs.h_in, bs.w_in, bs.width, bs.width, 3, bs.stride, 1));
      gs.push_back(make_geom(N, bs.h_out, bs.w_out, bs.width, bs.c_out, 1, 1, 0));
    }
    const void *u = cur;
    for (size_t j = 0; j < gs.size(); ++j) {
      PreUnit un;
      un.g = gs[j];
      un.w_off = L.off(T_CONVW, (int)j);
      un.gamma_off = L.off(T_GAMMA, (int)j);
      un.beta_off = L.off(T_BETA, (int)j);
      un.rmean_off = L.off(T_RMEAN, (int)j);
      un.rvar_off = L.off(T_RVAR, (int)j);
      un.u = u;
      un.a = A.take_act(un.rows() * un.g.C, es);
      un.h = A.take_act((int64_t)N * un.g.P * un.g.Q * un.g.K, es);
      float *p = A.take<float>((int64_t)4 * un.g.C);
      un.mean = p; un.invstd = p + un.g.C; un.scale = p + 2 * un.g.C; un.shift = p + 3 * un.g.C;
      const int64_t nf = (int64_t)un.g.K * un.g.R * un.g.S * un.g.C;
      un.wT = A.take_act(nf, es);
      if (lp) un.wlp = A.take_act(nf, es);
      track(un.g, true);
      u = un.h;
      pb.units.push_back(un);
    }
    pb.has_ds = bs.has_ds;
    if (bs.has_ds) {
      pb.dsg = make_geom(N, bs.h_in, bs.w_in, bs.c_in, bs.c_out, 1, bs.stride, 0);
      pb.ds_w_off = L.off(T_CONVW, 3);
      const int64_t nf = (int64_t)bs.c_out * bs.c_in;
      pb.ds_wT = A.take_act(nf, es);
      if (lp) pb.ds_wlp = A.take_act(nf, es);
      track(pb.dsg, false);
    }
    pb.out = pb.units.back().h;
    cur = pb.out;
  }
  RESIST_TRY(shape_rc);
  const BlockShape &last = net.blocks[blocks[nblocks - 1]];
  P->feat_in = cur;
  P->feat_hw = last.h_out * last.w_out;
  P->head_rows = (int64_t)N * P->feat_hw;
  {
    float *p = A.take<float>((int64_t)4 * net.head_c);
    P->hmean = p; P->hinvstd = p + net.head_c; P->hscale = p + 2 * net.head_c; P->hshift = p + 3 * net.head_c;
    max_c = std::max(max_c, net.head_c);
    const int J = net.d.num_classes;
    P->pooled = A.take<float>((int64_t)N * net.head_c);
    P->dpooled = A.take<float>((int64_t)N * net.head_c);
    P->z = A.take<float>((int64_t)N * J);
    P->dz = A.take<float>((int64_t)N * J);
    P->row_loss = A.take<float>(N);
  }
  P->gbuf[0] = A.take_act(max_act, es);
  P->gbuf[1] = A.take_act(max_act, es);
  P->sc = A.take_act(max_act, es);
  P->dsgrad = A.take_act(max_act, es);
  P->dy0 = A.take_act(max_act, es);
  P->dy1 = A.take_act(max_act, es);
  P->da = A.take_act(max_act, es);
  P->splitk = A.take<float>(max_splitk);
  P->stats = A.take<float>(max_stats);
  P->bn_scratch = A.take<double>(bn_scratch_doubles(max_c));
  P->own_grads.resize(nblocks + 2);
  for (int i = 0; i < nblocks + 2; ++i) P->own_grads[i] = A.take<float>(P->layouts[i].n_trainable);
  P->bytes = (A.off + 255) & ~(int64_t)255;
  return RESIST_OK;
}

BnBufs pre_bn_bufs(const PreUnit &un, float *params, float *grads) {
  BnBufs b{};
  b.gamma = params + un.gamma_off;
  b.beta = params + un.beta_off;
  b.rmean = params + un.rmean_off;
  b.rvar = params + un.rvar_off;
  b.mean = un.mean; b.invstd = un.invstd; b.scale = un.scale; b.shift = un.shift;
  b.dgamma = grads + un.gamma_off;
  b.dbeta = grads + un.beta_off;
  return b;
}

int local_step_preact(const resist_model_desc *desc, const int32_t *blocks, int32_t nblocks, void *const *block_params,
                      void *const *block_momentum, void *const *block_grads, const float *x, const int32_t *labels,
                      int32_t batch, float lr, float momentum, float weight_decay, void *workspace, int64_t workspace_bytes,
                      float *loss_out, hipStream_t st) {
  PrePlan P;
  RESIST_TRY(build_preact_plan(desc, blocks, nblocks, batch, workspace, &P));
  if (workspace_bytes < P.bytes) return set_error(RESIST_EWORKSPACE, "workspace has %lld bytes, %lld needed", (long long)workspace_bytes, (long long)P.bytes);
  const Net &net = P.net;
  const int nslots = nblocks + 2, N = batch, dt = net.d.compute_dtype;
  const float eps = net.d.bn_eps, bnm = net.d.bn_momentum;
  auto params = [&](int slot) { return (float *)block_params[slot]; };
  auto grads = [&](int slot) { return block_grads ? (float *)block_grads[slot] : P.own_grads[slot]; };
  double step_flops = 0;
  for (PreBlock &pb : P.blocks) {
    for (PreUnit &un : pb.units) step_flops += 3.0 * geom_flops(un.g);
    if (pb.has_ds) step_flops += 3.0 * geom_flops(pb.dsg);
  }
  WgradSide wg(st, dt, P.splitk, step_flops);
  {
    std::vector<FilterPrep> prep;
    for (PreBlock &pb : P.blocks) {
      float *pp = params(pb.slot);
      for (PreUnit &un : pb.units) prep.push_back(FilterPrep{un.g, pp + un.w_off, un.wlp, un.wT});
      if (pb.has_ds) prep.push_back(FilterPrep{pb.dsg, pp + pb.ds_w_off, pb.ds_wlp, pb.ds_wT});
    }
    RESIST_TRY(wg.prepare(prep));
  }
  auto fwd_filter = [&](const float *w, const void *wlp) -> const void * { return dt == DT_F32 ? (const void *)w : wlp; };

  // ================= forward =================
  const int K0 = net.d.width[0];
  const int taps = net.stem_rs * net.stem_rs * net.d.in_c;
  StatParts parts;   // number of per-tile sums the last statistics-taking convolution left in P.stats
  RESIST_TRY(pad_rows(dt, params(0) + P.stem_w_off, P.wpad, K0, taps, P.kpad, st));
  RESIST_TRY(stem_forward(net, dt, N, P.kpad, x, P.wpad, P.x0, P.stats, &parts, st));
  for (PreBlock &pb : P.blocks) {
    float *pp = params(pb.slot), *gg = grads(pb.slot);
    const size_t n = pb.units.size();
    for (size_t j = 0; j < n; ++j) {
      PreUnit &un = pb.units[j];
      BnBufs b = pre_bn_bufs(un, pp, gg);
      RESIST_TRY(bn_finalize(P.stats, parts, un.rows(), un.g.C, b, eps, bnm, P.bn_scratch, st));
      RESIST_TRY(bn_apply(dt, un.u, un.rows(), un.g.C, b, nullptr, nullptr, true, un.a, st));
      if (j == 0 && pb.has_ds)
        RESIST_TRY(conv_fwd(pb.dsg, dt, un.a, fwd_filter(pp + pb.ds_w_off, pb.ds_wlp), P.sc, nullptr, nullptr, nullptr, st));
      const void *addend = j + 1 == n ? (pb.has_ds ? (const void *)P.sc : pb.x) : nullptr;
      RESIST_TRY(conv_fwd(un.g, dt, un.a, fwd_filter(pp + un.w_off, un.wlp), un.h, addend, P.stats, &parts, st));
    }
  }
  const int J = net.d.num_classes, CH = net.head_c;
  const int hs = nslots - 1;
  const BlockLayout &HL = P.layouts[hs];
  float *hp = params(hs), *hg = grads(hs);
  BnBufs hb{};
  hb.gamma = hp + HL.off(T_GAMMA, 0); hb.beta = hp + HL.off(T_BETA, 0);
  hb.rmean = hp + HL.off(T_RMEAN, 0); hb.rvar = hp + HL.off(T_RVAR, 0);
  hb.mean = P.hmean; hb.invstd = P.hinvstd; hb.scale = P.hscale; hb.shift = P.hshift;
  hb.dgamma = hg + HL.off(T_GAMMA, 0); hb.dbeta = hg + HL.off(T_BETA, 0);
  float *fcw = hp + HL.off(T_FCW, 0), *fcb = hp + HL.off(T_FCB, 0);
  RESIST_TRY(bn_finalize(P.stats, parts, P.head_rows, CH, hb, eps, bnm, P.bn_scratch, st));
  RESIST_TRY(bn_apply(dt, P.feat_in, P.head_rows, CH, hb, nullptr, nullptr, true, P.da, st));
  RESIST_TRY(avgpool_fwd(dt, P.da, P.pooled, N, P.feat_hw, CH, st));
  RESIST_TRY(fc_fwd_f32(P.pooled, fcw, fcb, P.z, N, CH, J, st));
  RESIST_TRY(softmax_ce_f32(P.z, labels, P.dz, P.row_loss, N, J, st));

  // ================= backward =================
  RESIST_TRY(fc_bwd_dx_f32(P.dz, fcw, P.dpooled, N, CH, J, st));
  RESIST_TRY(wg.off_chain([&](hipStream_t s) {
    RESIST_TRY(mean_loss_f32(P.row_loss, loss_out, N, s));
    return fc_bwd_params_f32(P.dz, P.pooled, hg + HL.off(T_FCW, 0), hg + HL.off(T_FCB, 0), N, CH, J, s);
  }));
  RESIST_TRY(avgpool_bwd(dt, P.dpooled, nullptr, P.da, N, P.feat_hw, CH, st));
  int gi = 0;
  RESIST_TRY(wg.filters_ready());
  RESIST_TRY(bn_backward(dt, P.da, true, P.feat_in, P.head_rows, CH, hb, P.gbuf[gi], nullptr, P.bn_scratch, st));
  for (int bi = (int)P.blocks.size() - 1; bi >= 0; --bi) {
    PreBlock &pb = P.blocks[bi];
    float *pp = params(pb.slot), *gg = grads(pb.slot);
    void *G = P.gbuf[gi], *Gn = P.gbuf[gi ^ 1];
    const void *gcur = G;
    void *dy = P.dy0, *dy_other = P.dy1;
    for (int j = (int)pb.units.size() - 1; j >= 0; --j) {
      PreUnit &un = pb.units[j];
      RESIST_TRY(wg.launch(un.g, gcur, un.a, gg + un.w_off));
      const void *addend = nullptr;
      if (j == 0 && pb.has_ds) {
        // the shortcut convolution reads the same a_1: its data gradient joins the branch's
        RESIST_TRY(wg.launch(pb.dsg, G, un.a, gg + pb.ds_w_off));
        RESIST_TRY(conv_dgrad(pb.dsg, dt, G, pb.ds_wT, P.dsgrad, nullptr, nullptr, st));
        addend = P.dsgrad;
      }
      RESIST_TRY(conv_dgrad(un.g, dt, gcur, un.wT, P.da, addend, nullptr, st));
      BnBufs b = pre_bn_bufs(un, pp, gg);
      if (j > 0) {
        RESIST_TRY(wg.before_write(dy));
        RESIST_TRY(bn_backward(dt, P.da, true, un.u, un.rows(), un.g.C, b, dy, nullptr, P.bn_scratch, st));
        gcur = dy;
        std::swap(dy, dy_other);
      } else {
        // gradient w.r.t. the block input: through BN_1, plus the identity shortcut's share
        RESIST_TRY(wg.before_write(Gn));
        RESIST_TRY(bn_backward(dt, P.da, true, un.u, un.rows(), un.g.C, b, Gn, pb.has_ds ? nullptr : G, P.bn_scratch, st));
      }
    }
    gi ^= 1;
  }
  RESIST_TRY(wg.launch_stem(net, N, P.kpad, P.gbuf[gi], x, P.dwpad));
  RESIST_TRY(unpad_rows_f32(P.dwpad, grads(0) + P.stem_w_off, K0, taps, P.kpad, wg.stream()));
  RESIST_TRY(wg.join());

  // ================= update =================
  std::vector<SgdSeg> segs;
  for (int i = 0; i < nslots; ++i)
    segs.push_back(SgdSeg{params(i), (float *)block_momentum[i], grads(i), P.layouts[i].n_trainable});
  return sgd_momentum_f32(segs, lr, momentum, weight_decay, st);
}

BnBufs bn_bufs(const ConvLayer &c, float *params, float *grads) {
  BnBufs b;
  b.gamma = params + c.gamma_off;
  b.beta = params + c.beta_off;
  b.rmean = params + c.rmean_off;
  b.rvar = params + c.rvar_off;
  b.mean = c.mean;
  b.invstd = c.invstd;
  b.scale = c.scale;
  b.shift = c.shift;
  b.dgamma = grads + c.gamma_off;
  b.dbeta = grads + c.beta_off;
  return b;
}

}  // namespace
}  // namespace resist

using namespace resist;

extern "C" int resist_workspace_bytes(const resist_model_desc *desc, const int32_t *blocks, int32_t nblocks,
                                      int32_t batch, int64_t *bytes) {
  if (!bytes) return set_error(RESIST_EINVAL, "bytes is NULL");
  if (desc && desc->block_kind >= 2) {
    PrePlan Q;
    RESIST_TRY(build_preact_plan(desc, blocks, nblocks, batch, nullptr, &Q));
    *bytes = Q.bytes;
    return RESIST_OK;
  }
  StepPlan P;
  RESIST_TRY(build_plan(desc, blocks, nblocks, batch, nullptr, &P));
  *bytes = P.bytes;
  return RESIST_OK;
}

extern "C" int resist_local_step(const resist_model_desc *desc, const int32_t *blocks, int32_t nblocks,
                                 void *const *block_params, void *const *block_momentum, void *const *block_grads,
                                 const float *x, const int32_t *labels, int32_t batch, float lr, float momentum,
                                 float weight_decay, void *workspace, int64_t workspace_bytes, float *loss_out,
                                 void *hip_stream) {
  if (!block_params || !block_momentum || !x || !labels || !workspace || !loss_out)
    return set_error(RESIST_EINVAL, "NULL argument");
  if (((uintptr_t)workspace & 15) || ((uintptr_t)x & 15)) return set_error(RESIST_EINVAL, "workspace and x must be 16-byte aligned");
  if (desc && desc->block_kind >= 2) {
    if (nblocks < 0) return set_error(RESIST_EINVAL, "nblocks");
    for (int i = 0; i < nblocks + 2; ++i) {
      if (!block_params[i] || !block_momentum[i] || (block_grads && !block_grads[i]))
        return set_error(RESIST_EINVAL, "buffer %d is NULL", i);
      if (((uintptr_t)block_params[i] & 15) || ((uintptr_t)block_momentum[i] & 15) || (block_grads && ((uintptr_t)block_grads[i] & 15)))
        return set_error(RESIST_EINVAL, "buffer %d is not 16-byte aligned", i);
    }
    return local_step_preact(desc, blocks, nblocks, block_params, block_momentum, block_grads, x, labels, batch, lr, momentum,
                             weight_decay, workspace, workspace_bytes, loss_out, (hipStream_t)hip_stream);
  }
  StepPlan P;
  RESIST_TRY(build_plan(desc, blocks, nblocks, batch, workspace, &P));
  if (workspace_bytes < P.bytes) return set_error(RESIST_EWORKSPACE, "workspace has %lld bytes, %lld needed", (long long)workspace_bytes, (long long)P.bytes);
  const int nslots = nblocks + 2;
  for (int i = 0; i < nslots; ++i) {
    if (!block_params[i] || !block_momentum[i] || (block_grads && !block_grads[i]))
      return set_error(RESIST_EINVAL, "buffer %d is NULL", i);
    if (((uintptr_t)block_params[i] & 15) || ((uintptr_t)block_momentum[i] & 15) || (block_grads && ((uintptr_t)block_grads[i] & 15)))
      return set_error(RESIST_EINVAL, "buffer %d is not 16-byte aligned", i);
  }
  hipStream_t st = (hipStream_t)hip_stream;
  const Net &net = P.net;
  const int N = batch;
  const float eps = net.d.bn_eps, bnm = net.d.bn_momentum;
  auto params = [&](int slot) { return (float *)block_params[slot]; };
  auto grads = [&](int slot) { return block_grads ? (float *)block_grads[slot] : P.own_grads[slot]; };

  const int dt = net.d.compute_dtype;
  double step_flops = 0;
  for (BlockPlan &bp : P.blocks) {
    for (ConvLayer &c : bp.convs) step_flops += 3.0 * geom_flops(c.g);
    if (bp.has_ds) step_flops += 3.0 * geom_flops(bp.ds.g);
  }
  WgradSide wg(st, dt, P.splitk, step_flops);
  // every filter once, up front: the transpose the data gradient reads and, in bf16 mode, the copy
  // the forward convolution multiplies with (fp32 mode multiplies the master itself)
  {
    std::vector<FilterPrep> prep;
    for (BlockPlan &bp : P.blocks) {
      float *pp = params(bp.slot);
      for (ConvLayer &c : bp.convs) prep.push_back(FilterPrep{c.g, pp + c.w_off, c.wlp, c.wT});
      if (bp.has_ds) prep.push_back(FilterPrep{bp.ds.g, pp + bp.ds.w_off, bp.ds.wlp, bp.ds.wT});
    }
    RESIST_TRY(wg.prepare(prep));
  }
  auto fwd_filter = [&](const ConvLayer &c, const float *w) -> const void * { return dt == DT_F32 ? (const void *)w : c.wlp; };

  // ================= forward =================
  {
    ConvLayer &s = P.stem;
    const int K0 = net.d.width[0];
    const int taps = net.stem_rs * net.stem_rs * net.d.in_c;
    RESIST_TRY(pad_rows(dt, params(0) + s.w_off, P.wpad, K0, taps, P.kpad, st));
    StatParts parts;
    RESIST_TRY(stem_forward(net, dt, N, P.kpad, x, P.wpad, s.y, P.stats, &parts, st));
    BnBufs b = bn_bufs(s, params(0), grads(0));
    RESIST_TRY(bn_finalize(P.stats, parts, s.M(), K0, b, eps, bnm, P.bn_scratch, st));
    RESIST_TRY(bn_apply(dt, s.y, s.M(), K0, b, nullptr, nullptr, true, s.a, st));
    if (net.d.stem_kind == 1)
      RESIST_TRY(maxpool_fwd(dt, s.a, P.stem_pool, P.stem_argmax, N, net.stem_h, net.stem_w, K0, net.body_h, net.body_w, st));
  }
  for (BlockPlan &bp : P.blocks) {
    float *pp = params(bp.slot), *gg = grads(bp.slot);
    // The shortcut convolution and its BN statistics depend on the block input only: on the second stream they
    // run next to the residual branch (with statistics scratch of their own), and the chain meets them at the
    // block's last BN.
    hipEvent_t ds_done = nullptr;
    const bool ds_aside = bp.has_ds && wg.side.on();
    if (ds_aside) {
      ConvLayer &d = bp.ds;
      RESIST_TRY(wg.off_chain([&](hipStream_t s) {
        StatParts parts;
        RESIST_TRY(conv_fwd(d.g, dt, d.in, fwd_filter(d, pp + d.w_off), d.y, nullptr, P.stats_ds, &parts, s));
        return bn_finalize(P.stats_ds, parts, d.M(), d.g.K, bn_bufs(d, pp, gg), eps, bnm, P.bn_scratch_ds, s);
      }));
      RESIST_TRY(wg.side.mark(&ds_done));
    }
    for (size_t j = 0; j < bp.convs.size(); ++j) {
      ConvLayer &c = bp.convs[j];
      StatParts parts;
      RESIST_TRY(conv_fwd(c.g, dt, c.in, fwd_filter(c, pp + c.w_off), c.y, nullptr, P.stats, &parts, st));
      BnBufs b = bn_bufs(c, pp, gg);
      RESIST_TRY(bn_finalize(P.stats, parts, c.M(), c.g.K, b, eps, bnm, P.bn_scratch, st));
      if (c.a) RESIST_TRY(bn_apply(dt, c.y, c.M(), c.g.K, b, nullptr, nullptr, true, c.a, st));
    }
    ConvLayer &last = bp.convs.back();
    BnBufs bl = bn_bufs(last, pp, gg);
    if (bp.has_ds) {
      ConvLayer &d = bp.ds;
      BnBufs bd = bn_bufs(d, pp, gg);
      if (ds_aside) {
        RESIST_TRY(wg.side.main_wait(ds_done));
      } else {
        StatParts parts;
        RESIST_TRY(conv_fwd(d.g, dt, d.in, fwd_filter(d, pp + d.w_off), d.y, nullptr, P.stats, &parts, st));
        RESIST_TRY(bn_finalize(P.stats, parts, d.M(), d.g.K, bd, eps, bnm, P.bn_scratch, st));
      }
      RESIST_TRY(bn_apply(dt, last.y, last.M(), last.g.K, bl, d.y, &bd, true, bp.out, st));
    } else {
      RESIST_TRY(bn_apply(dt, last.y, last.M(), last.g.K, bl, bp.in, nullptr, true, bp.out, st));
    }
  }
  const int J = net.d.num_classes, CH = net.head_c;
  const int hs = nslots - 1;
  const BlockLayout &HL = P.layouts[hs];
  float *fcw = params(hs) + HL.off(T_FCW, 0), *fcb = params(hs) + HL.off(T_FCB, 0);
  RESIST_TRY(avgpool_fwd(dt, P.feat, P.pooled, N, P.feat_hw, CH, st));
  RESIST_TRY(fc_fwd_f32(P.pooled, fcw, fcb, P.z, N, CH, J, st));
  RESIST_TRY(softmax_ce_f32(P.z, labels, P.dz, P.row_loss, N, J, st));

  // ================= backward =================
  RESIST_TRY(wg.filters_ready());
  RESIST_TRY(fc_bwd_dx_f32(P.dz, fcw, P.dpooled, N, CH, J, st));
  RESIST_TRY(wg.off_chain([&](hipStream_t s) {
    RESIST_TRY(mean_loss_f32(P.row_loss, loss_out, N, s));
    return fc_bwd_params_f32(P.dz, P.pooled, grads(hs) + HL.off(T_FCW, 0), grads(hs) + HL.off(T_FCB, 0), N, CH, J, s);
  }));
  // The gradient w.r.t. a block's output is stored already taken through that block's final ReLU: the
  // kernel that produces it (the mean-pool backward, or the first convolution's data gradient of the
  // block after it) reads the block output once and zeroes the gradient where it is not positive, so
  // the two BN backward passes behind it need no mask tensor and no masked copy is written.
  // In bf16 mode a stride-1 data gradient also takes the first pass of the BN backward that consumes its
  // output (per-row-tile sums in P.stats, free during the backward pass): one launch and one read of the
  // gradient less per BN, in a mode where the backward chain, not the matrix cores, sets the step time.
  const bool fuse_bn = bn_fusion_mode() == 2 || (bn_fusion_mode() == 1 && dt == DT_BF16);
  StatParts pre{};        // P.stats holds the first pass for the BN that ends the block below
  bool have_pre = false;
  int gi = 0;
  void *G = P.gbuf[gi];
  RESIST_TRY(avgpool_bwd(dt, P.dpooled, P.feat, G, N, P.feat_hw, CH, st));
  for (int bi = (int)P.blocks.size() - 1; bi >= 0; --bi) {
    BlockPlan &bp = P.blocks[bi];
    float *pp = params(bp.slot), *gg = grads(bp.slot);
    void *Gn = P.gbuf[gi ^ 1];
    const int nc = (int)bp.convs.size();
    ConvLayer &last = bp.convs[nc - 1];
    BnBufs bl = bn_bufs(last, pp, gg);
    // the last BN of the residual branch
    RESIST_TRY(wg.before_write(P.dy0));
    RESIST_TRY(bn_backward(dt, G, false, last.y, last.M(), last.g.K, bl, P.dy0, nullptr, P.bn_scratch, st,
                           have_pre ? P.stats : nullptr, pre));
    have_pre = false;
    if (bp.has_ds) {
      // shortcut branch: BN and 1x1 convolution; its data gradient initialises Gn
      ConvLayer &d = bp.ds;
      BnBufs bd = bn_bufs(d, pp, gg);
      RESIST_TRY(wg.before_write(P.gm));
      RESIST_TRY(bn_backward(dt, G, false, d.y, d.M(), d.g.K, bd, P.gm, nullptr, P.bn_scratch, st));
      RESIST_TRY(wg.launch(d.g, P.gm, d.in, gg + d.w_off));
      RESIST_TRY(conv_dgrad(d.g, dt, P.gm, d.wT, Gn, nullptr, nullptr, st));
    }
    void *dy = P.dy0, *dy_other = P.dy1;
    for (int j = nc - 1; j >= 0; --j) {
      ConvLayer &c = bp.convs[j];
      RESIST_TRY(wg.launch(c.g, dy, c.in, gg + c.w_off));
      if (j > 0) {
        ConvLayer &prev = bp.convs[j - 1];
        BnBufs bp_ = bn_bufs(prev, pp, gg);
        StatParts sp{};
        const BnBwdFuse f{prev.y, bp_, true, P.stats, &sp};
        const bool fz = fuse_bn && c.g.stride == 1;
        RESIST_TRY(conv_dgrad(c.g, dt, dy, c.wT, P.da, nullptr, nullptr, st, fz ? &f : nullptr));
        RESIST_TRY(wg.before_write(dy_other));
        RESIST_TRY(bn_backward(dt, P.da, true, prev.y, prev.M(), prev.g.K, bp_, dy_other, nullptr, P.bn_scratch, st,
                               fz ? P.stats : nullptr, sp));
        std::swap(dy, dy_other);
      } else {
        // gradient w.r.t. the block input = branch + shortcut (the identity shortcut passes G itself),
        // taken through the ReLU that ends the block before (the stem's ReLU is handled by its own BN backward)
        const bool fz = fuse_bn && bi > 0 && c.g.stride == 1;
        if (fz) {
          // its output is the (masked) gradient of the block below's output: first pass of that block's last BN
          BlockPlan &below = P.blocks[bi - 1];
          ConvLayer &bl_last = below.convs.back();
          const BnBwdFuse f{bl_last.y, bn_bufs(bl_last, params(below.slot), grads(below.slot)), false, P.stats, &pre};
          RESIST_TRY(conv_dgrad(c.g, dt, dy, c.wT, Gn, bp.has_ds ? Gn : G, bp.in, st, &f));
        } else {
          RESIST_TRY(conv_dgrad(c.g, dt, dy, c.wT, Gn, bp.has_ds ? Gn : G, bi > 0 ? bp.in : nullptr, st));
        }
        have_pre = fz;
      }
    }
    gi ^= 1;
    G = Gn;
  }
  {
    ConvLayer &s = P.stem;
    const int K0 = net.d.width[0];
    const int taps = net.stem_rs * net.stem_rs * net.d.in_c;
    const void *Gs = G;
    if (net.d.stem_kind == 1) {
      RESIST_TRY(maxpool_bwd(dt, G, P.stem_argmax, P.da, N, net.stem_h, net.stem_w, K0, net.body_h, net.body_w, st));
      Gs = P.da;
    }
    BnBufs b = bn_bufs(s, params(0), grads(0));
    RESIST_TRY(wg.before_write(P.dy0));
    RESIST_TRY(bn_backward(dt, Gs, true, s.y, s.M(), K0, b, P.dy0, nullptr, P.bn_scratch, st));
    RESIST_TRY(wg.launch_stem(net, N, P.kpad, P.dy0, x, P.dwpad));
    RESIST_TRY(unpad_rows_f32(P.dwpad, grads(0) + s.w_off, K0, taps, P.kpad, wg.stream()));
  }
  RESIST_TRY(wg.join());

  // ================= update =================
  std::vector<SgdSeg> segs;
  for (int i = 0; i < nslots; ++i)
    segs.push_back(SgdSeg{params(i), (float *)block_momentum[i], grads(i), P.layouts[i].n_trainable});
  RESIST_TRY(sgd_momentum_f32(segs, lr, momentum, weight_decay, st));
  return RESIST_OK;
}

namespace resist {
namespace {

// test-time forward of a pre-activation network: out = shortcut + s * conv_n(a_n); the scale is folded
// into a copy of the last convolution's filter
struct PreForwardPlan {
  Net net;
  std::vector<BlockLayout> layouts;
  int kpad = 0;
  ConvGeom stem;
  void *wpad = nullptr;
  std::vector<PreBlock> blocks;
  void *abuf = nullptr, *sc = nullptr;
  float *affine = nullptr, *pooled = nullptr, *dz = nullptr, *row_loss = nullptr;
  const void *feat_in = nullptr;
  int feat_hw = 0;
  int64_t bytes = 0;
};

int build_preact_forward_plan(const resist_model_desc *desc, const int32_t *blocks, int32_t nblocks, int32_t batch, void *ws,
                              PreForwardPlan *P) {
  RESIST_TRY(build_net(desc, &P->net));
  const Net &net = P->net;
  RESIST_TRY(check_block_list(net, blocks, nblocks, batch));
  const int B = (int)net.blocks.size();
  const int N = batch, es = esize(net.d.compute_dtype);
  Arena A(ws);
  P->layouts.resize(nblocks + 2);
  RESIST_TRY(block_layout(net, -1, &P->layouts[0]));
  for (int i = 0; i < nblocks; ++i) RESIST_TRY(block_layout(net, blocks[i], &P->layouts[i + 1]));
  RESIST_TRY(block_layout(net, B, &P->layouts[nblocks + 1]));
  const int taps = net.stem_rs * net.stem_rs * net.d.in_c;
  P->kpad = (taps + 31) / 32 * 32;
  const int K0 = net.d.width[0];
  P->stem = make_geom(N, net.stem_h, net.stem_w, P->kpad, K0, 1, 1, 0);
  if (stem_scratch_floats(net, N, P->kpad) == 0) return RESIST_ESHAPE;
  int64_t max_act = (int64_t)N * net.stem_h * net.stem_w * K0;
  int max_c = std::max(K0, net.head_c);
  P->blocks.resize(nblocks);
  for (int i = 0; i < nblocks; ++i) {
    const BlockShape &bs = net.blocks[blocks[i]];
    const BlockLayout &L = P->layouts[i + 1];
    PreBlock &pb = P->blocks[i];
    pb.slot = i + 1;
    std::vector<ConvGeom> gs;
    if (!net.bottleneck) {
      gs.push_back(make_geom(N, bs.h_in, bs.w_in, bs.c_in, bs.width, 3, bs.stride, 1));
      gs.push_back(make_geom(N, bs.h_out, bs.w_out, bs.width, bs.c_out, 3, 1, 1));
    } else {
      gs.push_back(make_geom(N, bs.h_in, bs.w_in, bs.c_in, bs.width, 1, 1, 0));
      gs.push_back(make_geom(N, bs.h_in, bs.w_in, bs.width, bs.width, 3, bs.stride, 1));
      gs.push_back(make_geom(N, bs.h_out, bs.w_out, bs.width, bs.c_out, 1, 1, 0));
    }
    for (size_t j = 0; j < gs.size(); ++j) {
      PreUnit un;
      un.g = gs[j];
      un.w_off = L.off(T_CONVW, (int)j);
      un.gamma_off = L.off(T_GAMMA, (int)j);
      un.beta_off = L.off(T_BETA, (int)j);
      un.rmean_off = L.off(T_RMEAN, (int)j);
      un.rvar_off = L.off(T_RVAR, (int)j);
      // a copy of the filter in the compute type; the last unit's always (it carries the branch scale)
      if (net.d.compute_dtype == DT_BF16 || j + 1 == gs.size())
        un.wlp = A.take_act((int64_t)un.g.K * un.g.R * un.g.S * un.g.C, es);
      RESIST_TRY(conv_check(un.g, net.d.compute_dtype));
      max_act = std::max<int64_t>(max_act, (int64_t)N * un.g.P * un.g.Q * un.g.K);
      max_act = std::max<int64_t>(max_act, un.rows() * un.g.C);
      max_c = std::max(max_c, std::max(un.g.C, un.g.K));
      pb.units.push_back(un);
    }
    pb.has_ds = bs.has_ds;
    if (bs.has_ds) {
      pb.dsg = make_geom(N, bs.h_in, bs.w_in, bs.c_in, bs.c_out, 1, bs.stride, 0);
      pb.ds_w_off = L.off(T_CONVW, 3);
      if (net.d.compute_dtype == DT_BF16) pb.ds_wlp = A.take_act((int64_t)bs.c_out * bs.c_in, es);
    }
  }
  P->wpad = A.take_act((int64_t)K0 * P->kpad, es);
  // the residual stream alternates between two buffers, the branch between two more
  void *ubuf[2] = {A.take_act(max_act, es), A.take_act(max_act, es)};
  void *hbuf[2] = {A.take_act(max_act, es), A.take_act(max_act, es)};
  P->abuf = A.take_act(max_act, es);
  P->sc = A.take_act(max_act, es);
  const void *cur = ubuf[0];
  int ui = 1;
  for (PreBlock &pb : P->blocks) {
    pb.x = cur;
    const void *u = cur;
    for (size_t j = 0; j < pb.units.size(); ++j) {
      PreUnit &un = pb.units[j];
      un.u = u;
      un.a = P->abuf;
      un.h = j + 1 == pb.units.size() ? ubuf[ui] : hbuf[j & 1];
      u = un.h;
    }
    pb.out = ubuf[ui];
    cur = pb.out;
    ui ^= 1;
  }
  P->feat_in = cur;
  const BlockShape &last = net.blocks[blocks[nblocks - 1]];
  P->feat_hw = last.h_out * last.w_out;
  P->affine = A.take<float>((int64_t)2 * max_c);
  P->pooled = A.take<float>((int64_t)N * net.head_c);
  P->dz = A.take<float>((int64_t)N * net.d.num_classes);
  P->row_loss = A.take<float>(N);
  P->bytes = (A.off + 255) & ~(int64_t)255;
  return RESIST_OK;
}

int forward_preact(const resist_model_desc *desc, const int32_t *blocks, int32_t nblocks, void *const *block_params,
                   const float *branch_scale, const float *x, int32_t batch, void *workspace, int64_t workspace_bytes,
                   float *logits_out, const int32_t *labels, float *loss_out, hipStream_t st) {
  PreForwardPlan P;
  RESIST_TRY(build_preact_forward_plan(desc, blocks, nblocks, batch, workspace, &P));
  if (workspace_bytes < P.bytes) return set_error(RESIST_EWORKSPACE, "workspace has %lld bytes, %lld needed", (long long)workspace_bytes, (long long)P.bytes);
  const Net &net = P.net;
  const int nslots = nblocks + 2, N = batch, dt = net.d.compute_dtype;
  const float eps = net.d.bn_eps;
  auto params = [&](int slot) { return (float *)block_params[slot]; };
  {
    std::vector<FilterPrep> prep;
    for (size_t bi = 0; bi < P.blocks.size(); ++bi) {
      PreBlock &pb = P.blocks[bi];
      float *pp = params(pb.slot);
      for (size_t j = 0; j < pb.units.size(); ++j) {
        PreUnit &un = pb.units[j];
        if (!un.wlp) continue;
        FilterPrep f{un.g, pp + un.w_off, un.wlp, nullptr};
        if (j + 1 == pb.units.size() && branch_scale) f.scale = branch_scale[bi];
        prep.push_back(f);
      }
      if (pb.ds_wlp) prep.push_back(FilterPrep{pb.dsg, pp + pb.ds_w_off, pb.ds_wlp, nullptr});
    }
    RESIST_TRY(prepare_filters(prep, dt, st));
  }
  const int K0 = net.d.width[0];
  const int taps = net.stem_rs * net.stem_rs * net.d.in_c;
  RESIST_TRY(pad_rows(dt, params(0) + P.layouts[0].off(T_CONVW, 0), P.wpad, K0, taps, P.kpad, st));
  RESIST_TRY(stem_forward(net, dt, N, P.kpad, x, P.wpad, const_cast<void *>(P.blocks[0].x), nullptr, nullptr, st));
  for (PreBlock &pb : P.blocks) {
    float *pp = params(pb.slot);
    const size_t n = pb.units.size();
    for (size_t j = 0; j < n; ++j) {
      PreUnit &un = pb.units[j];
      BnBufs b{};
      b.gamma = pp + un.gamma_off; b.beta = pp + un.beta_off; b.rmean = pp + un.rmean_off; b.rvar = pp + un.rvar_off;
      b.scale = P.affine; b.shift = P.affine + un.g.C;
      RESIST_TRY(bn_eval_affine(un.g.C, b, eps, 1.f, st));
      RESIST_TRY(bn_apply(dt, un.u, un.rows(), un.g.C, b, nullptr, nullptr, true, un.a, st));
      if (j == 0 && pb.has_ds) {
        const void *wd = dt == DT_F32 ? (const void *)(pp + pb.ds_w_off) : pb.ds_wlp;
        RESIST_TRY(conv_fwd(pb.dsg, dt, un.a, wd, P.sc, nullptr, nullptr, nullptr, st));
      }
      const void *wf = un.wlp ? un.wlp : (const void *)(pp + un.w_off);
      const void *addend = j + 1 == n ? (pb.has_ds ? (const void *)P.sc : pb.x) : nullptr;
      RESIST_TRY(conv_fwd(un.g, dt, un.a, wf, un.h, addend, nullptr, nullptr, st));
    }
  }
  const int J = net.d.num_classes, CH = net.head_c;
  const BlockLayout &HL = P.layouts[nslots - 1];
  float *hp = params(nslots - 1);
  BnBufs hb{};
  hb.gamma = hp + HL.off(T_GAMMA, 0); hb.beta = hp + HL.off(T_BETA, 0);
  hb.rmean = hp + HL.off(T_RMEAN, 0); hb.rvar = hp + HL.off(T_RVAR, 0);
  hb.scale = P.affine; hb.shift = P.affine + CH;
  RESIST_TRY(bn_eval_affine(CH, hb, eps, 1.f, st));
  RESIST_TRY(bn_apply(dt, P.feat_in, (int64_t)N * P.feat_hw, CH, hb, nullptr, nullptr, true, P.abuf, st));
  RESIST_TRY(avgpool_fwd(dt, P.abuf, P.pooled, N, P.feat_hw, CH, st));
  RESIST_TRY(fc_fwd_f32(P.pooled, hp + HL.off(T_FCW, 0), hp + HL.off(T_FCB, 0), logits_out, N, CH, J, st));
  if (labels) {
    RESIST_TRY(softmax_ce_f32(logits_out, labels, P.dz, P.row_loss, N, J, st));
    RESIST_TRY(mean_loss_f32(P.row_loss, loss_out, N, st));
  }
  return RESIST_OK;
}

}  // namespace
}  // namespace resist

extern "C" int resist_forward_workspace_bytes(const resist_model_desc *desc, const int32_t *blocks, int32_t nblocks,
                                              int32_t batch, int64_t *bytes) {
  if (!bytes) return set_error(RESIST_EINVAL, "bytes is NULL");
  if (desc && desc->block_kind >= 2) {
    PreForwardPlan Q;
    RESIST_TRY(build_preact_forward_plan(desc, blocks, nblocks, batch, nullptr, &Q));
    *bytes = Q.bytes;
    return RESIST_OK;
  }
  ForwardPlan P;
  RESIST_TRY(build_forward_plan(desc, blocks, nblocks, batch, nullptr, &P));
  *bytes = P.bytes;
  return RESIST_OK;
}

extern "C" int resist_forward(const resist_model_desc *desc, const int32_t *blocks, int32_t nblocks,
                              void *const *block_params, const float *branch_scale, const float *x, int32_t batch,
                              void *workspace, int64_t workspace_bytes, float *logits_out, const int32_t *labels,
                              float *loss_out, void *hip_stream) {
  if (!block_params || !x || !workspace || !logits_out) return set_error(RESIST_EINVAL, "NULL argument");
  if ((labels == nullptr) != (loss_out == nullptr)) return set_error(RESIST_EINVAL, "labels and loss_out go together");
  if (((uintptr_t)workspace & 15) || ((uintptr_t)x & 15) || ((uintptr_t)logits_out & 15))
    return set_error(RESIST_EINVAL, "workspace, x and logits_out must be 16-byte aligned");
  if (desc && desc->block_kind >= 2) {
    if (nblocks < 0) return set_error(RESIST_EINVAL, "nblocks");
    for (int i = 0; i < nblocks + 2; ++i)
      if (!block_params[i] || ((uintptr_t)block_params[i] & 15)) return set_error(RESIST_EINVAL, "buffer %d is NULL or not 16-byte aligned", i);
    return forward_preact(desc, blocks, nblocks, block_params, branch_scale, x, batch, workspace, workspace_bytes, logits_out,
                          labels, loss_out, (hipStream_t)hip_stream);
  }
  ForwardPlan P;
  RESIST_TRY(build_forward_plan(desc, blocks, nblocks, batch, workspace, &P));
  if (workspace_bytes < P.bytes) return set_error(RESIST_EWORKSPACE, "workspace has %lld bytes, %lld needed", (long long)workspace_bytes, (long long)P.bytes);
  const int nslots = nblocks + 2;
  for (int i = 0; i < nslots; ++i)
    if (!block_params[i] || ((uintptr_t)block_params[i] & 15)) return set_error(RESIST_EINVAL, "buffer %d is NULL or not 16-byte aligned", i);
  hipStream_t st = (hipStream_t)hip_stream;
  const Net &net = P.net;
  const int N = batch, dt = net.d.compute_dtype;
  const float eps = net.d.bn_eps;
  auto params = [&](int slot) { return (float *)block_params[slot]; };
  if (dt == DT_BF16) {
    std::vector<FilterPrep> prep;
    for (BlockPlan &bp : P.blocks) {
      float *pp = params(bp.slot);
      for (ConvLayer &c : bp.convs) prep.push_back(FilterPrep{c.g, pp + c.w_off, c.wlp, nullptr});
      if (bp.has_ds) prep.push_back(FilterPrep{bp.ds.g, pp + bp.ds.w_off, bp.ds.wlp, nullptr});
    }
    RESIST_TRY(prepare_filters(prep, dt, st));
  }
  auto filter = [&](const ConvLayer &c, const float *w) -> const void * { return dt == DT_F32 ? (const void *)w : c.wlp; };
  {
    ConvLayer &s = P.stem;
    const int K0 = net.d.width[0];
    const int taps = net.stem_rs * net.stem_rs * net.d.in_c;
    RESIST_TRY(pad_rows(dt, params(0) + s.w_off, P.wpad, K0, taps, P.kpad, st));
    RESIST_TRY(stem_forward(net, dt, N, P.kpad, x, P.wpad, s.y, nullptr, nullptr, st));
    BnBufs b = bn_eval_bufs(s, params(0), P.affine[0]);
    RESIST_TRY(bn_eval_affine(K0, b, eps, 1.f, st));
    RESIST_TRY(bn_apply(dt, s.y, s.M(), K0, b, nullptr, nullptr, true, s.a, st));
    if (net.d.stem_kind == 1)
      RESIST_TRY(maxpool_fwd(dt, s.a, P.stem_pool, P.stem_argmax, N, net.stem_h, net.stem_w, K0, net.body_h, net.body_w, st));
  }
  for (size_t bi = 0; bi < P.blocks.size(); ++bi) {
    BlockPlan &bp = P.blocks[bi];
    float *pp = params(bp.slot);
    const float scale = branch_scale ? branch_scale[bi] : 1.f;
    const size_t nc = bp.convs.size();
    BnBufs bl{};
    for (size_t j = 0; j < nc; ++j) {
      ConvLayer &c = bp.convs[j];
      RESIST_TRY(conv_fwd(c.g, dt, c.in, filter(c, pp + c.w_off), c.y, nullptr, nullptr, nullptr, st));
      BnBufs b = bn_eval_bufs(c, pp, P.affine[0]);
      RESIST_TRY(bn_eval_affine(c.g.K, b, eps, j + 1 == nc ? scale : 1.f, st));
      if (c.a) RESIST_TRY(bn_apply(dt, c.y, c.M(), c.g.K, b, nullptr, nullptr, true, c.a, st));
      else bl = b;
    }
    ConvLayer &last = bp.convs.back();
    if (bp.has_ds) {
      ConvLayer &d = bp.ds;
      RESIST_TRY(conv_fwd(d.g, dt, d.in, filter(d, pp + d.w_off), d.y, nullptr, nullptr, nullptr, st));
      BnBufs bd = bn_eval_bufs(d, pp, P.affine[1]);
      RESIST_TRY(bn_eval_affine(d.g.K, bd, eps, 1.f, st));
      RESIST_TRY(bn_apply(dt, last.y, last.M(), last.g.K, bl, d.y, &bd, true, bp.out, st));
    } else {
      RESIST_TRY(bn_apply(dt, last.y, last.M(), last.g.K, bl, bp.in, nullptr, true, bp.out, st));
    }
  }
  const int J = net.d.num_classes, CH = net.head_c;
  const BlockLayout &HL = P.layouts[nslots - 1];
  float *fcw = params(nslots - 1) + HL.off(T_FCW, 0), *fcb = params(nslots - 1) + HL.off(T_FCB, 0);
  RESIST_TRY(avgpool_fwd(dt, P.feat, P.pooled, N, P.feat_hw, CH, st));
  RESIST_TRY(fc_fwd_f32(P.pooled, fcw, fcb, logits_out, N, CH, J, st));
  if (labels) {
    RESIST_TRY(softmax_ce_f32(logits_out, labels, P.dz, P.row_loss, N, J, st));
    RESIST_TRY(mean_loss_f32(P.row_loss, loss_out, N, st));
  }
  return RESIST_OK;
}

extern "C" int resist_aggregate(const resist_model_desc *desc, int32_t S, const int32_t *sub_offsets,
                                const int32_t *sub_blocks, void *const *const *sub_block_params,
                                void *const *global_block_params, void *hip_stream) {
  Net net;
  RESIST_TRY(build_net(desc, &net));
  const int B = (int)net.blocks.size();
  if (S < 1 || !sub_offsets || !sub_blocks || !sub_block_params || !global_block_params)
    return set_error(RESIST_EINVAL, "NULL argument or S < 1");
  if (S > 16) return set_error(RESIST_EUNSUPPORTED, "S=%d: at most 16 sub-ResNets supported", S);
  std::vector<AggSeg> segs(B + 2);
  for (int key = -1; key <= B; ++key) {
    BlockLayout L;
    RESIST_TRY(block_layout(net, key, &L));
    AggSeg &g = segs[key + 1];
    g.dst = (float *)global_block_params[key + 1];
    g.count = 0;
    g.n = L.n_total;
    if (!g.dst) return set_error(RESIST_EINVAL, "global buffer %d is NULL", key + 1);
  }
  for (int s = 0; s < S; ++s) {
    const int n_s = sub_offsets[s + 1] - sub_offsets[s];
    if (n_s < 0) return set_error(RESIST_EINVAL, "sub_offsets not ascending");
    if (!sub_block_params[s]) return set_error(RESIST_EINVAL, "sub_block_params[%d] is NULL", s);
    auto add = [&](int key, const void *p) -> int {
      if (!p) return set_error(RESIST_EINVAL, "sub-ResNet %d: buffer for block %d is NULL", s, key);
      AggSeg &g = segs[key + 1];
      g.src[g.count++] = (const float *)p;
      return RESIST_OK;
    };
    RESIST_TRY(add(-1, sub_block_params[s][0]));
    for (int i = 0; i < n_s; ++i) {
      const int b = sub_blocks[sub_offsets[s] + i];
      if (b < 0 || b >= B) return set_error(RESIST_EINVAL, "sub-ResNet %d holds block %d outside [0,%d)", s, b, B);
      if (i > 0 && b <= sub_blocks[sub_offsets[s] + i - 1]) return set_error(RESIST_EINVAL, "sub-ResNet %d: blocks not ascending", s);
      RESIST_TRY(add(b, sub_block_params[s][1 + i]));
    }
    RESIST_TRY(add(B, sub_block_params[s][1 + n_s]));
  }
  return aggregate_f32(segs, (hipStream_t)hip_stream);
}
