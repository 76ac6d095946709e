// Host-side description of the global ResNet, parameter-buffer layout, and the random
// layer-wise split into sub-ResNets (Sec. 2.2 of the paper).  No device code here.
#include <stdarg.h>
#include <stdio.h>

#include <algorithm>

#include "internal.h"

namespace resist {

static thread_local char g_err[512] = "";

int set_error(int code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

static int out_dim(int in, int k, int stride, int pad) { return (in + 2 * pad - k) / stride + 1; }

int build_net(const resist_model_desc *d, Net *net) {
  if (!d) return set_error(RESIST_EINVAL, "model description is NULL");
  if (d->block_kind < 0 || d->block_kind > 3) return set_error(RESIST_EINVAL, "block_kind %d", d->block_kind);
  if (d->block_kind >= 2 && d->stem_kind != 0)
    return set_error(RESIST_EUNSUPPORTED, "pre-activation networks take the 3x3 stem (stem_kind 0)");
  if (d->stem_kind < 0 || d->stem_kind > 1) return set_error(RESIST_EINVAL, "stem_kind %d", d->stem_kind);
  if (d->compute_dtype < 0 || d->compute_dtype > 1) return set_error(RESIST_EINVAL, "compute_dtype %d", d->compute_dtype);
  if (d->num_stages < 1 || d->num_stages > RESIST_MAX_STAGES) return set_error(RESIST_EINVAL, "num_stages %d", d->num_stages);
  if (d->in_c < 1 || d->in_c > 4 || d->in_h < 1 || d->in_w < 1) return set_error(RESIST_ESHAPE, "input %dx%dx%d", d->in_c, d->in_h, d->in_w);
  if (d->num_classes < 2) return set_error(RESIST_EINVAL, "num_classes %d", d->num_classes);
  if (!(d->bn_eps > 0.f) || !(d->bn_momentum >= 0.f && d->bn_momentum <= 1.f)) return set_error(RESIST_EINVAL, "bn_eps/bn_momentum");
  for (int i = 0; i < d->num_stages; ++i) {
    if (d->width[i] < 16 || d->width[i] % 16) return set_error(RESIST_ESHAPE, "width[%d]=%d must be a positive multiple of 16", i, d->width[i]);
    if (d->blocks[i] < 1) return set_error(RESIST_ESHAPE, "blocks[%d]=%d", i, d->blocks[i]);
  }
  net->d = *d;
  net->preact = d->block_kind >= 2;
  net->bottleneck = (d->block_kind & 1) != 0;
  net->expansion = net->bottleneck ? 4 : 1;
  net->stem_rs = d->stem_kind == 0 ? 3 : 7;
  net->stem_stride = d->stem_kind == 0 ? 1 : 2;
  net->stem_pad = d->stem_kind == 0 ? 1 : 3;
  net->stem_h = out_dim(d->in_h, net->stem_rs, net->stem_stride, net->stem_pad);
  net->stem_w = out_dim(d->in_w, net->stem_rs, net->stem_stride, net->stem_pad);
  net->body_h = d->stem_kind == 0 ? net->stem_h : out_dim(net->stem_h, 3, 2, 1);
  net->body_w = d->stem_kind == 0 ? net->stem_w : out_dim(net->stem_w, 3, 2, 1);
  if (net->body_h < 1 || net->body_w < 1) return set_error(RESIST_ESHAPE, "input too small for the stem");
  net->blocks.clear();
  net->stage_first.clear();
  int c_in = d->width[0], h = net->body_h, w = net->body_w;
  for (int s = 0; s < d->num_stages; ++s) {
    net->stage_first.push_back((int)net->blocks.size());
    for (int b = 0; b < d->blocks[s]; ++b) {
      BlockShape bs;
      bs.stage = s; bs.index = b;
      bs.c_in = c_in; bs.width = d->width[s]; bs.c_out = d->width[s] * net->expansion;
      bs.stride = (b == 0 && s > 0) ? 2 : 1;
      bs.has_ds = b == 0 && (bs.stride != 1 || bs.c_in != bs.c_out);
      bs.h_in = h; bs.w_in = w;
      bs.h_out = out_dim(h, 3, bs.stride, 1); bs.w_out = out_dim(w, 3, bs.stride, 1);
      if (bs.stride == 2 && ((h & 1) || (w & 1)))
        return set_error(RESIST_ESHAPE, "stage %d enters with odd spatial size %dx%d", s, h, w);
      if (bs.h_out < 1 || bs.w_out < 1) return set_error(RESIST_ESHAPE, "spatial size vanishes at stage %d", s);
      net->blocks.push_back(bs);
      c_in = bs.c_out; h = bs.h_out; w = bs.w_out;
    }
  }
  net->head_c = c_in;
  return RESIST_OK;
}

static int64_t pad4(int64_t n) { return (n + 3) & ~(int64_t)3; }

static void push(BlockLayout *L, int kind, int layer, int64_t count, int d0, int d1 = 0, int d2 = 0, int d3 = 0) {
  TensorSlot s{kind, layer, L->n_total, count, {d0, d1, d2, d3}};
  L->slots.push_back(s);
  L->n_total += pad4(count);
}

int block_layout(const Net &net, int block, BlockLayout *L) {
  const int B = (int)net.blocks.size();
  if (block < -1 || block > B) return set_error(RESIST_EINVAL, "block %d outside [-1,%d]", block, B);
  L->slots.clear();
  L->n_total = 0;
  std::vector<std::pair<int, int>> bns;   // (layer, channels)
  auto conv_bn = [&](int layer, int K, int R, int C) {
    push(L, T_CONVW, layer, (int64_t)K * R * R * C, K, R, R, C);
    push(L, T_GAMMA, layer, K, K);
    push(L, T_BETA, layer, K, K);
    bns.push_back({layer, K});
  };
  // pre-activation: the BN of layer j sits before convolution j and has its input channels
  auto bn_conv = [&](int layer, int K, int R, int C) {
    push(L, T_GAMMA, layer, C, C);
    push(L, T_BETA, layer, C, C);
    push(L, T_CONVW, layer, (int64_t)K * R * R * C, K, R, R, C);
    bns.push_back({layer, C});
  };
  if (net.preact) {
    if (block == -1) {
      push(L, T_CONVW, 0, (int64_t)net.d.width[0] * net.stem_rs * net.stem_rs * net.d.in_c, net.d.width[0], net.stem_rs,
           net.stem_rs, net.d.in_c);
    } else if (block == B) {
      push(L, T_GAMMA, 0, net.head_c, net.head_c);
      push(L, T_BETA, 0, net.head_c, net.head_c);
      bns.push_back({0, net.head_c});
      push(L, T_FCW, 0, (int64_t)net.d.num_classes * net.head_c, net.d.num_classes, net.head_c);
      push(L, T_FCB, 0, net.d.num_classes, net.d.num_classes);
    } else {
      const BlockShape &b = net.blocks[block];
      if (!net.bottleneck) {
        bn_conv(0, b.width, 3, b.c_in);
        bn_conv(1, b.c_out, 3, b.width);
      } else {
        bn_conv(0, b.width, 1, b.c_in);
        bn_conv(1, b.width, 3, b.width);
        bn_conv(2, b.c_out, 1, b.width);
      }
      if (b.has_ds) push(L, T_CONVW, 3, (int64_t)b.c_out * b.c_in, b.c_out, 1, 1, b.c_in);
    }
  } else if (block == -1) {
    conv_bn(0, net.d.width[0], net.stem_rs, net.d.in_c);
  } else if (block == B) {
    push(L, T_FCW, 0, (int64_t)net.d.num_classes * net.head_c, net.d.num_classes, net.head_c);
    push(L, T_FCB, 0, net.d.num_classes, net.d.num_classes);
  } else {
    const BlockShape &b = net.blocks[block];
    if (!net.bottleneck) {
      conv_bn(0, b.width, 3, b.c_in);
      conv_bn(1, b.c_out, 3, b.width);
    } else {
      conv_bn(0, b.width, 1, b.c_in);
      conv_bn(1, b.width, 3, b.width);
      conv_bn(2, b.c_out, 1, b.width);
    }
    if (b.has_ds) conv_bn(3, b.c_out, 1, b.c_in);
  }
  L->n_trainable = L->n_total;
  for (auto &p : bns) {
    push(L, T_RMEAN, p.first, p.second, p.second);
    push(L, T_RVAR, p.first, p.second, p.second);
  }
  return RESIST_OK;
}

// splitmix64: the sequence generator behind the block permutation
struct SplitMix64 {
  uint64_t s;
  uint64_t next() {
    s += 0x9E3779B97F4A7C15ull;
    uint64_t z = s;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
  }
};

}  // namespace resist

using namespace resist;

extern "C" const char *resist_last_error(void) { return g_err; }

extern "C" int resist_num_blocks(const resist_model_desc *desc, int32_t *num_blocks) {
  Net net;
  RESIST_TRY(build_net(desc, &net));
  if (!num_blocks) return set_error(RESIST_EINVAL, "num_blocks is NULL");
  *num_blocks = (int32_t)net.blocks.size();
  return RESIST_OK;
}

extern "C" int resist_block_param_count(const resist_model_desc *desc, int32_t block, int64_t *n_total,
                                        int64_t *n_trainable) {
  Net net;
  RESIST_TRY(build_net(desc, &net));
  BlockLayout L;
  RESIST_TRY(block_layout(net, block, &L));
  if (n_total) *n_total = L.n_total;
  if (n_trainable) *n_trainable = L.n_trainable;
  return RESIST_OK;
}

extern "C" int resist_block_layout(const resist_model_desc *desc, int32_t block, resist_tensor_info *out,
                                   int32_t cap, int32_t *n_tensors) {
  Net net;
  RESIST_TRY(build_net(desc, &net));
  BlockLayout L;
  RESIST_TRY(block_layout(net, block, &L));
  if (!n_tensors) return set_error(RESIST_EINVAL, "n_tensors is NULL");
  if (cap < 0 || (cap > 0 && !out)) return set_error(RESIST_EINVAL, "bad out/cap");
  *n_tensors = (int32_t)L.slots.size();
  for (int i = 0; i < cap && i < (int)L.slots.size(); ++i) {
    const TensorSlot &s = L.slots[i];
    out[i].kind = s.kind; out[i].layer = s.layer; out[i].offset = s.offset; out[i].count = s.count;
    for (int j = 0; j < 4; ++j) out[i].dims[j] = s.dims[j];
  }
  return RESIST_OK;
}

extern "C" int resist_partition(const resist_model_desc *desc, const uint8_t *partitionable, int32_t S,
                                int32_t min_depth, uint64_t seed, uint64_t round, int32_t *sub_offsets,
                                int32_t *sub_blocks, int32_t cap, int32_t *owner_count) {
  Net net;
  RESIST_TRY(build_net(desc, &net));
  const int B = (int)net.blocks.size();
  if (S < 1) return set_error(RESIST_EINVAL, "S=%d must be >= 1", S);
  if (min_depth < 0) return set_error(RESIST_EINVAL, "min_depth=%d must be >= 0", min_depth);
  if (!sub_offsets || !sub_blocks || !owner_count || cap < 0) return set_error(RESIST_EINVAL, "NULL output or negative cap");
  // dealt = the partitionable blocks, fixed = everything else (kept by every sub-ResNet)
  std::vector<int> dealt_ids, fixed_ids;
  for (int b = 0; b < B; ++b) {
    bool is_first = std::find(net.stage_first.begin(), net.stage_first.end(), b) != net.stage_first.end();
    bool p = partitionable ? partitionable[b] != 0 : !is_first;
    (p ? dealt_ids : fixed_ids).push_back(b);
  }
  const int64_t P = (int64_t)dealt_ids.size();
  int64_t D = 0;
  if (P > 0) D = std::max<int64_t>((P + S - 1) / S, std::min<int64_t>(min_depth, P));
  const int64_t per_sub = (int64_t)fixed_ids.size() + D;
  if (per_sub * S > cap) return set_error(RESIST_EWORKSPACE, "sub_blocks needs %lld entries, cap=%d", (long long)(per_sub * S), cap);
  // random permutation of positions 0..P-1 (Fisher-Yates, top index down)
  std::vector<int> order(P);
  for (int64_t i = 0; i < P; ++i) order[i] = (int)i;
  SplitMix64 rng{seed ^ (round * 0x9E3779B97F4A7C15ull)};
  for (int64_t i = P - 1; i >= 1; --i) {
    uint64_t j = rng.next() % (uint64_t)(i + 1);
    std::swap(order[i], order[j]);
  }
  for (int b = 0; b < B; ++b) owner_count[b] = 0;
  std::vector<uint8_t> held(P);
  int32_t w = 0;
  for (int s = 0; s < S; ++s) {
    sub_offsets[s] = w;
    std::fill(held.begin(), held.end(), 0);
    for (int64_t j = 0; j < D; ++j) {
      int64_t slot = (s + j * (int64_t)S) % P;
      while (held[order[slot]]) slot = (slot + 1) % P;     // D <= P, so a free one exists
      held[order[slot]] = 1;
    }
    const int32_t start = w;
    for (int b : fixed_ids) sub_blocks[w++] = b;
    for (int64_t i = 0; i < P; ++i)
      if (held[i]) sub_blocks[w++] = dealt_ids[i];
    std::sort(sub_blocks + start, sub_blocks + w);
    for (int32_t i = start; i < w; ++i) owner_count[sub_blocks[i]]++;
  }
  sub_offsets[S] = w;
  return RESIST_OK;
}
