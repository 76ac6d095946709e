// Driver for the sanitizer build of the library's host-only code (model.cpp: model description,
// block layouts, and the random layer-wise split of Sec. 2.2): g++ -fsanitize=address,undefined, no GPU.
// Every output array is an exactly-sized heap block, so a write one past any end is reported; besides
// that the driver checks what must hold for every split: equal sizes, ascending block lists, every
// fixed block in every sub-ResNet, owner counts that add up, nothing written past `cap`.
#include <cstdio>
#include <cstdlib>
#include <memory>
#include <vector>

#include "resist.h"

namespace {
int failures = 0;
#define EXPECT(cond)                                                          \
  do {                                                                        \
    if (!(cond)) { std::fprintf(stderr, "line %d: %s\n", __LINE__, #cond); ++failures; } \
  } while (0)

resist_model_desc model(int kind, int stem, int hw, std::vector<int> widths, std::vector<int> blocks, int classes) {
  resist_model_desc d{};
  d.block_kind = kind; d.stem_kind = stem; d.in_c = 3; d.in_h = hw; d.in_w = hw;
  d.num_stages = (int)widths.size();
  for (size_t i = 0; i < widths.size(); ++i) { d.width[i] = widths[i]; d.blocks[i] = blocks[i]; }
  d.num_classes = classes; d.compute_dtype = 0; d.bn_eps = 1e-5f; d.bn_momentum = 0.1f;
  return d;
}

void check_layouts(const resist_model_desc &d) {
  int32_t B = 0;
  EXPECT(resist_num_blocks(&d, &B) == RESIST_OK);
  for (int b = -1; b <= B; ++b) {
    int64_t total = 0, trainable = 0;
    EXPECT(resist_block_param_count(&d, b, &total, &trainable) == RESIST_OK);
    int32_t n = 0;
    EXPECT(resist_block_layout(&d, b, nullptr, 0, &n) == RESIST_OK);
    std::unique_ptr<resist_tensor_info[]> info(new resist_tensor_info[n]);
    EXPECT(resist_block_layout(&d, b, info.get(), n, &n) == RESIST_OK);
    int64_t end = 0;
    for (int i = 0; i < n; ++i) {
      EXPECT(info[i].offset >= end && info[i].offset % 4 == 0 && info[i].count > 0);
      end = info[i].offset + info[i].count;
    }
    EXPECT(end <= total && trainable <= total);
    // a capacity smaller than the number of tensors: only `cap` entries may be written
    if (n > 1) {
      std::unique_ptr<resist_tensor_info[]> few(new resist_tensor_info[n - 1]);
      int32_t m = 0;
      EXPECT(resist_block_layout(&d, b, few.get(), n - 1, &m) == RESIST_OK && m == n);
    }
  }
  int64_t t = 0;
  EXPECT(resist_block_param_count(&d, B + 1, &t, &t) != RESIST_OK);
  EXPECT(resist_block_param_count(&d, -2, &t, &t) != RESIST_OK);
}

void check_partition(const resist_model_desc &d, int S, int min_depth, uint64_t seed, uint64_t round, bool paper_mask) {
  int32_t B = 0;
  EXPECT(resist_num_blocks(&d, &B) == RESIST_OK);
  std::unique_ptr<uint8_t[]> mask(new uint8_t[B]);
  int first = 0, fixed = 0;
  std::vector<int> is_first(B, 0);
  for (int s = 0; s < d.num_stages; ++s) { is_first[first] = 1; first += d.blocks[s]; }
  for (int b = 0; b < B; ++b) {
    // the paper's rule: only the non-strided blocks of the third section are dealt
    const int third_lo = d.num_stages >= 3 ? d.blocks[0] + d.blocks[1] : B;
    const int third_hi = d.num_stages >= 3 ? third_lo + d.blocks[2] : B;
    mask[b] = paper_mask ? (b > third_lo && b < third_hi) : !is_first[b];
    fixed += !mask[b];
  }
  const int P = B - fixed;
  const int D = P > 0 ? std::max((P + S - 1) / S, std::min(min_depth, P)) : 0;
  const int need = S * (fixed + D);
  std::unique_ptr<int32_t[]> offs(new int32_t[S + 1]), blocks(new int32_t[need]), owner(new int32_t[B]);
  EXPECT(resist_partition(&d, paper_mask ? mask.get() : nullptr, S, min_depth, seed, round, offs.get(), blocks.get(), need,
                          owner.get()) == RESIST_OK);
  std::vector<int> count(B, 0);
  for (int s = 0; s < S; ++s) {
    EXPECT(offs[s + 1] - offs[s] == fixed + D);
    for (int i = offs[s]; i < offs[s + 1]; ++i) {
      EXPECT(blocks[i] >= 0 && blocks[i] < B);
      EXPECT(i == offs[s] || blocks[i] > blocks[i - 1]);
      if (blocks[i] >= 0 && blocks[i] < B) ++count[blocks[i]];
    }
  }
  for (int b = 0; b < B; ++b) {
    EXPECT(owner[b] == count[b] && owner[b] >= (P > 0 && S * D >= P ? 1 : 0));
    if (!mask[b]) EXPECT(owner[b] == S);
  }
  if (need > 0) {   // one entry short: refused, nothing written
    std::unique_ptr<int32_t[]> small(new int32_t[need - 1]);
    EXPECT(resist_partition(&d, paper_mask ? mask.get() : nullptr, S, min_depth, seed, round, offs.get(), small.get(), need - 1,
                            owner.get()) == RESIST_EWORKSPACE);
  }
}
}  // namespace

int main() {
  const std::vector<resist_model_desc> models = {
      model(0, 0, 16, {16}, {2}, 10),                            // tiny
      model(0, 0, 32, {64, 128, 256, 512}, {3, 4, 23, 3}, 100),  // CIFAR-shaped
      model(1, 1, 224, {64, 128, 256, 512}, {3, 4, 6, 3}, 1000), // ImageNet-shaped bottleneck
      model(2, 0, 32, {64, 128, 256, 512}, {3, 4, 23, 3}, 10),   // pre-activation basic
      model(3, 0, 16, {16, 32}, {2, 3}, 7),                      // pre-activation bottleneck
      model(0, 0, 8, {16, 32, 64}, {1, 1, 1}, 3)};               // nothing to deal
  for (const auto &d : models) {
    check_layouts(d);
    for (int S : {1, 2, 3, 4, 8, 16})
      for (int md : {0, 4, 5, 10, 1000})
        for (uint64_t seed : {0ull, 1ull, 0xFFFFFFFFFFFFFFFFull})
          for (bool paper : {false, true}) check_partition(d, S, md, seed, seed % 3, paper);
  }
  // argument errors come back as statuses
  resist_model_desc d = models[1];
  int32_t x[64], y[64], z[64];
  EXPECT(resist_partition(&d, nullptr, 0, 0, 0, 0, x, y, 64, z) == RESIST_EINVAL);
  EXPECT(resist_partition(&d, nullptr, 2, -1, 0, 0, x, y, 64, z) == RESIST_EINVAL);
  EXPECT(resist_partition(nullptr, nullptr, 2, 0, 0, 0, x, y, 64, z) != RESIST_OK);
  d.width[1] = 100;
  int32_t B = 0;
  EXPECT(resist_num_blocks(&d, &B) == RESIST_ESHAPE);
  if (failures == 0) std::printf("host code: clean\n");
  return failures ? 1 : 0;
}
