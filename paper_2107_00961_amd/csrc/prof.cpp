// Optional per-kernel timing with HIP events on the caller's stream (off by default).
// When enabled, every kernel launch of the library is bracketed by two events; reading the
// statistics synchronises on them.  Host-side objects only: no device memory is allocated.
#include <string.h>

#include <mutex>

#include "internal.h"

namespace resist {
namespace prof {
namespace {
struct Rec { hipEvent_t a, b; int kind; double flops, bytes; };
std::mutex g_mu;
bool g_on = false;
std::vector<std::string> g_names;
std::vector<Rec> g_recs;
std::vector<hipEvent_t> g_pool;

hipEvent_t get_event() {
  if (!g_pool.empty()) {
    hipEvent_t e = g_pool.back();
    g_pool.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}
}  // namespace

bool enabled() { return g_on; }

int kind(const char *label) {
  std::lock_guard<std::mutex> lk(g_mu);
  for (size_t i = 0; i < g_names.size(); ++i)
    if (g_names[i] == label) return (int)i;
  g_names.push_back(label);
  return (int)g_names.size() - 1;
}

Scope::Scope(const char *label, double flops, double bytes, hipStream_t st) : st_(st), idx_(-1) {
  if (!g_on) return;
  const int k = kind(label);
  std::lock_guard<std::mutex> lk(g_mu);
  Rec r{get_event(), get_event(), k, flops, bytes};
  if (!r.a || !r.b) return;
  if (hipEventRecord(r.a, st) != hipSuccess) return;
  g_recs.push_back(r);
  idx_ = (int)g_recs.size() - 1;
}

Scope::~Scope() {
  if (idx_ < 0) return;
  std::lock_guard<std::mutex> lk(g_mu);
  (void)hipEventRecord(g_recs[idx_].b, st_);
}

}  // namespace prof
}  // namespace resist

using namespace resist;

extern "C" int resist_profile_enable(int on) {
  std::lock_guard<std::mutex> lk(prof::g_mu);
  for (auto &r : prof::g_recs) {
    prof::g_pool.push_back(r.a);
    prof::g_pool.push_back(r.b);
  }
  prof::g_recs.clear();
  prof::g_on = on != 0;
  return RESIST_OK;
}

extern "C" int resist_profile_read(resist_kernel_stat *out, int32_t cap, int32_t *n) {
  if (!n || cap < 0 || (cap > 0 && !out)) return set_error(RESIST_EINVAL, "bad out/cap/n");
  std::lock_guard<std::mutex> lk(prof::g_mu);
  std::vector<resist_kernel_stat> acc(prof::g_names.size());
  for (size_t i = 0; i < acc.size(); ++i) {
    memset(&acc[i], 0, sizeof(acc[i]));
    strncpy(acc[i].name, prof::g_names[i].c_str(), sizeof(acc[i].name) - 1);
  }
  for (auto &r : prof::g_recs) {
    RESIST_CHECK_HIP(hipEventSynchronize(r.b));
    float ms = 0.f;
    RESIST_CHECK_HIP(hipEventElapsedTime(&ms, r.a, r.b));
    acc[r.kind].launches += 1;
    acc[r.kind].ms += ms;
    acc[r.kind].flops += r.flops;
    acc[r.kind].bytes += r.bytes;
  }
  int32_t m = 0;
  for (auto &s : acc) {
    if (s.launches == 0) continue;
    if (m < cap) out[m] = s;
    ++m;
  }
  *n = m;
  return RESIST_OK;
}
