// A second HIP stream for work that is off the critical path of a step.  In the backward pass the
// weight gradient of a layer is needed only by the parameter update at the very end, while the data
// gradient and the BN backward kernels form the chain every earlier layer waits for: running the
// weight gradients on a side stream lets the short, latency-bound kernels of the chain overlap with
// them.  One side stream (default priority, non-blocking) and a ring of events per device, created
// on first use and kept until the process ends.
#include <atomic>
#include <mutex>

#include "internal.h"

namespace resist {
namespace {

constexpr int kMaxDevices = 16;
constexpr int kRing = 256;   // a wait captures the record that precedes it, so an event may be reused later

struct DeviceSide {
  hipStream_t stream = nullptr;
  hipEvent_t ring[kRing] = {};
  int next = 0;
};
DeviceSide g_side[kMaxDevices];
std::mutex g_mu;
std::atomic<int> g_overlap{1};
std::atomic<int> g_bn_fusion{1};

}  // namespace

int overlap_mode() { return g_overlap.load(); }

extern "C" int resist_set_overlap(int32_t mode) {
  if (mode < 0 || mode > 2) return set_error(RESIST_EINVAL, "overlap mode %d: 0 (off), 1 (steps with enough work) or 2 (always)", mode);
  g_overlap.store(mode);
  return RESIST_OK;
}

int bn_fusion_mode() { return g_bn_fusion.load(); }

extern "C" int resist_set_bn_fusion(int32_t mode) {
  if (mode < 0 || mode > 2) return set_error(RESIST_EINVAL, "BN fusion mode %d: 0 (never), 1 (bf16 steps) or 2 (always)", mode);
  g_bn_fusion.store(mode);
  return RESIST_OK;
}

SideStream::SideStream(hipStream_t main, bool enable) : main_(main), side_(nullptr), dev_(-1) {
  if (!enable) return;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return;
  std::lock_guard<std::mutex> lock(g_mu);
  DeviceSide &d = g_side[dev];
  if (!d.stream && hipStreamCreateWithFlags(&d.stream, hipStreamNonBlocking) != hipSuccess) {
    d.stream = nullptr;
    (void)hipGetLastError();
    return;   // no side stream: everything stays on the caller's stream
  }
  side_ = d.stream;
  dev_ = dev;
}

hipEvent_t SideStream::take() {
  std::lock_guard<std::mutex> lock(g_mu);
  DeviceSide &d = g_side[dev_];
  hipEvent_t &e = d.ring[d.next];
  d.next = (d.next + 1) % kRing;
  if (!e && hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) e = nullptr;
  return e;
}

int SideStream::fork() {
  if (!side_) return RESIST_OK;
  hipEvent_t e = take();
  if (!e) return set_error(RESIST_EHIP, "event creation failed");
  RESIST_CHECK_HIP(hipEventRecord(e, main_));
  RESIST_CHECK_HIP(hipStreamWaitEvent(side_, e, 0));
  return RESIST_OK;
}

int SideStream::mark(hipEvent_t *ev) {
  *ev = nullptr;
  if (!side_) return RESIST_OK;
  hipEvent_t e = take();
  if (!e) return set_error(RESIST_EHIP, "event creation failed");
  RESIST_CHECK_HIP(hipEventRecord(e, side_));
  *ev = e;
  return RESIST_OK;
}

int SideStream::main_wait(hipEvent_t ev) {
  if (!side_ || !ev) return RESIST_OK;
  RESIST_CHECK_HIP(hipStreamWaitEvent(main_, ev, 0));
  return RESIST_OK;
}

int SideStream::join() {
  if (!side_) return RESIST_OK;
  hipEvent_t e = nullptr;
  RESIST_TRY(mark(&e));
  return main_wait(e);
}

}  // namespace resist
