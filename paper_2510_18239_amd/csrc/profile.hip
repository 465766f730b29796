// Optional per-kernel timing: when switched on, each main kernel is launched with a start and a stop
// event of its own (hipExtLaunchKernel), which carry the dispatch's begin and end time stamps, so a caller
// can read that kernel's own duration (without the small pack / merge kernels around it and without the
// gaps between launches).  Off by default; costs nothing then.  Creates events and, in collect, waits for them.
#include "../../include/lime.h"
#include "common.hpp"

#include <atomic>
#include <mutex>
#include <vector>

namespace lime {
namespace {
struct Span {
  int kernel;
  hipEvent_t start, stop;
};
std::mutex g_mu;
std::atomic<bool> g_on{false};  // read without the lock on every launch
std::vector<Span> g_spans;
std::vector<hipEvent_t> g_pool;

hipEvent_t take_event() {
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

bool profile_events(int kernel, hipEvent_t* start, hipEvent_t* stop) {
  if (!g_on.load(std::memory_order_relaxed)) return false;
  std::lock_guard<std::mutex> lock(g_mu);
  Span sp{kernel, take_event(), take_event()};
  if (!sp.start || !sp.stop) return false;
  g_spans.push_back(sp);
  *start = sp.start, *stop = sp.stop;
  return true;
}
}  // namespace lime

extern "C" {
#pragma GCC visibility push(default)

void lime_profile_enable(int32_t on) {
  std::lock_guard<std::mutex> lock(lime::g_mu);
  lime::g_on = on != 0;
}

int32_t lime_profile_collect(int32_t kernel, float* ms, int32_t capacity) {
  std::lock_guard<std::mutex> lock(lime::g_mu);
  int32_t n = 0;
  std::vector<lime::Span> keep;
  for (lime::Span& sp : lime::g_spans) {
    if (sp.kernel != kernel) {
      keep.push_back(sp);
      continue;
    }
    float t = 0.f;
    if (hipEventSynchronize(sp.stop) == hipSuccess && hipEventElapsedTime(&t, sp.start, sp.stop) == hipSuccess &&
        ms != nullptr && n < capacity)
      ms[n++] = t;
    lime::g_pool.push_back(sp.start);
    lime::g_pool.push_back(sp.stop);
  }
  lime::g_spans.swap(keep);
  return n;
}

#pragma GCC visibility pop
}
