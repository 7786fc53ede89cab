// Per-process caches of what the launchers would otherwise ask the HIP runtime on every call:
// the compute-unit count of a device, and which kernels already had their dynamic-LDS limit
// raised on which device.  Both are thread-safe; after the first call on a device a launcher
// costs one hipGetDevice (a thread-local read) and a short table scan.
#include <atomic>
#include <cstdlib>
#include <mutex>
#include <utility>
#include <vector>

#include "a2d_common.hpp"

namespace a2d {
namespace {

constexpr int kMaxDevices = 64;
std::atomic<int> g_cus[kMaxDevices];                       // 0 = not asked yet
std::mutex g_mu;
std::vector<std::pair<int, const void*>> g_prepared;       // (device, kernel): limit already raised
std::atomic<int> g_force_generic{-1};                      // -1 = environment not read yet

// kernel trace of the calling host thread (a2d_debug_trace)
thread_local hipEvent_t* t_trace_events = nullptr;
thread_local int t_trace_cap = 0;
thread_local int t_trace_used = 0;

}  // namespace

hipError_t device_cus(int* cus) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const bool cached = dev >= 0 && dev < kMaxDevices;
  int c = cached ? g_cus[dev].load(std::memory_order_relaxed) : 0;
  if (c <= 0) {
    e = hipDeviceGetAttribute(&c, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    if (c <= 0) return hipErrorInvalidDevice;
    if (cached) g_cus[dev].store(c, std::memory_order_relaxed);
  }
  *cus = c;
  return hipSuccess;
}

hipError_t ensure_dynamic_lds(const void* kernel, int bytes) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const std::pair<int, const void*> key(dev, kernel);
  {
    std::lock_guard<std::mutex> lock(g_mu);
    for (const auto& p : g_prepared)
      if (p == key) return hipSuccess;
  }
  // (two threads may both get here for the same kernel: setting the attribute twice is harmless)
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e != hipSuccess) return e;
  std::lock_guard<std::mutex> lock(g_mu);
  g_prepared.push_back(key);
  return hipSuccess;
}

bool force_generic() {
  int v = g_force_generic.load(std::memory_order_relaxed);
  if (v < 0) {
    const char* e = getenv("A2D_FORCE_GENERIC");       // read once per process
    v = (e && e[0] == '1') ? 1 : 0;
    int expected = -1;
    if (!g_force_generic.compare_exchange_strong(expected, v)) v = expected;   // a setter came first
  }
  return v != 0;
}

void set_force_generic(bool on) { g_force_generic.store(on ? 1 : 0); }

void trace_set(hipEvent_t* events, int n) {
  t_trace_events = (events && n > 0) ? events : nullptr;
  t_trace_cap = t_trace_events ? n : 0;
  t_trace_used = 0;
}
int trace_count() { return t_trace_used; }
void trace_mark(hipStream_t s) {
  if (!t_trace_events || t_trace_used >= t_trace_cap) return;
  if (hipEventRecord(t_trace_events[t_trace_used], s) == hipSuccess) ++t_trace_used;
}

}  // namespace a2d
