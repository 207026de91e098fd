// Optional per-kernel timing (slkv_profile_begin / slkv_profile_end): every timed launch carries its
// own start / stop events (hipExtLaunchKernelGGL), so a record is the kernel's execution time.
#include <hip/hip_runtime.h>

#include <atomic>
#include <mutex>
#include <vector>

#include "slkv_internal.h"

namespace {
struct Rec {
  int id;
  hipEvent_t a, b;
};
std::mutex g_mu;
std::atomic<bool> g_on{false};   // read without the lock on the launch path
std::vector<Rec> g_pool;   // events created by slkv_profile_begin
size_t g_used = 0;
}  // namespace

namespace {
thread_local int tl_kernel_id = -1;   // kernel named by the innermost ScopedKernelTimer of this thread
}

namespace slkv {

ScopedKernelTimer::ScopedKernelTimer(int id, void*) : prev_(tl_kernel_id) { tl_kernel_id = id; }

ScopedKernelTimer::~ScopedKernelTimer() { tl_kernel_id = prev_; }

bool profile_events(void** start_event, void** stop_event) {
  if (tl_kernel_id < 0 || !g_on.load(std::memory_order_relaxed)) return false;
  std::lock_guard<std::mutex> lk(g_mu);
  if (!g_on.load(std::memory_order_relaxed) || g_used >= g_pool.size()) return false;
  Rec& r = g_pool[g_used++];
  r.id = tl_kernel_id;
  *start_event = (void*)r.a;
  *stop_event = (void*)r.b;
  return true;
}

}  // namespace slkv

using namespace slkv;

extern "C" slkv_status slkv_profile_begin(int32_t max_records) {
  clear_error();
  if (max_records < 1 || max_records > (1 << 20)) return fail(SLKV_ERR_BAD_ARG, "max_records outside 1..2^20");
  std::lock_guard<std::mutex> lk(g_mu);
  while ((int)g_pool.size() < max_records) {
    Rec r;
    r.id = -1;
    if (hipEventCreate(&r.a) != hipSuccess || hipEventCreate(&r.b) != hipSuccess)
      return fail(SLKV_ERR_HIP, "hipEventCreate failed");
    g_pool.push_back(r);
  }
  g_used = 0;
  g_on = true;
  return SLKV_OK;
}

extern "C" slkv_status slkv_profile_end(slkv_kernel_time* h_records, int32_t capacity, int32_t* count) {
  clear_error();
  if (!count) return fail(SLKV_ERR_NULL, "count is NULL");
  std::lock_guard<std::mutex> lk(g_mu);
  g_on = false;
  int n = 0;
  for (size_t i = 0; i < g_used; ++i) {
    if (hipEventSynchronize(g_pool[i].b) != hipSuccess) return fail(SLKV_ERR_HIP, "hipEventSynchronize failed");
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, g_pool[i].a, g_pool[i].b) != hipSuccess)
      return fail(SLKV_ERR_HIP, "hipEventElapsedTime failed");
    if (h_records && n < capacity) {
      h_records[n].kernel = g_pool[i].id;
      h_records[n].ms = ms;
    }
    ++n;
  }
  *count = n;
  g_used = 0;
  return SLKV_OK;
}
