// Declarations shared by the host and device translation units of libslkv.
#ifndef SLKV_INTERNAL_H
#define SLKV_INTERNAL_H

#include <stdint.h>

#include "slkv.h"

namespace slkv {

constexpr int kMaxRows = 512;         // (Hq/Hkv) * w rows scored per KV head
constexpr int kMaxPool = 63;          // widest pooling window
constexpr int kMaxSegPerLaunch = 64;  // (sequence, KV head) segments described per kernel launch

// Sets the calling thread's error detail and returns `s`.
slkv_status fail(slkv_status s, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

// Rows kept for a segment of n tokens, window w and capacity cap (Algorithm 3).
int64_t kept_rows(int64_t n, int64_t w, int64_t cap);

// Checks everything in the descriptor that can be checked on the host.
slkv_status validate_desc(const slkv_layer_desc* d);
slkv_status validate_ragged_desc(const slkv_ragged_desc* d);

// Kernel timing (slkv_profile_begin / _end).  A ScopedKernelTimer names the kernel that the
// launches inside its scope belong to; while profiling is on, profile_events() hands such a
// launch a pair of events that the launch itself carries (start and end of the kernel's own
// execution, without the launch gap an event recorded on the stream would include).
class ScopedKernelTimer {
 public:
  explicit ScopedKernelTimer(int kernel_id, void* stream = nullptr);
  ~ScopedKernelTimer();
 private:
  int prev_;
};
// False when profiling is off, no kernel is named or the record pool is used up.
bool profile_events(void** start_event, void** stop_event);

}  // namespace slkv

#endif
