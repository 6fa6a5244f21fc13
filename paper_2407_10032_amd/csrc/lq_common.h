// Shared host-side helpers of the LeanQuant HIP library: error text, argument
// checks, launch checks.  No device code and no arithmetic of the method here.
#pragma once

#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>

#include <mutex>

#include "../../include/leanquant.h"

namespace lq {

// Thread-local error text returned by lq_last_error().
char* error_buffer();
lq_status fail(lq_status code, const char* fmt, ...);

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Side streams (two) and a few events each, per host thread and device, created on first use and
// kept for the life of the thread.  Calls use it to run independent kernel chains side by
// side with the caller's stream (fork and join through events, so the work is still
// ordered after everything enqueued before the call and before everything enqueued after
// it).  Returns nullptr if the objects cannot be created; callers then stay on one stream.
struct SideStream {
  hipStream_t stream;
  hipEvent_t fork[4];   // recorded on the caller's stream, waited on by the side stream
  hipEvent_t join;      // recorded on the side stream, waited on by the caller's stream
};
SideStream* side_stream(int which = 0);   // which: 0 or 1

// One-time set-up per device (kernel attributes such as the dynamic LDS limit), safe when
// several host threads enter a call for the first time together and when one process drives
// several devices.  Usage:
//   static lq::DeviceOnce once_flag;
//   if (lq::DeviceOnceGuard once(once_flag); once.first()) { ...set up...; once.done(); }
// The guard holds the flag's mutex for its lifetime; a set-up that fails (early return) is
// tried again by the next call.
constexpr int MAX_DEVICES = 16;
struct DeviceOnce {
  std::mutex m;
  bool done[MAX_DEVICES] = {};
};
class DeviceOnceGuard {
 public:
  explicit DeviceOnceGuard(DeviceOnce& o) : o_(o), lk_(o.m) {
    if (hipGetDevice(&dev_) != hipSuccess || dev_ < 0 || dev_ >= MAX_DEVICES) dev_ = -1;
  }
  bool first() const { return dev_ < 0 || !o_.done[dev_]; }
  void done() { if (dev_ >= 0) o_.done[dev_] = true; }
 private:
  DeviceOnce& o_;
  std::unique_lock<std::mutex> lk_;
  int dev_ = -1;
};

// Resolve Eq. 8's shrink limit t for the given parameters; returns < 0 if invalid.
int resolve_t(const lq_params* P);
// Validate the fields every call shares; returns LQ_OK or sets the error text.
lq_status check_params(const lq_params* P, int64_t c);

}  // namespace lq

#define LQ_CHECK_HIP(expr)                                                                   \
  do {                                                                                       \
    hipError_t _e = (expr);                                                                  \
    if (_e != hipSuccess)                                                                    \
      return lq::fail(LQ_ERR_HIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(_e),     \
                      __FILE__, __LINE__);                                                   \
  } while (0)

#define LQ_CHECK_LAUNCH(name)                                                                \
  do {                                                                                       \
    hipError_t _e = hipGetLastError();                                                       \
    if (_e != hipSuccess)                                                                    \
      return lq::fail(LQ_ERR_HIP, "launch of %s failed: %s", name, hipGetErrorString(_e));   \
  } while (0)
