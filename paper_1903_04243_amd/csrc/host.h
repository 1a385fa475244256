// Host-side helpers shared by the sources that implement the C ABI: the per-thread error text, the
// name under which the kernels being enqueued are timed, and the launch-and-check macro.
#pragma once

#include "../../include/pfg.h"
#include "common.h"

namespace pfg {

// Stores a printf-style message as the calling thread's last error and returns code.
int fail(int code, const char *fmt, ...);
void clear_error();
// Family name recorded for the kernels enqueued next on this thread (per-kernel timing).
void set_timing_family(const char *name);

constexpr int64_t kMaxRows = 0x7fffffffLL;          // folded iteration index m = b * S + s
constexpr int64_t kMaxElems = (int64_t)1 << 46;     // per tensor

// Checks of a dense network that every entry point shares: sizes, activation, dtype, then the
// weight pointers.  Both return a pfg_status and record the error text.
int check_mlp(const pfg_mlp *net);
int check_mlp_weights(const pfg_mlp *net);

inline float *ws_at(void *ws, size_t off) {
  return reinterpret_cast<float *>(static_cast<char *>(ws) + off);
}

}  // namespace pfg

#define PFG_LAUNCH(name, expr)                                                                \
  do {                                                                                        \
    ::pfg::set_timing_family(name);                                                           \
    hipError_t e_ = (expr);                                                                   \
    if (e_ != hipSuccess)                                                                     \
      return ::pfg::fail(-6 /* PFG_ERR_DEVICE */, "%s: %s", name, hipGetErrorString(e_));     \
  } while (0)
