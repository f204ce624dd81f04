// Internal helpers shared by the library's translation units (error reporting, launch checks,
// workspace carving). Nothing here is exported.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "../../include/hgnn.h"

namespace hgnn {

int32_t set_error(int32_t code, const char* fmt, ...);

#define HGNN_REQUIRE(cond, code, ...)                         \
  do {                                                        \
    if (!(cond)) return ::hgnn::set_error((code), __VA_ARGS__); \
  } while (0)

#define HGNN_HIP(expr)                                                                      \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess)                                                                   \
      return ::hgnn::set_error(HGNN_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

#define HGNN_LAUNCH_CHECK(name)                                                             \
  do {                                                                                      \
    hipError_t e_ = hipGetLastError();                                                      \
    if (e_ != hipSuccess)                                                                   \
      return ::hgnn::set_error(HGNN_ERR_HIP, "launch of %s failed: %s", name,               \
                               hipGetErrorString(e_));                                      \
  } while (0)

#define HGNN_TRY(expr)            \
  do {                            \
    int32_t s_ = (expr);          \
    if (s_ != HGNN_OK) return s_; \
  } while (0)

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// Wait for a stream by polling: the calls that hand a count or an error to the host sit in the middle of a step,
// where the wake-up latency of a blocking wait would leave the GPU idle.
inline hipError_t wait_stream(hipStream_t st) {
  hipError_t e;
  while ((e = hipStreamQuery(st)) == hipErrorNotReady) {
  }
  return e;
}

// Carves aligned sub-buffers out of a caller workspace; `used()` is what a size query reports.
struct Carver {
  char* base;
  size_t off = 0;
  explicit Carver(void* p) : base(static_cast<char*>(p)) {}
  template <typename T>
  T* take(size_t count) {
    T* r = reinterpret_cast<T*>(base ? base + off : nullptr);
    off += align_up(count * sizeof(T));
    return r;
  }
  size_t used() const { return off; }
};

inline bool valid_H(int H) { return H == 64 || H == 128 || H == 256; }

// compute units of the current device (asked once)
inline int num_cus() {
  static int n = 0;
  if (n == 0) {
    hipDeviceProp_t prop;
    int dev = 0;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
      n = prop.multiProcessorCount;
    if (n <= 0) n = 256;
  }
  return n;
}

// device-wide exclusive prefix sum of n int32 values; out has n+1 entries (out[n] = total).
// scratch must hold scan_scratch_ints(n) ints.
size_t scan_scratch_ints(int64_t n);
int32_t exclusive_scan_i32(hipStream_t st, const int32_t* in, int32_t* out, int64_t n, int32_t* scratch);

}  // namespace hgnn
