// The library-owned side stream of the reverse pass (internal; defined in layer.hip): weight gradients and bias sums
// feed nothing downstream, so they are forked onto it and joined before the call returns.
#pragma once

#include "common.h"

namespace hgnn {

struct SideStream {
  hipStream_t s = nullptr;
  hipEvent_t ev[8] = {};
  bool ok = false;
};
SideStream& side_stream();          // created on first use (default priority, non-blocking)
bool side_stream_enabled(bool fragment_path);   // hgnn_set_side_stream / HGNN_SIDE_STREAM, else the library's choice per path
int32_t stream_after(hipStream_t to, hipStream_t from, hipEvent_t ev);   // `to` waits for what `from` holds so far

}  // namespace hgnn
