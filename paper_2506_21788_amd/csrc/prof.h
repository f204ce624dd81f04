// Optional timing of kernel classes with HIP events on the launch stream (internal). A ProfScope
// around a launch records a start/stop event pair when its tag is enabled; otherwise it costs one
// load and a branch.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace hgnn {

enum ProfTag : int {
  PT_NEIGH_SETUP = 0,   // per-graph metadata, binning, scans
  PT_NEIGH_COUNT,       // candidate walk, counting pass
  PT_NEIGH_FILL,        // candidate walk, fill pass
  PT_NEIGH_EMIT,        // in-row ranking + edge emission
  PT_NEIGH_TRANSPOSE,   // source-sorted plan
  PT_PACK,              // weight packing
  PT_GEMM_NODE,         // row-tile GEMM over atoms / graphs
  PT_WGRAD_NODE,        // transposed GEMM over atoms / graphs (+ its partial reduction)
  PT_WGRAD_EDGE,        // transposed GEMM over edges (+ its partial reduction)
  PT_COLSUM,            // column sums (bias and vector gradients)
  PT_SEG_FWD,           // destination-sorted segmented reduction of messages
  PT_SEGSUM_DST,        // destination-sorted segmented sum (backward)
  PT_SEGSUM_SRC,        // source-sorted (transpose) segmented sum (backward)
  PT_HEAD_OUT,          // head output layers
  PT_POOL,
  PT_EMBED,
  PT_MISC,
  PT_EDGE_FUSED_FWD,    // fused gather + GEMM + segmented reduction (forward)
  PT_EDGE_FUSED_BWD,    // fused backward edge kernels
  PT_FRAG_GEMM_EDGE,    // fragment path (widths other than 64 / 128 / 256): per-edge H x H products (z2 = a1 W2, g_a1 = g_z2 W2^T)
  PT_FRAG_WGRAD_EDGE,   // fragment path (widths other than 64 / 128 / 256): g_W2 = a1^T g_z2 (+ its partial reduction)
  PT_EDGE_ELEM,         // fragment path (widths other than 64 / 128 / 256): element-wise edge kernels (a1, g_z2, g_z1)
  PT_TO_FRAG,           // fragment path (widths other than 64 / 128 / 256): row-major -> fragment conversions of atom tensors
  PT_COUNT
};

extern uint64_t g_prof_mask;
void prof_record(int tag, hipStream_t st, bool start);

struct ProfScope {
  int tag;
  hipStream_t st;
  bool on;
  ProfScope(int t, hipStream_t s) : tag(t), st(s), on((g_prof_mask >> t) & 1ull) {
    if (on) prof_record(tag, st, true);
  }
  ~ProfScope() {
    if (on) prof_record(tag, st, false);
  }
};

}  // namespace hgnn
