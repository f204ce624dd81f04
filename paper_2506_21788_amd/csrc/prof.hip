// Kernel-class timing with HIP events (see prof.h) and its exported control functions.
#include "prof.h"

#include <vector>

#include "common.h"

namespace hgnn {

uint64_t g_prof_mask = 0;

namespace {
struct Rec {
  int tag;
  hipEvent_t a, b;
};
std::vector<Rec> g_recs;
std::vector<hipEvent_t> g_pool;
double g_ms[PT_COUNT];
long long g_n[PT_COUNT];

hipEvent_t get_event() {
  if (!g_pool.empty()) {
    hipEvent_t e = g_pool.back();
    g_pool.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  (void)hipEventCreate(&e);
  return e;
}

const char* const kNames[PT_COUNT] = {
    "neigh_setup", "neigh_count", "neigh_fill", "neigh_emit", "neigh_transpose", "pack", "gemm_node",
    "wgrad_node", "wgrad_edge", "colsum", "seg_fwd", "segsum_dst", "segsum_src", "head_out", "pool", "embed",
    "misc", "edge_fused_fwd", "edge_fused_bwd", "frag_gemm_edge", "frag_wgrad_edge", "edge_elementwise", "to_frag"};
}  // namespace

void prof_record(int tag, hipStream_t st, bool start) {
  if (start) {
    Rec r{tag, get_event(), get_event()};
    (void)hipEventRecord(r.a, st);
    g_recs.push_back(r);
  } else {
    // scopes nest like a stack: close the innermost open record of this tag
    for (size_t k = g_recs.size(); k-- > 0;) {
      if (g_recs[k].tag == tag) {
        (void)hipEventRecord(g_recs[k].b, st);
        break;
      }
    }
  }
}

}  // namespace hgnn

using namespace hgnn;

extern "C" int32_t hgnn_profile_begin(uint64_t tag_mask) {
  for (auto& r : g_recs) {
    g_pool.push_back(r.a);
    g_pool.push_back(r.b);
  }
  g_recs.clear();
  for (int t = 0; t < PT_COUNT; ++t) {
    g_ms[t] = 0.0;
    g_n[t] = 0;
  }
  g_prof_mask = tag_mask;
  return HGNN_OK;
}

extern "C" int32_t hgnn_profile_end(void* stream) {
  g_prof_mask = 0;
  HGNN_HIP(hipStreamSynchronize(static_cast<hipStream_t>(stream)));
  for (auto& r : g_recs) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) {
      g_ms[r.tag] += ms;
      g_n[r.tag] += 1;
    }
    g_pool.push_back(r.a);
    g_pool.push_back(r.b);
  }
  g_recs.clear();
  return HGNN_OK;
}

extern "C" int32_t hgnn_profile_num_tags(void) { return PT_COUNT; }

extern "C" const char* hgnn_profile_tag_name(int32_t tag) {
  return (tag >= 0 && tag < PT_COUNT) ? kNames[tag] : "";
}

extern "C" int32_t hgnn_profile_read(int32_t tag, int64_t* launches_host, double* total_ms_host) {
  HGNN_REQUIRE(tag >= 0 && tag < PT_COUNT, HGNN_ERR_BAD_SHAPE, "unknown profile tag %d", tag);
  HGNN_REQUIRE(launches_host && total_ms_host, HGNN_ERR_NULLPTR, "profile_read: null pointer");
  *launches_host = g_n[tag];
  *total_ms_host = g_ms[tag];
  return HGNN_OK;
}
