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

// ---------------------------------------------------------------------------------------------
// Matrix-core rate probe (instrumentation): every wavefront runs `iters` rounds of four independent
// 32x32 matrix-core instructions on registers only, so the kernel measures what the matrix pipes sustain
// (to set the published peak beside a measured one). Returns the number of floating-point operations issued.
// ---------------------------------------------------------------------------------------------
namespace hgnn {
typedef float probe_f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 probe_bf16x8 __attribute__((ext_vector_type(8)));

template <bool BF16>
__global__ void __launch_bounds__(256) k_mfma_probe(int iters, float* sink) {
  probe_f32x16 acc[4];
#pragma unroll
  for (int k = 0; k < 4; ++k)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[k][v] = 0.f;
  const float seed = 1.0f + (float)(threadIdx.x & 7) * 0.125f;
  probe_bf16x8 a, b;
#pragma unroll
  for (int t = 0; t < 8; ++t) { a[t] = (__bf16)seed; b[t] = (__bf16)(0.5f * seed); }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if constexpr (BF16) acc[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[k], 0, 0, 0);
      else acc[k] = __builtin_amdgcn_mfma_f32_32x32x2f32(seed, 0.5f * seed, acc[k], 0, 0, 0);
    }
  }
  float s = 0.f;
#pragma unroll
  for (int k = 0; k < 4; ++k)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += acc[k][v];
  if (s == 12345.678f) sink[0] = s;   // keeps the loop alive; never true in practice
}
}  // namespace hgnn

extern "C" int64_t hgnn_mfma_probe(void* stream, int32_t dtype, int32_t workgroups, int32_t iters, float* sink) {
  if (workgroups <= 0 || iters <= 0 || !sink) return 0;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const bool bf16 = dtype == 1;
  if (bf16) hgnn::k_mfma_probe<true><<<dim3((unsigned)workgroups), 256, 0, st>>>(iters, sink);
  else hgnn::k_mfma_probe<false><<<dim3((unsigned)workgroups), 256, 0, st>>>(iters, sink);
  if (hipGetLastError() != hipSuccess) return 0;
  const int64_t per_instr = bf16 ? 2LL * 32 * 32 * 16 : 2LL * 32 * 32 * 2;
  return (int64_t)workgroups * 4 /*wavefronts*/ * iters * 4 * per_instr;
}

// ---------------------------------------------------------------------------------------------
// Load-path rate probe (instrumentation): what the vector memory path (16-byte loads per lane, 1 KiB per wavefront
// instruction, eight in flight) and the LDS (ds_read_b128) deliver per compute unit, to set beside the operand
// traffic of the matrix kernels.
// kind 0: wavefront w reads 1 KiB chunks of a device buffer cyclically: window > 0: chunks w * window .. + window - 1;
//         window == 0: its equal share of the buffer (a buffer far larger than the caches streams from HBM, one of a
//         few MB stays in the L2); window < 0: every wavefront the same first -window chunks (they stay in the L1)
// kind 1: every wavefront reads eight 1 KiB pieces of a 32 KiB LDS array per round
// ---------------------------------------------------------------------------------------------
namespace hgnn {
typedef unsigned probe_u32x4 __attribute__((ext_vector_type(4)));

__global__ void __launch_bounds__(256) k_load_probe_global(int iters, long window, const char* __restrict__ buf,
                                                           long nchunks, unsigned* sink) {
  const int lane = threadIdx.x & 63;
  const long w = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  const long nwaves = (long)gridDim.x * 4;
  const long own = nchunks / nwaves >= 8 ? nchunks / nwaves : 8;       // window == 0: an equal share of the buffer
  const long span = window > 0 ? window : window < 0 ? -window : own;
  const long first = window > 0 ? (w * window) % nchunks : window < 0 ? 0 : (w * own) % nchunks;
  probe_u32x4 acc = {0u, 0u, 0u, 0u};
  long pos = 0;
  for (int it = 0; it < iters; ++it) {
    probe_u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      long c = first + (pos + u) % span;
      if (c >= nchunks) c -= nchunks;
      v[u] = *reinterpret_cast<const probe_u32x4*>(buf + c * 1024 + lane * 16);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u];
    pos = (pos + 8) % span;
  }
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u) sink[0] = acc[0];   // keeps the loads alive
}

__global__ void __launch_bounds__(256) k_load_probe_lds(int iters, unsigned* sink) {
  __shared__ __align__(16) probe_u32x4 lds[2048];   // 32 KiB
  for (int i = threadIdx.x; i < 2048; i += 256) lds[i] = probe_u32x4{(unsigned)i, 1u, 2u, 3u};
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  probe_u32x4 acc = {0u, 0u, 0u, 0u};
  for (int it = 0; it < iters; ++it) {
    probe_u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = lds[((it + wave * 8 + u * 4) & 31) * 64 + lane];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u];
  }
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u) sink[0] = acc[0];
}
// kind 2: as kind 0 with window == 0, but the eight 1 KiB chunks of a round go from memory straight into the LDS
// (16 bytes per lane, lane l of a wavefront lands at its 16 l of the 1 KiB piece), without passing through registers.
// Every round one piece is compared with a plain load of the same chunk; sink[1] counts the mismatching lanes.
__global__ void __launch_bounds__(256) k_load_probe_to_lds(int iters, const char* __restrict__ buf, long nchunks,
                                                           unsigned* sink) {
  __shared__ __align__(16) probe_u32x4 lds[4 * 8 * 64];   // 8 KiB per wavefront
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const long w = (long)blockIdx.x * 4 + wave;
  const long nwaves = (long)gridDim.x * 4;
  const long own = nchunks / nwaves >= 8 ? nchunks / nwaves : 8;
  const long first = (w * own) % nchunks;
  probe_u32x4 acc = {0u, 0u, 0u, 0u};
  unsigned bad = 0;
  long pos = 0;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      long c = first + (pos + u) % own;
      if (c >= nchunks) c -= nchunks;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(buf + c * 1024 + lane * 16),
                                       (__attribute__((address_space(3))) void*)&lds[(wave * 8 + u) * 64], 16, 0, 0);
    }
    __syncthreads();   // waits for the loads of every wavefront
    const int u = it & 7;
    const probe_u32x4 got = lds[(wave * 8 + u) * 64 + lane];
    acc ^= got;
    if (it < 16) {     // the check costs a second load: first rounds only
      long c = first + (pos + u) % own;
      if (c >= nchunks) c -= nchunks;
      const probe_u32x4 want = *reinterpret_cast<const probe_u32x4*>(buf + c * 1024 + lane * 16);
      bad += (got[0] != want[0]) | (got[1] != want[1]) | (got[2] != want[2]) | (got[3] != want[3]);
    }
    __syncthreads();   // the piece has been read before the next round overwrites it
    pos = (pos + 8) % own;
  }
  if (bad) atomicAdd(&sink[1], bad);
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u) sink[0] = acc[0];
}
}  // namespace hgnn

extern "C" int64_t hgnn_load_probe(void* stream, int32_t kind, int32_t workgroups, int32_t iters, int64_t window_chunks,
                                   const void* buf, int64_t buf_bytes, void* sink) {
  if (workgroups <= 0 || iters <= 0 || !sink) return 0;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (kind == 0) {
    const long nchunks = buf_bytes / 1024;
    const long aw = window_chunks < 0 ? -window_chunks : window_chunks;
    if (!buf || nchunks < 8 || aw > nchunks || (aw > 0 && aw < 8)) return 0;
    hgnn::k_load_probe_global<<<dim3((unsigned)workgroups), 256, 0, st>>>(iters, window_chunks, static_cast<const char*>(buf),
                                                                          nchunks, static_cast<unsigned*>(sink));
  } else if (kind == 1) {
    hgnn::k_load_probe_lds<<<dim3((unsigned)workgroups), 256, 0, st>>>(iters, static_cast<unsigned*>(sink));
  } else if (kind == 2) {
    const long nchunks = buf_bytes / 1024;
    if (!buf || nchunks < 8) return 0;
    hgnn::k_load_probe_to_lds<<<dim3((unsigned)workgroups), 256, 0, st>>>(iters, static_cast<const char*>(buf), nchunks,
                                                                          static_cast<unsigned*>(sink));
  } else {
    return 0;
  }
  if (hipGetLastError() != hipSuccess) return 0;
  return (int64_t)workgroups * 4 * iters * 8 * 1024;
}
