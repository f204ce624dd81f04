// hgnn_mp_layer_fwd / hgnn_mp_layer_bwd: host-side sequencing of one message-passing layer.
//
// The first edge linear layer is split by linearity,
//     W1^T [h_i ; h_j ; d2] = (h W1a)_i + (h W1b)_j + d2 * w1d,
// so its two H x H products are done once per ATOM (P = h W1a + b1, Q = h W1b) and each edge only
// gathers and adds two rows. The per-edge matrix work is then the single H x H product with W2.
// The reverse pass mirrors this: the gradient with respect to z1 is reduced per destination (g_P)
// and per source (g_Q, through the source-sorted plan) and the W1 products run per atom again.
#include <cstdlib>

#include "edge_fused.h"
#include "edgeops.h"
#include "gemm.h"
#include "side.h"
#include "wide.h"

namespace hgnn {

struct LayerOff {  // element offsets into the flat weight buffer (k edge attributes: W1 has 2H + k rows)
  long W1, b1, W2, b2, wx, W3, b3, W4, b4, total;
  explicit LayerOff(long H, long k = 1) {
    long o = 0;
    W1 = o; o += (2 * H + k) * H;
    b1 = o; o += H;
    W2 = o; o += H * H;
    b2 = o; o += H;
    wx = o; o += H;
    W3 = o; o += 2 * H * H;
    b3 = o; o += H;
    W4 = o; o += H * H;
    b4 = o; o += H;
    total = o;
  }
};

struct LayerSaved {
  float* PQ;    // [N,2H] fp32  P = h W1a + b1 | Q = h W1b   (or the same as bf16 pairs, [N,H] words)
  void* z2_vm;  // [E32,H] z2, v-major fragment order (bf16 or fp32)
  void* a1_pk;  // [E32,H] silu(z1), operand-packed fragment order (bf16 or fp32); null with bf16 pairs and the single
                // d2 attribute, where the reverse pass recomputes it
  float* M;     // [N,H]
  float* z3;    // [N,H]
  float* xe;    // [E] x_e = wx . m_e (written only when the caller may ask for edge gradients)
  size_t bytes;
};

// a1 is recomputed (not stored) where the weight-gradient kernel can rebuild it from the gathers alone
// a1 = silu(z1) is not stored but recomputed by the W2-gradient kernel: bf16 pairs (H = 256), and fp32 operands at
// H = 128, with the squared length as the only edge attribute
static bool a1_recomputed(int H, bool bf16, int k) { return (edge_pairs(H, bf16) || (!bf16 && H == 128)) && k == 1; }

static LayerSaved carve_saved(void* p, int N, int64_t E, int H, bool bf16, int k = 1) {
  Carver c(p);
  LayerSaved s;
  const size_t eb = frag_rows(E) * H * (bf16 ? 2 : 4);
  s.PQ = c.take<float>((size_t)N * 2 * H);
  s.z2_vm = c.take<char>(eb);
  s.a1_pk = a1_recomputed(H, bf16, k) ? nullptr : c.take<char>(eb);
  s.M = c.take<float>((size_t)N * H);
  s.z3 = c.take<float>((size_t)N * H);
  s.xe = c.take<float>((size_t)E + 4);
  s.bytes = c.used();
  return s;
}

struct LayerWs {
  void* packed;    // 6 blocks
  void* packed_x3; // fp32 operands: W2 (forward) or W2^T (reverse) as three bf16 planes for the fused edge kernels
  void* gz2_pk;    // [E32,H] operand-packed
  void* gz1_vm;    // [E32,H] v-major (bf16 or fp32)
  float* cvec;     // [E]
  float* g_z3;     // [N,H]
  float* g_hM;     // [N,2H]
  unsigned* gM_pk; // [N,H/2] words: g_M as bf16 pairs (only when the fused kernels gather pairs)
  float* g_PQ;     // [N,2H]
  float* partial;  // split-K / column-sum partials of the main stream
  float* partial2; // partials of the W2 gradient
  float* partial3; // partials of the atom-level weight gradients
  float* cs_partial;  // column-sum partials of the node weight-gradient kernel (side stream)
  float* attrpart;    // partials of the attribute rows of g_W1 (k > 1 only)
  float* dpart;       // per-unit partials of the destination sums formed inside the reverse edge kernel
  size_t bytes;
};

static LayerWs carve_ws(void* p, int N, int64_t E, int H, bool bf16, int k = 1) {
  Carver c(p);
  LayerWs w;
  w.packed = c.take<char>(6 * packed_block_bytes(H, bf16));
  w.packed_x3 = bf16 ? nullptr : c.take<char>(packed_x3_bytes(H));
  w.gz2_pk = c.take<char>(frag_rows(E) * H * (bf16 ? 2 : 4));
  w.gz1_vm = c.take<char>(frag_rows(E) * H * (bf16 ? 2 : 4));
  w.cvec = c.take<float>((size_t)E + 4);
  w.g_z3 = c.take<float>((size_t)N * H);
  w.g_hM = c.take<float>((size_t)N * 2 * H);
  w.gM_pk = c.take<unsigned>((size_t)N * (H / 2));
  w.g_PQ = c.take<float>((size_t)N * 2 * H);
  // three regions of their own: the reductions of a reverse pass run as one launch at its end, so the partials of
  // the edge kernel, of the W2 gradient and of the atom-level weight gradients all live until then
  const size_t pc = colsum_partial_floats(H, N, 1), pe = edge_bwd_colpart_floats(H);
  w.partial = c.take<float>(pc > pe ? pc : pe);
  w.partial2 = c.take<float>(wgrad_frag_partial_floats(H));
  w.partial3 = c.take<float>(wgrad_partial_floats(H, N, 5, 1));   // the layer's five atom-level blocks in one launch
  w.cs_partial = c.take<float>(wgrad_colsum_partial_floats(H, N));
  w.attrpart = k > 1 ? c.take<float>(edge_bwd_attrpart_floats(H)) : nullptr;
  w.dpart = edge_bwd_sums_dst(H, bf16) && k <= 1 ? c.take<float>(edge_bwd_dpart_floats(E, H)) : nullptr;
  w.bytes = c.used();
  return w;
}

// Weight gradients are off the critical path of the reverse pass (nothing downstream reads them), so they run
// on a library-owned side stream (default priority) that forks from and joins the caller's stream through
// events: they overlap the latency-bound kernels of the main chain. Everything stays asynchronous to the host.
SideStream& side_stream() {
  static SideStream ss;
  if (!ss.ok) {
    bool good = hipStreamCreateWithFlags(&ss.s, hipStreamNonBlocking) == hipSuccess;
    for (auto& e : ss.ev) good = good && hipEventCreateWithFlags(&e, hipEventDisableTiming) == hipSuccess;
    ss.ok = good;
  }
  return ss;
}
// `to` waits for everything enqueued on `from` so far
int32_t stream_after(hipStream_t to, hipStream_t from, hipEvent_t ev) {
  HGNN_HIP(hipEventRecord(ev, from));
  HGNN_HIP(hipStreamWaitEvent(to, ev, 0));
  return HGNN_OK;
}

// -2: not read yet (then the environment variable HGNN_SIDE_STREAM decides: "0" = off, "1" = on, anything else or
// unset = the library's choice); -1: the library's choice; 0 / 1: set by the caller.
// The library's choice: on for the fragment path (its many atom-level launches leave compute units idle that the
// weight gradients fill: config 6 13.18 against 13.31 ms per step), off for the fused kernels, every one of which
// fills the chip by itself (config 1 0.93 against 1.03 ms, config 5 32.2 against 32.6 ms, configs 2-4 the same
// either way).
static int g_side_mode = -2;
static int side_setting() {
  if (g_side_mode == -2) {
    const char* e = getenv("HGNN_SIDE_STREAM");
    g_side_mode = (e && e[0] == '0') ? 0 : ((e && e[0] == '1') ? 1 : -1);
  }
  return g_side_mode;
}
bool side_stream_enabled(bool fragment_path) {
  const int s = side_setting();
  return s < 0 ? fragment_path : s != 0;
}

static int32_t check_layer_args(int N, int64_t E, int H, int dtype) {
  HGNN_REQUIRE(N >= 0 && E >= 0, HGNN_ERR_BAD_SHAPE, "negative N or E");
  HGNN_REQUIRE(E <= 2147483647LL - 128, HGNN_ERR_OVERFLOW, "edge count does not fit the 32-bit edge indices");
  // the edge kernels gather rows of [N,2H] fp32 node tensors at 32-bit byte offsets
  HGNN_REQUIRE((int64_t)N * 2 * H * 4 < (1ll << 32), HGNN_ERR_OVERFLOW,
               "N * 2H * 4 bytes must stay below 4 GiB (N = %d, H = %d)", N, H);
  HGNN_REQUIRE(dtype == HGNN_F32 || dtype == HGNN_BF16, HGNN_ERR_BAD_SHAPE, "unknown dtype %d", dtype);
  HGNN_REQUIRE(valid_H(H) || wide_H(H), HGNN_ERR_BAD_SHAPE, "H must lie in 1..1024 (got %d)", H);
  HGNN_REQUIRE(!wide_H(H) || dtype == HGNN_BF16, HGNN_ERR_UNIMPLEMENTED,
               "widths other than 64, 128, 256 run with bf16 operands only (H = %d)", H);
  return HGNN_OK;
}

}  // namespace hgnn

using namespace hgnn;

extern "C" int32_t hgnn_set_side_stream(int32_t enable) {
  const int32_t before = side_setting();
  g_side_mode = enable < 0 ? -1 : (enable ? 1 : 0);
  return before;
}

static int32_t layer_sizes(int32_t N, int64_t E, int32_t H, int32_t k, int32_t dtype, size_t* ws_bytes_host,
                           size_t* saved_bytes_host) {
  HGNN_TRY(check_layer_args(N, E, H, dtype));
  HGNN_REQUIRE(ws_bytes_host && saved_bytes_host, HGNN_ERR_NULLPTR, "null size pointer");
  if (wide_H(H)) {
    wide_layer_sizes(N, E, H, k, ws_bytes_host, saved_bytes_host);
    return HGNN_OK;
  }
  *ws_bytes_host = carve_ws(nullptr, N, E, H, dtype == HGNN_BF16, k).bytes;
  *saved_bytes_host = carve_saved(nullptr, N, E, H, dtype == HGNN_BF16, k).bytes;
  return HGNN_OK;
}

extern "C" int32_t hgnn_mp_layer_workspace_bytes(int32_t N, int64_t E, int32_t H, int32_t dtype,
                                                 size_t* ws_bytes_host, size_t* saved_bytes_host) {
  return layer_sizes(N, E, H, 1, dtype, ws_bytes_host, saved_bytes_host);
}

// Scratch behind the workspace proper for calls without a saved buffer: the saved tensors and two [N,3] vectors
static size_t unsaved_extra_bytes(int N, int64_t E, int H, bool bf16, int k) {
  return carve_saved(nullptr, N, E, H, bf16, k).bytes + 2 * align_up((size_t)N * 3 * sizeof(float));
}

// Everything of the forward pass that the reverse pass needs again (P|Q, z2 (a1), M, z3), written to `s`; also v_out.
// Packs its own weight blocks into w.packed: 0 W1a, 1 W1b, 2 W2, 3 W3a, 4 W3b, 5 W4.
// keep_xe: also keep x_e = wx . m_e per edge (fused kernels only; the fragment path always does)
// k == 1: `attr` is the single per-edge attribute (the squared length); k > 1: [E,k] attributes, bf16 operands
// h_out (optional): also h' = h + silu(z3) W4 + b4, formed by the kernel that forms z3 while its tile is on the chip
static int32_t layer_fwd_core(hipStream_t st, int32_t N, int64_t E, int32_t H, int32_t k, bool bf16, float alpha,
                              const int32_t* row_ptr, const int32_t* dst, const int32_t* col, const float* attr,
                              const float* rvec, const float* h_in, const float* v_in, const float* W, float* v_out,
                              const LayerWs& w, const LayerSaved& s, bool keep_xe, float* h_out) {
  const LayerOff o(H, k);
  PackArgs pk;
  pk.src = W;
  pk.dst = w.packed;
  pk.nblocks = 6;
  const long HH = (long)H * H;
  pk.d[0] = {o.W1, H, 1};
  pk.d[1] = {o.W1 + HH, H, 1};
  pk.d[2] = {o.W2, H, 1};
  pk.d[3] = {o.W3, H, 1};
  pk.d[4] = {o.W3 + HH, H, 1};
  pk.d[5] = {o.W4, H, 1};
  pk.x3_dst = w.packed_x3; pk.x3_desc = 2;   // fp32 operands: W2 also as three bf16 planes
  HGNN_TRY(launch_pack(st, H, bf16, pk));

  {  // P | Q
    GemmArgs g;
    g.A[0] = h_in; g.lda[0] = H; g.nkc = 1;
    g.B = w.packed; g.blk[0][0] = 0; g.blk[0][1] = 1; g.ncb = 2;
    g.M = N;
    g.bias = W + o.b1; g.bias_cb_mask = 1;
    g.C = s.PQ; g.ldc = 2 * H;
    if (edge_pairs(H, bf16)) {
      g.Cpair = reinterpret_cast<unsigned*>(s.PQ); g.ldpair = H; g.pair_cb_mask = 3;
      g.pair_off[0] = 0; g.pair_off[1] = H / 2;
    }
    HGNN_TRY(launch_gemm_chain(st, H, bf16, nullptr, g, 0));   // h is staged once for both halves
  }
  {  // per edge: a1 = silu(P[dst] + Q[col] + d2*w1d), z2 = a1 W2 + b2   (one fused kernel)
    EdgeFwdArgs e;
    e.E = E; e.dst = dst; e.col = col;
    if (k > 1) { e.d2 = nullptr; e.attr = attr; e.k = k; e.W1a = W + o.W1 + 2 * HH; }
    else e.d2 = attr;
    e.PQ = s.PQ; e.w1d = W + o.W1 + 2 * HH;
    e.W2p = static_cast<const char*>(w.packed) + 2 * packed_block_bytes(H, bf16);
    if (!bf16) e.W2p = w.packed_x3;
    e.b2 = W + o.b2;
    e.a1_pk = s.a1_pk; e.z2_vm = s.z2_vm;
    HGNN_TRY(launch_edge_fwd(st, H, bf16, e));
  }
  HGNN_TRY(launch_seg_fwd_vm(st, H, bf16, N, row_ptr, s.z2_vm, rvec, W + o.wx, alpha, v_in, s.M, v_out,
                             keep_xe ? s.xe : nullptr));
  {  // z3 = [h ; M] W3 + b3
    GemmArgs g;
    g.A[0] = h_in; g.lda[0] = H; g.A[1] = s.M; g.lda[1] = H; g.nkc = 2;
    g.B = w.packed; g.blk[0][0] = 3; g.blk[1][0] = 4;
    g.M = N;
    g.bias = W + o.b3; g.bias_cb_mask = 1;
    g.C = s.z3; g.ldc = H;
    if (h_out) {  // h' = h + silu(z3) W4 + b4 from the same tile
      GemmArgs g2;
      g2.B = w.packed; g2.blk[0][0] = 5;
      g2.M = N;
      g2.bias = W + o.b4; g2.bias_cb_mask = 1;
      g2.add1 = h_in; g2.ldadd1 = H;
      g2.C = h_out; g2.ldc = H;
      HGNN_TRY(launch_gemm_chain(st, H, bf16, &g, g2, 1));
    } else {
      HGNN_TRY(launch_gemm(st, H, bf16, g));
    }
  }
  return HGNN_OK;
}

static int32_t mp_layer_fwd_impl(void* stream, int32_t N, int64_t E, int32_t H, int32_t k, int32_t dtype, float alpha,
                                 const int32_t* row_ptr, const int32_t* dst, const int32_t* col, const float* d2,
                                 const float* rvec, const float* h_in, const float* v_in, const float* W, float* h_out,
                                 float* v_out, void* saved, size_t saved_bytes, void* ws, size_t ws_bytes, bool keep_xe) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  HGNN_TRY(check_layer_args(N, E, H, dtype));
  if (N == 0) return HGNN_OK;
  HGNN_REQUIRE(row_ptr && h_in && v_in && W && h_out && v_out && ws, HGNN_ERR_NULLPTR, "mp_layer_fwd: null pointer");
  HGNN_REQUIRE(E == 0 || (dst && col && d2 && rvec), HGNN_ERR_NULLPTR, "mp_layer_fwd: null edge array");
  HGNN_REQUIRE(h_out != h_in, HGNN_ERR_BAD_SHAPE, "h_out may not alias h_in");
  if (wide_H(H)) {
    HGNN_REQUIRE(saved != nullptr, HGNN_ERR_UNIMPLEMENTED,
                 "mp_layer_fwd without a saved buffer exists at H = 64, 128, 256 only (H = %d)", H);
    size_t need_ws, need_saved;
    wide_layer_sizes(N, E, H, 1, &need_ws, &need_saved);
    HGNN_REQUIRE(ws_bytes >= need_ws, HGNN_ERR_WORKSPACE_TOO_SMALL, "mp_layer workspace: need %zu bytes, got %zu", need_ws, ws_bytes);
    HGNN_REQUIRE(saved_bytes >= need_saved, HGNN_ERR_WORKSPACE_TOO_SMALL, "mp_layer saved buffer: need %zu bytes, got %zu", need_saved, saved_bytes);
    WideLayerArgs a;
    a.N = N; a.E = E; a.H = H; a.alpha = alpha;
    a.row_ptr = row_ptr; a.dst = dst; a.col = col; a.d2 = d2; a.rvec = rvec;
    a.h_in = h_in; a.v_in = v_in; a.W = W; a.h_out = h_out; a.v_out = v_out;
    a.saved = saved; a.ws = ws;
    return wide_layer_fwd(st, a);
  }
  const bool bf16 = dtype == HGNN_BF16;
  LayerWs w = carve_ws(ws, N, E, H, bf16, k);
  if (saved == nullptr) {
    // nothing is kept for the reverse pass: the intermediates live behind the workspace proper for this call only
    const size_t need = w.bytes + unsaved_extra_bytes(N, E, H, bf16, k);
    HGNN_REQUIRE(ws_bytes >= need, HGNN_ERR_WORKSPACE_TOO_SMALL,
                 "mp_layer workspace without a saved buffer: need %zu bytes (workspace + saved size), got %zu", need, ws_bytes);
    saved = static_cast<char*>(ws) + w.bytes;
    saved_bytes = ws_bytes - w.bytes;
  }
  LayerSaved s = carve_saved(saved, N, E, H, bf16, k);
  HGNN_REQUIRE(ws_bytes >= w.bytes, HGNN_ERR_WORKSPACE_TOO_SMALL, "mp_layer workspace: need %zu bytes, got %zu", w.bytes, ws_bytes);
  HGNN_REQUIRE(saved_bytes >= s.bytes, HGNN_ERR_WORKSPACE_TOO_SMALL, "mp_layer saved buffer: need %zu bytes, got %zu", s.bytes, saved_bytes);
  const LayerOff o(H, k);
  HGNN_TRY(layer_fwd_core(st, N, E, H, k, bf16, alpha, row_ptr, dst, col, d2, rvec, h_in, v_in, W, v_out, w, s, keep_xe, h_out));
  return HGNN_OK;
}

extern "C" int32_t hgnn_mp_layer_fwd(void* stream, int32_t N, int64_t E, int32_t H, int32_t dtype, float alpha,
                                     const int32_t* row_ptr, const int32_t* dst, const int32_t* col,
                                     const float* d2, const float* rvec, const float* h_in, const float* v_in,
                                     const float* W, float* h_out, float* v_out, void* saved, size_t saved_bytes,
                                     void* ws, size_t ws_bytes) {
  return mp_layer_fwd_impl(stream, N, E, H, 1, dtype, alpha, row_ptr, dst, col, d2, rvec, h_in, v_in, W, h_out, v_out, saved,
                           saved_bytes, ws, ws_bytes, false);
}

// g_d2 / g_rvec (optional, fused kernels): gradient with respect to d2 and to the edge vectors; the forward pass must
// have kept x_e
static int32_t mp_layer_bwd_impl(void* stream, int32_t N, int64_t E, int32_t H, int32_t k, int32_t dtype, float alpha,
                                 const int32_t* row_ptr, const int32_t* dst, const int32_t* col, const float* d2,
                                 const float* rvec, const int32_t* colT_ptr, const int32_t* permT, const float* h_in,
                                 const float* W, const void* saved, size_t saved_bytes, const float* g_h_out,
                                 const float* g_v_out, float* g_h_in, float* g_v_in, float* gW, void* ws,
                                 size_t ws_bytes, float* g_d2, float* g_rvec) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  HGNN_TRY(check_layer_args(N, E, H, dtype));
  HGNN_REQUIRE(gW && W && ws, HGNN_ERR_NULLPTR, "mp_layer_bwd: null pointer");
  HGNN_REQUIRE(N == 0 || (row_ptr && colT_ptr && h_in && g_h_out && g_v_out && g_h_in && g_v_in),
               HGNN_ERR_NULLPTR, "mp_layer_bwd: null pointer");
  HGNN_REQUIRE(E == 0 || (dst && col && d2 && rvec && permT), HGNN_ERR_NULLPTR, "mp_layer_bwd: null edge array");
  HGNN_REQUIRE(N == 0 || g_h_in != g_h_out, HGNN_ERR_BAD_SHAPE, "g_h_in may not alias g_h_out");
  if (N == 0) return launch_fill_f32(st, gW, LayerOff(H, k).total, 0.f);
  if (wide_H(H)) {
    HGNN_REQUIRE(saved != nullptr, HGNN_ERR_UNIMPLEMENTED,
                 "mp_layer_bwd without a saved buffer exists at H = 64, 128, 256 only (H = %d)", H);
    size_t need_ws, need_saved;
    wide_layer_sizes(N, E, H, 1, &need_ws, &need_saved);
    HGNN_REQUIRE(ws_bytes >= need_ws, HGNN_ERR_WORKSPACE_TOO_SMALL, "mp_layer workspace: need %zu bytes, got %zu", need_ws, ws_bytes);
    HGNN_REQUIRE(saved_bytes >= need_saved, HGNN_ERR_WORKSPACE_TOO_SMALL, "mp_layer saved buffer: need %zu bytes, got %zu", need_saved, saved_bytes);
    WideLayerArgs a;
    a.N = N; a.E = E; a.H = H; a.alpha = alpha;
    a.row_ptr = row_ptr; a.dst = dst; a.col = col; a.d2 = d2; a.rvec = rvec;
    a.colT_ptr = colT_ptr; a.permT = permT;
    a.h_in = h_in; a.W = W; a.g_h_out = g_h_out; a.g_v_out = g_v_out; a.g_h_in = g_h_in; a.g_v_in = g_v_in; a.gW = gW;
    a.saved = const_cast<void*>(saved); a.ws = ws;
    return wide_layer_bwd(st, a);
  }
  const bool bf16 = dtype == HGNN_BF16;
  LayerWs w = carve_ws(ws, N, E, H, bf16, k);
  const bool recompute = saved == nullptr;
  if (recompute) {
    HGNN_REQUIRE(g_d2 == nullptr && g_rvec == nullptr, HGNN_ERR_BAD_SHAPE,
                 "edge gradients need the saved buffer of hgnn_mp_layer_attr_fwd");
    const size_t need = w.bytes + unsaved_extra_bytes(N, E, H, bf16, k);
    HGNN_REQUIRE(ws_bytes >= need, HGNN_ERR_WORKSPACE_TOO_SMALL,
                 "mp_layer workspace without a saved buffer: need %zu bytes (workspace + saved size), got %zu", need, ws_bytes);
    saved = static_cast<char*>(ws) + w.bytes;
    saved_bytes = ws_bytes - w.bytes;
  }
  LayerSaved s = carve_saved(const_cast<void*>(saved), N, E, H, bf16, k);
  HGNN_REQUIRE(ws_bytes >= w.bytes, HGNN_ERR_WORKSPACE_TOO_SMALL, "mp_layer workspace: need %zu bytes, got %zu", w.bytes, ws_bytes);
  HGNN_REQUIRE(saved_bytes >= s.bytes, HGNN_ERR_WORKSPACE_TOO_SMALL, "mp_layer saved buffer: need %zu bytes, got %zu", s.bytes, saved_bytes);
  const LayerOff o(H, k);
  const long HH = (long)H * H;
  if (recompute) {
    // the forward pass of this layer once more, up to z3 (its v' goes to scratch; the input v does not matter for
    // anything the reverse pass reads, so any valid [N,3] array serves)
    float* v_scratch = reinterpret_cast<float*>(static_cast<char*>(const_cast<void*>(saved)) + s.bytes);
    HGNN_TRY(layer_fwd_core(st, N, E, H, k, bf16, alpha, row_ptr, dst, col, d2, rvec, h_in, g_v_out, W, v_scratch, w, s, false, nullptr));
  }

  // transposed blocks: 0 W4^T, 1 W3a^T, 2 W3b^T, 3 W2^T, 4 W1a^T, 5 W1b^T
  PackArgs pk;
  pk.src = W;
  pk.dst = w.packed;
  pk.nblocks = 6;
  pk.d[0] = {o.W4, 1, H};
  pk.d[1] = {o.W3, 1, H};
  pk.d[2] = {o.W3 + HH, 1, H};
  pk.d[3] = {o.W2, 1, H};
  pk.d[4] = {o.W1, 1, H};
  pk.d[5] = {o.W1 + HH, 1, H};
  pk.x3_dst = w.packed_x3; pk.x3_desc = 3;   // fp32 operands: W2^T also as three bf16 planes
  HGNN_TRY(launch_pack(st, H, bf16, pk));

  SideStream& ss = side_stream();
  HGNN_REQUIRE(ss.ok, HGNN_ERR_HIP, "could not create the side stream");
  hipStream_t sx = side_stream_enabled(false) ? ss.s : st;
  HGNN_TRY(stream_after(sx, st, ss.ev[0]));   // inputs of this call are ready on the side stream too
  // one stream: the four reductions of split partials below (edge kernel sums, W2 gradient, atom-level weight
  // gradients and their bias sums) run as one launch at the end; nothing in this call reads their results
  ReduceQueueScope reductions(st, sx == st);

  // every gradient field is written below even when there is nothing to sum over
  {  // g_z3 = (g_h' W4^T) * silu'(z3), and from the same tile [g_h' + g_h(a) | g_M] = g_z3 W3^T (+ g_h' on the first half)
    GemmArgs g;
    g.A[0] = g_h_out; g.lda[0] = H;
    g.B = w.packed; g.blk[0][0] = 0;
    g.M = N;
    g.mul = s.z3; g.ldmul = H; g.mul_is_z = 1;
    g.C = w.g_z3; g.ldc = H;
    GemmArgs g2;
    g2.B = w.packed; g2.blk[0][0] = 1; g2.blk[0][1] = 2; g2.ncb = 2;
    g2.M = N;
    g2.add1 = g_h_out; g2.ldadd1 = H; g2.add1_cb_mask = 1;
    g2.C = w.g_hM; g2.ldc = 2 * H;
    if (edge_pairs(H, bf16)) {   // the g_M half goes out as bf16 pairs for the fused edge kernel
      g2.Cpair = w.gM_pk; g2.ldpair = H / 2; g2.pair_cb_mask = 2; g2.pair_off[1] = 0;
      g2.pair_scale = alpha;   // the pair form carries alpha * g_M
    }
    HGNN_TRY(launch_gemm_chain(st, H, bf16, &g, g2, 0));
  }
  // edge part: c_e, then g_z2 -> (x W2^T) -> g_z1 with the per-column sums. The fused edge kernel fills
  // every CU by itself, so the side stream is drained first instead of competing with it.
  HGNN_TRY(launch_edge_cvec(st, E, dst, rvec, g_v_out, alpha, w.cvec));
  HGNN_TRY(stream_after(st, sx, ss.ev[5]));
  // With bf16 pairs, or fp32 operands at H = 128, the reverse edge kernel also sums g_z1 per destination (out of the
  // tile it holds in LDS). The gradient with respect to d2 (on request: the dot of every g_z1 row with the d2 row of
  // W1) is then formed by the source-sorted pass, which reads every edge's row exactly once as well.
  // HGNN_DSUM_IN_KERNEL=0 keeps the separate destination-sorted pass (for comparing the two).
  const char* dsum_env = getenv("HGNN_DSUM_IN_KERNEL");
  DsumFix dfix{nullptr, nullptr, nullptr, 0};
  const bool dsum_in_kernel = edge_bwd_sums_dst(H, bf16) && k <= 1 && N > 0 && !(dsum_env && dsum_env[0] == '0');
  {
    EdgeBwdArgs e;
    e.E = E; e.dst = dst; e.col = col;
    if (k > 1) {
      e.d2 = nullptr; e.attr = d2; e.k = k; e.W1a = W + o.W1 + 2 * HH;
      e.attrpart = w.attrpart; e.g_W1a = gW + o.W1 + 2 * HH;
    } else {
      e.d2 = d2;
    }
    e.PQ = s.PQ; e.w1d = W + o.W1 + 2 * HH;
    e.W2Tp = static_cast<const char*>(w.packed) + 3 * packed_block_bytes(H, bf16);
    if (!bf16) e.W2Tp = w.packed_x3;
    e.z2_vm = s.z2_vm;
    if (edge_pairs(H, bf16)) { e.gM = w.gM_pk; e.ldgM = H / 2; }
    else { e.gM = w.g_hM + H; e.ldgM = 2 * H; }
    e.cvec = w.cvec; e.wx = W + o.wx; e.alpha = alpha;
    e.gz2_pk = w.gz2_pk; e.gz1_vm = w.gz1_vm;
    e.colpart = w.partial;
    e.g_b2 = gW + o.b2; e.g_wx = gW + o.wx; e.g_w1d = k > 1 ? nullptr : gW + o.W1 + 2 * HH;
    if (dsum_in_kernel) {
      e.gP = w.g_PQ; e.ldgP = 2 * H; e.dpart = w.dpart; e.row_ptr = row_ptr; e.N = N;
      dfix = edge_bwd_dsum_fix(e);   // the source-sorted sum below adds the partials on its way
    }
    HGNN_TRY(launch_edge_bwd(st, H, bf16, e));
  }
  HGNN_TRY(stream_after(sx, st, ss.ev[2]));
  // side: g_W2 = a1^T g_z2 streams while the main stream runs the two segment sums
  if (a1_recomputed(H, bf16, k) && !bf16)
    HGNN_TRY(launch_wgrad_frag_recompute32(sx, H, E, dst, col, d2, reinterpret_cast<const float*>(s.PQ),
                                           W + o.W1 + 2 * HH, w.gz2_pk, w.partial2, gW + o.W2));
  else if (a1_recomputed(H, bf16, k))
    HGNN_TRY(launch_wgrad_frag_recompute(sx, H, E, dst, col, d2, s.PQ, W + o.W1 + 2 * HH, w.gz2_pk, w.partial2,
                                         gW + o.W2));
  else
    HGNN_TRY(launch_wgrad_frag(sx, H, bf16, E, s.a1_pk, w.gz2_pk, w.partial2, gW + o.W2));
  // g_P (and, on request, the gradient with respect to d2: the dot of every g_z1 row with the d2 row of W1)
  if (dsum_in_kernel) {
    // g_P left the edge kernel already
  } else if (k > 1) {
    // several attributes: the gradient with respect to them (on request) is a pass of its own over g_z1
    HGNN_TRY(launch_segsum_vm(st, H, bf16, N, row_ptr, nullptr, w.gz1_vm, w.g_PQ, 2 * H, PT_SEGSUM_DST));
    if (g_d2) HGNN_TRY(launch_gattr_vm(st, H, E, w.gz1_vm, W + o.W1 + 2 * HH, k, g_d2));
  } else {
    HGNN_TRY(launch_segsum_vm(st, H, bf16, N, row_ptr, nullptr, w.gz1_vm, w.g_PQ, 2 * H, PT_SEGSUM_DST,
                              W + o.W1 + 2 * HH, g_d2));
  }
  if (g_rvec) HGNN_TRY(launch_edge_grvec(st, E, dst, s.xe, g_v_out, alpha, g_rvec));
  if (dsum_in_kernel)   // g_Q, the rows of g_P that cross tiles, and g_d2 where it is asked for
    HGNN_TRY(launch_segsum_vm(st, H, bf16, N, colT_ptr, permT, w.gz1_vm, w.g_PQ + H, 2 * H, PT_SEGSUM_SRC,
                              g_d2 ? W + o.W1 + 2 * HH : nullptr, g_d2, &dfix));
  else
    HGNN_TRY(launch_segsum_vm(st, H, bf16, N, colT_ptr, permT, w.gz1_vm, w.g_PQ + H, 2 * H, PT_SEGSUM_SRC));  // g_Q
  {  // g_h = (g_h' + g_h(a)) + g_P W1a^T + g_Q W1b^T
    GemmArgs g;
    g.A[0] = w.g_PQ; g.lda[0] = 2 * H; g.A[1] = w.g_PQ + H; g.lda[1] = 2 * H; g.nkc = 2;
    g.B = w.packed; g.blk[0][0] = 4; g.blk[1][0] = 5;
    g.M = N;
    g.add1 = w.g_hM; g.ldadd1 = 2 * H;
    g.C = g_h_in; g.ldc = H;
    HGNN_TRY(launch_gemm(st, H, bf16, g));
  }
  {  // the three atom-level weight gradients of the layer and their bias sums in one launch, once all their operands
     // exist: gW4 = silu(z3)^T g_h', gb4 | gW3 = [h ; M]^T g_z3, gb3 | gW1a = h^T g_P, gW1b = h^T g_Q, gb1 = sum_i g_P_i
    HGNN_TRY(stream_after(sx, st, ss.ev[3]));
    WgradArgs j[3];
    j[0].A[0] = s.z3; j[0].lda[0] = H; j[0].a_silu = 1;
    j[0].B[0] = g_h_out; j[0].ldb[0] = H;
    j[0].dest[0] = gW + o.W4;
    j[0].colsum_dest[0] = gW + o.b4;
    j[1].A[0] = h_in; j[1].lda[0] = H; j[1].A[1] = s.M; j[1].lda[1] = H; j[1].nA = 2;
    j[1].B[0] = w.g_z3; j[1].ldb[0] = H;
    j[1].dest[0] = gW + o.W3; j[1].dest[1] = gW + o.W3 + HH;
    j[1].colsum_dest[0] = gW + o.b3;
    j[2].A[0] = h_in; j[2].lda[0] = H;
    j[2].B[0] = w.g_PQ; j[2].ldb[0] = 2 * H; j[2].B[1] = w.g_PQ + H; j[2].ldb[1] = 2 * H; j[2].nB = 2;
    j[2].dest[0] = gW + o.W1; j[2].dest[1] = gW + o.W1 + HH;
    j[2].colsum_dest[0] = gW + o.b1;
    for (auto& a : j) a.M = N;
    j[0].partial = w.partial3; j[0].colsum_partial = w.cs_partial;
    HGNN_TRY(launch_wgrad_multi(sx, H, bf16, j, 3));
  }
  {
    ProfScope ps(PT_MISC, st);
    if (g_v_in != g_v_out && N > 0) {   // g_v passes through: a reduction of one partial is a copy (joins the launch below)
      float* dest[4] = {g_v_in, nullptr, nullptr, nullptr};
      HGNN_TRY(launch_reduce_partials(st, g_v_out, 1, 1, (long)N * 3, dest, 1, 0));
    }
    HGNN_TRY(reductions.flush());
  }
  HGNN_TRY(stream_after(st, sx, ss.ev[4]));   // join: the caller's stream now also orders after every gradient
  return HGNN_OK;
}

extern "C" int32_t hgnn_mp_layer_bwd(void* stream, int32_t N, int64_t E, int32_t H, int32_t dtype, float alpha,
                                     const int32_t* row_ptr, const int32_t* dst, const int32_t* col,
                                     const float* d2, const float* rvec, const int32_t* colT_ptr,
                                     const int32_t* permT, const float* h_in, const float* W, const void* saved,
                                     size_t saved_bytes, const float* g_h_out, const float* g_v_out,
                                     float* g_h_in, float* g_v_in, float* gW, void* ws, size_t ws_bytes) {
  return mp_layer_bwd_impl(stream, N, E, H, 1, dtype, alpha, row_ptr, dst, col, d2, rvec, colT_ptr, permT, h_in, W, saved,
                           saved_bytes, g_h_out, g_v_out, g_h_in, g_v_in, gW, ws, ws_bytes, nullptr, nullptr);
}

// ---------------------------------------------------------------------------------------------
// the layer with k edge attributes in place of d2 (fragment path; one attribute at H = 64 / 128 / 256: the fused kernels)
// ---------------------------------------------------------------------------------------------
static int32_t check_attr_args(int N, int64_t E, int H, int k, int dtype) {
  HGNN_REQUIRE(N >= 0 && E >= 0, HGNN_ERR_BAD_SHAPE, "negative N or E");
  HGNN_REQUIRE(E <= 2147483647LL - 256, HGNN_ERR_OVERFLOW, "edge count does not fit the 32-bit edge indices");
  HGNN_REQUIRE(dtype == HGNN_F32 || dtype == HGNN_BF16, HGNN_ERR_BAD_SHAPE, "unknown dtype %d", dtype);
  HGNN_REQUIRE(H >= 1 && H <= 1024, HGNN_ERR_BAD_SHAPE, "H must lie in 1..1024 (got %d)", H);
  HGNN_REQUIRE(k >= 1 && k <= WIDE_MAX_ATTR, HGNN_ERR_BAD_SHAPE, "k must lie in 1..%d (got %d)", WIDE_MAX_ATTR, k);
  HGNN_REQUIRE(dtype == HGNN_BF16 || (k == 1 && valid_H(H)), HGNN_ERR_UNIMPLEMENTED,
               "layers with several edge attributes, or of a width other than 64, 128, 256, run with bf16 operands only");
  return HGNN_OK;
}
// every width the fused kernels serve (several attributes: bf16 operands, which check_attr_args has made sure of)
static bool attr_on_fused_kernels(int H, int k) { (void)k; return valid_H(H); }

extern "C" int32_t hgnn_mp_layer_attr_workspace_bytes(int32_t N, int64_t E, int32_t H, int32_t k, int32_t dtype,
                                                      size_t* ws_bytes_host, size_t* saved_bytes_host) {
  HGNN_TRY(check_attr_args(N, E, H, k, dtype));
  HGNN_REQUIRE(ws_bytes_host && saved_bytes_host, HGNN_ERR_NULLPTR, "null size pointer");
  if (attr_on_fused_kernels(H, k)) return layer_sizes(N, E, H, k, dtype, ws_bytes_host, saved_bytes_host);
  wide_layer_sizes(N, E, H, k, ws_bytes_host, saved_bytes_host);
  return HGNN_OK;
}

extern "C" int32_t hgnn_mp_layer_attr_fwd(void* stream, int32_t N, int64_t E, int32_t H, int32_t k, int32_t dtype,
                                          float alpha, const int32_t* row_ptr, const int32_t* dst, const int32_t* col,
                                          const float* attr, const float* rvec, const float* h_in, const float* v_in,
                                          const float* W, float* h_out, float* v_out, void* saved, size_t saved_bytes,
                                          void* ws, size_t ws_bytes) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  HGNN_TRY(check_attr_args(N, E, H, k, dtype));
  if (attr_on_fused_kernels(H, k))
    return mp_layer_fwd_impl(stream, N, E, H, k, dtype, alpha, row_ptr, dst, col, attr, rvec, h_in, v_in, W, h_out, v_out,
                             saved, saved_bytes, ws, ws_bytes, true);
  if (N == 0) return HGNN_OK;
  HGNN_REQUIRE(row_ptr && h_in && v_in && W && h_out && v_out && ws && saved, HGNN_ERR_NULLPTR, "mp_layer_attr_fwd: null pointer");
  HGNN_REQUIRE(E == 0 || (dst && col && attr && rvec), HGNN_ERR_NULLPTR, "mp_layer_attr_fwd: null edge array");
  HGNN_REQUIRE(h_out != h_in, HGNN_ERR_BAD_SHAPE, "h_out may not alias h_in");
  size_t need_ws, need_saved;
  wide_layer_sizes(N, E, H, k, &need_ws, &need_saved);
  HGNN_REQUIRE(ws_bytes >= need_ws, HGNN_ERR_WORKSPACE_TOO_SMALL, "mp_layer workspace: need %zu bytes, got %zu", need_ws, ws_bytes);
  HGNN_REQUIRE(saved_bytes >= need_saved, HGNN_ERR_WORKSPACE_TOO_SMALL, "mp_layer saved buffer: need %zu bytes, got %zu", need_saved, saved_bytes);
  WideLayerArgs a;
  a.N = N; a.E = E; a.H = H; a.alpha = alpha;
  a.row_ptr = row_ptr; a.dst = dst; a.col = col; a.attr = attr; a.k = k; a.rvec = rvec;
  a.h_in = h_in; a.v_in = v_in; a.W = W; a.h_out = h_out; a.v_out = v_out;
  a.saved = saved; a.ws = ws;
  return wide_layer_fwd(st, a);
}

extern "C" int32_t hgnn_mp_layer_attr_bwd(void* stream, int32_t N, int64_t E, int32_t H, int32_t k, int32_t dtype,
                                          float alpha, const int32_t* row_ptr, const int32_t* dst, const int32_t* col,
                                          const float* attr, const float* rvec, const int32_t* colT_ptr,
                                          const int32_t* permT, const float* h_in, const float* W, const void* saved,
                                          size_t saved_bytes, const float* g_h_out, const float* g_v_out, float* g_h_in,
                                          float* g_v_in, float* gW, float* g_attr, float* g_rvec, void* ws,
                                          size_t ws_bytes) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  HGNN_TRY(check_attr_args(N, E, H, k, dtype));
  if (attr_on_fused_kernels(H, k))
    return mp_layer_bwd_impl(stream, N, E, H, k, dtype, alpha, row_ptr, dst, col, attr, rvec, colT_ptr, permT, h_in, W,
                             saved, saved_bytes, g_h_out, g_v_out, g_h_in, g_v_in, gW, ws, ws_bytes, g_attr, g_rvec);
  HGNN_REQUIRE(gW && W && ws, HGNN_ERR_NULLPTR, "mp_layer_attr_bwd: null pointer");
  HGNN_REQUIRE(N == 0 || (row_ptr && colT_ptr && h_in && saved && g_h_out && g_v_out && g_h_in && g_v_in),
               HGNN_ERR_NULLPTR, "mp_layer_attr_bwd: null pointer");
  HGNN_REQUIRE(E == 0 || (dst && col && attr && rvec && permT), HGNN_ERR_NULLPTR, "mp_layer_attr_bwd: null edge array");
  HGNN_REQUIRE(N == 0 || g_h_in != g_h_out, HGNN_ERR_BAD_SHAPE, "g_h_in may not alias g_h_out");
  if (N == 0) return launch_fill_f32(st, gW, 6L * H * H + (5L + k) * H, 0.f);
  size_t need_ws, need_saved;
  wide_layer_sizes(N, E, H, k, &need_ws, &need_saved);
  HGNN_REQUIRE(ws_bytes >= need_ws, HGNN_ERR_WORKSPACE_TOO_SMALL, "mp_layer workspace: need %zu bytes, got %zu", need_ws, ws_bytes);
  HGNN_REQUIRE(saved_bytes >= need_saved, HGNN_ERR_WORKSPACE_TOO_SMALL, "mp_layer saved buffer: need %zu bytes, got %zu", need_saved, saved_bytes);
  WideLayerArgs a;
  a.N = N; a.E = E; a.H = H; a.alpha = alpha;
  a.row_ptr = row_ptr; a.dst = dst; a.col = col; a.attr = attr; a.k = k; a.rvec = rvec;
  a.colT_ptr = colT_ptr; a.permT = permT;
  a.h_in = h_in; a.W = W; a.g_h_out = g_h_out; a.g_v_out = g_v_out; a.g_h_in = g_h_in; a.g_v_in = g_v_in; a.gW = gW;
  a.g_attr = g_attr; a.g_rvec = g_rvec;
  a.saved = const_cast<void*>(saved); a.ws = ws;
  return wide_layer_bwd(st, a);
}
