// hgnn_mp_layer_fwd / hgnn_mp_layer_bwd: host-side sequencing of one message-passing layer.
//
// The first edge linear layer is split by linearity,
//     W1^T [h_i ; h_j ; d2] = (h W1a)_i + (h W1b)_j + d2 * w1d,
// so its two H x H products are done once per ATOM (P = h W1a + b1, Q = h W1b) and each edge only
// gathers and adds two rows. The per-edge matrix work is then the single H x H product with W2.
// The reverse pass mirrors this: the gradient with respect to z1 is reduced per destination (g_P)
// and per source (g_Q, through the source-sorted plan) and the W1 products run per atom again.
#include "edgeops.h"
#include "gemm.h"

namespace hgnn {

struct LayerOff {  // element offsets into the flat weight buffer
  long W1, b1, W2, b2, wx, W3, b3, W4, b4, total;
  explicit LayerOff(long H) {
    long o = 0;
    W1 = o; o += (2 * H + 1) * H;
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
  float* PQ;  // [N,2H]  P = h W1a + b1 | Q = h W1b
  float* z2;  // [E,H]
  float* M;   // [N,H]
  float* z3;  // [N,H]
  size_t bytes;
};

static LayerSaved carve_saved(void* p, int N, int64_t E, int H) {
  Carver c(p);
  LayerSaved s;
  s.PQ = c.take<float>((size_t)N * 2 * H);
  s.z2 = c.take<float>((size_t)E * H);
  s.M = c.take<float>((size_t)N * H);
  s.z3 = c.take<float>((size_t)N * H);
  s.bytes = c.used();
  return s;
}

struct LayerWs {
  void* packed;    // 6 blocks
  float* a1;       // [E,H]
  float* s1;       // [E,H]  silu'(z1), overwritten in place by g_z1
  float* g_z2;     // [E,H]
  float* cvec;     // [E]
  float* g_z3;     // [N,H]
  float* g_hM;     // [N,2H]
  float* g_PQ;     // [N,2H]
  float* partial;  // split-K / column-sum partials
  size_t bytes;
};

static LayerWs carve_ws(void* p, int N, int64_t E, int H, bool bf16) {
  Carver c(p);
  LayerWs w;
  w.packed = c.take<char>(6 * packed_block_bytes(H, bf16));
  w.a1 = c.take<float>((size_t)E * H);
  w.s1 = c.take<float>((size_t)E * H);
  w.g_z2 = c.take<float>((size_t)E * H);
  w.cvec = c.take<float>((size_t)E + 1);
  w.g_z3 = c.take<float>((size_t)N * H);
  w.g_hM = c.take<float>((size_t)N * 2 * H);
  w.g_PQ = c.take<float>((size_t)N * 2 * H);
  const int64_t mx = E > N ? E : N;
  size_t pf = wgrad_partial_floats(H, mx, 2, 1);
  size_t cf = colsum_partial_floats(H, mx, 1);
  w.partial = c.take<float>(pf > cf ? pf : cf);
  w.bytes = c.used();
  return w;
}

static int32_t check_layer_args(int N, int64_t E, int H, int dtype) {
  HGNN_REQUIRE(N >= 0 && E >= 0, HGNN_ERR_BAD_SHAPE, "negative N or E");
  HGNN_REQUIRE(E < (1ll << 31) / 1, HGNN_ERR_OVERFLOW, "edge count does not fit int32");
  HGNN_REQUIRE(valid_H(H), HGNN_ERR_BAD_SHAPE, "H must be 64, 128 or 256 (got %d)", H);
  HGNN_REQUIRE(dtype == HGNN_F32 || dtype == HGNN_BF16, HGNN_ERR_BAD_SHAPE, "unknown dtype %d", dtype);
  return HGNN_OK;
}

}  // namespace hgnn

using namespace hgnn;

extern "C" int32_t hgnn_mp_layer_workspace_bytes(int32_t N, int64_t E, int32_t H, int32_t dtype,
                                                 size_t* ws_bytes_host, size_t* saved_bytes_host) {
  HGNN_TRY(check_layer_args(N, E, H, dtype));
  HGNN_REQUIRE(ws_bytes_host && saved_bytes_host, HGNN_ERR_NULLPTR, "null size pointer");
  *ws_bytes_host = carve_ws(nullptr, N, E, H, dtype == HGNN_BF16).bytes;
  *saved_bytes_host = carve_saved(nullptr, N, E, H).bytes;
  return HGNN_OK;
}

extern "C" int32_t hgnn_mp_layer_fwd(void* stream, int32_t N, int64_t E, int32_t H, int32_t dtype, float alpha,
                                     const int32_t* row_ptr, const int32_t* dst, const int32_t* col,
                                     const float* d2, const float* rvec, const float* h_in, const float* v_in,
                                     const float* W, float* h_out, float* v_out, void* saved, size_t saved_bytes,
                                     void* ws, size_t ws_bytes) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  HGNN_TRY(check_layer_args(N, E, H, dtype));
  if (N == 0) return HGNN_OK;
  HGNN_REQUIRE(row_ptr && h_in && v_in && W && h_out && v_out && ws, HGNN_ERR_NULLPTR, "mp_layer_fwd: null pointer");
  HGNN_REQUIRE(E == 0 || (dst && col && d2 && rvec), HGNN_ERR_NULLPTR, "mp_layer_fwd: null edge array");
  HGNN_REQUIRE(saved != nullptr, HGNN_ERR_UNIMPLEMENTED,
               "mp_layer_fwd without a saved buffer (recompute in backward) is not implemented");
  HGNN_REQUIRE(h_out != h_in, HGNN_ERR_BAD_SHAPE, "h_out may not alias h_in");
  const bool bf16 = dtype == HGNN_BF16;
  LayerWs w = carve_ws(ws, N, E, H, bf16);
  LayerSaved s = carve_saved(saved, N, E, H);
  HGNN_REQUIRE(ws_bytes >= w.bytes, HGNN_ERR_WORKSPACE_TOO_SMALL, "mp_layer workspace: need %zu bytes, got %zu", w.bytes, ws_bytes);
  HGNN_REQUIRE(saved_bytes >= s.bytes, HGNN_ERR_WORKSPACE_TOO_SMALL, "mp_layer saved buffer: need %zu bytes, got %zu", s.bytes, saved_bytes);
  const LayerOff o(H);

  // packed blocks: 0 W1a, 1 W1b, 2 W2, 3 W3a, 4 W3b, 5 W4
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
  HGNN_TRY(launch_pack(st, H, bf16, pk));

  {  // P | Q
    GemmArgs g;
    g.A[0] = h_in; g.lda[0] = H; g.nkc = 1;
    g.B = w.packed; g.blk[0][0] = 0; g.blk[0][1] = 1; g.ncb = 2;
    g.M = N;
    g.bias = W + o.b1; g.bias_cb_mask = 1;
    g.C = s.PQ; g.ldc = 2 * H;
    HGNN_TRY(launch_gemm(st, H, bf16, g));
  }
  if (E > 0) {
    HGNN_TRY(launch_edge_pre(st, H, E, dst, col, d2, s.PQ, W + o.W1 + 2 * HH, w.a1, nullptr));
    GemmArgs g;
    g.A[0] = w.a1; g.lda[0] = H;
    g.B = w.packed; g.blk[0][0] = 2;
    g.M = (int)E;
    g.bias = W + o.b2; g.bias_cb_mask = 1;
    g.C = s.z2; g.ldc = H;
    HGNN_TRY(launch_gemm(st, H, bf16, g));
  }
  HGNN_TRY(launch_seg_fwd(st, H, N, row_ptr, s.z2, rvec, W + o.wx, alpha, v_in, s.M, v_out));
  {  // z3 = [h ; M] W3 + b3
    GemmArgs g;
    g.A[0] = h_in; g.lda[0] = H; g.A[1] = s.M; g.lda[1] = H; g.nkc = 2;
    g.B = w.packed; g.blk[0][0] = 3; g.blk[1][0] = 4;
    g.M = N;
    g.bias = W + o.b3; g.bias_cb_mask = 1;
    g.C = s.z3; g.ldc = H;
    HGNN_TRY(launch_gemm(st, H, bf16, g));
  }
  {  // h' = h + silu(z3) W4 + b4
    GemmArgs g;
    g.A[0] = s.z3; g.lda[0] = H; g.a_silu = 1;
    g.B = w.packed; g.blk[0][0] = 5;
    g.M = N;
    g.bias = W + o.b4; g.bias_cb_mask = 1;
    g.add1 = h_in; g.ldadd1 = H;
    g.C = h_out; g.ldc = H;
    HGNN_TRY(launch_gemm(st, H, bf16, g));
  }
  return HGNN_OK;
}

extern "C" int32_t hgnn_mp_layer_bwd(void* stream, int32_t N, int64_t E, int32_t H, int32_t dtype, float alpha,
                                     const int32_t* row_ptr, const int32_t* dst, const int32_t* col,
                                     const float* d2, const float* rvec, const int32_t* colT_ptr,
                                     const int32_t* permT, const float* h_in, const float* W, const void* saved,
                                     size_t saved_bytes, const float* g_h_out, const float* g_v_out,
                                     float* g_h_in, float* g_v_in, float* gW, void* ws, size_t ws_bytes) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  HGNN_TRY(check_layer_args(N, E, H, dtype));
  HGNN_REQUIRE(gW && W && ws, HGNN_ERR_NULLPTR, "mp_layer_bwd: null pointer");
  HGNN_REQUIRE(N == 0 || (row_ptr && colT_ptr && h_in && saved && g_h_out && g_v_out && g_h_in && g_v_in),
               HGNN_ERR_NULLPTR, "mp_layer_bwd: null pointer");
  HGNN_REQUIRE(E == 0 || (dst && col && d2 && rvec && permT), HGNN_ERR_NULLPTR, "mp_layer_bwd: null edge array");
  HGNN_REQUIRE(N == 0 || g_h_in != g_h_out, HGNN_ERR_BAD_SHAPE, "g_h_in may not alias g_h_out");
  if (N == 0) return launch_fill_f32(st, gW, LayerOff(H).total, 0.f);
  const bool bf16 = dtype == HGNN_BF16;
  LayerWs w = carve_ws(ws, N, E, H, bf16);
  LayerSaved s = carve_saved(const_cast<void*>(saved), N, E, H);
  HGNN_REQUIRE(ws_bytes >= w.bytes, HGNN_ERR_WORKSPACE_TOO_SMALL, "mp_layer workspace: need %zu bytes, got %zu", w.bytes, ws_bytes);
  HGNN_REQUIRE(saved_bytes >= s.bytes, HGNN_ERR_WORKSPACE_TOO_SMALL, "mp_layer saved buffer: need %zu bytes, got %zu", s.bytes, saved_bytes);
  const LayerOff o(H);
  const long HH = (long)H * H;

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
  HGNN_TRY(launch_pack(st, H, bf16, pk));

  // every gradient field is written below even when there is nothing to sum over
  {  // g_z3 = (g_h' W4^T) * silu'(z3)
    GemmArgs g;
    g.A[0] = g_h_out; g.lda[0] = H;
    g.B = w.packed; g.blk[0][0] = 0;
    g.M = N;
    g.mul = s.z3; g.ldmul = H; g.mul_is_z = 1;
    g.C = w.g_z3; g.ldc = H;
    HGNN_TRY(launch_gemm(st, H, bf16, g));
  }
  {  // gW4 = silu(z3)^T g_h' ; gb4
    WgradArgs a;
    a.A[0] = s.z3; a.lda[0] = H; a.a_silu = 1;
    a.B[0] = g_h_out; a.ldb[0] = H;
    a.M = N;
    a.dest[0] = gW + o.W4;
    a.partial = w.partial;
    HGNN_TRY(launch_wgrad(st, H, bf16, a));
    ColsumArgs c;
    c.X = g_h_out; c.ldx = H; c.M = N; c.dest = gW + o.b4; c.partial = w.partial;
    HGNN_TRY(launch_colsum(st, H, c));
  }
  {  // [g_h(a) | g_M] = g_z3 W3^T
    GemmArgs g;
    g.A[0] = w.g_z3; g.lda[0] = H;
    g.B = w.packed; g.blk[0][0] = 1; g.blk[0][1] = 2; g.ncb = 2;
    g.M = N;
    g.C = w.g_hM; g.ldc = 2 * H;
    HGNN_TRY(launch_gemm(st, H, bf16, g));
  }
  {  // gW3 = [h ; M]^T g_z3 ; gb3
    WgradArgs a;
    a.A[0] = h_in; a.lda[0] = H; a.A[1] = s.M; a.lda[1] = H; a.nA = 2;
    a.B[0] = w.g_z3; a.ldb[0] = H;
    a.M = N;
    a.dest[0] = gW + o.W3; a.dest[1] = gW + o.W3 + HH;
    a.partial = w.partial;
    HGNN_TRY(launch_wgrad(st, H, bf16, a));
    ColsumArgs c;
    c.X = w.g_z3; c.ldx = H; c.M = N; c.dest = gW + o.b3; c.partial = w.partial;
    HGNN_TRY(launch_colsum(st, H, c));
  }
  // edge part
  HGNN_TRY(launch_edge_gz2(st, H, E, dst, rvec, s.z2, w.g_hM + H, 2 * H, g_v_out, W + o.wx, alpha, w.g_z2, w.cvec));
  {
    ColsumArgs c;  // g_wx = sum_e c_e * m_e
    c.X = s.z2; c.ldx = H; c.f_silu = 1; c.w = w.cvec; c.M = E; c.dest = gW + o.wx; c.partial = w.partial;
    HGNN_TRY(launch_colsum(st, H, c));
    ColsumArgs c2;  // gb2
    c2.X = w.g_z2; c2.ldx = H; c2.M = E; c2.dest = gW + o.b2; c2.partial = w.partial;
    HGNN_TRY(launch_colsum(st, H, c2));
  }
  HGNN_TRY(launch_edge_pre(st, H, E, dst, col, d2, s.PQ, W + o.W1 + 2 * HH, w.a1, w.s1));
  {  // gW2 = a1^T g_z2
    WgradArgs a;
    a.A[0] = w.a1; a.lda[0] = H;
    a.B[0] = w.g_z2; a.ldb[0] = H;
    a.M = E;
    a.dest[0] = gW + o.W2;
    a.partial = w.partial;
    HGNN_TRY(launch_wgrad(st, H, bf16, a));
  }
  if (E > 0) {  // g_z1 = (g_z2 W2^T) * silu'(z1), in place over s1
    GemmArgs g;
    g.A[0] = w.g_z2; g.lda[0] = H;
    g.B = w.packed; g.blk[0][0] = 3;
    g.M = (int)E;
    g.mul = w.s1; g.ldmul = H;
    g.C = w.s1; g.ldc = H;
    HGNN_TRY(launch_gemm(st, H, bf16, g));
  }
  float* g_z1 = w.s1;
  HGNN_TRY(launch_segsum(st, H, N, row_ptr, nullptr, g_z1, w.g_PQ, 2 * H));       // g_P: per destination
  HGNN_TRY(launch_segsum(st, H, N, colT_ptr, permT, g_z1, w.g_PQ + H, 2 * H));    // g_Q: per source
  {
    ColsumArgs c;  // g_w1d = sum_e d2_e * g_z1_e
    c.X = g_z1; c.ldx = H; c.w = d2; c.M = E; c.dest = gW + o.W1 + 2 * HH; c.partial = w.partial;
    HGNN_TRY(launch_colsum(st, H, c));
    ColsumArgs c2;  // gb1 = sum_i g_P_i
    c2.X = w.g_PQ; c2.ldx = 2 * H; c2.M = N; c2.dest = gW + o.b1; c2.partial = w.partial;
    HGNN_TRY(launch_colsum(st, H, c2));
  }
  {  // gW1a = h^T g_P ; gW1b = h^T g_Q
    WgradArgs a;
    a.A[0] = h_in; a.lda[0] = H;
    a.B[0] = w.g_PQ; a.ldb[0] = 2 * H; a.B[1] = w.g_PQ + H; a.ldb[1] = 2 * H; a.nB = 2;
    a.M = N;
    a.dest[0] = gW + o.W1; a.dest[1] = gW + o.W1 + HH;
    a.partial = w.partial;
    HGNN_TRY(launch_wgrad(st, H, bf16, a));
  }
  if (N > 0) {  // g_h = g_h' + g_h(a) + g_P W1a^T + g_Q W1b^T
    GemmArgs g;
    g.A[0] = w.g_PQ; g.lda[0] = 2 * H; g.A[1] = w.g_PQ + H; g.lda[1] = 2 * H; g.nkc = 2;
    g.B = w.packed; g.blk[0][0] = 4; g.blk[1][0] = 5;
    g.M = N;
    g.add1 = g_h_out; g.ldadd1 = H;
    g.add2 = w.g_hM; g.ldadd2 = 2 * H;
    g.C = g_h_in; g.ldc = H;
    HGNN_TRY(launch_gemm(st, H, bf16, g));
  }
  if (g_v_in != g_v_out) HGNN_TRY(launch_copy_f32(st, g_v_out, g_v_in, (int64_t)N * 3));
  return HGNN_OK;
}
