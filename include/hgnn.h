/*
 * libhgnn -- one GPU's share of a HydraGNN multi-task pre-training step on MI355X (gfx950).
 *
 * The step (paper: shared message-passing stack, then one decoding branch per dataset, each branch
 * split into an energy-per-atom head and an atomic-force head; sections "Two-level hierarchical MTL
 * architecture" and "Multi-task parallelism"; EGNN backbone named in section "Numerical Results"):
 *
 *   radius graph -> embedding -> L x message-passing layer -> mean pool -> per-source heads
 *   and the reverse pass of all of it.
 *
 * Conventions
 *  - Plain C ABI. Every function returns an hgnn_status (0 = ok, negative = error) and never throws.
 *    hgnn_last_error_string() gives the text of the calling thread's last error.
 *  - Unless a name ends in _host, every pointer is a DEVICE pointer to a contiguous row-major array,
 *    aligned to 16 bytes. The caller owns every buffer (inputs, outputs, saved activations and
 *    workspaces); the library allocates no device memory and keeps no pointer after a call returns.
 *  - `stream` is a hipStream_t passed as void*. Calls only enqueue work on it, except where a
 *    function is documented to synchronise.
 *  - Index type is int32. N atoms, G graphs, E directed edges, H hidden width, S sources.
 *    Edge e = (i <- j, s): i = dst[e] is the destination atom, j = col[e] the source atom, s the
 *    integer lattice shift applied to j.
 *  - The fused kernels serve H = 64, 128 and 256 (tile granularity of the matrix cores) with a head width equal to
 *    H; every other width up to 1024 takes the fragment-GEMM kernels (bf16 operands only). Each entry point states
 *    what it accepts.
 *  - dtype selects the GEMM operand type: HGNN_F32 (fp32 matrix cores) or HGNN_BF16 (operands rounded
 *    to bf16 on load, fp32 accumulation). Activations, aggregation, biases and SiLU stay fp32.
 *  - Gradient outputs are overwritten, not accumulated, unless said otherwise.
 *  - Results are deterministic: no floating-point atomics anywhere, all reductions in a fixed order.
 */
#ifndef HGNN_H
#define HGNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  HGNN_OK = 0,
  HGNN_ERR_NULLPTR = -1,
  HGNN_ERR_BAD_SHAPE = -2,
  HGNN_ERR_BAD_OFFSETS = -3,
  HGNN_ERR_BAD_CELL = -4,
  HGNN_ERR_BAD_SOURCE_ID = -5,
  HGNN_ERR_WORKSPACE_TOO_SMALL = -6,
  HGNN_ERR_OVERFLOW = -7,
  HGNN_ERR_HIP = -8,
  HGNN_ERR_UNIMPLEMENTED = -9
} hgnn_status;

enum { HGNN_F32 = 0, HGNN_BF16 = 1 };
enum { HGNN_POOL_SUM = 0, HGNN_POOL_MEAN = 1 };
enum { HGNN_ZMAX = 94 }; /* embedding table has HGNN_ZMAX+1 rows */

const char* hgnn_last_error_string(void);
int32_t hgnn_version(void);

/* ---------------------------------------------------------------------------------------------
 * Radius graph (the "radius graphs of atomistic structures" the shared message-passing stack runs
 * on; the paper gives no construction).
 *
 * Edge (i <- j, s) exists when i, j belong to the same graph, (j,s) != (i,0) and, in float32 with
 * every operation rounded on its own (no fused multiply-add):
 *      t = (s1*a + s2*b) + s3*c ;  rvec = pos_i - (pos_j + t) ;  d2 = (rx*rx + ry*ry) + rz*rz < rc*rc
 * a, b, c = rows of cell[g]. Graphs with pbc[g] == 0 (or cell == NULL) only have s = 0. For periodic
 * graphs every image within the cutoff is found provided the atoms lie inside the cell (fractional
 * coordinates in [0,1) up to rounding); self images (j == i, s != 0) are edges. No neighbour cap.
 * Output order: by i, then j, then s1, s2, s3 ascending -- a destination-sorted CSR.
 *
 * Two calls: _count fills row_ptr and returns E; the caller allocates the edge arrays; _fill writes
 * them. `ws` (hgnn_radius_graph_workspace_bytes) carries state from _count to _fill and must not be
 * touched in between. `tmp` (8*E bytes) is scratch of _fill only.
 *
 * _count SYNCHRONISES the stream (it has to hand E to the host) and reports input errors:
 * graph_off not starting at 0 / not non-decreasing / not ending at N -> BAD_OFFSETS; a periodic graph
 * with |det cell| < 1e-6 A^3, or one that would need more than 127 images in a direction, or an atom of a periodic
 * graph outside its cell (a fractional coordinate outside [-1e-5, 1 + 1e-5]) -> BAD_CELL;
 * E >= 2^31 -> OVERFLOW; rc <= 0 -> BAD_SHAPE. All of them are found on the device and reported after that one
 * synchronisation; the outputs are undefined then. _fill only enqueues work and may be called again after one _count.
 * ------------------------------------------------------------------------------------------- */
int32_t hgnn_radius_graph_workspace_bytes(int32_t N, int32_t G, size_t* bytes_host);

int32_t hgnn_radius_graph_count(void* stream, int32_t N, int32_t G,
                                const float* pos /*[N,3]*/, const int32_t* graph_off /*[G+1]*/,
                                const float* cell /*[G,3,3] or NULL*/, const uint8_t* pbc /*[G] or NULL*/,
                                float rc, void* ws, size_t ws_bytes,
                                int32_t* row_ptr /*out [N+1]*/, int64_t* E_host /*out, host*/);

int32_t hgnn_radius_graph_fill(void* stream, int32_t N, int32_t G,
                               const float* pos, const int32_t* graph_off,
                               const float* cell, const uint8_t* pbc, float rc,
                               void* ws, size_t ws_bytes, void* tmp, size_t tmp_bytes /*>= 8*E*/,
                               const int32_t* row_ptr /*in [N+1]*/, int64_t E,
                               int32_t* dst /*out [E]*/, int32_t* col /*out [E]*/,
                               int8_t* shift /*out [E,3]*/, float* d2 /*out [E]*/,
                               float* rvec /*out [E,3]*/, int32_t* edge_graph_ptr /*out [G+1]*/,
                               int32_t* colT_ptr /*out [N+1]*/, int32_t* permT /*out [E]*/);
/* colT_ptr / permT: the same edges regrouped by source atom j (edge ids ascending inside each
 * group); the reverse pass reduces over them. edge_graph_ptr[g] = first edge of graph g. */

/* ---------------------------------------------------------------------------------------------
 * Embedding: h0[i,:] = emb[Z[i],:]  (input node features = learnable table indexed by atomic
 * number, 0 <= Z <= HGNN_ZMAX). _bwd: g_emb[z,:] = sum over atoms with Z == z of g_h[i,:], summed in
 * atom order (chunks of atoms are reduced first, then the chunks in order); ws is scratch of
 * hgnn_embed_bwd_workspace_bytes(N, H) bytes. 1 <= H <= 1024 (vector kernels at 64 / 128 / 256).
 * ------------------------------------------------------------------------------------------- */
int32_t hgnn_embed_fwd(void* stream, int32_t N, int32_t H, const int32_t* Z,
                       const float* emb /*[ZMAX+1,H]*/, float* h /*out [N,H]*/);
int32_t hgnn_embed_bwd_workspace_bytes(int32_t N, int32_t H, size_t* ws_bytes_host);
int32_t hgnn_embed_bwd(void* stream, int32_t N, int32_t H, const int32_t* Z,
                       const float* g_h /*[N,H]*/, float* g_emb /*out [ZMAX+1,H]*/,
                       void* ws, size_t ws_bytes);

/* hgnn_embed_bwd for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): same arguments without the workspace, same kernels, same result bit for bit. The
 * scratch is an array of HGNN_EMBED_BWD_STATIC_MAX_BYTES built into the library's device code (every GPU the library
 * runs on holds it until the process ends); the call allocates and frees nothing. WORKSPACE_TOO_SMALL when
 * hgnn_embed_bwd_workspace_bytes(N, H) exceeds that size (ceil(N / 2048) * 95 * H * 4 bytes: e.g. N <= 176,128 at
 * H = 256); use hgnn_embed_bwd then. All calls on one GPU share that array: calls that overlap on one GPU (two
 * streams, two threads) race; calls on one stream are ordered and safe. Only enqueues work. */
enum { HGNN_EMBED_BWD_STATIC_MAX_BYTES = 8 << 20 };
int32_t hgnn_embed_bwd_static(void* stream, int32_t N, int32_t H, const int32_t* Z,
                              const float* g_h /*[N,H]*/, float* g_emb /*out [ZMAX+1,H]*/);

/* ---------------------------------------------------------------------------------------------
 * One message-passing layer of the shared stack (EGNN layer, positions held fixed):
 *   edge  e=(i<-j): m_e = silu(W2^T silu(W1^T [h_i ; h_j ; d2_e] + b1) + b2),  x_e = wx . m_e
 *   atom  i:        M_i = alpha * sum_{e in row i} m_e
 *                   v'_i = v_i + alpha * sum_{e in row i} x_e * rvec_e
 *                   h'_i = h_i + W4^T silu(W3^T [h_i ; M_i] + b3) + b4
 * W is one flat float32 buffer, matrices row-major [in,out]:
 *   W1[(2H+1),H] b1[H] W2[H,H] b2[H] wx[H] W3[2H,H] b3[H] W4[H,H] b4[H]     (6H^2 + 6H floats)
 * gW of _bwd has the same layout. `saved` (size from the workspace query) is written by _fwd and
 * read by _bwd of the same layer; `ws` is scratch. Rows with no edge get M_i = 0, v'_i = v_i.
 * saved == NULL (both calls; H = 64, 128, 256 only): nothing is kept between the two calls and _bwd runs the forward
 * pass of the layer once more to get what it needs (one more edge pass per layer in exchange for saved_bytes of
 * memory per layer: 0.8 GB per layer on a 1.2 M-edge batch at H = 256). `ws` must then hold ws_bytes + saved_bytes
 * + 512 + 24 N bytes of the query; the results are bit for bit those of the calls with a saved buffer.
 * _bwd takes g_h_out = dL/dh', g_v_out = dL/dv' and writes g_h_in = dL/dh, g_v_in = dL/dv and gW.
 * d2 and rvec are constants of the step (no gradient with respect to positions).
 * h_out may not alias h_in; g_h_in may not alias g_h_out.
 * H is 64, 128 or 256 (either dtype), or any other width in 1..1024 with dtype HGNN_BF16 (the paper's backbone has
 * 866 hidden units, section "Numerical Results"; such widths are padded to a multiple of 128 inside the library and
 * float32 operands are UNIMPLEMENTED for them).
 * Errors: BAD_SHAPE for any other H or an unknown dtype; OVERFLOW if E > 2^31 - 129 or
 * N * 2H * 4 bytes reaches 4 GiB (the edge kernels index edges and gathered rows with 32 bits);
 * WORKSPACE_TOO_SMALL if ws / saved are smaller than the query says; UNIMPLEMENTED if saved == NULL at another
 * width.
 * _bwd may enqueue weight-gradient work on a stream the library creates once (default priority). It
 * forks from and joins `stream` through events inside the call, so for the caller everything is
 * ordered on `stream`; the call that creates that stream must not run under stream capture.
 * hgnn_set_side_stream(enable): 1 = always use that stream, 0 = keep all work on `stream` (e.g. to time kernels
 * in isolation), -1 = the library's choice (the default: used at widths other than 64 / 128 / 256, where many small
 * atom-level launches leave compute units idle, not used by the fused kernels, which fill the chip by themselves).
 * The environment variable HGNN_SIDE_STREAM = 0 / 1, read before the first call, sets the same. Returns the previous
 * setting (-1 / 0 / 1). The results do not depend on it bit for bit.
 * _bwd needs dst sorted ascending and consistent with row_ptr (a destination-sorted CSR, as hgnn_radius_graph_fill
 * writes it): with bf16 operands at H = 256 and with float32 operands at H = 128 the reverse edge kernel sums the
 * gradients of an atom's incoming edges as runs of consecutive edges with equal dst. The environment variable
 * HGNN_DSUM_IN_KERNEL = 0, read at every call, makes those sums a pass of its own over the edge tensor again (for
 * comparing the two forms; the results then differ in the last places, both orders of addition are fixed).
 * The library keeps per-process state without locks: call it from one host thread at a time.
 * ------------------------------------------------------------------------------------------- */
int32_t hgnn_set_side_stream(int32_t enable);

int32_t hgnn_mp_layer_workspace_bytes(int32_t N, int64_t E, int32_t H, int32_t dtype,
                                      size_t* ws_bytes_host, size_t* saved_bytes_host);

int32_t hgnn_mp_layer_fwd(void* stream, int32_t N, int64_t E, int32_t H, int32_t dtype, float alpha,
                          const int32_t* row_ptr, const int32_t* dst, const int32_t* col,
                          const float* d2, const float* rvec,
                          const float* h_in /*[N,H]*/, const float* v_in /*[N,3]*/,
                          const float* W, float* h_out /*[N,H]*/, float* v_out /*[N,3]*/,
                          void* saved, size_t saved_bytes, void* ws, size_t ws_bytes);

int32_t hgnn_mp_layer_bwd(void* stream, int32_t N, int64_t E, int32_t H, int32_t dtype, float alpha,
                          const int32_t* row_ptr, const int32_t* dst, const int32_t* col,
                          const float* d2, const float* rvec,
                          const int32_t* colT_ptr, const int32_t* permT,
                          const float* h_in, const float* W, const void* saved, size_t saved_bytes,
                          const float* g_h_out /*[N,H]*/, const float* g_v_out /*[N,3]*/,
                          float* g_h_in /*out [N,H]*/, float* g_v_in /*out [N,3]*/,
                          float* gW /*out, layout of W*/, void* ws, size_t ws_bytes);

/* ---------------------------------------------------------------------------------------------
 * The same layer with k edge attributes in place of d2: the edge input is [h_i ; h_j ; attr_e] of width 2H + k
 * and W1 has 2H + k rows (rows 2H .. 2H+k-1 act on the attributes; everything after W1 in W and gW moves
 * accordingly: (6H^2 + (5 + k) H floats). attr is [E,k] float32, a constant of the step like d2.
 * hgnn_edge_rbf fills it with a radial basis of the edge length d = sqrt(d2) (the paper names no basis; this is the
 * usual Gaussian expansion with a smooth cutoff):
 *   attr[e][j] = exp(-gamma (d - mu_j)^2) * (cos(pi d / rc) + 1) / 2,  mu_j = j rc / (k-1),  gamma = ((k-1) / rc)^2
 * 2 <= k <= 16 there; the layer takes 1 <= k <= 16 and any attributes. 1 <= H <= 1024. With several attributes, or at
 * a width other than 64 / 128 / 256, this variant runs through the fragment-GEMM kernels: dtype HGNN_BF16 only (HGNN_F32
 * -> UNIMPLEMENTED). One attribute (k = 1, e.g. attr = d2) at H = 64 / 128 / 256 runs on the fused kernels of
 * hgnn_mp_layer_* with either dtype, and differs from those calls only in the edge gradients below. Other arguments,
 * side stream, errors and aliasing rules as for hgnn_mp_layer_*. Only enqueue work.
 * _bwd can also hand out what position gradients are made of (both optional, NULL = not wanted):
 *   g_attr [E,k]  gradient with respect to the edge attributes, g_attr[e][j] = sum_c g_z1[e][c] W1[2H + j][c]
 *   g_rvec [E,3]  gradient with respect to the edge vectors through v', g_rvec_e = alpha (wx . m_e) g_v_out[dst_e]
 * (they need what hgnn_mp_layer_attr_fwd keeps in `saved`: pair _attr_bwd with _attr_fwd, not with hgnn_mp_layer_fwd).
 * ------------------------------------------------------------------------------------------- */
int32_t hgnn_edge_rbf(void* stream, int64_t E, const float* d2 /*[E]*/, int32_t k, float rc,
                      float* attr /*out [E,k]*/);

int32_t hgnn_mp_layer_attr_workspace_bytes(int32_t N, int64_t E, int32_t H, int32_t k, int32_t dtype,
                                           size_t* ws_bytes_host, size_t* saved_bytes_host);

int32_t hgnn_mp_layer_attr_fwd(void* stream, int32_t N, int64_t E, int32_t H, int32_t k, int32_t dtype, float alpha,
                               const int32_t* row_ptr, const int32_t* dst, const int32_t* col,
                               const float* attr /*[E,k]*/, const float* rvec,
                               const float* h_in /*[N,H]*/, const float* v_in /*[N,3]*/,
                               const float* W, float* h_out /*[N,H]*/, float* v_out /*[N,3]*/,
                               void* saved, size_t saved_bytes, void* ws, size_t ws_bytes);

int32_t hgnn_mp_layer_attr_bwd(void* stream, int32_t N, int64_t E, int32_t H, int32_t k, int32_t dtype, float alpha,
                               const int32_t* row_ptr, const int32_t* dst, const int32_t* col,
                               const float* attr /*[E,k]*/, const float* rvec,
                               const int32_t* colT_ptr, const int32_t* permT,
                               const float* h_in, const float* W, const void* saved, size_t saved_bytes,
                               const float* g_h_out /*[N,H]*/, const float* g_v_out /*[N,3]*/,
                               float* g_h_in /*out [N,H]*/, float* g_v_in /*out [N,3]*/,
                               float* gW /*out, layout of W*/, float* g_attr /*out [E,k] or NULL*/,
                               float* g_rvec /*out [E,3] or NULL*/, void* ws, size_t ws_bytes);

/* ---------------------------------------------------------------------------------------------
 * Atoms that move between layers, and gradients with respect to positions. The paper's backbone is the E(n)-GNN
 * (section "Numerical Results"), whose layers also update the coordinates: here the equivariant channel v is read as
 * the displacement of every atom from its input position, x_i = x0_i + v_i. The neighbour list (and the periodic image
 * of every edge) stays that of the input positions; before every layer
 *   hgnn_edge_geometry_fwd:  rvec_e = rvec0_e + (v[dst_e] - v[col_e]),  d2_e = |rvec_e|^2
 * gives the layer its edge vectors and lengths (v = 0: those of the neighbour search). In the reverse pass
 *   hgnn_edge_rbf_bwd:       g_d2_e = sum_j g_attr[e][j] d attr_j / d d2   (basis of hgnn_edge_rbf; edges of length 0
 *                            give inf / nan: distinct atoms never coincide)
 *   hgnn_edge_geometry_bwd:  g_r_e = g_rvec_e + 2 g_d2_e rvec_e            (g_d2 NULL: g_r = g_rvec)
 *                            g_r_sum_e += g_r_e                             (optional)
 *                            g_v[i] += sum_{e: dst_e = i} g_r_e - sum_{e: col_e = i} g_r_e   (optional, fixed order)
 * turn a layer's g_attr / g_rvec into the gradient with respect to the displacements that entered the layer (add it to
 * the layer's g_v_in when the atoms move) and accumulate the gradient with respect to rvec0; one last call with
 * g_rvec = that sum, g_d2 = NULL and a zeroed g_v gives the gradient with respect to the input positions. The negative
 * of that gradient for dL/dE = atoms per graph, dL/dF = 0 is the conservative force -dE/dx.
 * g_r may alias g_rvec; g_r_sum may alias neither. row_ptr / colT_ptr / permT as produced by hgnn_radius_graph_fill.
 * float32 throughout. Only enqueue work.
 * ------------------------------------------------------------------------------------------- */
int32_t hgnn_edge_geometry_fwd(void* stream, int32_t N, int64_t E, const float* rvec0 /*[E,3]*/,
                               const float* v /*[N,3]*/, const int32_t* dst, const int32_t* col,
                               float* rvec /*out [E,3]*/, float* d2 /*out [E]*/);

int32_t hgnn_edge_rbf_bwd(void* stream, int64_t E, const float* d2 /*[E]*/, int32_t k, float rc,
                          const float* g_attr /*[E,k]*/, float* g_d2 /*out [E]*/);

int32_t hgnn_edge_geometry_bwd(void* stream, int32_t N, int64_t E, const int32_t* row_ptr, const int32_t* colT_ptr,
                               const int32_t* permT, const float* rvec /*[E,3]*/, const float* g_rvec /*[E,3]*/,
                               const float* g_d2 /*[E] or NULL*/, float* g_r /*out [E,3]*/,
                               float* g_r_sum /*in/out [E,3] or NULL*/, float* g_v /*in/out [N,3] or NULL*/);

/* ---------------------------------------------------------------------------------------------
 * Pooling over the contiguous atoms of each graph: p_g = sum or mean of h_i (mean gives the
 * "energy per atom" target of the paper its per-atom normalisation). Empty graphs give 0.
 * _bwd: g_h_i (+)= g_p[g(i)] (/ n_g);  accumulate != 0 adds into g_h instead of overwriting it.
 * 1 <= H <= 1024.
 * ------------------------------------------------------------------------------------------- */
int32_t hgnn_pool_by_graph_fwd(void* stream, int32_t N, int32_t G, int32_t H, int32_t mode,
                               const int32_t* graph_off, const float* h, float* p /*out [G,H]*/);
int32_t hgnn_pool_by_graph_bwd(void* stream, int32_t N, int32_t G, int32_t H, int32_t mode,
                               const int32_t* graph_off, const float* g_p, float* g_h /*[N,H]*/,
                               int32_t accumulate);

/* ---------------------------------------------------------------------------------------------
 * Two-level multi-task decoder, all S branches resident on this GPU. Graph g is decoded by branch
 * s = source_id[g] and by no other (the heads of different sources never exchange anything in the
 * forward pass: paper, section "Multi-task parallelism"):
 *   e_g = We2_s . silu(We1_s^T p_g + be1_s) + be2_s                       (energy per atom)
 *   q_i = Wf2_s . silu(Wf1_s^T h_i + bf1_s) + bf2_s ,  F_i = q_i * v_i     (atomic force)
 * Whead: S branches back to back, each  We1[H,Hh] be1[Hh] We2[Hh] be2[1] Wf1[H,Hh] bf1[Hh] Wf2[Hh]
 * bf2[1]. gWhead has the same layout; a branch with no graph in the batch gets exactly zero.
 * H in {64, 128, 256} with Hh = H runs with either dtype; any other H, Hh in 1..1024 is the D = 1 case of
 * hgnn_multihead_deep_* below (HGNN_BF16 only).
 *
 * hgnn_multihead_plan groups graphs and their atoms by source (stable): plan is an int32 array of
 * hgnn_multihead_plan_ints(N,G,S) entries laid out as
 *   grp_graph_ptr[S+1] | graph_perm[G] | grp_atom_ptr[S+1] | atom_perm[N] | atom_graph[N] | internal
 * It SYNCHRONISES the stream and returns BAD_SOURCE_ID if some source_id is outside [0,S).
 * ------------------------------------------------------------------------------------------- */
int64_t hgnn_multihead_plan_ints(int32_t N, int32_t G, int32_t S);
int32_t hgnn_multihead_plan(void* stream, int32_t N, int32_t G, int32_t S,
                            const int32_t* graph_off, const int32_t* source_id,
                            int32_t* plan /*out*/);

int32_t hgnn_multihead_decode_workspace_bytes(int32_t N, int32_t G, int32_t H, int32_t Hh, int32_t S,
                                              int32_t dtype, size_t* ws_bytes_host,
                                              size_t* saved_bytes_host);

int32_t hgnn_multihead_decode_fwd(void* stream, int32_t N, int32_t G, int32_t H, int32_t Hh, int32_t S,
                                  int32_t dtype, const int32_t* plan,
                                  const float* p /*[G,H]*/, const float* h /*[N,H]*/,
                                  const float* v /*[N,3]*/, const float* Whead,
                                  float* energy /*out [G]*/, float* force /*out [N,3]*/,
                                  void* saved, size_t saved_bytes, void* ws, size_t ws_bytes);

int32_t hgnn_multihead_decode_bwd(void* stream, int32_t N, int32_t G, int32_t H, int32_t Hh, int32_t S,
                                  int32_t dtype, const int32_t* plan,
                                  const float* p, const float* h, const float* v, const float* Whead,
                                  const void* saved, size_t saved_bytes,
                                  const float* g_energy /*[G]*/, const float* g_force /*[N,3]*/,
                                  float* g_p /*out [G,H]*/, float* g_h /*out [N,H]*/,
                                  float* g_v /*out [N,3]*/, float* gWhead /*out*/,
                                  void* ws, size_t ws_bytes);

/* ---------------------------------------------------------------------------------------------
 * The same decoder with D fully connected hidden layers per head (paper, section "Numerical Results": every
 * dataset-specific head has three layers of 889 units), silu after each hidden layer:
 *   a_0 = p_g (energy head) or h_i (force head);  a_l = silu(W_l^T a_{l-1} + b_l), l = 1..D;  out = wo . a_D + bo
 *   e_g = out of the energy head,  F_i = (out of the force head) * v_i
 * Whead: S branches back to back, each the energy head then the force head, a head being
 *   W_1[H,Hh] b_1[Hh]  W_l[Hh,Hh] b_l[Hh] (l = 2..D)  wo[Hh] bo[1]
 * (D = 1 is the layout of hgnn_multihead_decode_*). gWhead has the same layout; a branch with no graph in the
 * batch gets exactly zero. plan, p, h, v, energy, force, saved, ws and the gradients are as for
 * hgnn_multihead_decode_*. 1 <= H, Hh <= 1024 (any value), 1 <= D <= 8, 1 <= S <= 1024; dtype must be HGNN_BF16
 * (HGNN_F32 -> UNIMPLEMENTED). Errors otherwise as for hgnn_multihead_decode_*. Only enqueues work.
 * ------------------------------------------------------------------------------------------- */
int32_t hgnn_multihead_deep_workspace_bytes(int32_t N, int32_t G, int32_t H, int32_t Hh, int32_t D, int32_t S,
                                            int32_t dtype, size_t* ws_bytes_host, size_t* saved_bytes_host);

int32_t hgnn_multihead_deep_fwd(void* stream, int32_t N, int32_t G, int32_t H, int32_t Hh, int32_t D, int32_t S,
                                int32_t dtype, const int32_t* plan,
                                const float* p /*[G,H]*/, const float* h /*[N,H]*/, const float* v /*[N,3]*/,
                                const float* Whead, float* energy /*out [G]*/, float* force /*out [N,3]*/,
                                void* saved, size_t saved_bytes, void* ws, size_t ws_bytes);

int32_t hgnn_multihead_deep_bwd(void* stream, int32_t N, int32_t G, int32_t H, int32_t Hh, int32_t D, int32_t S,
                                int32_t dtype, const int32_t* plan,
                                const float* p, const float* h, const float* v, const float* Whead,
                                const void* saved, size_t saved_bytes,
                                const float* g_energy /*[G]*/, const float* g_force /*[N,3]*/,
                                float* g_p /*out [G,H]*/, float* g_h /*out [N,H]*/, float* g_v /*out [N,3]*/,
                                float* gWhead /*out*/, void* ws, size_t ws_bytes);

/* ---------------------------------------------------------------------------------------------
 * AdamW update of a flat float32 parameter buffer (paper, training setup: the optimiser is AdamW, learning rate 1e-3;
 * the update itself is the published algorithm, Adam with decoupled weight decay):
 *   m <- beta1 m + (1-beta1) g;  v <- beta2 v + (1-beta2) g*g;
 *   w <- w - lr * ( (m / (1-beta1^step)) / (sqrt(v / (1-beta2^step)) + eps) + weight_decay * w )
 * w, m, v [n] are updated in place, g [n] is read; all device pointers, 16-byte aligned; m and v start at zero
 * and `step` counts the updates from 1. The layer and head weight buffers of this library are flat, so one call
 * per buffer (or one call over a buffer that holds them all) updates the model. Only enqueues work.
 * Errors: BAD_SHAPE for n < 0, step < 1 or a beta outside [0,1); NULLPTR for a null buffer with n > 0.
 * ------------------------------------------------------------------------------------------- */
int32_t hgnn_adamw_step(void* stream, int64_t n, float* w, const float* g, float* m, float* v,
                        int32_t step, double lr, double beta1, double beta2, double eps, double weight_decay);

/* ---------------------------------------------------------------------------------------------
 * Instrumentation (for benchmarks; not part of the method): time classes of kernels with HIP events
 * recorded on the launch stream. _begin enables the classes whose bit is set in tag_mask and clears
 * earlier records; _end SYNCHRONISES the stream and accumulates; _read returns how many launches of
 * a class were timed and their total duration. Not thread safe; costs two event records per timed
 * launch and nothing for classes that are not enabled.
 * ------------------------------------------------------------------------------------------- */
int32_t hgnn_profile_begin(uint64_t tag_mask);
int32_t hgnn_profile_end(void* stream);
int32_t hgnn_profile_num_tags(void);
const char* hgnn_profile_tag_name(int32_t tag);
int32_t hgnn_profile_read(int32_t tag, int64_t* launches_host, double* total_ms_host);

#ifdef __cplusplus
}
#endif
#endif /* HGNN_H */
