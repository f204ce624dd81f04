// Views into the routing plan that hgnn_multihead_plan writes (internal).
#pragma once

#include <cstdint>

namespace hgnn {

struct PlanView {
  int32_t *grp_graph_ptr, *graph_perm, *grp_atom_ptr, *atom_perm, *atom_graph, *graph_src, *graph_dst_off, *status;
  int32_t *cur_graph, *cur_atom;   // [S] each: running cursors of the stable placement
  int64_t ints;
};

template <typename T>
static PlanView plan_view(T* plan, int N, int G, int S) {
  PlanView v;
  int32_t* p = const_cast<int32_t*>(plan);
  int64_t o = 0;
  v.grp_graph_ptr = p + o; o += S + 1;
  v.graph_perm = p + o; o += G;
  v.grp_atom_ptr = p + o; o += S + 1;
  v.atom_perm = p + o; o += N;
  v.atom_graph = p + o; o += N;
  v.graph_src = p + o; o += G;
  v.graph_dst_off = p + o; o += G;
  v.status = p + o; o += 4;
  v.cur_graph = p + o; o += S;
  v.cur_atom = p + o; o += S;
  v.ints = o;
  return v;
}

}  // namespace hgnn
