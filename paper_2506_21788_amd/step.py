"""Harness around the binding: owns the device buffers of one batch and issues the library calls of
one training step in order. No arithmetic happens here -- torch is the allocator and the stream."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


def _dev(a, dtype=None):
    t = torch.as_tensor(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda().contiguous()


def _bytes(n):
    return torch.empty(max(int(n), 16), dtype=torch.uint8, device="cuda")


class Graph:
    """Device-resident radius graph of a batch (destination-sorted CSR + transpose plan)."""

    def __init__(self, pos, graph_off, cell, pbc, rc):
        self.N = int(pos.shape[0])
        self.G = int(graph_off.shape[0] - 1)
        self.rc = float(rc)
        self.pos, self.graph_off, self.cell, self.pbc = pos, graph_off, cell, pbc
        self.ws = _bytes(B.radius_graph_workspace_bytes(self.N, self.G))
        self.row_ptr = torch.empty(self.N + 1, dtype=torch.int32, device="cuda")
        self.E = None

    def build(self):
        N, G = self.N, self.G
        E = B.radius_graph_count(N, G, self.pos, self.graph_off, self.cell, self.pbc, self.rc, self.ws, self.row_ptr)
        if self.E != E:
            i32 = dict(dtype=torch.int32, device="cuda")
            f32 = dict(dtype=torch.float32, device="cuda")
            self.E = E
            self.tmp = _bytes(8 * E)
            self.dst = torch.empty(E, **i32)
            self.col = torch.empty(E, **i32)
            self.shift = torch.empty((E, 3), dtype=torch.int8, device="cuda")
            self.d2 = torch.empty(E, **f32)
            self.rvec = torch.empty((E, 3), **f32)
            self.edge_graph_ptr = torch.empty(G + 1, **i32)
            self.colT_ptr = torch.empty(N + 1, **i32)
            self.permT = torch.empty(E, **i32)
        B.radius_graph_fill(N, G, self.pos, self.graph_off, self.cell, self.pbc, self.rc, self.ws, self.tmp,
                            self.row_ptr, E, self.dst, self.col, self.shift, self.d2, self.rvec,
                            self.edge_graph_ptr, self.colT_ptr, self.permT)
        return self

    def to_numpy(self):
        keys = ("row_ptr", "dst", "col", "shift", "d2", "rvec", "edge_graph_ptr", "colT_ptr", "permT")
        out = {k: getattr(self, k).cpu().numpy() for k in keys}
        out["E"] = self.E
        return out


class HotPath:
    """One GPU's share of a training step on one batch: graph -> embed -> L layers -> pool -> heads,
    forward and backward. Inputs are numpy arrays (uploaded once); outputs stay on the device."""

    def __init__(self, batch, rc, H, L, S, dtype, emb, layer_weights, head_weights, alpha=None, Hh=None, D=None,
                 rbf_k=None, move=False, pos_grad=False, keep_grads=False):
        """D: hidden layers per head (the deep-head entry points); None: the one-hidden-layer heads.
        rbf_k: number of radial-basis edge attributes that take the place of d2 (None: d2 itself).
        move: the atoms move between layers (x = x0 + v): edge vectors, lengths and attributes are recomputed
        before every layer. pos_grad (implied by move): backward() also leaves the gradient with respect to the input
        positions in g_pos. Both run the layers through the edge-attribute entry points (bf16 operands).
        keep_grads: backward() keeps the gradient with respect to every layer's input (g_h[l], g_v[l], l = 0..L) instead
        of ping-ponging between two buffers."""
        self.keep_grads = bool(keep_grads)
        self.move = bool(move)
        self.pos_grad = bool(pos_grad or move)
        self.k = rbf_k if rbf_k is not None else (1 if self.pos_grad else None)   # None: the plain layer calls
        self.N, self.G, self.H, self.L, self.S = batch.N, batch.G, H, L, S
        self.Hh = H if Hh is None else Hh
        self.D = D
        self.rbf_k = rbf_k
        self.rc = float(rc)
        self.dtype = {"f32": B.F32, "bf16": B.BF16}[dtype]
        self.pos = _dev(batch.pos, torch.float32)
        self.Z = _dev(batch.Z, torch.int32)
        self.graph_off = _dev(batch.graph_off, torch.int32)
        self.cell = _dev(batch.cell, torch.float32)
        self.pbc = _dev(batch.pbc, torch.uint8)
        self.source_id = _dev(batch.source_id, torch.int32)
        self.emb = _dev(emb, torch.float32)
        self.W = [_dev(w, torch.float32) for w in layer_weights]
        self.Whead = _dev(head_weights, torch.float32)
        self.alpha = alpha
        self.graph = Graph(self.pos, self.graph_off, self.cell, self.pbc, rc)
        self._alloc_E = None
        self.plan = torch.empty(B.multihead_plan_ints(self.N, self.G, S), dtype=torch.int32, device="cuda")
        self.build_plan()

    @classmethod
    def from_problem(cls, P, alpha=None, **kw):
        """P: a problem dict of hgnn_inputs (batch, hyper-parameters hp, emb, Ws, Wh)."""
        b, hp = P["batch"], P["hp"]
        return cls(b, hp["rc"], hp["H"], hp["L"], hp["S"], hp["dtype"], P["emb"], P["Ws"], P["Wh"], alpha=alpha,
                   Hh=hp.get("Hh"), D=hp.get("D"), rbf_k=hp.get("rbf_k"), move=hp.get("move", False),
                   pos_grad=hp.get("pos_grad", False), **kw)

    def build_plan(self):
        """Routing of graphs and atoms to their source's branch (depends on the batch only)."""
        B.multihead_plan(self.N, self.G, self.S, self.graph_off, self.source_id, self.plan)

    # -- graph ---------------------------------------------------------------------------------
    def build_graph(self):
        self.graph.build()
        if self.alpha is None:
            self.alpha = 1.0 / max(1.0, self.graph.E / max(1, self.N))
        self._alloc(self.graph.E)
        return self.graph

    def _alloc(self, E):
        if self._alloc_E == E:
            return
        N, G, H, L, S = self.N, self.G, self.H, self.L, self.S
        f32 = dict(dtype=torch.float32, device="cuda")
        if self.k is None:
            ws_b, saved_b = B.mp_layer_workspace_bytes(N, E, H, self.dtype)
        else:
            ws_b, saved_b = B.mp_layer_attr_workspace_bytes(N, E, H, self.k, self.dtype)
            En = max(E, 1)
            nl = L if self.move else 1            # per-layer geometry only when the atoms move
            if self.move:
                self.rvec_l = [torch.empty((En, 3), **f32) for _ in range(L)]
                self.d2_l = [torch.empty(En, **f32) for _ in range(L)]
            if self.rbf_k is not None:
                self.attr_l = [torch.empty((En, self.k), **f32) for _ in range(nl)]
            if self.pos_grad:
                self.g_attr = torch.empty((En, self.k), **f32)
                self.g_d2 = torch.empty(En, **f32)
                self.g_rvec = torch.empty((En, 3), **f32)
                self.g_r0 = torch.empty((En, 3), **f32)
                self.g_pos = torch.empty((N, 3), **f32)
        if self.D is None:
            hws_b, hsaved_b = B.multihead_decode_workspace_bytes(N, G, H, self.Hh, S, self.dtype)
        else:
            hws_b, hsaved_b = B.multihead_deep_workspace_bytes(N, G, H, self.Hh, self.D, S, self.dtype)
        self.ws = _bytes(max(ws_b, hws_b, B.embed_bwd_workspace_bytes(N, H)))
        self.saved = [_bytes(saved_b) for _ in range(L)]
        self.hsaved = _bytes(hsaved_b)
        self.h = [torch.empty((N, H), **f32) for _ in range(L + 1)]
        self.v = [torch.zeros((N, 3), **f32) for _ in range(L + 1)]   # v[0] stays zero: v^0 = 0
        self.p = torch.empty((G, H), **f32)
        self.energy = torch.empty(G, **f32)
        self.force = torch.empty((N, 3), **f32)
        self.g_p = torch.empty((G, H), **f32)
        ng = L + 1 if self.keep_grads else 2
        self.g_h = [torch.empty((N, H), **f32) for _ in range(ng)]
        self.g_v = [torch.empty((N, 3), **f32) for _ in range(ng)]
        self.gW = [torch.empty_like(w) for w in self.W]
        self.gWhead = torch.empty_like(self.Whead)
        self.g_emb = torch.empty_like(self.emb)
        self._alloc_E = E

    # -- forward / backward ----------------------------------------------------------------------
    def forward(self):
        g, N, G, H = self.graph, self.N, self.G, self.H
        B.embed_fwd(N, H, self.Z, self.emb, self.h[0])
        for l in range(self.L):
            if self.k is None:
                B.mp_layer_fwd(N, g.E, H, self.dtype, self.alpha, g.row_ptr, g.dst, g.col, g.d2, g.rvec,
                               self.h[l], self.v[l], self.W[l], self.h[l + 1], self.v[l + 1], self.saved[l], self.ws)
                continue
            if self.move:
                B.edge_geometry_fwd(N, g.E, g.rvec, self.v[l], g.dst, g.col, self.rvec_l[l], self.d2_l[l])
            if self.rbf_k is not None and (self.move or l == 0):
                B.edge_rbf(g.E, self._d2(l), self.k, self.rc, self.attr_l[l])
            B.mp_layer_attr_fwd(N, g.E, H, self.k, self.dtype, self.alpha, g.row_ptr, g.dst, g.col, self._attr(l),
                                self._rvec(l), self.h[l], self.v[l], self.W[l], self.h[l + 1], self.v[l + 1],
                                self.saved[l], self.ws)
        B.pool_by_graph_fwd(N, G, H, B.POOL_MEAN, self.graph_off, self.h[-1], self.p)
        if self.D is None:
            B.multihead_decode_fwd(N, G, H, self.Hh, self.S, self.dtype, self.plan, self.p, self.h[-1], self.v[-1],
                                   self.Whead, self.energy, self.force, self.hsaved, self.ws)
        else:
            B.multihead_deep_fwd(N, G, H, self.Hh, self.D, self.S, self.dtype, self.plan, self.p, self.h[-1],
                                 self.v[-1], self.Whead, self.energy, self.force, self.hsaved, self.ws)

    # geometry and attributes of layer l (those of the neighbour search unless the atoms move)
    def _rvec(self, l):
        return self.rvec_l[l] if self.move else self.graph.rvec

    def _d2(self, l):
        return self.d2_l[l] if self.move else self.graph.d2

    def _attr(self, l):
        if self.rbf_k is None:
            return self._d2(l)                       # one attribute per edge: the squared length, [E] = [E,1]
        return self.attr_l[l if self.move else 0]

    def backward(self, g_energy, g_force):
        g, N, G, H, L = self.graph, self.N, self.G, self.H, self.L
        # buffer that holds the gradient with respect to h[l] / v[l]
        at = (lambda l: l) if self.keep_grads else (lambda l: (L - l) % 2)
        top = at(L)
        if self.D is None:
            B.multihead_decode_bwd(N, G, H, self.Hh, self.S, self.dtype, self.plan, self.p, self.h[-1], self.v[-1],
                                   self.Whead, self.hsaved, g_energy, g_force, self.g_p, self.g_h[top], self.g_v[top],
                                   self.gWhead, self.ws)
        else:
            B.multihead_deep_bwd(N, G, H, self.Hh, self.D, self.S, self.dtype, self.plan, self.p, self.h[-1],
                                 self.v[-1], self.Whead, self.hsaved, g_energy, g_force, self.g_p, self.g_h[top],
                                 self.g_v[top], self.gWhead, self.ws)
        B.pool_by_graph_bwd(N, G, H, B.POOL_MEAN, self.graph_off, self.g_p, self.g_h[top], True)
        for l in reversed(range(self.L)):
            cur, nxt = at(l + 1), at(l)
            if self.k is None:
                B.mp_layer_bwd(N, g.E, H, self.dtype, self.alpha, g.row_ptr, g.dst, g.col, g.d2, g.rvec, g.colT_ptr,
                               g.permT, self.h[l], self.W[l], self.saved[l], self.g_h[cur], self.g_v[cur],
                               self.g_h[nxt], self.g_v[nxt], self.gW[l], self.ws)
            else:
                pg = self.pos_grad
                B.mp_layer_attr_bwd(N, g.E, H, self.k, self.dtype, self.alpha, g.row_ptr, g.dst, g.col, self._attr(l),
                                    self._rvec(l), g.colT_ptr, g.permT, self.h[l], self.W[l], self.saved[l],
                                    self.g_h[cur], self.g_v[cur], self.g_h[nxt], self.g_v[nxt], self.gW[l],
                                    self.ws, g_attr=self.g_attr if pg else None, g_rvec=self.g_rvec if pg else None)
                if pg:
                    if l == self.L - 1:
                        self.g_r0.zero_()
                    if self.rbf_k is not None:
                        B.edge_rbf_bwd(g.E, self._d2(l), self.k, self.rc, self.g_attr, self.g_d2)
                    g_d2 = self.g_d2 if self.rbf_k is not None else self.g_attr   # k = 1: the attribute is d2
                    B.edge_geometry_bwd(N, g.E, g.row_ptr, g.colT_ptr, g.permT, self._rvec(l), self.g_rvec, g_d2,
                                        self.g_rvec, self.g_r0, self.g_v[nxt] if self.move else None)
        if self.pos_grad:
            # rvec0 = x0[dst] - x0[col] - image shift: the summed edge-vector gradients land on the input positions
            self.g_pos.zero_()
            if self.L > 0:
                B.edge_geometry_bwd(N, g.E, g.row_ptr, g.colT_ptr, g.permT, None, self.g_r0, None, self.g_rvec, None,
                                    self.g_pos)
        B.embed_bwd(N, H, self.Z, self.g_h[at(0)], self.g_emb, self.ws)
        self.g_h0, self.g_v0 = self.g_h[at(0)], self.g_v[at(0)]

    def step(self, g_energy, g_force, with_graph=True):
        """One whole step. with_graph: everything that depends on the batch is rebuilt as for a new batch (radius
        graph and routing plan)."""
        if with_graph:
            # the plan first: both calls wait for the stream once, and the second wait is short when nothing but the
            # counting pass of the graph sits between them; the filling pass then runs ahead of the forward pass
            self.build_plan()
            self.build_graph()
        self.forward()
        self.backward(g_energy, g_force)

    # -- HIP graph of forward + backward (graph prebuilt) ------------------------------------------
    def capture(self, g_energy, g_force):
        """Record forward() + backward(g_energy, g_force) into a HIP graph and return it (replay() launches it).

        Both only enqueue kernels and event fork/joins of the library's side stream, all of which a stream capture
        records. Everything that allocates or sets kernel attributes happens on first use, so one eager step runs
        first. The graph reads and writes this object's buffers and the two gradient tensors given here: refill
        those in place before a replay. The radius graph is not part of it (its count call synchronises)."""
        self.forward()
        self.backward(g_energy, g_force)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.forward()
            self.backward(g_energy, g_force)
        return graph
