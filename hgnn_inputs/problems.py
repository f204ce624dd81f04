"""A "problem" = one seeded batch together with every weight buffer and the upstream gradients of one step, as the
dict both the CPU oracle's tests and the GPU harness / benchmark start from. Draws and layouts only."""
from __future__ import annotations

import numpy as np

from .configs import make_config
from .structures import concat_graphs
from .weights import (init_deep_head_weights, init_embedding, init_head_weights, init_layer_weights,
                      upstream_grads)


def make_weights(seed, H, L, S, N, G, Hh=None, D=None, k=1):
    """Hh, D: head width and hidden layers per head (None: the plain heads, one hidden layer of width H).
    k: edge attributes per edge (1: the squared distance)."""
    ss = np.random.SeedSequence(seed).spawn(3)
    rw = np.random.default_rng(ss[1])
    rg = np.random.default_rng(ss[2])
    emb = init_embedding(rw, H)
    Ws = [init_layer_weights(rw, H, k=k) for _ in range(L)]
    Wh = init_head_weights(rw, H, H, S) if D is None else init_deep_head_weights(rw, H, Hh, D, S)
    gE, gF = upstream_grads(rg, G, N)
    return emb, Ws, Wh, gE, gF


def problem_from_config(name, rbf_k=None, move=False, pos_grad=False, **over):
    """rbf_k: run the config with that many radial-basis edge attributes in place of d2. move: the atoms move between
    layers; pos_grad: the reverse pass also gives the position gradient."""
    batch, hp = make_config(name, **over)
    if rbf_k:
        hp["rbf_k"] = int(rbf_k)
    if move or pos_grad:
        hp.update(move=bool(move), pos_grad=True)
    emb, Ws, Wh, gE, gF = make_weights(hp["seed"], hp["H"], hp["L"], hp["S"], batch.N, batch.G, hp.get("Hh"),
                                       hp.get("D"), hp.get("rbf_k") or 1)
    return dict(batch=batch, hp=hp, emb=emb, Ws=Ws, Wh=Wh, gE=gE, gF=gF)


def problem_from_batch(batch, rc, H, L, S, dtype, seed=0, Hh=None, D=None, rbf_k=None, move=False, pos_grad=False):
    """move: the atoms move between layers; pos_grad: the reverse pass also gives the position gradient."""
    emb, Ws, Wh, gE, gF = make_weights(seed, H, L, S, batch.N, batch.G, Hh, D, rbf_k or 1)
    hp = dict(rc=rc, H=H, L=L, S=S, dtype=dtype, seed=seed, name="custom")
    if rbf_k:
        hp["rbf_k"] = rbf_k
    if move or pos_grad:
        hp.update(move=bool(move), pos_grad=True)
    if D is not None:
        hp.update(Hh=Hh, D=D)
    return dict(batch=batch, hp=hp, emb=emb, Ws=Ws, Wh=Wh, gE=gE, gF=gF)


def sub_batch(b, graphs):
    """The listed graphs of a batch as a batch of their own (same atoms, cells, sources)."""
    gl = [(b.pos[b.graph_off[g]:b.graph_off[g + 1]], b.Z[b.graph_off[g]:b.graph_off[g + 1]],
           b.cell[g] if b.pbc[g] else None) for g in graphs]
    return concat_graphs(gl, b.source_id[graphs])


def sub_problem(P, graphs):
    """The problem restricted to the listed graphs: their structures and upstream gradients, the same weights."""
    b = P["batch"]
    graphs = np.asarray(graphs)
    atoms = np.concatenate([np.arange(b.graph_off[g], b.graph_off[g + 1]) for g in graphs]) if len(graphs) else \
        np.zeros(0, np.int64)
    return dict(P, batch=sub_batch(b, graphs), gE=P["gE"][graphs], gF=P["gF"][atoms]), atoms
