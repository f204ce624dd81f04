"""Shared helpers of the GPU parity tests: build a seeded problem, run the oracle, run the library."""
from __future__ import annotations

import numpy as np

import oracle
from hgnn_inputs import (init_deep_head_weights, init_embedding, init_head_weights, init_layer_weights,
                         make_config, upstream_grads)

TOL = {  # norm-wise L-inf relative error (max|a-b| / max|b|) against the float64 oracle
    "f32": dict(fwd=1e-5, grad=1e-4),
    "bf16": dict(fwd=2e-2, grad=2e-2),
}


def relerr(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    assert a.shape == b.shape, (a.shape, b.shape)
    if b.size == 0:
        return 0.0
    den = np.max(np.abs(b))
    num = np.max(np.abs(a - b))
    return float(num / den) if den > 0 else float(num)


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


def oracle_graph(P):
    b, hp = P["batch"], P["hp"]
    return oracle.radius_graph(b.pos, b.graph_off, b.cell, b.pbc, hp["rc"])


def oracle_step(P, graph, alpha, grads=True, keep_layers=False):
    b, hp = P["batch"], P["hp"]
    geom = hp.get("pos_grad", False)
    rbf = (hp["rbf_k"], hp["rc"]) if hp.get("rbf_k") and geom else None
    attr = oracle.edge_rbf(graph["d2"], hp["rbf_k"], hp["rc"]) if hp.get("rbf_k") and not geom else None
    return oracle.step_fwd_bwd(b.Z, b.graph_off, b.source_id, graph, P["emb"].astype(np.float64),
                               [w.astype(np.float64) for w in P["Ws"]], P["Wh"].astype(np.float64),
                               hp.get("Hh", hp["H"]), hp["S"], alpha,
                               P["gE"].astype(np.float64) if grads else None,
                               P["gF"].astype(np.float64) if grads else None, keep_layers=keep_layers, D=hp.get("D"),
                               attr=attr, rbf=rbf, move=hp.get("move", False), pos_grad=geom)


def gpu_hotpath(P, alpha=None):
    from paper_2506_21788_amd.step import HotPath
    b, hp = P["batch"], P["hp"]
    return HotPath(b, hp["rc"], hp["H"], hp["L"], hp["S"], hp["dtype"], P["emb"], P["Ws"], P["Wh"], alpha=alpha,
                   Hh=hp.get("Hh"), D=hp.get("D"), rbf_k=hp.get("rbf_k"), move=hp.get("move", False),
                   pos_grad=hp.get("pos_grad", False))


def assert_graph_equal(got, want):
    assert got["E"] == want["E"], (got["E"], want["E"])
    for k in ("row_ptr", "dst", "col", "shift", "edge_graph_ptr", "colT_ptr", "permT"):
        assert np.array_equal(got[k], want[k]), k
    # float outputs are produced by the same individually rounded float32 operations: bit-exact
    assert np.array_equal(got["d2"].view(np.uint32), want["d2"].view(np.uint32)), "d2"
    assert np.array_equal(got["rvec"].view(np.uint32), want["rvec"].view(np.uint32)), "rvec"


def sub_batch(b, graphs):
    """The listed graphs of a batch as a batch of their own (same atoms, cells, sources)."""
    from hgnn_inputs import concat_graphs
    gl = [(b.pos[b.graph_off[g]:b.graph_off[g + 1]], b.Z[b.graph_off[g]:b.graph_off[g + 1]],
           b.cell[g] if b.pbc[g] else None) for g in graphs]
    return concat_graphs(gl, b.source_id[graphs])
