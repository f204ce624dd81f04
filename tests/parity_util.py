"""Shared helpers of the GPU parity tests: build a seeded problem, run the oracle, run the library."""
from __future__ import annotations

import numpy as np

import oracle
from hgnn_inputs import (make_weights, problem_from_batch, problem_from_config, sub_batch,  # noqa: F401
                         sub_problem)

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


def gpu_hotpath(P, alpha=None, **kw):
    from paper_2506_21788_amd.step import HotPath
    return HotPath.from_problem(P, alpha=alpha, **kw)


def assert_graph_equal(got, want):
    assert got["E"] == want["E"], (got["E"], want["E"])
    for k in ("row_ptr", "dst", "col", "shift", "edge_graph_ptr", "colT_ptr", "permT"):
        assert np.array_equal(got[k], want[k]), k
    # float outputs are produced by the same individually rounded float32 operations: bit-exact
    assert np.array_equal(got["d2"].view(np.uint32), want["d2"].view(np.uint32)), "d2"
    assert np.array_equal(got["rvec"].view(np.uint32), want["rvec"].view(np.uint32)), "rvec"


def oracle_layer_by_row_blocks(h, v, g, Wflat, alpha, g_h_out, g_v_out, nblocks):
    """One layer, forward and reverse, by the oracle, evaluated over blocks of destination rows so that the edge
    tensors of a large graph never exist all at once. g: the graph arrays (row_ptr, dst, col, d2, rvec).

    Forward: row i of (h', v') depends on h, v and on the edges of row i only. Reverse: the layer's reverse pass is
    linear in (g_h_out, g_v_out), so the upstream gradients masked to a block of rows give that block's additive
    share of every gradient (tests/test_oracle_model.py pins that additivity); the shares are summed in float64.
    Each block runs on the atoms it touches only (its rows and the sources of their edges), renumbered.
    Returns h', v', g_h, g_v, dict of weight gradients."""
    h = np.asarray(h, np.float64)
    v = np.asarray(v, np.float64)
    g_h_out = np.asarray(g_h_out, np.float64)
    g_v_out = np.asarray(g_v_out, np.float64)
    N = h.shape[0]
    row_ptr = g["row_ptr"]
    bounds = np.linspace(0, N, nblocks + 1).astype(np.int64)
    h_out, v_out = np.empty_like(h), np.empty_like(v)
    g_h, g_v, gW = np.zeros_like(h), np.zeros_like(v), None
    for r0, r1 in zip(bounds[:-1], bounds[1:]):
        if r1 == r0:
            continue
        e0, e1 = int(row_ptr[r0]), int(row_ptr[r1])
        dst, col = g["dst"][e0:e1].astype(np.int64), g["col"][e0:e1].astype(np.int64)
        atoms = np.union1d(np.arange(r0, r1), col)                 # sorted; the block's rows are among them
        ldst, lcol = np.searchsorted(atoms, dst), np.searchsorted(atoms, col)
        own = np.searchsorted(atoms, np.arange(r0, r1))
        ho, vo, cache = oracle.mp_layer_fwd(h[atoms], v[atoms], ldst, lcol, g["d2"][e0:e1], g["rvec"][e0:e1], Wflat,
                                            alpha)
        h_out[r0:r1], v_out[r0:r1] = ho[own], vo[own]
        gh_m, gv_m = np.zeros((len(atoms), h.shape[1])), np.zeros((len(atoms), 3))
        gh_m[own], gv_m[own] = g_h_out[r0:r1], g_v_out[r0:r1]
        gh_b, gv_b, gW_b = oracle.mp_layer_bwd(cache, gh_m, gv_m)
        g_h[atoms] += gh_b
        g_v[atoms] += gv_b
        gW = gW_b if gW is None else {k: gW[k] + gW_b[k] for k in gW}
        del cache
    return h_out, v_out, g_h, g_v, gW
