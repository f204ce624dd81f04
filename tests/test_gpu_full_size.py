"""GPU parity at the sizes and in the launch configuration bench.py times: every gradient field of configs 4, 5
and 6 against the oracle, which is evaluated piecewise (graph group by graph group, or over blocks of destination
rows) and summed in float64 (needs a GPU)."""
import sys

import numpy as np
import pytest

import oracle
from hgnn_inputs import HEAD_FIELDS, LAYER_FIELDS, layer_field_slices
from oracle.model import pack_fields
from parity_util import (TOL, gpu_hotpath, oracle_graph, oracle_layer_by_row_blocks, oracle_step,
                         problem_from_config, relerr, sub_problem)

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def _run(name, **kw):
    import torch
    P = problem_from_config(name)
    hpth = gpu_hotpath(P, **kw)
    hpth.build_graph()
    hpth.forward()
    hpth.backward(torch.as_tensor(P["gE"]).cuda(), torch.as_tensor(P["gF"]).cuda())
    torch.cuda.synchronize()
    return P, hpth


def _field_errors(prefix, got_flat, want_flat, H, k=1):
    return {f"{prefix}.{n}": relerr(got_flat[lo:hi], want_flat[lo:hi]) for n, (lo, hi, _) in
            layer_field_slices(H, k).items()}


def _check(errs, tol):
    for n, e in errs.items():
        assert e <= tol, (n, e)


def _groups(b, edges_per_group, deg):
    """Consecutive graphs grouped so that a group holds about edges_per_group edges."""
    groups, cur, n = [], [], 0
    for g in range(b.G):
        cur.append(g)
        n += int(b.graph_off[g + 1] - b.graph_off[g])
        if n * deg >= edges_per_group:
            groups.append(np.asarray(cur))
            cur, n = [], 0
    if cur:
        groups.append(np.asarray(cur))
    return groups


def _whole_step_by_graph_groups(name, edges_per_group):
    """A graph's outputs depend on that graph only and every weight gradient is a sum over graphs, so the oracle runs
    the whole step on one group of graphs at a time: outputs are compared graph by graph, gradients after summing."""
    P, hpth = _run(name)
    b, hp = P["batch"], P["hp"]
    H, L = hp["H"], hp["L"]
    G = hpth.graph.to_numpy()
    say(name, "N", b.N, "G", b.G, "E", G["E"], "alpha", hpth.alpha)
    got = dict(energy=hpth.energy.cpu().numpy(), force=hpth.force.cpu().numpy(), h=hpth.h[-1].cpu().numpy(),
               g_h0=hpth.g_h0.cpu().numpy())
    want = {k: np.zeros(a.shape) for k, a in got.items()}
    g_layers = [np.zeros(w.shape, np.float64) for w in P["Ws"]]
    g_heads, g_emb = np.zeros(P["Wh"].shape), np.zeros(P["emb"].shape)
    for graphs in _groups(b, edges_per_group, G["E"] / max(b.N, 1)):
        Ps, atoms = sub_problem(P, graphs)
        og = oracle_graph(Ps)
        # the group's edges, bit-exact (atom numbers relative to the group's first atom)
        a0 = int(b.graph_off[graphs[0]])
        e0, e1 = int(G["edge_graph_ptr"][graphs[0]]), int(G["edge_graph_ptr"][graphs[-1] + 1])
        assert e1 - e0 == og["E"]
        assert np.array_equal(G["row_ptr"][atoms[0]:atoms[-1] + 2] - e0, og["row_ptr"])
        assert np.array_equal(G["dst"][e0:e1] - a0, og["dst"]) and np.array_equal(G["col"][e0:e1] - a0, og["col"])
        assert np.array_equal(G["shift"][e0:e1], og["shift"])
        assert np.array_equal(G["d2"][e0:e1].view(np.uint32), og["d2"].view(np.uint32))
        assert np.array_equal(G["rvec"][e0:e1].view(np.uint32), og["rvec"].view(np.uint32))
        w = oracle_step(Ps, og, hpth.alpha)
        want["energy"][graphs] = w["energy"]
        for k in ("force", "h", "g_h0"):
            want[k][atoms] = w[k]
        for l in range(L):
            g_layers[l] += w["g_layers"][l]
        g_heads += w["g_heads"]
        g_emb += w["g_emb"]
        say(name, "graphs", graphs[0], "..", graphs[-1], "edges", og["E"])
    ct, pt = oracle.transpose_plan(G["col"], b.N)
    assert np.array_equal(ct, G["colT_ptr"]) and np.array_equal(pt, G["permT"])
    assert np.array_equal(G["edge_graph_ptr"], G["row_ptr"][b.graph_off])
    tol = TOL[hp["dtype"]]
    ferrs = {k: relerr(got[k], want[k]) for k in ("energy", "force", "h")}
    gerrs = dict(g_h0=relerr(got["g_h0"], want["g_h0"]), g_emb=relerr(hpth.g_emb.cpu().numpy(), g_emb),
                 g_heads=relerr(hpth.gWhead.cpu().numpy(), g_heads))
    for l in range(L):
        gerrs.update(_field_errors(f"gW{l}", hpth.gW[l].cpu().numpy(), g_layers[l], H))
    say(name, "whole step", {n: f"{e:.2e}" for n, e in {**ferrs, **gerrs}.items()})
    _check(ferrs, tol["fwd"])
    _check(gerrs, tol["grad"])


def test_cfg4_whole_step_every_gradient():
    """Config 4 (~40k atoms, ~1.2M edges, bf16, 5 sources): every edge, output and gradient field."""
    _whole_step_by_graph_groups("cfg4", 150000)


# ------------------------------------------------------------------------------------------------
# layer by layer on the library's own layer inputs and upstream gradients (kept by the harness)
# ------------------------------------------------------------------------------------------------
_kept = {}


def _kept_run(name):
    """One step of a config with every layer's input and upstream gradient kept, as host arrays."""
    if name not in _kept:
        _kept.clear()                     # one config's arrays at a time
        P, hpth = _run(name, keep_grads=True)
        G = hpth.graph.to_numpy()
        L = P["hp"]["L"]
        r = dict(P=P, G=G, alpha=hpth.alpha, h=[t.cpu().numpy() for t in hpth.h], v=[t.cpu().numpy() for t in hpth.v],
                 g_h=[t.cpu().numpy() for t in hpth.g_h], g_v=[t.cpu().numpy() for t in hpth.g_v],
                 gW=[t.cpu().numpy() for t in hpth.gW], gWhead=hpth.gWhead.cpu().numpy(), g_emb=hpth.g_emb.cpu().numpy(),
                 p=hpth.p.cpu().numpy(), energy=hpth.energy.cpu().numpy(), force=hpth.force.cpu().numpy(),
                 g_p=hpth.g_p.cpu().numpy())
        assert len(r["g_h"]) == L + 1
        _kept[name] = r
        del hpth
    return _kept[name]


def _layer_at_full_size(name, l, nblocks):
    r = _kept_run(name)
    P = r["P"]
    hp = P["hp"]
    tol = TOL[hp["dtype"]]
    say(name, "layer", l, "E", r["G"]["E"])
    h_out, v_out, g_h, g_v, gW = oracle_layer_by_row_blocks(r["h"][l], r["v"][l], r["G"], P["Ws"][l].astype(np.float64),
                                                            r["alpha"], r["g_h"][l + 1], r["g_v"][l + 1], nblocks)
    ferrs = dict(h=relerr(r["h"][l + 1], h_out), v=relerr(r["v"][l + 1], v_out))
    gerrs = dict(g_h=relerr(r["g_h"][l], g_h), g_v=relerr(r["g_v"][l], g_v))
    gerrs.update(_field_errors("gW", r["gW"][l], pack_fields(gW, LAYER_FIELDS), hp["H"]))
    say(name, "layer", l, {n: f"{e:.2e}" for n, e in {**ferrs, **gerrs}.items()})
    _check(ferrs, tol["fwd"])
    _check(gerrs, tol["grad"])


def _heads_and_embedding_at_full_size(name):
    """Pooling, heads (forward and reverse) and the embedding gradient on the library's own last-layer features."""
    r = _kept_run(name)
    P = r["P"]
    b, hp = P["batch"], P["hp"]
    tol = TOL[hp["dtype"]]
    L = hp["L"]
    p = oracle.pool_fwd(r["h"][L], b.graph_off)
    Wh = P["Wh"].astype(np.float64)
    if hp.get("D") is None:
        e, f, hc = oracle.heads_fwd(p, r["h"][L], r["v"][L], b.graph_off, b.source_id, Wh, hp["H"], hp["S"])
        g_p, g_h, g_v, gheads = oracle.heads_bwd(hc, P["gE"], P["gF"])
        g_heads = np.concatenate([pack_fields(d, HEAD_FIELDS) for d in gheads])
    else:
        e, f, hc = oracle.heads_deep_fwd(p, r["h"][L], r["v"][L], b.graph_off, b.source_id, Wh, hp["Hh"], hp["D"],
                                         hp["S"])
        g_p, g_h, g_v, g_heads = oracle.heads_deep_bwd(hc, P["gE"], P["gF"])
    g_h = g_h + oracle.pool_bwd(g_p, b.graph_off, b.N)
    ferrs = dict(p=relerr(r["p"], p), energy=relerr(r["energy"], e), force=relerr(r["force"], f))
    gerrs = dict(g_p=relerr(r["g_p"], g_p), g_h=relerr(r["g_h"][L], g_h), g_v=relerr(r["g_v"][L], g_v),
                 g_heads=relerr(r["gWhead"], g_heads),
                 g_emb=relerr(r["g_emb"], oracle.embed_bwd(b.Z, r["g_h"][0], P["emb"].shape[0])))
    say(name, "heads", {n: f"{e:.2e}" for n, e in {**ferrs, **gerrs}.items()})
    _check(ferrs, tol["fwd"])
    _check(gerrs, tol["grad"])


@pytest.mark.parametrize("l", [0, 1, 2])
def test_cfg5_layer_every_gradient(l):
    """Config 5 (80,000 atoms, ~7.2M edges, fp32, H = 128): one layer at full size, all rows and all gradient fields."""
    _layer_at_full_size("cfg5", l, 32)


def test_cfg5_heads_and_embedding_gradients():
    _heads_and_embedding_at_full_size("cfg5")


@pytest.mark.parametrize("l", [0, 1, 2, 3])
def test_cfg6_layer_every_gradient(l):
    """Config 6 (the paper's model shape: H = 866, ~254k edges, bf16): one layer at full size."""
    _layer_at_full_size("cfg6", l, 8)


def test_cfg6_heads_and_embedding_gradients():
    _heads_and_embedding_at_full_size("cfg6")
