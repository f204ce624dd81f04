"""Atoms that move between layers, gradients with respect to positions and conservative forces (needs a GPU):
the geometry entry points one by one, the layer's edge gradients, and whole steps against the float64 oracle."""
import numpy as np
import pytest

import oracle
from hgnn_inputs import small_mixed_batch
from hgnn_inputs.weights import init_layer_weights
from parity_util import TOL, gpu_hotpath, oracle_graph, oracle_step, problem_from_batch, relerr
from test_gpu_layer_sizes import _edges

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


def _dev(a):
    import torch
    return torch.as_tensor(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("N,E", [(40, 0), (1, 5), (300, 4097), (5000, 150001)])
def test_edge_geometry_forward_and_reverse(N, E):
    import torch
    from paper_2506_21788_amd import binding as B
    say("edge geometry", N, E)
    rng = np.random.default_rng(N + E)
    row_ptr, dst, col, _, rvec0 = _edges(rng, N, E)
    colT_ptr, permT = oracle.transpose_plan(col, N)
    v = (0.2 * rng.standard_normal((N, 3))).astype(np.float32)
    rvec = torch.full((max(E, 1), 3), float("nan"), device="cuda")
    d2 = torch.full((max(E, 1),), float("nan"), device="cuda")
    B.edge_geometry_fwd(N, E, _dev(rvec0), _dev(v), _dev(dst), _dev(col), rvec, d2)
    torch.cuda.synchronize()
    want_r, want_d2 = oracle.edge_geometry(rvec0, v, dst, col)
    if E:
        assert relerr(rvec.cpu().numpy()[:E], want_r) <= TOL["f32"]["fwd"]
        assert relerr(d2.cpu().numpy()[:E], want_d2) <= TOL["f32"]["fwd"]
    g_rvec = rng.standard_normal((E, 3)).astype(np.float32)
    g_d2 = rng.standard_normal(E).astype(np.float32)
    g_sum0 = rng.standard_normal((E, 3)).astype(np.float32)
    g_v0 = rng.standard_normal((N, 3)).astype(np.float32)
    g_r = torch.full((max(E, 1), 3), float("nan"), device="cuda")
    g_sum, g_v = _dev(g_sum0 if E else np.zeros((1, 3), np.float32)), _dev(g_v0)
    r32 = want_r.astype(np.float32)
    B.edge_geometry_bwd(N, E, _dev(row_ptr), _dev(colT_ptr), _dev(permT.astype(np.int32)),
                        _dev(r32 if E else np.zeros((1, 3), np.float32)),
                        _dev(g_rvec if E else np.zeros((1, 3), np.float32)),
                        _dev(g_d2 if E else np.zeros(1, np.float32)), g_r, g_sum, g_v)
    torch.cuda.synchronize()
    want_gr, want_gv = oracle.edge_geometry_bwd(r32.astype(np.float64), g_rvec, g_d2, dst, col, N)
    if E:
        assert relerr(g_r.cpu().numpy()[:E], want_gr) <= TOL["f32"]["grad"]
        assert relerr(g_sum.cpu().numpy()[:E], g_sum0 + want_gr) <= TOL["f32"]["grad"]     # accumulates
    assert relerr(g_v.cpu().numpy(), g_v0 + want_gv) <= TOL["f32"]["grad"]                  # accumulates
    if E:
        # without g_d2 and without the sum: plain signed incidence sums; the result may overwrite g_rvec
        g_in = _dev(g_rvec)
        g_v2 = torch.zeros((N, 3), device="cuda")
        B.edge_geometry_bwd(N, E, _dev(row_ptr), _dev(colT_ptr), _dev(permT.astype(np.int32)), None, g_in, None, g_in,
                            None, g_v2)
        torch.cuda.synchronize()
        _, want2 = oracle.edge_geometry_bwd(np.zeros((E, 3)), g_rvec, np.zeros(E), dst, col, N)
        assert np.array_equal(g_in.cpu().numpy(), g_rvec)
        assert relerr(g_v2.cpu().numpy(), want2) <= TOL["f32"]["grad"]


@pytest.mark.parametrize("E,k", [(0, 4), (1000, 2), (70001, 16)])
def test_edge_rbf_reverse_and_cutoff(E, k):
    import torch
    from paper_2506_21788_amd import binding as B
    say("edge rbf reverse", E, k)
    rc = 5.0
    rng = np.random.default_rng(E + k)
    d = rng.uniform(0.3, 1.2 * rc, size=E)          # a fifth of the edges lie beyond the cutoff (moved atoms)
    d2 = (d * d).astype(np.float32)
    ga = rng.standard_normal((E, k)).astype(np.float32)
    attr = torch.full((max(E, 1), k), float("nan"), device="cuda")
    g_d2 = torch.full((max(E, 1),), float("nan"), device="cuda")
    B.edge_rbf(E, _dev(d2 if E else np.zeros(1, np.float32)), k, rc, attr)
    B.edge_rbf_bwd(E, _dev(d2 if E else np.zeros(1, np.float32)), k, rc, _dev(ga if E else np.zeros((1, k), np.float32)), g_d2)
    torch.cuda.synchronize()
    if E == 0:
        return
    got_a, got_g = attr.cpu().numpy(), g_d2.cpu().numpy()
    out = np.sqrt(d2.astype(np.float64)) >= rc
    assert out.any() and np.all(got_a[out] == 0.0) and np.all(got_g[out] == 0.0)
    assert relerr(got_a, oracle.edge_rbf(d2, k, rc)) <= TOL["f32"]["fwd"]
    assert relerr(got_g, oracle.edge_rbf_bwd(d2, k, rc, ga)) <= TOL["f32"]["grad"]


@pytest.mark.parametrize("N,E,H,k,dtype", [(300, 5000, 866, 8, "bf16"), (200, 3001, 256, 16, "bf16"),
                                           (64, 700, 333, 1, "bf16"), (100, 1500, 64, 4, "bf16"), (50, 0, 128, 5, "bf16"),
                                           (100, 900, 1024, 2, "bf16"),
                                           # one attribute (the squared length) at the widths of the fused kernels
                                           (200, 3001, 128, 1, "f32"), (300, 5003, 256, 1, "bf16"), (100, 1500, 64, 1, "f32"),
                                           (150, 2000, 256, 1, "f32"), (90, 1100, 128, 1, "bf16"), (40, 0, 64, 1, "f32")])
def test_layer_edge_gradients(N, E, H, k, dtype):
    """g_attr and g_rvec of the layer's reverse pass, and with them every other output of the layer."""
    import torch
    from paper_2506_21788_amd import binding as B
    say("layer edge gradients", N, E, H, k, dtype)
    dt = {"f32": B.F32, "bf16": B.BF16}[dtype]
    rc = 5.0
    rng = np.random.default_rng(N + E + H + k)
    row_ptr, dst, col, d2, rvec = _edges(rng, N, E)
    d2 = np.minimum(d2, np.float32(rc * rc))
    attr = oracle.edge_rbf(d2, k, rc).astype(np.float32) if k > 1 else d2[:, None].copy()
    colT_ptr, permT = oracle.transpose_plan(col, N)
    W = init_layer_weights(rng, H, k=k).astype(np.float32)
    h = rng.standard_normal((N, H)).astype(np.float32)
    v = (rng.standard_normal((N, 3)) * 0.3).astype(np.float32)
    gh = rng.standard_normal((N, H)).astype(np.float32)
    gv = rng.standard_normal((N, 3)).astype(np.float32)
    alpha = 1.0 / max(1.0, E / N)
    ws_b, saved_b = B.mp_layer_attr_workspace_bytes(N, E, H, k, dt)
    ws = torch.empty(ws_b, dtype=torch.uint8, device="cuda")
    saved = torch.empty(saved_b, dtype=torch.uint8, device="cuda")
    t = dict(row_ptr=_dev(row_ptr), dst=_dev(dst), col=_dev(col), attr=_dev(attr if E else np.zeros((1, k), np.float32)),
             rvec=_dev(rvec if E else np.zeros((1, 3), np.float32)), colT=_dev(colT_ptr),
             permT=_dev(permT.astype(np.int32)), h=_dev(h), v=_dev(v), W=_dev(W), gh=_dev(gh), gv=_dev(gv))
    h_out, v_out = torch.empty_like(t["h"]), torch.empty_like(t["v"])
    g_h, g_v, gW = torch.empty_like(t["h"]), torch.empty_like(t["v"]), torch.empty_like(t["W"])
    g_attr = torch.full((max(E, 1), k), float("nan"), device="cuda")
    g_rvec = torch.full((max(E, 1), 3), float("nan"), device="cuda")
    B.mp_layer_attr_fwd(N, E, H, k, dt, alpha, t["row_ptr"], t["dst"], t["col"], t["attr"], t["rvec"], t["h"],
                        t["v"], t["W"], h_out, v_out, saved, ws)
    B.mp_layer_attr_bwd(N, E, H, k, dt, alpha, t["row_ptr"], t["dst"], t["col"], t["attr"], t["rvec"], t["colT"],
                        t["permT"], t["h"], t["W"], saved, t["gh"], t["gv"], g_h, g_v, gW, ws, g_attr=g_attr,
                        g_rvec=g_rvec)
    torch.cuda.synchronize()
    ho, vo, cache = oracle.mp_layer_fwd(h, v, dst, col, d2, rvec, W.astype(np.float64), alpha, attr=attr)
    gho, gvo, gWo, want_ga, want_gr = oracle.mp_layer_bwd(cache, gh, gv, edge_grads=True)
    tol = TOL[dtype]
    errs = dict(h=relerr(h_out.cpu().numpy(), ho), v=relerr(v_out.cpu().numpy(), vo))
    gerrs = dict(g_h=relerr(g_h.cpu().numpy(), gho), g_v=relerr(g_v.cpu().numpy(), gvo))
    got = oracle.unpack_layer(gW.cpu().numpy(), H, k)
    for name, want in gWo.items():
        gerrs["gW." + name] = relerr(got[name], want)
    if E:
        got_ga, got_gr = g_attr.cpu().numpy(), g_rvec.cpu().numpy()
        assert np.all(np.isfinite(got_ga)) and np.all(np.isfinite(got_gr))
        gerrs.update(g_attr=relerr(got_ga, want_ga), g_rvec=relerr(got_gr, want_gr))
    say("  ", {n: f"{e:.1e}" for n, e in {**errs, **gerrs}.items()})
    for n, e in errs.items():
        assert e <= tol["fwd"], (n, e)
    for n, e in gerrs.items():
        assert e <= tol["grad"], (n, e)


def _compare_geometry_step(P, label):
    import torch
    from hgnn_inputs import layer_field_slices
    hp = P["hp"]
    tol = TOL[hp["dtype"]]
    og = oracle_graph(P)
    hpth = gpu_hotpath(P)
    hpth.build_graph()
    want = oracle_step(P, og, hpth.alpha)
    hpth.forward()
    hpth.backward(torch.as_tensor(P["gE"]).cuda(), torch.as_tensor(P["gF"]).cuda())
    torch.cuda.synchronize()
    errs = dict(h=relerr(hpth.h[-1].cpu().numpy(), want["h"]), v=relerr(hpth.v[-1].cpu().numpy(), want["v"]),
                energy=relerr(hpth.energy.cpu().numpy(), want["energy"]),
                force=relerr(hpth.force.cpu().numpy(), want["force"]))
    gerrs = dict(g_pos=relerr(hpth.g_pos.cpu().numpy(), want["g_pos"]),
                 g_emb=relerr(hpth.g_emb.cpu().numpy(), want["g_emb"]),
                 g_heads=relerr(hpth.gWhead.cpu().numpy(), want["g_heads"]))
    for l in range(hp["L"]):
        got = hpth.gW[l].cpu().numpy()
        for name, (lo, hi, _) in layer_field_slices(hp["H"], hp.get("rbf_k") or 1).items():
            gerrs[f"gW{l}.{name}"] = relerr(got[lo:hi], want["g_layers"][l][lo:hi])
    say(label, {n: f"{e:.2e}" for n, e in {**errs, **gerrs}.items()})
    for n, e in errs.items():
        assert e <= tol["fwd"], (n, e)
    for n, e in gerrs.items():
        assert e <= tol["grad"], (n, e)
    return hpth, want


@pytest.mark.parametrize("H,k,move,dtype", [(128, None, False, "bf16"), (128, 8, True, "bf16"), (866, None, True, "bf16"),
                                            (100, 16, False, "bf16"), (256, 4, True, "bf16"),
                                            # the squared length alone at the fused kernels' widths: float32 operands too
                                            (64, None, True, "f32"), (128, None, False, "f32"), (256, None, True, "f32"),
                                            (256, None, True, "bf16")])
def test_step_with_position_gradients(H, k, move, dtype):
    say("step with position gradients", H, k, move, dtype)
    b = small_mixed_batch(21, n_mol=5, n_cry=4, S=3, mol_atoms=(3, 40), cry_atoms=(2, 30))
    P = problem_from_batch(b, 4.5, H, 3, 3, dtype, seed=H + (k or 0), rbf_k=k, move=move, pos_grad=True)
    hpth, want = _compare_geometry_step(P, f"H={H} k={k} move={move} {dtype}")
    # no net force on any structure
    g_pos = hpth.g_pos.cpu().numpy()
    scale = np.max(np.abs(g_pos))
    for g in range(b.G):
        lo, hi = int(b.graph_off[g]), int(b.graph_off[g + 1])
        assert np.max(np.abs(g_pos[lo:hi].sum(axis=0))) <= 1e-4 * max(1.0, scale) * max(1, hi - lo)


def test_step_with_position_gradients_without_edges():
    """Cutoff below every distance: no edges, nothing moves, the position gradient is zero."""
    import torch
    say("position gradients, no edges")
    b = small_mixed_batch(22, n_mol=4, n_cry=0, S=2, mol_atoms=(2, 6))
    P = problem_from_batch(b, 0.05, 128, 2, 2, "bf16", seed=3, rbf_k=4, move=True)
    hpth, _ = _compare_geometry_step(P, "no edges")
    assert hpth.graph.E == 0
    assert torch.all(hpth.g_pos == 0) and torch.all(hpth.v[-1] == 0)


@pytest.mark.parametrize("move", [False, True])
def test_conservative_forces(move):
    """F = -dE/dx: the reverse pass seeded with minus the atom counts on the energies and nothing on the force head."""
    import torch
    say("conservative forces, move =", move)
    b = small_mixed_batch(23, n_mol=4, n_cry=4, S=3, mol_atoms=(3, 30), cry_atoms=(2, 24))
    P = problem_from_batch(b, 4.5, 128, 2, 3, "bf16", seed=9, rbf_k=8, move=move, pos_grad=True)
    hp = P["hp"]
    og = oracle_graph(P)
    hpth = gpu_hotpath(P)
    hpth.build_graph()
    n_at = np.diff(b.graph_off).astype(np.float32)
    hpth.forward()
    hpth.backward(torch.as_tensor(-n_at).cuda(), torch.zeros((b.N, 3), device="cuda"))
    torch.cuda.synchronize()
    e, F = oracle.conservative_forces(b.Z, b.graph_off, b.source_id, og, P["emb"].astype(np.float64),
                                      [w.astype(np.float64) for w in P["Ws"]], P["Wh"].astype(np.float64), hp["H"],
                                      hp["S"], hpth.alpha, rbf=(hp["rbf_k"], hp["rc"]), move=move)
    errs = dict(energy=relerr(hpth.energy.cpu().numpy(), e), F=relerr(hpth.g_pos.cpu().numpy(), F))
    say("  ", {n: f"{v:.2e}" for n, v in errs.items()})
    assert errs["energy"] <= TOL["bf16"]["fwd"] and errs["F"] <= TOL["bf16"]["grad"]


@pytest.mark.parametrize("name,move", [("cfg2", True), ("cfg3", False), ("cfg1", True)])
def test_configs_with_position_gradients(name, move):
    """Whole benchmark configs (config 2: 128 molecules, five sources, float32; config 3: periodic crystals with images
    and self images, bf16; config 1: float32, H = 64) with position gradients, with and without moving atoms."""
    from parity_util import problem_from_config
    say("config with position gradients", name, move)
    P = problem_from_config(name, move=move, pos_grad=True)
    hpth, want = _compare_geometry_step(P, f"{name} move={move}")
    b = P["batch"]
    g_pos = hpth.g_pos.cpu().numpy()
    scale = np.max(np.abs(g_pos))
    for g in range(b.G):    # no net force on any structure, periodic ones included
        lo, hi = int(b.graph_off[g]), int(b.graph_off[g + 1])
        assert np.max(np.abs(g_pos[lo:hi].sum(axis=0))) <= 1e-4 * max(1.0, scale) * max(1, hi - lo)
