"""Decoding heads with D hidden layers (the paper's three layers of 889 units) against the oracle (needs a GPU)."""
import numpy as np
import pytest

import oracle
from hgnn_inputs import deep_head_field_slices, deep_head_weight_count, init_deep_head_weights
from parity_util import TOL, relerr

pytestmark = pytest.mark.gpu


def _run(G, atoms, H, Hh, D, S, seed, sources=None):
    import torch
    from paper_2506_21788_amd import binding as B
    rng = np.random.default_rng(seed)
    n = rng.integers(atoms[0], atoms[1] + 1, size=G)
    graph_off = np.zeros(G + 1, np.int32)
    graph_off[1:] = np.cumsum(n)
    N = int(graph_off[-1])
    src = rng.choice(np.arange(S) if sources is None else np.asarray(sources), size=G).astype(np.int32)
    h = rng.standard_normal((N, H)).astype(np.float32)
    v = (rng.standard_normal((N, 3)) * 0.5).astype(np.float32)
    p = oracle.pool_fwd(h, graph_off).astype(np.float32)
    Wh = init_deep_head_weights(rng, H, Hh, D, S)
    gE = rng.standard_normal(G).astype(np.float32)
    gF = rng.standard_normal((N, 3)).astype(np.float32)
    dev = lambda a: torch.as_tensor(a).cuda()
    t = dict(graph_off=dev(graph_off), src=dev(src), h=dev(h), v=dev(v), p=dev(p), Wh=dev(Wh), gE=dev(gE), gF=dev(gF))
    plan = torch.empty(B.multihead_plan_ints(N, G, S), dtype=torch.int32, device="cuda")
    B.multihead_plan(N, G, S, t["graph_off"], t["src"], plan)
    ws_b, sv_b = B.multihead_deep_workspace_bytes(N, G, H, Hh, D, S, B.BF16)
    ws = torch.empty(ws_b, dtype=torch.uint8, device="cuda")
    sv = torch.empty(sv_b, dtype=torch.uint8, device="cuda")
    f32 = dict(dtype=torch.float32, device="cuda")
    energy, force = torch.empty(G, **f32), torch.empty((N, 3), **f32)
    g_p, g_h, g_v = torch.empty((G, H), **f32), torch.empty((N, H), **f32), torch.empty((N, 3), **f32)
    gWh = torch.full_like(t["Wh"], float("nan"))
    B.multihead_deep_fwd(N, G, H, Hh, D, S, B.BF16, plan, t["p"], t["h"], t["v"], t["Wh"], energy, force, sv, ws)
    B.multihead_deep_bwd(N, G, H, Hh, D, S, B.BF16, plan, t["p"], t["h"], t["v"], t["Wh"], sv, t["gE"], t["gF"],
                         g_p, g_h, g_v, gWh, ws)
    torch.cuda.synchronize()
    eo, fo, c = oracle.heads_deep_fwd(p, h, v, graph_off, src, Wh.astype(np.float64), Hh, D, S)
    gpo, gho, gvo, gWo = oracle.heads_deep_bwd(c, gE, gF)
    tol = TOL["bf16"]
    errs = dict(energy=relerr(energy.cpu().numpy(), eo), force=relerr(force.cpu().numpy(), fo),
                g_p=relerr(g_p.cpu().numpy(), gpo), g_h=relerr(g_h.cpu().numpy(), gho),
                g_v=relerr(g_v.cpu().numpy(), gvo))
    got = gWh.cpu().numpy()
    assert np.all(np.isfinite(got)), "a gradient field was left unwritten"
    per = deep_head_weight_count(H, Hh, D)
    present = set(int(s) for s in src)
    for s in range(S):
        blk_got, blk_want = got[s * per:(s + 1) * per], gWo[s * per:(s + 1) * per]
        if s not in present:
            assert not blk_got.any() and not blk_want.any(), f"absent source {s} must get exactly zero"
            continue
        for name, (lo, hi, _) in deep_head_field_slices(H, Hh, D).items():
            errs[f"s{s}.{name}"] = relerr(blk_got[lo:hi], blk_want[lo:hi])
    worst = sorted(errs.items(), key=lambda kv: -kv[1])[:4]
    print(f"deep heads G={G} N={N} H={H} Hh={Hh} D={D} S={S}", {k: f"{e:.1e}" for k, e in worst}, flush=True)
    for k, e in errs.items():
        assert e <= (tol["fwd"] if k in ("energy", "force") else tol["grad"]), (k, e)


@pytest.mark.parametrize("G,atoms,H,Hh,D,S,sources", [
    (24, (3, 30), 866, 889, 3, 5, None),      # the paper's widths and depth, five sources
    (10, (1, 9), 64, 32, 1, 3, None),         # one hidden layer: the layout of the plain heads
    (12, (2, 40), 256, 300, 2, 2, None),
    (9, (1, 12), 130, 70, 4, 4, (0, 2)),      # two sources absent from the batch
    (700, (1, 2), 96, 128, 2, 2, None),       # more than 256 graphs per source: several row tiles per group
    (15, (0, 4), 200, 150, 3, 3, None),       # graphs without atoms (their energy is the head of a zero vector)
])
def test_deep_heads_match_the_oracle(G, atoms, H, Hh, D, S, sources):
    _run(G, atoms, H, Hh, D, S, seed=G + H + D, sources=sources)


def test_deep_heads_and_wide_layer_error_paths():
    """Argument errors come back as status codes from the host side; nothing is launched for them."""
    import torch
    from paper_2506_21788_amd import binding as B
    N, G, H, Hh, D, S = 20, 3, 300, 280, 2, 2
    f32 = dict(dtype=torch.float32, device="cuda")
    graph_off = torch.tensor([0, 7, 12, 20], dtype=torch.int32, device="cuda")
    src = torch.tensor([0, 1, 0], dtype=torch.int32, device="cuda")
    plan = torch.empty(B.multihead_plan_ints(N, G, S), dtype=torch.int32, device="cuda")
    B.multihead_plan(N, G, S, graph_off, src, plan)
    ws_b, sv_b = B.multihead_deep_workspace_bytes(N, G, H, Hh, D, S, B.BF16)
    ws = torch.empty(ws_b, dtype=torch.uint8, device="cuda")
    sv = torch.empty(sv_b, dtype=torch.uint8, device="cuda")
    from hgnn_inputs import deep_head_weight_count
    Wh = torch.zeros(S * deep_head_weight_count(H, Hh, D), **f32)
    p, h, v = torch.zeros((G, H), **f32), torch.zeros((N, H), **f32), torch.zeros((N, 3), **f32)
    e, f = torch.empty(G, **f32), torch.empty((N, 3), **f32)

    def code(call):
        with pytest.raises(B.HgnnError) as err:
            call()
        return err.value.code

    assert code(lambda: B.multihead_deep_fwd(N, G, H, Hh, D, S, B.BF16, plan, p, h, v, Wh, e, f, sv, ws[:1024])) == -6
    assert code(lambda: B.multihead_deep_fwd(N, G, H, Hh, D, S, B.BF16, plan, p, h, v, Wh, e, f, sv[:64], ws)) == -6
    assert code(lambda: B.multihead_deep_fwd(N, G, H, Hh, D, S, B.BF16, plan, p, None, v, Wh, e, f, sv, ws)) == -1
    assert code(lambda: B.multihead_deep_fwd(N, G, H, Hh, 9, S, B.BF16, plan, p, h, v, Wh, e, f, sv, ws)) == -2
    assert code(lambda: B.multihead_deep_fwd(N, G, H, Hh, D, S, B.F32, plan, p, h, v, Wh, e, f, sv, ws)) == -9
    B.multihead_deep_fwd(N, G, H, Hh, D, S, B.BF16, plan, p, h, v, Wh, e, f, sv, ws)   # the good call still works
    torch.cuda.synchronize()
    assert bool(torch.isfinite(e).all())
    # the layer at other widths than 64, 128, 256: float32 operands are not implemented, small buffers are refused
    assert code(lambda: B.mp_layer_workspace_bytes(N, 50, 300, B.F32)) == -9
    assert code(lambda: B.mp_layer_workspace_bytes(N, 50, 1025, B.BF16)) == -2
    assert code(lambda: B.mp_layer_workspace_bytes(N, 50, 0, B.BF16)) == -2
    lws, lsv = B.mp_layer_workspace_bytes(N, 0, 300, B.BF16)
    W = torch.zeros(6 * 300 * 300 + 6 * 300, **f32)
    row_ptr = torch.zeros(N + 1, dtype=torch.int32, device="cuda")
    h300, out = torch.zeros((N, 300), **f32), torch.empty((N, 300), **f32)
    assert code(lambda: B.mp_layer_fwd(N, 0, 300, B.BF16, 1.0, row_ptr, None, None, None, None, h300, v, W, out, f,
                                       torch.empty(lsv, dtype=torch.uint8, device="cuda"),
                                       torch.empty(64, dtype=torch.uint8, device="cuda"))) == -6
