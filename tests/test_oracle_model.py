"""Pins of the oracle's layer / pooling / decoder arithmetic against things other than itself."""
import math

import numpy as np
import pytest
import torch

import oracle
from hgnn_inputs import (LAYER_FIELDS, concat_graphs, head_field_slices, head_weight_count, init_embedding,
                         init_head_weights, init_layer_weights, layer_field_slices,
                         layer_weight_count, small_mixed_batch, upstream_grads)
from hgnn_inputs.structures import Batch


def make_problem(seed=0, H=8, Hh=6, L=2, S=3, rc=4.0, batch=None):
    b = batch if batch is not None else small_mixed_batch(seed, S=S)
    rng = np.random.default_rng(seed + 1000)
    g = oracle.radius_graph(b.pos, b.graph_off, b.cell, b.pbc, rc)
    emb = init_embedding(rng, H).astype(np.float64)
    Ws = [init_layer_weights(rng, H).astype(np.float64) for _ in range(L)]
    Wh = init_head_weights(rng, H, Hh, S).astype(np.float64)
    gE, gF = upstream_grads(rng, b.G, b.N)
    alpha = 1.0 / max(1.0, g["E"] / b.N)
    return dict(b=b, g=g, emb=emb, Ws=Ws, Wh=Wh, gE=gE.astype(np.float64), gF=gF.astype(np.float64),
                alpha=alpha, H=H, Hh=Hh, L=L, S=S, rc=rc)


def run(P, grads=True, **kw):
    b = kw.get("b", P["b"])
    return oracle.step_fwd_bwd(b.Z, b.graph_off, b.source_id, kw.get("g", P["g"]), kw.get("emb", P["emb"]),
                               kw.get("Ws", P["Ws"]), kw.get("Wh", P["Wh"]), P["Hh"], P["S"], P["alpha"],
                               P["gE"] if grads else None, P["gF"] if grads else None)


def no_borderline(g, rc, tol=1e-3):
    return np.all(np.abs(np.sqrt(g["d2"].astype(np.float64)) - rc) > tol)


# ---------------------------------------------------------------------------------------------
# forward: brute force with scalar Python loops on a tiny input
# ---------------------------------------------------------------------------------------------
def _silu(t):
    return t / (1.0 + math.exp(-t))


def scalar_forward(P):
    """Edge-by-edge, feature-by-feature evaluation reading the flat buffers by explicit index."""
    b, g, H, Hh, S = P["b"], P["g"], P["H"], P["Hh"], P["S"]
    N = b.N
    h = [[float(P["emb"][b.Z[i], k]) for k in range(H)] for i in range(N)]
    v = [[0.0] * 3 for _ in range(N)]
    for Wl in P["Ws"]:
        sl = layer_field_slices(H)
        o = {k: sl[k][0] for k in sl}
        M = [[0.0] * H for _ in range(N)]
        dv = [[0.0] * 3 for _ in range(N)]
        for e in range(g["E"]):
            i, j = int(g["dst"][e]), int(g["col"][e])
            d2 = float(g["d2"][e])
            a1 = []
            for n in range(H):
                t = float(Wl[o["b1"] + n])
                for k in range(H):
                    t += h[i][k] * Wl[o["W1"] + k * H + n]
                    t += h[j][k] * Wl[o["W1"] + (H + k) * H + n]
                t += d2 * Wl[o["W1"] + 2 * H * H + n]
                a1.append(_silu(t))
            x = 0.0
            for n in range(H):
                t = float(Wl[o["b2"] + n])
                for k in range(H):
                    t += a1[k] * Wl[o["W2"] + k * H + n]
                m = _silu(t)
                M[i][n] += m
                x += Wl[o["wx"] + n] * m
            for c in range(3):
                dv[i][c] += x * float(g["rvec"][e, c])
        hn = []
        for i in range(N):
            u = []
            for n in range(H):
                t = float(Wl[o["b3"] + n])
                for k in range(H):
                    t += h[i][k] * Wl[o["W3"] + k * H + n]
                    t += P["alpha"] * M[i][k] * Wl[o["W3"] + (H + k) * H + n]
                u.append(_silu(t))
            row = []
            for n in range(H):
                t = h[i][n] + float(Wl[o["b4"] + n])
                for k in range(H):
                    t += u[k] * Wl[o["W4"] + k * H + n]
                row.append(t)
            hn.append(row)
            for c in range(3):
                v[i][c] += P["alpha"] * dv[i][c]
        h = hn
    per = head_weight_count(H, Hh)
    hs = head_field_slices(H, Hh)
    energy, force = [], [[0.0] * 3 for _ in range(N)]
    for gi in range(b.G):
        base = int(b.source_id[gi]) * per
        lo, hi = int(b.graph_off[gi]), int(b.graph_off[gi + 1])
        p = [sum(h[i][k] for i in range(lo, hi)) / (hi - lo) for k in range(H)]
        e = float(P["Wh"][base + hs["be2"][0]])
        for n in range(Hh):
            t = float(P["Wh"][base + hs["be1"][0] + n])
            for k in range(H):
                t += p[k] * P["Wh"][base + hs["We1"][0] + k * Hh + n]
            e += _silu(t) * P["Wh"][base + hs["We2"][0] + n]
        energy.append(e)
        for i in range(lo, hi):
            q = float(P["Wh"][base + hs["bf2"][0]])
            for n in range(Hh):
                t = float(P["Wh"][base + hs["bf1"][0] + n])
                for k in range(H):
                    t += h[i][k] * P["Wh"][base + hs["Wf1"][0] + k * Hh + n]
                q += _silu(t) * P["Wh"][base + hs["Wf2"][0] + n]
            for c in range(3):
                force[i][c] = q * v[i][c]
    return np.array(h), np.array(v), np.array(energy), np.array(force)


def test_forward_equals_scalar_brute_force():
    P = make_problem(seed=3, H=4, Hh=3, L=2, S=2, rc=3.2,
                     batch=small_mixed_batch(3, n_mol=2, n_cry=1, S=2, mol_atoms=(3, 6), cry_atoms=(2, 4)))
    assert 20 < P["g"]["E"] < 2000
    out = run(P, grads=False)
    h, v, e, f = scalar_forward(P)
    assert np.allclose(out["h"], h, rtol=1e-12, atol=1e-12)
    assert np.allclose(out["v"], v, rtol=1e-12, atol=1e-12)
    assert np.allclose(out["energy"], e, rtol=1e-12, atol=1e-12)
    assert np.allclose(out["force"], f, rtol=1e-12, atol=1e-12)
    assert np.abs(f).max() > 1e-4


# ---------------------------------------------------------------------------------------------
# aggregation = dense adjacency product; adjoint identity
# ---------------------------------------------------------------------------------------------
def test_aggregation_equals_dense_adjacency_product():
    P = make_problem(seed=4)
    b, g = P["b"], P["g"]
    h0 = oracle.embed_fwd(b.Z, P["emb"])
    _, v1, c = oracle.mp_layer_fwd(h0, np.zeros((b.N, 3)), g["dst"], g["col"], g["d2"], g["rvec"],
                                   P["Ws"][0], P["alpha"])
    A = np.zeros((b.N, g["E"]))
    for e in range(g["E"]):
        A[g["dst"][e], e] = 1.0
    assert np.allclose(c["M"], P["alpha"] * (A @ c["m"]), rtol=1e-13, atol=1e-13)
    x = c["m"] @ oracle.unpack_layer(P["Ws"][0], P["H"])["wx"]
    assert np.allclose(v1, P["alpha"] * (A @ (x[:, None] * g["rvec"])), rtol=1e-13, atol=1e-13)
    # adjoint identity <scatter(m), y> = <m, gather(y)>
    y = np.random.default_rng(0).standard_normal((b.N, P["H"]))
    assert np.isclose(np.sum((A @ c["m"]) * y), np.sum(c["m"] * y[g["dst"]]))


# ---------------------------------------------------------------------------------------------
# symmetries
# ---------------------------------------------------------------------------------------------
def random_rotation(rng):
    q, r = np.linalg.qr(rng.standard_normal((3, 3)))
    q = q * np.sign(np.diag(r))
    if np.linalg.det(q) < 0:
        q[:, 0] = -q[:, 0]
    return q


def transformed(P, pos=None, cell=None, perm=None, gperm=None):
    b = P["b"]
    nb = Batch(pos=(b.pos if pos is None else pos).astype(np.float32), Z=b.Z.copy(),
               graph_off=b.graph_off.copy(), cell=(b.cell if cell is None else cell).astype(np.float32),
               pbc=b.pbc.copy(), source_id=b.source_id.copy())
    if perm is not None:
        nb.pos, nb.Z = nb.pos[perm], nb.Z[perm]
    if gperm is not None:
        graphs = []
        for g in gperm:
            lo, hi = b.graph_off[g], b.graph_off[g + 1]
            graphs.append((nb.pos[lo:hi], nb.Z[lo:hi], nb.cell[g] if b.pbc[g] else None))
        nb = concat_graphs(graphs, b.source_id[gperm])
    g = oracle.radius_graph(nb.pos, nb.graph_off, nb.cell, nb.pbc, P["rc"], extra_images=1)
    return nb, g


def test_rotation_translation_invariance_and_force_equivariance():
    P = make_problem(seed=6, rc=3.6)
    assert no_borderline(P["g"], P["rc"])
    out = run(P, grads=False)
    rng = np.random.default_rng(9)
    R = random_rotation(rng)
    t = np.array([0.7, -0.3, 1.1])
    b = P["b"]
    pos2 = b.pos.astype(np.float64) @ R.T + t
    cell2 = b.cell.astype(np.float64) @ R.T
    nb, g2 = transformed(P, pos=pos2, cell=cell2)
    assert g2["E"] == P["g"]["E"] and np.array_equal(g2["col"], P["g"]["col"])
    out2 = run(P, grads=False, b=nb, g=g2)
    assert np.allclose(out2["energy"], out["energy"], rtol=1e-5, atol=1e-6)
    assert np.allclose(out2["h"], out["h"], rtol=1e-5, atol=1e-6)
    assert np.allclose(out2["force"], out["force"] @ R.T, rtol=1e-4, atol=1e-6)
    assert np.abs(out["force"]).max() > 1e-3
    # a rotated force differs from the unrotated one: the check above is not vacuous
    assert not np.allclose(out2["force"], out["force"], rtol=1e-2, atol=1e-4)


def test_permutation_equivariance():
    P = make_problem(seed=8)
    out = run(P, grads=False)
    b = P["b"]
    rng = np.random.default_rng(1)
    perm = np.arange(b.N)
    for g in range(b.G):
        lo, hi = b.graph_off[g], b.graph_off[g + 1]
        perm[lo:hi] = lo + rng.permutation(hi - lo)
    nb, g2 = transformed(P, perm=perm)
    out2 = run(P, grads=False, b=nb, g=g2)
    assert np.allclose(out2["energy"], out["energy"], rtol=1e-12)
    assert np.allclose(out2["force"], out["force"][perm], rtol=1e-10, atol=1e-12)
    # graph order
    gperm = rng.permutation(b.G)
    nb, g3 = transformed(P, gperm=gperm)
    out3 = run(P, grads=False, b=nb, g=g3)
    assert np.allclose(out3["energy"], out["energy"][gperm], rtol=1e-12)


def test_supercell_gives_same_energy_per_atom_and_duplicated_forces():
    rng = np.random.default_rng(2)
    from hgnn_inputs.structures import make_crystal
    pos, z, cell = make_crystal(rng, 5, 3.0, 5.0, 0.9, 1, 30, max_density=0.2)
    b1 = concat_graphs([(pos, z, cell)])
    pos2 = np.concatenate([pos, pos + cell[0]], axis=0)
    cell2 = cell.copy()
    cell2[0] *= 2
    b2 = concat_graphs([(pos2, np.concatenate([z, z]), cell2)])
    rc = 4.5
    P1 = make_problem(seed=1, S=1, rc=rc, batch=b1)
    g2 = oracle.radius_graph(b2.pos, b2.graph_off, b2.cell, b2.pbc, rc)
    assert no_borderline(P1["g"], rc, 1e-4)
    assert g2["E"] == 2 * P1["g"]["E"]
    assert np.array_equal(np.diff(g2["row_ptr"]), np.tile(np.diff(P1["g"]["row_ptr"]), 2))
    o1 = run(P1, grads=False)
    o2 = run(P1, grads=False, b=b2, g=g2)
    assert np.allclose(o2["energy"], o1["energy"], rtol=1e-6)
    assert np.allclose(o2["force"], np.tile(o1["force"], (2, 1)), rtol=1e-4, atol=1e-6)
    assert any(i == j for i, j in zip(P1["g"]["dst"], P1["g"]["col"]))   # self images were needed


# ---------------------------------------------------------------------------------------------
# layout conventions of W1 / W3 (which rows act on what)
# ---------------------------------------------------------------------------------------------
def test_weight_row_blocks_act_on_the_documented_inputs():
    P = make_problem(seed=10, L=1)
    b, g, H = P["b"], P["g"], P["H"]
    sl = layer_field_slices(H)
    rng = np.random.default_rng(0)
    h0 = rng.standard_normal((b.N, H))
    v0 = np.zeros((b.N, 3))

    def msgs(W, h):
        return oracle.mp_layer_fwd(h, v0, g["dst"], g["col"], g["d2"], g["rvec"], W, 1.0)[2]["m"]

    W = P["Ws"][0].copy()
    o = sl["W1"][0]
    # zero the block acting on the source: messages must not change when only source features change
    Wa = W.copy()
    Wa[o + H * H:o + 2 * H * H] = 0.0
    e = int(np.argmax(g["dst"] != g["col"]))
    h1 = h0.copy()
    h1[g["col"][e]] += 1.0
    rows_of_src = g["dst"] == g["col"][e]
    m0, m1 = msgs(Wa, h0), msgs(Wa, h1)
    assert np.allclose(m0[~rows_of_src], m1[~rows_of_src])
    assert not np.allclose(m0[rows_of_src], m1[rows_of_src])
    # zero the d2 row: messages independent of distances
    Wb = W.copy()
    Wb[o + 2 * H * H:o + 2 * H * H + H] = 0.0
    c0 = oracle.mp_layer_fwd(h0, v0, g["dst"], g["col"], g["d2"], g["rvec"], Wb, 1.0)[2]["m"]
    c1 = oracle.mp_layer_fwd(h0, v0, g["dst"], g["col"], g["d2"] * 2, g["rvec"], Wb, 1.0)[2]["m"]
    assert np.allclose(c0, c1)
    assert not np.allclose(msgs(W, h0), oracle.mp_layer_fwd(h0, v0, g["dst"], g["col"], g["d2"] * 2,
                                                            g["rvec"], W, 1.0)[2]["m"])
    # W2 = 0 and b2 = 0: no message, the layer reduces to the node MLP on [h ; 0], v unchanged
    Wc = W.copy()
    Wc[sl["W2"][0]:sl["W2"][1]] = 0.0
    Wc[sl["b2"][0]:sl["b2"][1]] = 0.0
    hout, vout, _ = oracle.mp_layer_fwd(h0, v0 + 1.0, g["dst"], g["col"], g["d2"], g["rvec"], Wc, 1.0)
    U = oracle.unpack_layer(Wc, H)
    z3 = h0 @ U["W3"][:H] + U["b3"]
    want = h0 + (z3 / (1 + np.exp(-z3))) @ U["W4"] + U["b4"]
    assert np.allclose(hout, want) and np.allclose(vout, v0 + 1.0)


# ---------------------------------------------------------------------------------------------
# decoder routing
# ---------------------------------------------------------------------------------------------
def test_equal_heads_equal_single_head_and_heads_are_independent():
    P = make_problem(seed=12, S=3)
    H, Hh = P["H"], P["Hh"]
    per = head_weight_count(H, Hh)
    one = P["Wh"][:per]
    Wsame = np.tile(one, 3)
    out3 = run(P, grads=False, Wh=Wsame)
    b = P["b"]
    P1 = dict(P, S=1)
    b1 = Batch(b.pos, b.Z, b.graph_off, b.cell, b.pbc, np.zeros_like(b.source_id))
    out1 = run(P1, grads=False, b=b1, Wh=one)
    assert np.allclose(out3["energy"], out1["energy"]) and np.allclose(out3["force"], out1["force"])
    # changing head t changes no output of graphs of another source
    t = int(b.source_id[0])
    W2 = P["Wh"].copy()
    W2[t * per:(t + 1) * per] += 0.3
    o0, o2 = run(P, grads=False), run(P, grads=False, Wh=W2)
    other = b.source_id != t
    assert other.any() and (~other).any()
    assert np.array_equal(o0["energy"][other], o2["energy"][other])
    assert not np.allclose(o0["energy"][~other], o2["energy"][~other])
    gid = np.searchsorted(b.graph_off, np.arange(b.N), side="right") - 1
    assert np.array_equal(o0["force"][other[gid]], o2["force"][other[gid]])


def test_routing_plan_by_python_loops():
    rng = np.random.default_rng(4)
    S, G = 4, 13
    src = rng.integers(0, S, size=G)
    sizes = rng.integers(1, 6, size=G)
    off = np.concatenate([[0], np.cumsum(sizes)])
    ggp, gperm, gap, aperm = oracle.routing_plan(src, off, S)
    want_g, want_a, gp, ap = [], [], [0], [0]
    for s in range(S):
        for g in range(G):
            if src[g] == s:
                want_g.append(g)
                want_a.extend(range(off[g], off[g + 1]))
        gp.append(len(want_g))
        ap.append(len(want_a))
    assert gperm.tolist() == want_g and aperm.tolist() == want_a
    assert ggp.tolist() == gp and gap.tolist() == ap
    with pytest.raises(ValueError):
        oracle.routing_plan(np.array([0, S]), np.array([0, 1, 2]), S)


def test_absent_source_has_exactly_zero_gradient():
    P = make_problem(seed=14, S=4)
    b = P["b"]
    src = b.source_id.copy()
    src[src == 2] = 1
    b2 = Batch(b.pos, b.Z, b.graph_off, b.cell, b.pbc, src)
    out = run(P, b=b2)
    per = head_weight_count(P["H"], P["Hh"])
    assert np.all(out["g_heads"][2 * per:3 * per] == 0.0)
    assert np.any(out["g_heads"][1 * per:2 * per] != 0.0)


# ---------------------------------------------------------------------------------------------
# backward: finite differences, autograd, linearity
# ---------------------------------------------------------------------------------------------
def loss_of(P, emb, Ws, Wh):
    o = run(P, grads=False, emb=emb, Ws=Ws, Wh=Wh)
    return float(np.sum(P["gE"] * o["energy"]) + np.sum(P["gF"] * o["force"]))


def test_backward_by_central_finite_differences_all_parameters():
    P = make_problem(seed=16, H=6, Hh=5, L=2, S=3)
    out = run(P)
    rng = np.random.default_rng(0)
    eps = 1e-6
    # one random direction over everything
    for trial in range(2):
        d_emb = rng.standard_normal(P["emb"].shape)
        d_Ws = [rng.standard_normal(w.shape) for w in P["Ws"]]
        d_Wh = rng.standard_normal(P["Wh"].shape)
        ana = (np.sum(out["g_emb"] * d_emb) + sum(np.sum(g * d) for g, d in zip(out["g_layers"], d_Ws))
               + np.sum(out["g_heads"] * d_Wh))
        lp = loss_of(P, P["emb"] + eps * d_emb, [w + eps * d for w, d in zip(P["Ws"], d_Ws)], P["Wh"] + eps * d_Wh)
        lm = loss_of(P, P["emb"] - eps * d_emb, [w - eps * d for w, d in zip(P["Ws"], d_Ws)], P["Wh"] - eps * d_Wh)
        num = (lp - lm) / (2 * eps)
        assert abs(num - ana) <= 1e-6 * max(1.0, abs(ana)), (num, ana)


def test_backward_by_finite_differences_field_by_field():
    """A direction confined to one field at a time: a wrong small field (a bias, wx) cannot hide."""
    P = make_problem(seed=17, H=5, Hh=4, L=2, S=2)
    out = run(P)
    rng = np.random.default_rng(1)
    eps = 1e-6
    H, Hh = P["H"], P["Hh"]
    for l in range(P["L"]):
        for name, (lo, hi, _) in layer_field_slices(H).items():
            d = np.zeros_like(P["Ws"][l])
            d[lo:hi] = rng.standard_normal(hi - lo)
            Wp = [w.copy() for w in P["Ws"]]
            Wm = [w.copy() for w in P["Ws"]]
            Wp[l] += eps * d
            Wm[l] -= eps * d
            num = (loss_of(P, P["emb"], Wp, P["Wh"]) - loss_of(P, P["emb"], Wm, P["Wh"])) / (2 * eps)
            ana = np.sum(out["g_layers"][l] * d)
            assert abs(num - ana) <= 2e-6 * max(1e-2, abs(ana)), (l, name, num, ana)
    per = head_weight_count(H, Hh)
    for s in range(P["S"]):
        for name, (lo, hi, _) in head_field_slices(H, Hh).items():
            d = np.zeros_like(P["Wh"])
            d[s * per + lo:s * per + hi] = rng.standard_normal(hi - lo)
            num = (loss_of(P, P["emb"], P["Ws"], P["Wh"] + eps * d)
                   - loss_of(P, P["emb"], P["Ws"], P["Wh"] - eps * d)) / (2 * eps)
            ana = np.sum(out["g_heads"] * d)
            assert abs(num - ana) <= 2e-6 * max(1e-2, abs(ana)), (s, name, num, ana)


def torch_loss(P, emb, Ws, Wh):
    """The forward written with torch ops; autograd then derives a backward that owes nothing to
    the oracle's hand-written reverse pass."""
    b, g, H, Hh, S = P["b"], P["g"], P["H"], P["Hh"], P["S"]
    dst = torch.as_tensor(g["dst"], dtype=torch.long)
    col = torch.as_tensor(g["col"], dtype=torch.long)
    d2 = torch.as_tensor(g["d2"], dtype=torch.float64)
    rvec = torch.as_tensor(g["rvec"], dtype=torch.float64)
    h = emb[torch.as_tensor(b.Z, dtype=torch.long)]
    v = torch.zeros(b.N, 3, dtype=torch.float64)
    silu = torch.nn.functional.silu
    for W in Ws:
        f = {k: W[lo:hi].reshape(shp) for k, (lo, hi, shp) in layer_field_slices(H).items()}
        m = silu(silu(torch.cat([h[dst], h[col], d2[:, None]], 1) @ f["W1"] + f["b1"]) @ f["W2"] + f["b2"])
        M = torch.zeros(b.N, H, dtype=torch.float64).index_add(0, dst, m) * P["alpha"]
        v = v + P["alpha"] * torch.zeros(b.N, 3, dtype=torch.float64).index_add(0, dst, (m @ f["wx"])[:, None] * rvec)
        h = h + silu(torch.cat([h, M], 1) @ f["W3"] + f["b3"]) @ f["W4"] + f["b4"]
    per = head_weight_count(H, Hh)
    loss = torch.zeros((), dtype=torch.float64)
    gE = torch.as_tensor(P["gE"])
    gF = torch.as_tensor(P["gF"])
    for gi in range(b.G):
        s = int(b.source_id[gi])
        f = {k: Wh[s * per + lo:s * per + hi].reshape(shp) for k, (lo, hi, shp) in head_field_slices(H, Hh).items()}
        lo, hi = int(b.graph_off[gi]), int(b.graph_off[gi + 1])
        e = silu(h[lo:hi].mean(0) @ f["We1"] + f["be1"]) @ f["We2"] + f["be2"][0]
        q = silu(h[lo:hi] @ f["Wf1"] + f["bf1"]) @ f["Wf2"] + f["bf2"][0]
        loss = loss + gE[gi] * e + torch.sum(gF[lo:hi] * (q[:, None] * v[lo:hi]))
    return loss


def test_backward_equals_torch_autograd():
    P = make_problem(seed=18, H=8, Hh=6, L=3, S=3)
    out = run(P)
    emb = torch.tensor(P["emb"], requires_grad=True)
    Ws = [torch.tensor(w, requires_grad=True) for w in P["Ws"]]
    Wh = torch.tensor(P["Wh"], requires_grad=True)
    loss = torch_loss(P, emb, Ws, Wh)
    loss.backward()
    o = run(P, grads=False)
    assert np.isclose(loss.item(), np.sum(P["gE"] * o["energy"]) + np.sum(P["gF"] * o["force"]), rtol=1e-12)

    def close(a, b):
        return np.max(np.abs(a - b)) <= 1e-10 * max(1.0, np.max(np.abs(b)))

    assert close(out["g_emb"], emb.grad.numpy())
    for l in range(P["L"]):
        assert close(out["g_layers"][l], Ws[l].grad.numpy()), l
    assert close(out["g_heads"], Wh.grad.numpy())


def test_gradient_of_a_batch_is_the_sum_over_its_halves():
    """What data-parallel averaging of the shared-layer gradients relies on."""
    P = make_problem(seed=20, S=2)
    b = P["b"]
    full = run(P)
    k = b.G // 2
    parts = []
    for lo_g, hi_g in ((0, k), (k, b.G)):
        graphs = [(b.pos[b.graph_off[g]:b.graph_off[g + 1]], b.Z[b.graph_off[g]:b.graph_off[g + 1]],
                   b.cell[g] if b.pbc[g] else None) for g in range(lo_g, hi_g)]
        nb = concat_graphs(graphs, b.source_id[lo_g:hi_g])
        a0, a1 = b.graph_off[lo_g], b.graph_off[hi_g]
        Ph = dict(P, b=nb, g=oracle.radius_graph(nb.pos, nb.graph_off, nb.cell, nb.pbc, P["rc"]),
                  gE=P["gE"][lo_g:hi_g], gF=P["gF"][a0:a1])
        parts.append(run(Ph))
    for l in range(P["L"]):
        assert np.allclose(full["g_layers"][l], parts[0]["g_layers"][l] + parts[1]["g_layers"][l], rtol=1e-10, atol=1e-12)
    assert np.allclose(full["g_heads"], parts[0]["g_heads"] + parts[1]["g_heads"], rtol=1e-10, atol=1e-12)
    assert np.allclose(full["g_emb"], parts[0]["g_emb"] + parts[1]["g_emb"], rtol=1e-10, atol=1e-12)


def test_parameter_count_with_all_heads_resident():
    """Memory with every branch on one device: P_s + N_h * P_h (paper, section 'Multi-task parallelism')."""
    H, Hh, L, S = 16, 12, 3, 5
    Ps = L * layer_weight_count(H)
    Ph = head_weight_count(H, Hh)
    assert layer_weight_count(H) == 6 * H * H + 6 * H
    assert Ph == 2 * (H * Hh + 2 * Hh + 1)
    rng = np.random.default_rng(0)
    total = sum(init_layer_weights(rng, H).size for _ in range(L)) + init_head_weights(rng, H, Hh, S).size
    assert total == Ps + S * Ph


def test_isolated_atom_keeps_v_and_gets_zero_aggregate():
    pos = np.array([[0, 0, 0], [1.0, 0, 0], [30.0, 0, 0]], dtype=np.float32)
    b = concat_graphs([(pos, np.array([1, 6, 8], np.int32))])
    P = make_problem(seed=2, S=1, rc=3.0, batch=b, L=1)
    assert P["g"]["E"] == 2 and np.diff(P["g"]["row_ptr"]).tolist() == [1, 1, 0]
    h0 = oracle.embed_fwd(b.Z, P["emb"])
    _, v, c = oracle.mp_layer_fwd(h0, np.ones((3, 3)), P["g"]["dst"], P["g"]["col"], P["g"]["d2"],
                                  P["g"]["rvec"], P["Ws"][0], 1.0)
    assert np.all(c["M"][2] == 0.0) and np.all(v[2] == 1.0) and np.any(c["M"][0] != 0.0)


# ---------------------------------------------------------------------------------------------
# heads with D hidden layers
# ---------------------------------------------------------------------------------------------
def _deep_problem(seed, H, Hh, D, S):
    from hgnn_inputs import init_deep_head_weights
    b = small_mixed_batch(seed, S=S)
    rng = np.random.default_rng(seed + 500)
    h = rng.standard_normal((b.N, H))
    v = rng.standard_normal((b.N, 3))
    p = oracle.pool_fwd(h, b.graph_off)
    Wh = init_deep_head_weights(rng, H, Hh, D, S).astype(np.float64)
    gE, gF = upstream_grads(rng, b.G, b.N)
    return b, h, v, p, Wh, gE.astype(np.float64), gF.astype(np.float64)


def test_deep_heads_with_one_hidden_layer_are_the_plain_heads():
    """D = 1 has the plain heads' buffer layout and must give their numbers (those are pinned by scalar loops)."""
    H, Hh, S = 7, 5, 3
    b, h, v, p, Wh, gE, gF = _deep_problem(31, H, Hh, 1, S)
    assert len(Wh) == S * head_weight_count(H, Hh)
    e1, f1, c1 = oracle.heads_fwd(p, h, v, b.graph_off, b.source_id, Wh, Hh, S)
    e2, f2, c2 = oracle.heads_deep_fwd(p, h, v, b.graph_off, b.source_id, Wh, Hh, 1, S)
    assert np.allclose(e1, e2, rtol=1e-13, atol=1e-13) and np.allclose(f1, f2, rtol=1e-13, atol=1e-13)
    gp1, gh1, gv1, gheads = oracle.heads_bwd(c1, gE, gF)
    flat1 = np.concatenate([np.concatenate([np.ravel(d[k]) for k in ("We1", "be1", "We2", "be2", "Wf1", "bf1", "Wf2", "bf2")])
                            for d in gheads])
    gp2, gh2, gv2, flat2 = oracle.heads_deep_bwd(c2, gE, gF)
    for x, y in ((gp1, gp2), (gh1, gh2), (gv1, gv2), (flat1, flat2)):
        assert np.allclose(x, y, rtol=1e-12, atol=1e-13)


def test_deep_heads_forward_by_scalar_loops():
    """Three hidden layers evaluated value by value, reading the flat buffer by explicit index."""
    from hgnn_inputs import deep_head_field_slices, deep_head_weight_count
    H, Hh, D, S = 4, 3, 3, 2
    b, h, v, p, Wh, _, _ = _deep_problem(32, H, Hh, D, S)
    energy, force, _ = oracle.heads_deep_fwd(p, h, v, b.graph_off, b.source_id, Wh, Hh, D, S)
    sl = deep_head_field_slices(H, Hh, D)
    per = deep_head_weight_count(H, Hh, D)

    def mlp(x, base, which):
        a = [float(t) for t in x]
        for l in range(1, D + 1):
            nin = H if l == 1 else Hh
            oW, ob = sl[f"{which}.W{l}"][0], sl[f"{which}.b{l}"][0]
            a = [_silu(float(Wh[base + ob + n]) + sum(a[k] * Wh[base + oW + k * Hh + n] for k in range(nin)))
                 for n in range(Hh)]
        return float(Wh[base + sl[f"{which}.bo"][0]]) + sum(a[n] * Wh[base + sl[f"{which}.wo"][0] + n] for n in range(Hh))

    for g in range(b.G):
        base = int(b.source_id[g]) * per
        assert abs(mlp(p[g], base, "e") - energy[g]) <= 1e-12 * max(1.0, abs(energy[g]))
        for i in range(int(b.graph_off[g]), int(b.graph_off[g + 1])):
            q = mlp(h[i], base, "f")
            assert np.allclose(q * v[i], force[i], rtol=1e-12, atol=1e-13)


def test_deep_heads_backward_equals_torch_autograd():
    from hgnn_inputs import deep_head_field_slices, deep_head_weight_count
    H, Hh, D, S = 6, 5, 3, 3
    b, h, v, p, Wh, gE, gF = _deep_problem(33, H, Hh, D, S)
    _, _, c = oracle.heads_deep_fwd(p, h, v, b.graph_off, b.source_id, Wh, Hh, D, S)
    g_p, g_h, g_v, g_W = oracle.heads_deep_bwd(c, gE, gF)
    sl = deep_head_field_slices(H, Hh, D)
    per = deep_head_weight_count(H, Hh, D)
    tp, th, tv, tW = (torch.tensor(x, requires_grad=True) for x in (p, h, v, Wh))
    silu = torch.nn.functional.silu
    loss = torch.zeros((), dtype=torch.float64)
    for g in range(b.G):
        s = int(b.source_id[g])
        lo, hi = int(b.graph_off[g]), int(b.graph_off[g + 1])
        f = {k: tW[s * per + a:s * per + e].reshape(shp) for k, (a, e, shp) in sl.items()}
        xe, xf = tp[g:g + 1], th[lo:hi]
        for l in range(1, D + 1):
            xe = silu(xe @ f[f"e.W{l}"] + f[f"e.b{l}"])
            xf = silu(xf @ f[f"f.W{l}"] + f[f"f.b{l}"])
        e = xe @ f["e.wo"] + f["e.bo"][0]
        q = xf @ f["f.wo"] + f["f.bo"][0]
        loss = loss + torch.as_tensor(gE[g]) * e[0] + torch.sum(torch.as_tensor(gF[lo:hi]) * (q[:, None] * tv[lo:hi]))
    loss.backward()
    for mine, ref in ((g_p, tp.grad), (g_h, th.grad), (g_v, tv.grad), (g_W, tW.grad)):
        ref = ref.numpy()
        assert np.max(np.abs(mine - ref)) <= 1e-10 * max(1.0, np.max(np.abs(ref)))


def test_whole_step_with_deep_heads_by_finite_differences():
    from hgnn_inputs import init_deep_head_weights
    P = make_problem(seed=34, H=6, Hh=5, L=2, S=3)
    D = 3
    rng = np.random.default_rng(7)
    Wh = init_deep_head_weights(rng, P["H"], P["Hh"], D, P["S"]).astype(np.float64)
    b = P["b"]

    def step(emb, Ws, Wh_, grads):
        return oracle.step_fwd_bwd(b.Z, b.graph_off, b.source_id, P["g"], emb, Ws, Wh_, P["Hh"], P["S"], P["alpha"],
                                   P["gE"] if grads else None, P["gF"] if grads else None, D=D)

    out = step(P["emb"], P["Ws"], Wh, True)
    d_emb = rng.standard_normal(P["emb"].shape)
    d_Ws = [rng.standard_normal(w.shape) for w in P["Ws"]]
    d_Wh = rng.standard_normal(Wh.shape)
    ana = (np.sum(out["g_emb"] * d_emb) + sum(np.sum(g * d) for g, d in zip(out["g_layers"], d_Ws))
           + np.sum(out["g_heads"] * d_Wh))
    eps = 1e-6

    def loss(sign):
        o = step(P["emb"] + sign * eps * d_emb, [w + sign * eps * d for w, d in zip(P["Ws"], d_Ws)],
                 Wh + sign * eps * d_Wh, False)
        return float(np.sum(P["gE"] * o["energy"]) + np.sum(P["gF"] * o["force"]))

    num = (loss(+1) - loss(-1)) / (2 * eps)
    assert abs(num - ana) <= 1e-6 * max(1.0, abs(ana)), (num, ana)


# ---------------------------------------------------------------------------------------------
# k edge attributes (radial basis of the edge length) in place of d^2
# ---------------------------------------------------------------------------------------------
def test_edge_rbf_closed_forms():
    k, rc = 7, 5.0
    mu = [j * rc / (k - 1) for j in range(k)]
    fc = lambda d: 0.5 * (math.cos(math.pi * d / rc) + 1.0)
    # at a centre the Gaussian is 1: only the cutoff envelope remains; at d = 0 that is 1, at d = rc it is 0
    a = oracle.edge_rbf(np.array([m * m for m in mu]), k, rc)
    for j in range(k):
        assert abs(a[j, j] - fc(mu[j])) <= 1e-15
    assert a[0, 0] == 1.0 and np.all(np.abs(a[-1]) <= 1e-30)
    # half way between two centres both Gaussians are exp(-1/4)
    mid = 0.5 * (mu[2] + mu[3])
    b = oracle.edge_rbf(np.array([mid * mid]), k, rc)[0]
    assert abs(b[2] - math.exp(-0.25) * fc(mid)) <= 1e-15 and abs(b[2] - b[3]) <= 1e-15
    # value by value with scalar arithmetic
    rng = np.random.default_rng(0)
    d = rng.uniform(0.0, rc, size=50)
    got = oracle.edge_rbf(d * d, k, rc)
    for e in range(50):
        for j in range(k):
            want = math.exp(-((k - 1) / rc) ** 2 * (d[e] - mu[j]) ** 2) * fc(d[e])
            assert abs(got[e, j] - want) <= 1e-14
    # smooth at the cutoff: the slope of every attribute vanishes there
    h = 1e-6
    lo = oracle.edge_rbf(np.array([(rc - h) ** 2]), k, rc)[0]
    assert np.all(np.abs(lo) <= 1e-10)


def test_layer_with_one_attribute_equal_to_d2_is_the_plain_layer():
    P = make_problem(seed=40, H=6, L=1)
    g, b = P["g"], P["b"]
    rng = np.random.default_rng(3)
    h = rng.standard_normal((b.N, P["H"]))
    v = rng.standard_normal((b.N, 3))
    a = oracle.mp_layer_fwd(h, v, g["dst"], g["col"], g["d2"], g["rvec"], P["Ws"][0], P["alpha"])
    c = oracle.mp_layer_fwd(h, v, g["dst"], g["col"], g["d2"], g["rvec"], P["Ws"][0], P["alpha"],
                            attr=np.asarray(g["d2"], dtype=np.float64)[:, None])
    assert np.array_equal(a[0], c[0]) and np.array_equal(a[1], c[1])


def test_layer_with_k_attributes_backward_equals_torch_autograd_and_finite_differences():
    P = make_problem(seed=41, H=5, L=1)
    g, b, H, k = P["g"], P["b"], P["H"], 4
    rng = np.random.default_rng(4)
    W = init_layer_weights(rng, H, k=k).astype(np.float64)
    assert len(W) == layer_weight_count(H, k) == (2 * H + k) * H + 5 * H + 3 * H * H + H * H
    h = rng.standard_normal((b.N, H))
    v = rng.standard_normal((b.N, 3))
    attr = oracle.edge_rbf(g["d2"], k, P["rc"])
    gh = rng.standard_normal((b.N, H))
    gv = rng.standard_normal((b.N, 3))
    ho, vo, cache = oracle.mp_layer_fwd(h, v, g["dst"], g["col"], g["d2"], g["rvec"], W, P["alpha"], attr=attr)
    g_h, g_v, gW = oracle.mp_layer_bwd(cache, gh, gv)
    # torch: the forward written with torch ops on the flat buffer
    sl = layer_field_slices(H, k)
    tW, th, tv = torch.tensor(W, requires_grad=True), torch.tensor(h, requires_grad=True), torch.tensor(v, requires_grad=True)
    f = {n: tW[lo:hi].reshape(shp) for n, (lo, hi, shp) in sl.items()}
    dst = torch.as_tensor(g["dst"], dtype=torch.long)
    col = torch.as_tensor(g["col"], dtype=torch.long)
    silu = torch.nn.functional.silu
    m = silu(silu(torch.cat([th[dst], th[col], torch.as_tensor(attr)], 1) @ f["W1"] + f["b1"]) @ f["W2"] + f["b2"])
    M = torch.zeros(b.N, H, dtype=torch.float64).index_add(0, dst, m) * P["alpha"]
    v2 = tv + P["alpha"] * torch.zeros(b.N, 3, dtype=torch.float64).index_add(
        0, dst, (m @ f["wx"])[:, None] * torch.as_tensor(g["rvec"], dtype=torch.float64))
    h2 = th + silu(torch.cat([th, M], 1) @ f["W3"] + f["b3"]) @ f["W4"] + f["b4"]
    assert np.allclose(h2.detach().numpy(), ho, rtol=1e-12, atol=1e-12)
    (torch.sum(h2 * torch.as_tensor(gh)) + torch.sum(v2 * torch.as_tensor(gv))).backward()
    flat = np.concatenate([np.ravel(gW[n]) for n in LAYER_FIELDS])
    for mine, ref in ((flat, tW.grad.numpy()), (g_h, th.grad.numpy()), (g_v, tv.grad.numpy())):
        assert np.max(np.abs(mine - ref)) <= 1e-10 * max(1.0, np.max(np.abs(ref)))
    # finite differences on the rows of W1 that act on the attributes
    lo = sl["W1"][0] + 2 * H * H
    d = np.zeros_like(W)
    d[lo:lo + k * H] = rng.standard_normal(k * H)
    eps = 1e-6

    def loss(Wx):
        a, c, _ = oracle.mp_layer_fwd(h, v, g["dst"], g["col"], g["d2"], g["rvec"], Wx, P["alpha"], attr=attr)
        return float(np.sum(a * gh) + np.sum(c * gv))

    num = (loss(W + eps * d) - loss(W - eps * d)) / (2 * eps)
    assert abs(num - np.sum(flat * d)) <= 1e-6 * max(1.0, abs(num))


# ---------------------------------------------------------------------------------------------
# atoms that move between layers, gradients with respect to the positions, conservative forces
# ---------------------------------------------------------------------------------------------
def test_edge_rbf_is_zero_from_the_cutoff_on_and_its_derivative_matches_finite_differences():
    k, rc = 6, 4.0
    beyond = oracle.edge_rbf(np.array([rc * rc, (rc + 0.3) ** 2, (1.9 * rc) ** 2]), k, rc)
    assert np.all(beyond == 0.0)
    g = oracle.edge_rbf_bwd(np.array([(rc + 0.3) ** 2]), k, rc, np.ones((1, k)))
    assert np.all(g == 0.0)
    rng = np.random.default_rng(5)
    d2 = rng.uniform(0.2, rc, size=40) ** 2
    ga = rng.standard_normal((40, k))
    got = oracle.edge_rbf_bwd(d2, k, rc, ga)
    eps = 1e-6
    num = np.sum(ga * (oracle.edge_rbf(d2 + eps, k, rc) - oracle.edge_rbf(d2 - eps, k, rc)), axis=1) / (2 * eps)
    assert np.max(np.abs(got - num)) <= 1e-7 * max(1.0, np.max(np.abs(num)))
    # at a centre mu_j the Gaussian is flat: only the envelope's slope is left, -(pi / 2 rc) sin(pi mu / rc) / (2 mu)
    j = 2
    mu = j * rc / (k - 1)
    e = np.zeros((1, k)); e[0, j] = 1.0
    want = -(math.pi / (2 * rc)) * math.sin(math.pi * mu / rc) / (2 * mu)
    assert abs(oracle.edge_rbf_bwd(np.array([mu * mu]), k, rc, e)[0] - want) <= 1e-15


def test_edge_geometry_and_its_reverse():
    P = make_problem(seed=50, H=4, L=1)
    g, b = P["g"], P["b"]
    rng = np.random.default_rng(6)
    v = 0.1 * rng.standard_normal((b.N, 3))
    rvec, d2 = oracle.edge_geometry(g["rvec"], v, g["dst"], g["col"])
    # zero displacement: the neighbour search's own vectors and lengths
    r0, d0 = oracle.edge_geometry(g["rvec"], np.zeros((b.N, 3)), g["dst"], g["col"])
    assert np.array_equal(r0, np.asarray(g["rvec"], dtype=np.float64))
    assert np.max(np.abs(d0 - g["d2"])) <= 1e-5
    # moving every atom of a graph by the same vector changes nothing; edge by edge with scalars
    shift = rng.standard_normal(3)
    r1, _ = oracle.edge_geometry(g["rvec"], v + shift, g["dst"], g["col"])
    assert np.max(np.abs(r1 - rvec)) <= 1e-14
    for e in range(0, g["E"], 7):
        i, j = int(g["dst"][e]), int(g["col"][e])
        for c in range(3):
            assert abs(rvec[e, c] - (float(g["rvec"][e, c]) + v[i, c] - v[j, c])) <= 1e-15
        assert abs(d2[e] - sum(rvec[e, c] ** 2 for c in range(3))) <= 1e-13
    # reverse against a dense signed incidence matrix
    g_rvec = rng.standard_normal((g["E"], 3))
    g_d2 = rng.standard_normal(g["E"])
    g_r, g_v = oracle.edge_geometry_bwd(rvec, g_rvec, g_d2, g["dst"], g["col"], b.N)
    B = np.zeros((b.N, g["E"]))
    B[g["dst"], np.arange(g["E"])] += 1.0
    B[g["col"], np.arange(g["E"])] -= 1.0          # a self-image edge (dst == col) cancels: its vector cannot change
    assert np.max(np.abs(g_v - B @ g_r)) <= 1e-12
    eps = 1e-6
    dv = rng.standard_normal((b.N, 3))
    f = lambda vv: (lambda r, q: float(np.sum(r * g_rvec) + np.sum(q * g_d2)))(*oracle.edge_geometry(g["rvec"], vv, g["dst"], g["col"]))
    num = (f(v + eps * dv) - f(v - eps * dv)) / (2 * eps)
    assert abs(num - np.sum(g_v * dv)) <= 1e-7 * max(1.0, abs(num))


def _moved_graph(g, delta):
    """The same neighbour list with every atom displaced by delta: edge vectors and lengths follow."""
    r = np.asarray(g["rvec"], dtype=np.float64) + delta[g["dst"]] - delta[g["col"]]
    out = dict(g)
    out["rvec"], out["d2"] = r, np.sum(r * r, axis=1)
    return out


def _f64_graph(g):
    return _moved_graph(g, np.zeros((int(max(g["dst"].max(), g["col"].max())) + 1, 3)))


@pytest.mark.parametrize("move,rbf", [(False, None), (True, None), (False, (5, 4.0)), (True, (5, 4.0))])
def test_position_gradient_by_finite_differences(move, rbf):
    P = make_problem(seed=51, H=6, Hh=5, L=3, S=3)
    b = P["b"]
    rng = np.random.default_rng(8)
    Ws = P["Ws"] if rbf is None else [init_layer_weights(rng, P["H"], k=rbf[0]).astype(np.float64) for _ in range(P["L"])]
    g0 = _f64_graph(P["g"])     # lengths consistent with the vectors to the last bit

    def step(g, grads):
        return oracle.step_fwd_bwd(b.Z, b.graph_off, b.source_id, g, P["emb"], Ws, P["Wh"], P["Hh"], P["S"],
                                   P["alpha"], P["gE"] if grads else None, P["gF"] if grads else None,
                                   move=move, rbf=rbf, pos_grad=True)

    out = step(g0, True)
    delta = rng.standard_normal((b.N, 3))
    eps = 1e-6
    loss = lambda o: float(np.sum(P["gE"] * o["energy"]) + np.sum(P["gF"] * o["force"]))
    num = (loss(step(_moved_graph(g0, eps * delta), False)) - loss(step(_moved_graph(g0, -eps * delta), False))) / (2 * eps)
    ana = float(np.sum(out["g_pos"] * delta))
    assert abs(num - ana) <= 1e-6 * max(1.0, abs(ana)), (num, ana)
    # no net force on any structure (moving a whole structure changes no edge vector) ...
    for gi in range(b.G):
        lo, hi = int(b.graph_off[gi]), int(b.graph_off[gi + 1])
        assert np.max(np.abs(out["g_pos"][lo:hi].sum(axis=0))) <= 1e-10 * max(1.0, np.max(np.abs(out["g_pos"])))
    # ... and the weight gradients are those of the step without position gradients when nothing moves
    if not move:
        ref = oracle.step_fwd_bwd(b.Z, b.graph_off, b.source_id, g0, P["emb"], Ws, P["Wh"], P["Hh"], P["S"],
                                  P["alpha"], P["gE"], P["gF"], rbf=rbf)
        assert all(np.array_equal(a, c) for a, c in zip(ref["g_layers"], out["g_layers"]))


def test_moving_atoms_weight_gradients_by_finite_differences_and_first_layer_equals_fixed_atoms():
    P = make_problem(seed=52, H=6, Hh=5, L=3, S=3)
    b = P["b"]
    g0 = _f64_graph(P["g"])
    rng = np.random.default_rng(9)

    def step(Ws, grads, move=True):
        return oracle.step_fwd_bwd(b.Z, b.graph_off, b.source_id, g0, P["emb"], Ws, P["Wh"], P["Hh"], P["S"],
                                   P["alpha"], P["gE"] if grads else None, P["gF"] if grads else None,
                                   move=move, keep_layers=True)

    out = step(P["Ws"], True)
    fixed = step(P["Ws"], False, move=False)
    # before the first layer nothing has moved; afterwards the features differ
    assert np.array_equal(out["hs"][1], fixed["hs"][1]) and not np.allclose(out["hs"][2], fixed["hs"][2])
    d_Ws = [rng.standard_normal(w.shape) for w in P["Ws"]]
    eps = 1e-6
    loss = lambda o: float(np.sum(P["gE"] * o["energy"]) + np.sum(P["gF"] * o["force"]))
    num = (loss(step([w + eps * d for w, d in zip(P["Ws"], d_Ws)], False))
           - loss(step([w - eps * d for w, d in zip(P["Ws"], d_Ws)], False))) / (2 * eps)
    ana = sum(float(np.sum(g * d)) for g, d in zip(out["g_layers"], d_Ws))
    assert abs(num - ana) <= 1e-6 * max(1.0, abs(ana)), (num, ana)


def test_moving_atoms_step_equals_torch_autograd():
    P = make_problem(seed=53, H=5, Hh=4, L=2, S=3)
    b, H, k, rc = P["b"], P["H"], 4, P["rc"]
    rng = np.random.default_rng(10)
    Ws = [init_layer_weights(rng, H, k=k).astype(np.float64) for _ in range(2)]
    g0 = _f64_graph(P["g"])
    out = oracle.step_fwd_bwd(b.Z, b.graph_off, b.source_id, g0, P["emb"], Ws, P["Wh"], P["Hh"], P["S"], P["alpha"],
                              P["gE"], P["gF"], move=True, rbf=(k, rc))
    # torch: positions as the differentiable leaf; edge vectors from positions and the image shifts of the list
    dst = torch.as_tensor(g0["dst"], dtype=torch.long)
    col = torch.as_tensor(g0["col"], dtype=torch.long)
    x0 = torch.tensor(np.asarray(b.pos, dtype=np.float64), requires_grad=True)
    t = torch.as_tensor(np.asarray(b.pos, dtype=np.float64)[g0["dst"]] - np.asarray(b.pos, dtype=np.float64)[g0["col"]]
                        - g0["rvec"])                     # image shift of every edge (a constant)
    tW = [torch.tensor(w, requires_grad=True) for w in Ws]
    silu = torch.nn.functional.silu
    h = torch.as_tensor(P["emb"])[torch.as_tensor(b.Z, dtype=torch.long)]
    x = x0
    sl = layer_field_slices(H, k)
    mu = torch.arange(k, dtype=torch.float64) * (rc / (k - 1))
    for w in tW:
        f = {n: w[lo:hi].reshape(shp) for n, (lo, hi, shp) in sl.items()}
        r = x[dst] - x[col] - t
        d = torch.sqrt(torch.sum(r * r, 1))
        fc = torch.where(d < rc, 0.5 * (torch.cos(math.pi * d / rc) + 1.0), torch.zeros_like(d))
        attr = torch.exp(-((k - 1) / rc) ** 2 * (d[:, None] - mu[None, :]) ** 2) * fc[:, None]
        m = silu(silu(torch.cat([h[dst], h[col], attr], 1) @ f["W1"] + f["b1"]) @ f["W2"] + f["b2"])
        M = torch.zeros(b.N, H, dtype=torch.float64).index_add(0, dst, m) * P["alpha"]
        x = x + P["alpha"] * torch.zeros(b.N, 3, dtype=torch.float64).index_add(0, dst, (m @ f["wx"])[:, None] * r)
        h = h + silu(torch.cat([h, M], 1) @ f["W3"] + f["b3"]) @ f["W4"] + f["b4"]
    assert np.max(np.abs((x - x0).detach().numpy() - out["v"])) <= 1e-12
    assert np.max(np.abs(h.detach().numpy() - out["h"])) <= 1e-11
    # the heads through the oracle's own reverse pass would be circular: seed the check at the layer outputs instead
    gh = rng.standard_normal((b.N, H))
    gv = rng.standard_normal((b.N, 3))
    (torch.sum(h * torch.as_tensor(gh)) + torch.sum((x - x0) * torch.as_tensor(gv))).backward()
    # oracle: the same seeds pushed through its layer / geometry reverse functions
    N = b.N
    vv = np.zeros((N, 3))
    hh = oracle.embed_fwd(b.Z, P["emb"])
    caches, geoms = [], []
    for w in Ws:
        rv, dd = oracle.edge_geometry(g0["rvec"], vv, g0["dst"], g0["col"])
        hh, vv, c = oracle.mp_layer_fwd(hh, vv, g0["dst"], g0["col"], dd, rv, w, P["alpha"], attr=oracle.edge_rbf(dd, k, rc))
        caches.append(c); geoms.append((rv, dd))
    g_h, g_v, g_r0, gWs = gh, gv, 0.0, []
    for c, (rv, dd) in zip(reversed(caches), reversed(geoms)):
        g_h, g_v, gW, g_attr, g_rvec = oracle.mp_layer_bwd(c, g_h, g_v, edge_grads=True)
        g_r, g_vg = oracle.edge_geometry_bwd(rv, g_rvec, oracle.edge_rbf_bwd(dd, k, rc, g_attr), g0["dst"], g0["col"], N)
        g_v = g_v + g_vg
        g_r0 = g_r0 + g_r
        gWs.append(np.concatenate([np.ravel(gW[n]) for n in LAYER_FIELDS]))
    gWs.reverse()
    g_pos = np.zeros((N, 3))
    np.add.at(g_pos, g0["dst"], g_r0)
    np.add.at(g_pos, g0["col"], -g_r0)
    # x - x0 does not depend on x0 directly, so torch's gradient at x0 is exactly the edge-vector path
    assert np.max(np.abs(g_pos - x0.grad.numpy())) <= 1e-10 * max(1.0, np.max(np.abs(g_pos)))
    for mine, ref in zip(gWs, tW):
        assert np.max(np.abs(mine - ref.grad.numpy())) <= 1e-10 * max(1.0, np.max(np.abs(mine)))


def test_conservative_forces_rotate_with_the_structure_and_match_energy_differences():
    P = make_problem(seed=54, H=6, Hh=5, L=2, S=3)
    b = P["b"]
    g0 = _f64_graph(P["g"])
    args = (b.Z, b.graph_off, b.source_id)
    rest = (P["emb"], P["Ws"], P["Wh"], P["Hh"], P["S"], P["alpha"])
    for move in (False, True):
        e, F = oracle.conservative_forces(*args, g0, *rest, move=move)
        # rotate every edge vector: energies stay, forces turn with the structure
        Q = np.linalg.qr(np.random.default_rng(11).standard_normal((3, 3)))[0]
        gq = dict(g0); gq["rvec"] = g0["rvec"] @ Q.T
        eq, Fq = oracle.conservative_forces(*args, gq, *rest, move=move)
        assert np.max(np.abs(eq - e)) <= 1e-12 and np.max(np.abs(Fq - F @ Q.T)) <= 1e-11 * max(1.0, np.max(np.abs(F)))
        # one atom pushed along one axis: total energy changes by -F . dx
        n_at = np.diff(b.graph_off)
        i, c, eps = 3, 1, 1e-6
        delta = np.zeros((b.N, 3)); delta[i, c] = eps
        ep = oracle.step_fwd_bwd(*args, _moved_graph(g0, delta), *rest, move=move)["energy"]
        em = oracle.step_fwd_bwd(*args, _moved_graph(g0, -delta), *rest, move=move)["energy"]
        num = -float(np.sum(n_at * (ep - em))) / (2 * eps)
        assert abs(num - F[i, c]) <= 1e-6 * max(1.0, abs(num)), (num, F[i, c])


def test_pooling_sum_and_mean_by_scalar_loops():
    """pool_fwd / pool_bwd in both modes against element-by-element Python arithmetic, with empty graphs; the reverse
    is the adjoint of the forward in either mode."""
    rng = np.random.default_rng(11)
    sizes = [2, 0, 5, 1, 0, 3]
    graph_off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    N, G, H = int(graph_off[-1]), len(sizes), 3
    h = rng.standard_normal((N, H))
    g_p = rng.standard_normal((G, H))
    for mean in (False, True):
        p = oracle.pool_fwd(h, graph_off, mean=mean)
        g_h = oracle.pool_bwd(g_p, graph_off, N, mean=mean)
        atom = 0
        for g, n in enumerate(sizes):
            for c in range(H):
                acc = 0.0
                for i in range(atom, atom + n):
                    acc += float(h[i, c])
                want = 0.0 if n == 0 else (acc / n if mean else acc)
                assert abs(p[g, c] - want) < 1e-14
                for i in range(atom, atom + n):
                    assert abs(g_h[i, c] - (float(g_p[g, c]) / n if mean else float(g_p[g, c]))) < 1e-15
            atom += n
        assert abs(np.sum(p * g_p) - np.sum(h * g_h)) < 1e-12
    # sum = mean times the atom count
    n_at = np.diff(graph_off)[:, None]
    assert np.allclose(oracle.pool_fwd(h, graph_off, mean=False), oracle.pool_fwd(h, graph_off, mean=True) * n_at)
