"""Message-passing layer, pooling and the two-level multi-task decoder, forward and reverse mode
(test infrastructure; see the package docstring). All arithmetic in float64.

The paper names the backbone (a stack of equivariant EGNN message-passing layers shared by all
sources, section "Numerical Results") and the decoder (one branch per dataset, each split into an
energy-per-atom head and an atomic-force head made of fully connected layers, section "Two-level
hierarchical MTL architecture"), and gives no formula. The layer below is the textbook E(n)-GNN
layer with the positions held fixed during the step:

  per edge e = (i <- j):   z1 = W1^T [h_i ; h_j ; d2_e] + b1     a1 = silu(z1)
                           z2 = W2^T a1 + b2                      m_e = silu(z2)
                           x_e = wx . m_e
  per atom i:              M_i  = alpha * sum_{e in row i} m_e
                           v'_i = v_i + alpha * sum_{e in row i} x_e * rvec_e   (equivariant channel)
                           z3 = W3^T [h_i ; M_i] + b3
                           h'_i = h_i + W4^T silu(z3) + b4
  pooling:                 p_g = mean_{i in g} h_i
  branch s = source_id[g]: e_g = We2_s . silu(We1_s^T p_g + be1_s) + be2_s          (energy per atom)
                           q_i = Wf2_s . silu(Wf1_s^T h_i + bf1_s) + bf2_s,   F_i = q_i * v_i

The force head is a stack of fully connected layers on the per-atom features, as the paper says;
multiplying its scalar output into the equivariant channel v_i is this build's reading of how an
invariant feature vector can give a force that rotates with the structure.
"""
from __future__ import annotations

import numpy as np

_LAYER_FIELDS = ("W1", "b1", "W2", "b2", "wx", "W3", "b3", "W4", "b4")
_HEAD_FIELDS = ("We1", "be1", "We2", "be2", "Wf1", "bf1", "Wf2", "bf2")


def unpack_layer(flat, H, k=1):
    """Views into one layer's flat buffer, in the documented field order (matrices are [in, out]).
    k: number of edge attributes (rows 2H .. 2H+k-1 of W1 act on them; k = 1: the squared distance)."""
    shapes = {"W1": (2 * H + k, H), "b1": (H,), "W2": (H, H), "b2": (H,), "wx": (H,),
              "W3": (2 * H, H), "b3": (H,), "W4": (H, H), "b4": (H,)}
    out, o = {}, 0
    for k in _LAYER_FIELDS:
        n = int(np.prod(shapes[k]))
        out[k] = np.asarray(flat[o:o + n]).reshape(shapes[k])
        o += n
    assert o == len(flat), "layer buffer has the wrong length"
    return out


def unpack_heads(flat, H, Hh, S):
    """List of S dicts, one per source branch."""
    shapes = {"We1": (H, Hh), "be1": (Hh,), "We2": (Hh,), "be2": (1,),
              "Wf1": (H, Hh), "bf1": (Hh,), "Wf2": (Hh,), "bf2": (1,)}
    per = sum(int(np.prod(s)) for s in shapes.values())
    assert len(flat) == per * S, "head buffer has the wrong length"
    out = []
    for s in range(S):
        d, o = {}, s * per
        for k in _HEAD_FIELDS:
            n = int(np.prod(shapes[k]))
            d[k] = np.asarray(flat[o:o + n]).reshape(shapes[k])
            o += n
        out.append(d)
    return out


def pack_fields(d, order):
    return np.concatenate([np.asarray(d[k], dtype=np.float64).ravel() for k in order])


def silu(t):
    return t / (1.0 + np.exp(-t))


def dsilu(t):
    s = 1.0 / (1.0 + np.exp(-t))
    return s * (1.0 + t * (1.0 - s))


# ---------------------------------------------------------------------------------------------
# embedding
# ---------------------------------------------------------------------------------------------
def embed_fwd(Z, emb):
    return np.asarray(emb, dtype=np.float64)[np.asarray(Z)]


def embed_bwd(Z, g_h, n_rows):
    g = np.zeros((n_rows, g_h.shape[1]), dtype=np.float64)
    np.add.at(g, np.asarray(Z), g_h)
    return g


# ---------------------------------------------------------------------------------------------
# radial basis of the edge length (the "k" edge attributes of an edge input [h_i ; h_j ; attr] of width 2H + k)
# ---------------------------------------------------------------------------------------------
def edge_rbf(d2, k, rc):
    """attr[e, j] = exp(-gamma (d_e - mu_j)^2) * fc(d_e),  d = sqrt(d2),  mu_j = j rc / (k - 1),
    gamma = ((k - 1) / rc)^2 (neighbouring Gaussians cross at exp(-1/4)),  fc(d) = (cos(pi d / rc) + 1) / 2
    (smooth cutoff: every attribute vanishes at d = rc).  k >= 2.  The paper names no basis: this is the usual
    Gaussian expansion of interatomic distances."""
    assert k >= 2
    d = np.sqrt(np.asarray(d2, dtype=np.float64))
    mu = np.arange(k, dtype=np.float64) * (rc / (k - 1))
    gamma = ((k - 1) / rc) ** 2
    fc = np.where(d < rc, 0.5 * (np.cos(np.pi * d / rc) + 1.0), 0.0)   # zero from the cutoff on (moved atoms)
    return np.exp(-gamma * (d[:, None] - mu[None, :]) ** 2) * fc[:, None]


def edge_rbf_bwd(d2, k, rc, g_attr):
    """g_d2[e] = sum_j g_attr[e, j] * d attr[e, j] / d d2_e, with d/d d2 = (1 / 2d) d/dd and
    d attr_j / dd = exp(-gamma (d - mu_j)^2) * (-2 gamma (d - mu_j) fc(d) + fc'(d)),
    fc'(d) = -(pi / 2 rc) sin(pi d / rc) inside the cutoff, 0 from the cutoff on.  d > 0 (distinct atoms)."""
    assert k >= 2
    d = np.sqrt(np.asarray(d2, dtype=np.float64))
    mu = np.arange(k, dtype=np.float64) * (rc / (k - 1))
    gamma = ((k - 1) / rc) ** 2
    inside = d < rc
    fc = np.where(inside, 0.5 * (np.cos(np.pi * d / rc) + 1.0), 0.0)
    dfc = np.where(inside, -(np.pi / (2.0 * rc)) * np.sin(np.pi * d / rc), 0.0)
    diff = d[:, None] - mu[None, :]
    dattr_dd = np.exp(-gamma * diff ** 2) * (-2.0 * gamma * diff * fc[:, None] + dfc[:, None])
    return np.sum(np.asarray(g_attr, dtype=np.float64) * dattr_dd, axis=1) / (2.0 * d)


# ---------------------------------------------------------------------------------------------
# edge geometry when the atoms move between layers (the E(n)-GNN coordinate update): the equivariant channel v is
# the displacement of every atom from its input position, x_i = x0_i + v_i, the neighbour list (with its periodic
# images) stays that of the input positions
# ---------------------------------------------------------------------------------------------
def edge_geometry(rvec0, v, dst, col):
    """rvec_e = rvec0_e + v[dst_e] - v[col_e] (rvec0: destination minus source image at the input positions),
    d2_e = |rvec_e|^2."""
    v = np.asarray(v, dtype=np.float64)
    rvec = np.asarray(rvec0, dtype=np.float64) + v[dst] - v[col]
    return rvec, np.sum(rvec * rvec, axis=1)


def edge_geometry_bwd(rvec, g_rvec, g_d2, dst, col, N):
    """Reverse of edge_geometry. Returns (g_r [E,3] = g_rvec + 2 g_d2 rvec, the gradient with respect to the edge
    vector through both of its uses; g_v [N,3] = sum over edges into i of g_r - sum over edges out of i of g_r)."""
    g_r = np.asarray(g_rvec, dtype=np.float64) + 2.0 * np.asarray(g_d2, dtype=np.float64)[:, None] * rvec
    g_v = np.zeros((N, 3), dtype=np.float64)
    np.add.at(g_v, dst, g_r)
    np.add.at(g_v, col, -g_r)
    return g_r, g_v


# ---------------------------------------------------------------------------------------------
# message-passing layer
# ---------------------------------------------------------------------------------------------
def mp_layer_fwd(h, v, dst, col, d2, rvec, Wflat, alpha, attr=None):
    """One layer. h [N,H], v [N,3]; dst/col [E] destination/source atom of each edge; d2 [E];
    rvec [E,3]; attr [E,k] (optional): edge attributes that take the place of d2 in the edge input,
    W1 then has 2H + k rows. Returns (h', v', cache-for-backward)."""
    h = np.asarray(h, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    N, H = h.shape
    d2 = np.asarray(d2, dtype=np.float64)
    eattr = d2[:, None] if attr is None else np.asarray(attr, dtype=np.float64)
    W = {k: np.asarray(a, dtype=np.float64) for k, a in unpack_layer(Wflat, H, eattr.shape[1]).items()}
    rvec = np.asarray(rvec, dtype=np.float64)
    xin = np.concatenate([h[dst], h[col], eattr], axis=1)                # [E, 2H+k]
    z1 = xin @ W["W1"] + W["b1"]
    a1 = silu(z1)
    z2 = a1 @ W["W2"] + W["b2"]
    m = silu(z2)
    x = m @ W["wx"]                                                      # [E]
    M = np.zeros((N, H), dtype=np.float64)
    np.add.at(M, dst, m)
    M *= alpha
    dv = np.zeros((N, 3), dtype=np.float64)
    np.add.at(dv, dst, x[:, None] * rvec)
    v_out = v + alpha * dv
    nin = np.concatenate([h, M], axis=1)                                 # [N, 2H]
    z3 = nin @ W["W3"] + W["b3"]
    u = silu(z3)
    h_out = h + u @ W["W4"] + W["b4"]
    cache = dict(h=h, dst=np.asarray(dst), col=np.asarray(col), d2=d2, rvec=rvec, W=W, alpha=alpha,
                 xin=xin, z1=z1, a1=a1, z2=z2, m=m, x=x, M=M, nin=nin, z3=z3, u=u)
    return h_out, v_out, cache


def mp_layer_bwd(cache, g_hout, g_vout, edge_grads=False):
    """Reverse mode of mp_layer_fwd. Returns (g_h, g_v, dict of weight gradients); with edge_grads also
    g_attr [E,k] (gradient with respect to the edge attributes, d2 when the layer took none) and g_rvec [E,3]
    (gradient with respect to the edge vectors through the update of v), from which position gradients follow."""
    c = cache
    W, alpha = c["W"], c["alpha"]
    dst, col, rvec = c["dst"], c["col"], c["rvec"]
    N, H = c["h"].shape
    g_hout = np.asarray(g_hout, dtype=np.float64)
    g_vout = np.asarray(g_vout, dtype=np.float64)
    gW = {}
    # h' = h + u W4 + b4
    gW["b4"] = g_hout.sum(axis=0)
    gW["W4"] = c["u"].T @ g_hout
    g_u = g_hout @ W["W4"].T
    g_z3 = g_u * dsilu(c["z3"])
    gW["b3"] = g_z3.sum(axis=0)
    gW["W3"] = c["nin"].T @ g_z3
    g_nin = g_z3 @ W["W3"].T
    g_h = g_hout + g_nin[:, :H]
    g_M = g_nin[:, H:]
    # v' = v + alpha sum x_e rvec_e ;  M = alpha sum m_e
    g_v = g_vout.copy()
    g_x = alpha * np.einsum("ec,ec->e", g_vout[dst], rvec)               # [E]
    g_m = alpha * g_M[dst] + g_x[:, None] * W["wx"][None, :]
    gW["wx"] = c["m"].T @ g_x
    g_z2 = g_m * dsilu(c["z2"])
    gW["b2"] = g_z2.sum(axis=0)
    gW["W2"] = c["a1"].T @ g_z2
    g_a1 = g_z2 @ W["W2"].T
    g_z1 = g_a1 * dsilu(c["z1"])
    gW["b1"] = g_z1.sum(axis=0)
    gW["W1"] = c["xin"].T @ g_z1
    g_xin = g_z1 @ W["W1"].T                                             # [E, 2H+1]
    np.add.at(g_h, dst, g_xin[:, :H])
    np.add.at(g_h, col, g_xin[:, H:2 * H])
    if edge_grads:
        g_rvec = alpha * c["x"][:, None] * g_vout[dst]
        return g_h, g_v, gW, g_xin[:, 2 * H:], g_rvec
    return g_h, g_v, gW


# ---------------------------------------------------------------------------------------------
# pooling (atoms of a graph are contiguous)
# ---------------------------------------------------------------------------------------------
def pool_fwd(h, graph_off, mean=True):
    h = np.asarray(h, dtype=np.float64)
    G = len(graph_off) - 1
    p = np.zeros((G, h.shape[1]), dtype=np.float64)
    for g in range(G):
        lo, hi = int(graph_off[g]), int(graph_off[g + 1])
        if hi > lo:
            p[g] = h[lo:hi].sum(axis=0) / ((hi - lo) if mean else 1.0)
    return p


def pool_bwd(g_p, graph_off, N, mean=True):
    g_p = np.asarray(g_p, dtype=np.float64)
    g_h = np.zeros((N, g_p.shape[1]), dtype=np.float64)
    for g in range(len(graph_off) - 1):
        lo, hi = int(graph_off[g]), int(graph_off[g + 1])
        if hi > lo:
            g_h[lo:hi] = g_p[g] / ((hi - lo) if mean else 1.0)
    return g_h


# ---------------------------------------------------------------------------------------------
# routing + heads
# ---------------------------------------------------------------------------------------------
def routing_plan(source_id, graph_off, S):
    """Stable grouping of graphs (and of their atoms) by source: the rows each branch decodes.

    Returns grp_graph_ptr[S+1], graph_perm[G], grp_atom_ptr[S+1], atom_perm[N], all int32."""
    source_id = np.asarray(source_id, dtype=np.int64)
    graph_off = np.asarray(graph_off, dtype=np.int64)
    if source_id.size and (source_id.min() < 0 or source_id.max() >= S):
        raise ValueError("source id out of range")
    graph_perm = np.argsort(source_id, kind="stable").astype(np.int32)
    gcnt = np.bincount(source_id, minlength=S)
    grp_graph_ptr = np.zeros(S + 1, dtype=np.int32)
    grp_graph_ptr[1:] = np.cumsum(gcnt)
    atom_lists = [np.arange(graph_off[g], graph_off[g + 1]) for g in graph_perm]
    atom_perm = (np.concatenate(atom_lists) if atom_lists else np.zeros(0)).astype(np.int32)
    acnt = np.zeros(S, dtype=np.int64)
    np.add.at(acnt, source_id, graph_off[1:] - graph_off[:-1])
    grp_atom_ptr = np.zeros(S + 1, dtype=np.int32)
    grp_atom_ptr[1:] = np.cumsum(acnt)
    return grp_graph_ptr, graph_perm, grp_atom_ptr, atom_perm


def heads_fwd(p, h, v, graph_off, source_id, Whead_flat, Hh, S):
    """Every graph is decoded by the branch of its own source and by no other."""
    p = np.asarray(p, dtype=np.float64)
    h = np.asarray(h, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    G, H = p.shape
    N = h.shape[0]
    heads = [{k: np.asarray(a, dtype=np.float64) for k, a in d.items()}
             for d in unpack_heads(Whead_flat, H, Hh, S)]
    energy = np.zeros(G, dtype=np.float64)
    q = np.zeros(N, dtype=np.float64)
    ze = np.zeros((G, Hh), dtype=np.float64)
    zf = np.zeros((N, Hh), dtype=np.float64)
    for g in range(G):
        w = heads[int(source_id[g])]
        lo, hi = int(graph_off[g]), int(graph_off[g + 1])
        ze[g] = p[g] @ w["We1"] + w["be1"]
        energy[g] = silu(ze[g]) @ w["We2"] + w["be2"][0]
        zf[lo:hi] = h[lo:hi] @ w["Wf1"] + w["bf1"]
        q[lo:hi] = silu(zf[lo:hi]) @ w["Wf2"] + w["bf2"][0]
    force = q[:, None] * v
    cache = dict(p=p, h=h, v=v, graph_off=np.asarray(graph_off), source_id=np.asarray(source_id),
                 heads=heads, ze=ze, zf=zf, q=q, Hh=Hh, S=S)
    return energy, force, cache


def heads_bwd(cache, g_energy, g_force):
    """Returns (g_p [G,H], g_h [N,H], g_v [N,3], list of S dicts of head-weight gradients)."""
    c = cache
    p, h, v = c["p"], c["h"], c["v"]
    G, H = p.shape
    N = h.shape[0]
    g_energy = np.asarray(g_energy, dtype=np.float64)
    g_force = np.asarray(g_force, dtype=np.float64)
    gheads = [{k: np.zeros_like(a) for k, a in w.items()} for w in c["heads"]]
    g_p = np.zeros_like(p)
    g_h = np.zeros_like(h)
    g_q = np.einsum("nc,nc->n", g_force, v)
    g_v = c["q"][:, None] * g_force
    for g in range(G):
        s = int(c["source_id"][g])
        w, gw = c["heads"][s], gheads[s]
        lo, hi = int(c["graph_off"][g]), int(c["graph_off"][g + 1])
        # energy head
        ae = silu(c["ze"][g])
        gw["be2"][0] += g_energy[g]
        gw["We2"] += g_energy[g] * ae
        g_ze = g_energy[g] * w["We2"] * dsilu(c["ze"][g])
        gw["be1"] += g_ze
        gw["We1"] += np.outer(p[g], g_ze)
        g_p[g] = w["We1"] @ g_ze
        # force head
        af = silu(c["zf"][lo:hi])
        gq = g_q[lo:hi]
        gw["bf2"][0] += gq.sum()
        gw["Wf2"] += af.T @ gq
        g_zf = gq[:, None] * w["Wf2"][None, :] * dsilu(c["zf"][lo:hi])
        gw["bf1"] += g_zf.sum(axis=0)
        gw["Wf1"] += h[lo:hi].T @ g_zf
        g_h[lo:hi] = g_zf @ w["Wf1"].T
    return g_p, g_h, g_v, gheads


# ---------------------------------------------------------------------------------------------
# heads with D fully connected hidden layers (in the paper's model every dataset-specific head has
# three of them, 889 units wide: section "Numerical Results")
# ---------------------------------------------------------------------------------------------
def deep_head_shapes(H, Hh, D):
    """Ordered (name, shape) list of one head: W1[H,Hh] b1[Hh], then Wl[Hh,Hh] bl[Hh] for l = 2..D,
    then the output layer wo[Hh] bo[1]. D = 1 is the layout of unpack_heads."""
    out = [("W1", (H, Hh)), ("b1", (Hh,))]
    for l in range(2, D + 1):
        out += [(f"W{l}", (Hh, Hh)), (f"b{l}", (Hh,))]
    out += [("wo", (Hh,)), ("bo", (1,))]
    return out


def unpack_deep_heads(flat, H, Hh, D, S):
    """List of S branches; a branch is {"e": head, "f": head}, a head maps field name -> array.
    Storage: branch after branch, in a branch the energy head then the force head."""
    shapes = deep_head_shapes(H, Hh, D)
    per_head = sum(int(np.prod(s)) for _, s in shapes)
    assert len(flat) == 2 * per_head * S, "head buffer has the wrong length"
    out, o = [], 0
    for _ in range(S):
        br = {}
        for which in ("e", "f"):
            d = {}
            for k, shp in shapes:
                n = int(np.prod(shp))
                d[k] = np.asarray(flat[o:o + n], dtype=np.float64).reshape(shp)
                o += n
            br[which] = d
        out.append(br)
    return out


def _mlp_fwd(x, w, D):
    """x [rows, in] through D hidden layers (silu after each) and the scalar output layer."""
    zs, acts = [], [x]
    for l in range(1, D + 1):
        z = acts[-1] @ w[f"W{l}"] + w[f"b{l}"]
        zs.append(z)
        acts.append(silu(z))
    return acts[-1] @ w["wo"] + w["bo"][0], zs, acts


def _mlp_bwd(g_out, w, gw, zs, acts, D):
    """Reverse of _mlp_fwd for upstream g_out [rows]; adds into gw, returns the gradient of x."""
    gw["bo"][0] += g_out.sum()
    gw["wo"] += acts[D].T @ g_out
    g_a = g_out[:, None] * w["wo"][None, :]
    for l in range(D, 0, -1):
        g_z = g_a * dsilu(zs[l - 1])
        gw[f"b{l}"] += g_z.sum(axis=0)
        gw[f"W{l}"] += acts[l - 1].T @ g_z
        g_a = g_z @ w[f"W{l}"].T
    return g_a


def heads_deep_fwd(p, h, v, graph_off, source_id, Whead_flat, Hh, D, S):
    """Like heads_fwd with D hidden layers per head: e_g = MLP_e,s(p_g), q_i = MLP_f,s(h_i), F_i = q_i v_i."""
    p = np.asarray(p, dtype=np.float64)
    h = np.asarray(h, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    G, H = p.shape
    N = h.shape[0]
    heads = unpack_deep_heads(Whead_flat, H, Hh, D, S)
    energy = np.zeros(G, dtype=np.float64)
    q = np.zeros(N, dtype=np.float64)
    per_graph = []
    for g in range(G):
        w = heads[int(source_id[g])]
        lo, hi = int(graph_off[g]), int(graph_off[g + 1])
        e, ze, ae = _mlp_fwd(p[g:g + 1], w["e"], D)
        energy[g] = e[0]
        qq, zf, af = _mlp_fwd(h[lo:hi], w["f"], D)
        q[lo:hi] = qq
        per_graph.append((ze, ae, zf, af))
    force = q[:, None] * v
    cache = dict(p=p, h=h, v=v, graph_off=np.asarray(graph_off), source_id=np.asarray(source_id), heads=heads,
                 per_graph=per_graph, q=q, Hh=Hh, D=D, S=S)
    return energy, force, cache


def heads_deep_bwd(cache, g_energy, g_force):
    """Returns (g_p [G,H], g_h [N,H], g_v [N,3], flat head-weight gradient in the layout of the weights)."""
    c = cache
    p, h, v, D = c["p"], c["h"], c["v"], c["D"]
    g_energy = np.asarray(g_energy, dtype=np.float64)
    g_force = np.asarray(g_force, dtype=np.float64)
    gheads = [{wh: {k: np.zeros_like(a) for k, a in br[wh].items()} for wh in ("e", "f")} for br in c["heads"]]
    g_p = np.zeros_like(p)
    g_h = np.zeros_like(h)
    g_q = np.einsum("nc,nc->n", g_force, v)
    g_v = c["q"][:, None] * g_force
    for g in range(p.shape[0]):
        s = int(c["source_id"][g])
        lo, hi = int(c["graph_off"][g]), int(c["graph_off"][g + 1])
        ze, ae, zf, af = c["per_graph"][g]
        g_p[g] = _mlp_bwd(g_energy[g:g + 1], c["heads"][s]["e"], gheads[s]["e"], ze, ae, D)[0]
        g_h[lo:hi] = _mlp_bwd(g_q[lo:hi], c["heads"][s]["f"], gheads[s]["f"], zf, af, D)
    H, Hh = p.shape[1], c["Hh"]
    order = [k for k, _ in deep_head_shapes(H, Hh, D)]
    flat = np.concatenate([gheads[s][wh][k].ravel() for s in range(c["S"]) for wh in ("e", "f") for k in order])
    return g_p, g_h, g_v, flat


# ---------------------------------------------------------------------------------------------
# whole step
# ---------------------------------------------------------------------------------------------
def step_fwd_bwd(Z, graph_off, source_id, graph, emb, layer_weights, head_weights, Hh, S, alpha,
                 g_energy=None, g_force=None, keep_layers=False, D=None, attr=None, move=False, rbf=None,
                 pos_grad=False):
    """Embedding -> L layers -> mean pool -> heads, then (if upstream gradients are given) the
    whole reverse pass. `graph` is the dict returned by oracle.radius_graph. D: hidden layers per
    head (None: the one-hidden-layer heads of heads_fwd). attr [E,k]: edge attributes in place of d2.
    rbf = (k, rc): the attributes are the radial basis of the current edge length (recomputed per layer when the
    atoms move). move: the atoms move between layers, x = x0 + v, edge vectors and lengths are recomputed before
    every layer. pos_grad (implied by move): the reverse pass also returns g_pos [N,3], the gradient with respect to
    the input positions through every edge vector and edge length."""
    H = emb.shape[1]
    N = len(Z)
    dst, col, d2_0, rvec0 = graph["dst"], graph["col"], graph["d2"], graph["rvec"]
    pos_grad = pos_grad or move
    h = embed_fwd(Z, emb)
    v = np.zeros((N, 3), dtype=np.float64)
    caches, hs, geoms = [], [h], []
    for Wl in layer_weights:
        if move:
            rvec, d2 = edge_geometry(rvec0, v, dst, col)
        else:
            rvec, d2 = np.asarray(rvec0, dtype=np.float64), np.asarray(d2_0, dtype=np.float64)
        a = edge_rbf(d2, rbf[0], rbf[1]) if rbf is not None else attr
        h, v, c = mp_layer_fwd(h, v, dst, col, d2, rvec, Wl, alpha, attr=a)
        caches.append(c)
        geoms.append((rvec, d2))
        if keep_layers:
            hs.append(h)
    p = pool_fwd(h, graph_off)
    if D is None:
        energy, force, hc = heads_fwd(p, h, v, graph_off, source_id, head_weights, Hh, S)
    else:
        energy, force, hc = heads_deep_fwd(p, h, v, graph_off, source_id, head_weights, Hh, D, S)
    out = dict(h=h, v=v, p=p, energy=energy, force=force, hs=hs)
    if g_energy is None:
        return out
    if D is None:
        g_p, g_h, g_v, gheads = heads_bwd(hc, g_energy, g_force)
        g_heads = np.concatenate([pack_fields(d, _HEAD_FIELDS) for d in gheads])
    else:
        g_p, g_h, g_v, g_heads = heads_deep_bwd(hc, g_energy, g_force)
    g_h = g_h + pool_bwd(g_p, graph_off, N)
    g_layers = []
    g_r0 = np.zeros((len(dst), 3), dtype=np.float64)
    for c, (rvec, d2) in zip(reversed(caches), reversed(geoms)):
        if not pos_grad:
            g_h, g_v, gW = mp_layer_bwd(c, g_h, g_v)
        else:
            g_h, g_v, gW, g_attr, g_rvec = mp_layer_bwd(c, g_h, g_v, edge_grads=True)
            if rbf is not None:
                g_d2 = edge_rbf_bwd(d2, rbf[0], rbf[1], g_attr)
            else:
                assert attr is None, "position gradients need attributes that are a function of the edge length"
                g_d2 = g_attr[:, 0]
            g_r, g_v_geom = edge_geometry_bwd(rvec, g_rvec, g_d2, dst, col, N)
            g_r0 += g_r
            if move:
                g_v = g_v + g_v_geom
        g_layers.append(pack_fields(gW, _LAYER_FIELDS))
    g_layers.reverse()
    out.update(
        g_emb=embed_bwd(Z, g_h, emb.shape[0]), g_layers=g_layers,
        g_heads=g_heads,
        g_h0=g_h, g_v0=g_v,
    )
    if pos_grad:
        # rvec0_e = x0[dst] - x0[col] - image shift: every layer's edge-vector gradient lands on the input positions
        g_pos = np.zeros((N, 3), dtype=np.float64)
        np.add.at(g_pos, dst, g_r0)
        np.add.at(g_pos, col, -g_r0)
        out["g_pos"] = g_pos
    return out


def conservative_forces(Z, graph_off, source_id, graph, emb, layer_weights, head_weights, Hh, S, alpha, **kw):
    """F_i = -d E_total / d x_i with E_total = sum over graphs of (atoms in the graph) x (energy per atom): the
    reverse pass seeded with the atom counts on the energies and nothing on the force head."""
    n_at = np.diff(np.asarray(graph_off)).astype(np.float64)
    out = step_fwd_bwd(Z, graph_off, source_id, graph, emb, layer_weights, head_weights, Hh, S, alpha,
                       g_energy=n_at, g_force=np.zeros((len(Z), 3)), pos_grad=True, **kw)
    return out["energy"], -out["g_pos"]
