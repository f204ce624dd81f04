"""Flat weight buffers (random init) and upstream gradients.

Layout of one message-passing layer (float32, matrices row-major [in, out]):
    W1[(2H+1), H]  rows 0..H-1 act on h_i (destination), H..2H-1 on h_j (source), row 2H on d^2
                   (with k edge attributes in place of d^2: W1[(2H+k), H], rows 2H..2H+k-1 on the attributes)
    b1[H]  W2[H,H]  b2[H]  wx[H]  W3[2H,H] (rows 0..H-1 on h_i, H..2H-1 on M_i)  b3[H]  W4[H,H]  b4[H]
Layout of one source's decoding branch:
    We1[H,Hh] be1[Hh] We2[Hh] be2[1]   (energy head)   Wf1[H,Hh] bf1[Hh] Wf2[Hh] bf2[1]   (force head)
All S branches are stored back to back.
Deep branch (D hidden layers per head; the paper's heads have three layers, 889 units wide): the energy head
then the force head, each  W1[H,Hh] b1[Hh]  Wl[Hh,Hh] bl[Hh] (l = 2..D)  wo[Hh] bo[1];  D = 1 is the layout above.
"""
from __future__ import annotations

import numpy as np

ZMAX = 94  # embedding table has ZMAX+1 rows, indexed by atomic number

LAYER_FIELDS = ("W1", "b1", "W2", "b2", "wx", "W3", "b3", "W4", "b4")
HEAD_FIELDS = ("We1", "be1", "We2", "be2", "Wf1", "bf1", "Wf2", "bf2")


def _layer_shapes(H, k=1):
    return {"W1": (2 * H + k, H), "b1": (H,), "W2": (H, H), "b2": (H,), "wx": (H,),
            "W3": (2 * H, H), "b3": (H,), "W4": (H, H), "b4": (H,)}


def _head_shapes(H, Hh):
    return {"We1": (H, Hh), "be1": (Hh,), "We2": (Hh,), "be2": (1,),
            "Wf1": (H, Hh), "bf1": (Hh,), "Wf2": (Hh,), "bf2": (1,)}


def _slices(shapes, order):
    out, o = {}, 0
    for k in order:
        n = int(np.prod(shapes[k]))
        out[k] = (o, o + n, shapes[k])
        o += n
    return out, o


def layer_field_slices(H, k=1):
    return _slices(_layer_shapes(H, k), LAYER_FIELDS)[0]


def head_field_slices(H, Hh):
    return _slices(_head_shapes(H, Hh), HEAD_FIELDS)[0]


def layer_weight_count(H, k=1):
    return _slices(_layer_shapes(H, k), LAYER_FIELDS)[1]


def head_weight_count(H, Hh):
    return _slices(_head_shapes(H, Hh), HEAD_FIELDS)[1]


def _fill(rng, shapes, order, fan_in, bias_scale):
    parts = []
    for k in order:
        shp = shapes[k]
        if k in fan_in:
            b = 1.0 / np.sqrt(fan_in[k])
            parts.append(rng.uniform(-b, b, size=shp).ravel())
        else:
            parts.append(rng.uniform(-bias_scale, bias_scale, size=shp).ravel())
    return np.concatenate(parts).astype(np.float32)


def init_layer_weights(rng, H, bias_scale=0.1, k=1):
    """U(-1/sqrt(fan_in), 1/sqrt(fan_in)) matrices; small non-zero biases so a dropped bias shows.
    k: edge attributes (W1 has 2H + k rows)."""
    fan = {"W1": 2 * H + k, "W2": H, "wx": H, "W3": 2 * H, "W4": H}
    return _fill(rng, _layer_shapes(H, k), LAYER_FIELDS, fan, bias_scale)


def init_head_weights(rng, H, Hh, S, bias_scale=0.1):
    fan = {"We1": H, "We2": Hh, "Wf1": H, "Wf2": Hh}
    return np.concatenate([_fill(rng, _head_shapes(H, Hh), HEAD_FIELDS, fan, bias_scale)
                           for _ in range(S)])


def deep_head_field_slices(H, Hh, D):
    """name -> (lo, hi, shape) inside one branch; names are "e.W1", "e.b1", ..., "e.wo", "e.bo", "f.W1", ..."""
    shapes, order = {}, []
    for which in ("e", "f"):
        shapes[f"{which}.W1"], shapes[f"{which}.b1"] = (H, Hh), (Hh,)
        order += [f"{which}.W1", f"{which}.b1"]
        for l in range(2, D + 1):
            shapes[f"{which}.W{l}"], shapes[f"{which}.b{l}"] = (Hh, Hh), (Hh,)
            order += [f"{which}.W{l}", f"{which}.b{l}"]
        shapes[f"{which}.wo"], shapes[f"{which}.bo"] = (Hh,), (1,)
        order += [f"{which}.wo", f"{which}.bo"]
    return _slices(shapes, order)[0]


def deep_head_weight_count(H, Hh, D):
    return 2 * (H * Hh + Hh + (D - 1) * (Hh * Hh + Hh) + Hh + 1)


def init_deep_head_weights(rng, H, Hh, D, S, bias_scale=0.1):
    sl = deep_head_field_slices(H, Hh, D)
    out = np.empty(S * deep_head_weight_count(H, Hh, D), dtype=np.float32)
    per = deep_head_weight_count(H, Hh, D)
    for s in range(S):
        for name, (lo, hi, shp) in sl.items():
            field = name.split(".")[1]
            if field[0] in "Ww":
                b = 1.0 / np.sqrt(shp[0])
                out[s * per + lo:s * per + hi] = rng.uniform(-b, b, size=hi - lo)
            else:
                out[s * per + lo:s * per + hi] = rng.uniform(-bias_scale, bias_scale, size=hi - lo)
    return out


def init_embedding(rng, H):
    return rng.standard_normal((ZMAX + 1, H)).astype(np.float32)


def upstream_grads(rng, G, N):
    """Seeded stand-in for dLoss/d(energy) [G] and dLoss/d(force) [N,3] (the loss is outside the path)."""
    return (rng.standard_normal(G).astype(np.float32),
            rng.standard_normal((N, 3)).astype(np.float32))
