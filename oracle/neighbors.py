"""Brute-force radius graph (test infrastructure; see the package docstring).

Definition. Graph g owns atoms graph_off[g]:graph_off[g+1]. A directed edge (i <- j, s) exists when
i and j are in the same graph, (j, s) != (i, 0), and

    t    = (s1*a + s2*b) + s3*c           lattice translation, a, b, c = rows of cell[g]
    rvec = pos_i - (pos_j + t)
    d2   = (rx*rx + ry*ry) + rz*rz  <  rc*rc

with every operation above carried out in float32 and rounded on its own (no fused multiply-add), so
that a second implementation can reproduce the list bit for bit. Non-periodic graphs only have
s = (0,0,0). For a periodic graph s runs over [-n1,n1] x [-n2,n2] x [-n3,n3] with
n_k = ceil(rc / h_k), h_k the distance between the two cell faces spanned by the other two lattice
vectors; that range is complete for atoms that lie inside the cell. Self-images (j = i, s != 0) are
edges. There is no cap on the number of neighbours.

Order of the list: by destination i, then source j, then s1, s2, s3, all ascending. This is the
"radius graph of an atomistic structure" that the paper's message-passing stack runs on; the paper
gives no construction, so the definition above is this build's reading.
"""
from __future__ import annotations

import numpy as np


def image_range(cell, rc, extra=0):
    """n_k = ceil(rc / h_k) for k = 1..3 (float64), plus `extra` (used by the completeness self-check)."""
    c = np.asarray(cell, dtype=np.float64)
    vol = abs(np.linalg.det(c))
    n = []
    for k in range(3):
        u, w = c[(k + 1) % 3], c[(k + 2) % 3]
        area = np.linalg.norm(np.cross(u, w))
        h = vol / area
        n.append(int(np.ceil(rc / h)) + int(extra))
    return tuple(n)


def _shift_table(cell32, nk):
    """All shifts in lexicographic (s1,s2,s3) order and their float32 translations t."""
    r1 = np.arange(-nk[0], nk[0] + 1)
    r2 = np.arange(-nk[1], nk[1] + 1)
    r3 = np.arange(-nk[2], nk[2] + 1)
    S = np.stack(np.meshgrid(r1, r2, r3, indexing="ij"), axis=-1).reshape(-1, 3)
    a, b, c = cell32[0], cell32[1], cell32[2]
    s1 = S[:, 0:1].astype(np.float32)
    s2 = S[:, 1:2].astype(np.float32)
    s3 = S[:, 2:3].astype(np.float32)
    t = (s1 * a[None, :] + s2 * b[None, :]) + s3 * c[None, :]        # float32, each op rounded
    assert t.dtype == np.float32
    return S.astype(np.int64), t


def radius_graph_rows(pos, graph_off, cell, pbc, rc, rows, extra_images=0):
    """Edges whose destination is one of `rows` (global atom indices), in list order.

    Returns a list with one tuple per requested row: (col int32[k], shift int8[k,3], d2 float32[k],
    rvec float32[k,3]).
    """
    pos = np.ascontiguousarray(pos, dtype=np.float32)
    graph_off = np.asarray(graph_off, dtype=np.int64)
    rc32 = np.float32(rc)
    rc2 = np.float32(rc32 * rc32)
    rows = np.asarray(rows, dtype=np.int64)
    gid = np.searchsorted(graph_off, rows, side="right") - 1
    out = [None] * len(rows)
    cache = {}
    for k, (i, g) in enumerate(zip(rows, gid)):
        g = int(g)
        if g not in cache:
            cache.clear()
            lo, hi = int(graph_off[g]), int(graph_off[g + 1])
            periodic = pbc is not None and cell is not None and bool(pbc[g])
            if periodic:
                c32 = np.asarray(cell[g], dtype=np.float32)
                nk = image_range(c32, float(rc), extra_images)
            else:
                c32 = np.zeros((3, 3), dtype=np.float32)
                nk = (0, 0, 0)
            S, t = _shift_table(c32, nk)
            q = pos[lo:hi, None, :] + t[None, :, :]                     # [n, ns, 3] float32
            zero_shift = int(np.nonzero(np.all(S == 0, axis=1))[0][0])
            cache[g] = (lo, hi, S, q, zero_shift)
        lo, hi, S, q, zero_shift = cache[g]
        r = pos[i][None, None, :] - q                                   # float32
        d2 = (r[..., 0] * r[..., 0] + r[..., 1] * r[..., 1]) + r[..., 2] * r[..., 2]
        keep = d2 < rc2
        keep[i - lo, zero_shift] = False
        jj, ss = np.nonzero(keep)                                       # j ascending, then shift index
        out[k] = ((jj + lo).astype(np.int32), S[ss].astype(np.int8), d2[jj, ss].astype(np.float32),
                  r[jj, ss].astype(np.float32))
    return out


def transpose_plan(col, N):
    """Edges regrouped by source atom: colT_ptr[N+1] and permT[E] (edge ids, ascending per source)."""
    col = np.asarray(col, dtype=np.int64)
    permT = np.argsort(col, kind="stable").astype(np.int32)
    cnt = np.bincount(col, minlength=N)
    colT_ptr = np.zeros(N + 1, dtype=np.int32)
    colT_ptr[1:] = np.cumsum(cnt)
    return colT_ptr, permT


def radius_graph(pos, graph_off, cell, pbc, rc, extra_images=0):
    """Whole-batch edge list as destination-sorted CSR plus the source-sorted transpose plan."""
    pos = np.ascontiguousarray(pos, dtype=np.float32)
    N = pos.shape[0]
    graph_off = np.asarray(graph_off, dtype=np.int64)
    G = len(graph_off) - 1
    per_row = radius_graph_rows(pos, graph_off, cell, pbc, rc, np.arange(N), extra_images)
    deg = np.array([len(r[0]) for r in per_row], dtype=np.int64)
    row_ptr = np.zeros(N + 1, dtype=np.int64)
    row_ptr[1:] = np.cumsum(deg)
    E = int(row_ptr[-1])
    if E >= 2 ** 31:
        raise OverflowError("edge count does not fit int32")
    if N:
        col = np.concatenate([r[0] for r in per_row]).astype(np.int32)
        shift = np.concatenate([r[1] for r in per_row]).astype(np.int8).reshape(-1, 3)
        d2 = np.concatenate([r[2] for r in per_row]).astype(np.float32)
        rvec = np.concatenate([r[3] for r in per_row]).astype(np.float32).reshape(-1, 3)
    else:
        col = np.zeros(0, np.int32)
        shift = np.zeros((0, 3), np.int8)
        d2 = np.zeros(0, np.float32)
        rvec = np.zeros((0, 3), np.float32)
    dst = np.repeat(np.arange(N, dtype=np.int32), deg)
    colT_ptr, permT = transpose_plan(col, N)
    return dict(
        row_ptr=row_ptr.astype(np.int32), col=col, shift=shift, d2=d2, rvec=rvec, dst=dst,
        edge_graph_ptr=row_ptr[graph_off[: G + 1]].astype(np.int32), colT_ptr=colT_ptr, permT=permT,
        E=E,
    )
