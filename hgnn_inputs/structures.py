"""Random atomistic structures: non-periodic molecules, triclinic crystals, large cubic bulk cells.

Everything here is rejection sampling of positions plus bookkeeping; nothing of the model.
Positions are float32 (the type the library's boundary takes); cells hold the lattice vectors a, b, c
as rows. Atoms of one graph are contiguous in the batch.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


@dataclass
class Batch:
    pos: np.ndarray          # [N,3] float32, Angstrom
    Z: np.ndarray            # [N]   int32 atomic numbers
    graph_off: np.ndarray    # [G+1] int32, graph g owns atoms graph_off[g]:graph_off[g+1]
    cell: np.ndarray         # [G,3,3] float32, rows = lattice vectors (zeros when not periodic)
    pbc: np.ndarray          # [G] uint8, 1 = periodic in all three lattice directions
    source_id: np.ndarray    # [G] int32 dataset/source of each graph
    meta: dict = field(default_factory=dict)

    @property
    def N(self) -> int:
        return int(self.pos.shape[0])

    @property
    def G(self) -> int:
        return int(self.graph_off.shape[0] - 1)


def _reject_sample_box(rng, n, side, dmin):
    """n points uniform in [0, side)^3, each redrawn while closer than dmin to an earlier one."""
    pts = np.empty((n, 3), dtype=np.float64)
    k = 0
    d2min = dmin * dmin
    while k < n:
        p = rng.uniform(0.0, side, size=3)
        if k and np.min(np.sum((pts[:k] - p) ** 2, axis=1)) < d2min:
            continue
        pts[k] = p
        k += 1
    return pts


def make_molecule(rng, n, side, dmin, z_choices, z_probs=None):
    """One non-periodic graph: (pos float32 [n,3], Z int32 [n])."""
    pts = _reject_sample_box(rng, n, side, dmin)
    z = rng.choice(np.asarray(z_choices, dtype=np.int32), size=n, p=z_probs).astype(np.int32)
    return pts.astype(np.float32), z


def cell_from_lengths_angles(a, b, c, alpha, beta, gamma):
    """Standard orientation: a along x, b in the xy-plane. Angles in radians. Rows are a, b, c."""
    ca, cb, cg = np.cos(alpha), np.cos(beta), np.cos(gamma)
    sg = np.sin(gamma)
    cx = cb
    cy = (ca - cb * cg) / sg
    cz2 = 1.0 - cx * cx - cy * cy
    if cz2 <= 0.0:
        return None
    return np.array(
        [[a, 0.0, 0.0], [b * cg, b * sg, 0.0], [c * cx, c * cy, c * np.sqrt(cz2)]], dtype=np.float64
    )


def draw_cell(rng, n, len_lo, len_hi, ang_lo_deg, ang_hi_deg, max_density, min_vol_factor=0.5):
    """Redraw lengths/angles until the cell is well conditioned and can hold n atoms."""
    while True:
        la, lb, lc = rng.uniform(len_lo, len_hi, size=3)
        al, be, ga = np.deg2rad(rng.uniform(ang_lo_deg, ang_hi_deg, size=3))
        ca, cb, cg = np.cos(al), np.cos(be), np.cos(ga)
        g2 = 1.0 + 2.0 * ca * cb * cg - ca * ca - cb * cb - cg * cg
        if g2 <= 0.0 or np.sqrt(g2) < min_vol_factor:
            continue
        cell = cell_from_lengths_angles(la, lb, lc, al, be, ga)
        if cell is None:
            continue
        vol = abs(np.linalg.det(cell))
        if n / vol > max_density:
            continue
        return cell


def make_crystal(rng, n, len_lo, len_hi, dmin, z_lo, z_hi, max_density=0.12,
                 ang_lo_deg=60.0, ang_hi_deg=120.0):
    """One periodic triclinic graph: (pos float32 [n,3], Z, cell float32 [3,3]).

    Fractional coordinates uniform in [0,1)^3, redrawn while any periodic image of an earlier atom
    (images -2..2 per direction) is closer than dmin.
    """
    r = np.arange(-2, 3)
    sh = np.stack(np.meshgrid(r, r, r, indexing="ij"), axis=-1).reshape(-1, 3).astype(np.float64)
    d2min = dmin * dmin
    while True:
        cell = draw_cell(rng, n, len_lo, len_hi, ang_lo_deg, ang_hi_deg, max_density)
        img = sh @ cell                               # [125,3]
        # an atom's own periodic images must not be closer than dmin either (tiny skewed cells)
        own = np.sum(img[np.any(sh != 0, axis=1)] ** 2, axis=1)
        if own.min() >= d2min:
            break
    pts = np.empty((n, 3), dtype=np.float64)
    k = 0
    while k < n:
        f = rng.uniform(0.0, 1.0, size=3)
        p = f @ cell
        if k:
            d = (pts[:k, None, :] + img[None, :, :]) - p
            if np.min(np.sum(d * d, axis=2)) < d2min:
                continue
        pts[k] = p
        k += 1
    pos32 = pts.astype(np.float32)
    cell32 = cell.astype(np.float32)
    z = rng.integers(z_lo, z_hi + 1, size=n).astype(np.int32)
    return pos32, z, cell32


def make_cubic_bulk(rng, n, density, dmin, z_lo, z_hi):
    """One large periodic cubic graph at the given number density, grid-accelerated rejection."""
    side = (n / density) ** (1.0 / 3.0)
    nb = max(1, int(np.floor(side / dmin)))
    w = side / nb
    buckets: dict = {}
    pts = np.empty((n, 3), dtype=np.float64)
    d2min = dmin * dmin
    k = 0
    while k < n:
        p = rng.uniform(0.0, side, size=3)
        b = np.minimum((p / w).astype(np.int64), nb - 1)
        ok = True
        for dx in (-1, 0, 1):
            for dy in (-1, 0, 1):
                for dz in (-1, 0, 1):
                    key = ((b[0] + dx) % nb, (b[1] + dy) % nb, (b[2] + dz) % nb)
                    lst = buckets.get(key)
                    if not lst:
                        continue
                    q = pts[lst]
                    d = q - p
                    d -= side * np.round(d / side)        # minimum image (side >> dmin)
                    if np.min(np.sum(d * d, axis=1)) < d2min:
                        ok = False
                        break
                if not ok:
                    break
            if not ok:
                break
        if not ok:
            continue
        pts[k] = p
        buckets.setdefault((int(b[0]), int(b[1]), int(b[2])), []).append(k)
        k += 1
    cell = np.eye(3, dtype=np.float64) * side
    pos32 = pts.astype(np.float32)
    # keep strictly inside the float32 cell
    side32 = np.float32(side)
    pos32 = np.minimum(pos32, np.nextafter(side32, np.float32(0.0)))
    z = rng.integers(z_lo, z_hi + 1, size=n).astype(np.int32)
    return pos32, z, cell.astype(np.float32)


def concat_graphs(graphs, source_ids=None, meta=None) -> Batch:
    """graphs: list of (pos, Z) or (pos, Z, cell). Periodic iff a cell is given."""
    pos = np.concatenate([g[0] for g in graphs], axis=0).astype(np.float32)
    z = np.concatenate([g[1] for g in graphs], axis=0).astype(np.int32)
    sizes = np.array([g[0].shape[0] for g in graphs], dtype=np.int64)
    off = np.zeros(len(graphs) + 1, dtype=np.int32)
    off[1:] = np.cumsum(sizes)
    cell = np.zeros((len(graphs), 3, 3), dtype=np.float32)
    pbc = np.zeros(len(graphs), dtype=np.uint8)
    for k, g in enumerate(graphs):
        if len(g) > 2 and g[2] is not None:
            cell[k] = g[2]
            pbc[k] = 1
    if source_ids is None:
        source_ids = np.zeros(len(graphs), dtype=np.int32)
    return Batch(pos=np.ascontiguousarray(pos), Z=z, graph_off=off, cell=cell, pbc=pbc,
                 source_id=np.asarray(source_ids, dtype=np.int32), meta=dict(meta or {}))
