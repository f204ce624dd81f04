"""Pins of the brute-force radius graph against things other than itself (CPU only)."""
import os

import numpy as np
import pytest
from scipy.spatial import cKDTree

import oracle
from hgnn_inputs import concat_graphs, make_config, small_mixed_batch

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def edge_set(g):
    return set(zip(g["dst"].tolist(), g["col"].tolist(), map(tuple, g["shift"].tolist())))


def kdtree_edges(batch, rc, band):
    """Independent construction: explicit float64 images + scipy KD-tree ball query.
    Returns (sure, maybe): pairs clearly inside the cutoff, and pairs within `band` of it."""
    sure, maybe = set(), set()
    for g in range(batch.G):
        lo, hi = int(batch.graph_off[g]), int(batch.graph_off[g + 1])
        P = batch.pos[lo:hi].astype(np.float64)
        if batch.pbc[g]:
            C = batch.cell[g].astype(np.float64)
            nk = np.array(oracle.image_range(C, rc)) + 1
            rng_ = [np.arange(-n, n + 1) for n in nk]
            S = np.stack(np.meshgrid(*rng_, indexing="ij"), -1).reshape(-1, 3)
        else:
            C = np.zeros((3, 3))
            S = np.zeros((1, 3), dtype=np.int64)
        img = (P[:, None, :] + (S @ C)[None, :, :]).reshape(-1, 3)
        tree = cKDTree(img)
        for i in range(hi - lo):
            for idx in tree.query_ball_point(P[i], rc + band):
                j, s = divmod(idx, len(S))
                if j == i and not S[s].any():
                    continue
                d = np.linalg.norm(img[idx] - P[i])
                key = (lo + i, lo + j, tuple(int(x) for x in S[s]))
                if d < rc - band:
                    sure.add(key)
                elif d < rc + band:
                    maybe.add(key)
    return sure, maybe


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_matches_kdtree_on_explicit_images(seed):
    b = small_mixed_batch(seed)
    rc = 5.0
    g = oracle.radius_graph(b.pos, b.graph_off, b.cell, b.pbc, rc)
    got = edge_set(g)
    sure, maybe = kdtree_edges(b, rc, 1e-4)
    assert sure <= got
    assert got <= (sure | maybe)
    assert len(got) > 50
    assert b.pbc.any() and not b.pbc.all()
    # self images must be present in some small cell
    assert any(i == j for (i, j, s) in got)


@pytest.mark.parametrize("seed", [0, 3])
def test_image_range_is_complete(seed):
    b = small_mixed_batch(seed)
    g0 = oracle.radius_graph(b.pos, b.graph_off, b.cell, b.pbc, 4.5)
    g1 = oracle.radius_graph(b.pos, b.graph_off, b.cell, b.pbc, 4.5, extra_images=1)
    for k in ("row_ptr", "col", "shift", "d2", "rvec", "dst", "colT_ptr", "permT"):
        assert np.array_equal(g0[k], g1[k]), k


def test_order_and_csr_consistency():
    b = small_mixed_batch(5)
    g = oracle.radius_graph(b.pos, b.graph_off, b.cell, b.pbc, 4.0)
    keys = list(zip(g["dst"].tolist(), g["col"].tolist(), *[g["shift"][:, k].tolist() for k in range(3)]))
    assert keys == sorted(keys) and len(set(keys)) == len(keys)
    # CSR pointers agree with dst
    for i in range(b.N):
        assert np.all(g["dst"][g["row_ptr"][i]:g["row_ptr"][i + 1]] == i)
    assert g["row_ptr"][-1] == g["E"] == len(g["col"])
    # edges never cross graphs; edge_graph_ptr brackets each graph's edges
    gid = np.searchsorted(b.graph_off, np.arange(b.N), side="right") - 1
    assert np.all(gid[g["dst"]] == gid[g["col"]])
    for k in range(b.G):
        e0, e1 = g["edge_graph_ptr"][k], g["edge_graph_ptr"][k + 1]
        assert np.all(gid[g["dst"][e0:e1]] == k)
    # d2 and rvec belong together and to the shift
    r = g["rvec"].astype(np.float64)
    assert np.allclose((r * r).sum(1), g["d2"], rtol=1e-6)
    for e in range(0, g["E"], 7):
        i, j, s = g["dst"][e], g["col"][e], g["shift"][e].astype(np.float64)
        C = b.cell[gid[i]].astype(np.float64)
        want = b.pos[i].astype(np.float64) - (b.pos[j].astype(np.float64) + s @ C)
        assert np.allclose(r[e], want, atol=1e-5)


def test_symmetry_of_the_edge_set():
    b = small_mixed_batch(7)
    g = oracle.radius_graph(b.pos, b.graph_off, b.cell, b.pbc, 4.0)
    es = edge_set(g)
    d2 = {k: v for k, v in zip(zip(g["dst"].tolist(), g["col"].tolist(),
                                   map(tuple, g["shift"].tolist())), g["d2"].tolist())}
    for (i, j, s) in es:
        rev = (j, i, tuple(-x for x in s))
        assert rev in es
        assert abs(d2[rev] - d2[(i, j, s)]) <= 1e-5 * d2[(i, j, s)]


def test_transpose_plan_by_python_loops():
    b = small_mixed_batch(11)
    g = oracle.radius_graph(b.pos, b.graph_off, b.cell, b.pbc, 3.5)
    buckets = [[] for _ in range(b.N)]
    for e, j in enumerate(g["col"].tolist()):
        buckets[j].append(e)
    flat = [e for lst in buckets for e in lst]
    assert flat == g["permT"].tolist()
    ptr = np.cumsum([0] + [len(x) for x in buckets])
    assert np.array_equal(ptr, g["colT_ptr"])


def _lattice(kind, a, reps):
    basis = {"sc": [[0, 0, 0]], "bcc": [[0, 0, 0], [.5, .5, .5]],
             "fcc": [[0, 0, 0], [0, .5, .5], [.5, 0, .5], [.5, .5, 0]]}[kind]
    pts = []
    for x in range(reps):
        for y in range(reps):
            for z in range(reps):
                for bb in basis:
                    pts.append([(x + bb[0]) * a, (y + bb[1]) * a, (z + bb[2]) * a])
    cell = np.eye(3) * a * reps
    return np.array(pts, dtype=np.float32), cell.astype(np.float32)


def test_coordination_shells_of_cubic_lattices():
    """Textbook shell counts (tests/golden/lattice_shells.txt) through periodic images of a ONE-cell
    lattice: every neighbour of the sc atom is a self image."""
    shells = {}
    for line in open(os.path.join(GOLD, "lattice_shells.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, d2, n = line.split()
        shells.setdefault(k, []).append((float(d2), int(n)))
    a = 2.0  # power of two: all distances exact in float32
    for kind, lst in shells.items():
        pos, cell = _lattice(kind, a, 1)
        b = concat_graphs([(pos, np.ones(len(pos), np.int32), cell)])
        rc = np.sqrt(max(d for d, _ in lst)) * a * 1.01
        g = oracle.radius_graph(b.pos, b.graph_off, b.cell, b.pbc, float(rc))
        for i in range(b.N):
            d2 = g["d2"][g["row_ptr"][i]:g["row_ptr"][i + 1]] / (a * a)
            for want_d2, want_n in lst:
                assert int(np.sum(np.abs(d2 - want_d2) < 1e-6)) == want_n, (kind, want_d2)
            # and nothing between the listed shells
            assert len(d2) == sum(n for d, n in lst if True)


def test_strict_cutoff_excludes_distance_equal_to_rc():
    pos, cell = _lattice("sc", 2.0, 1)
    b = concat_graphs([(pos, np.ones(1, np.int32), cell)])
    assert oracle.radius_graph(b.pos, b.graph_off, b.cell, b.pbc, 2.0)["E"] == 0
    assert oracle.radius_graph(b.pos, b.graph_off, b.cell, b.pbc, 2.0001)["E"] == 6


def test_mean_degree_closed_form_for_uniform_points():
    """Ideal-gas points in a periodic cube: expected degree = rho * 4/3 pi rc^3."""
    rng = np.random.default_rng(123)
    n, side, rc = 3000, 30.0, 4.0
    pos = rng.uniform(0, side, size=(n, 3)).astype(np.float32)
    b = concat_graphs([(pos, np.ones(n, np.int32), (np.eye(3) * side).astype(np.float32))])
    g = oracle.radius_graph(b.pos, b.graph_off, b.cell, b.pbc, rc)
    want = n / side ** 3 * 4.0 / 3.0 * np.pi * rc ** 3
    got = g["E"] / n
    # pair-count standard deviation ~ sqrt(pairs); 4 sigma
    sigma = 2.0 * np.sqrt(g["E"] / 2.0) / n
    assert abs(got - want) < 4 * sigma + 1e-3, (got, want)


def test_cubic_cell_equals_minimum_image_convention():
    rng = np.random.default_rng(5)
    n, side, rc = 150, 11.0, 5.0            # side > 2 rc: at most one image per pair
    pos = rng.uniform(0, side, size=(n, 3)).astype(np.float32)
    b = concat_graphs([(pos, np.ones(n, np.int32), (np.eye(3) * side).astype(np.float32))])
    g = oracle.radius_graph(b.pos, b.graph_off, b.cell, b.pbc, rc)
    P = pos.astype(np.float64)
    d = P[:, None, :] - P[None, :, :]
    d -= side * np.round(d / side)
    dist = np.sqrt((d * d).sum(-1))
    np.fill_diagonal(dist, np.inf)
    want = {(i, j) for i, j in zip(*np.nonzero(dist < rc - 1e-5))}
    maybe = {(i, j) for i, j in zip(*np.nonzero(np.abs(dist - rc) <= 1e-5))}
    got = list(zip(g["dst"].tolist(), g["col"].tolist()))
    assert len(set(got)) == len(got)
    assert want <= set(got) <= (want | maybe)
    e = np.arange(g["E"])
    assert np.allclose(np.sqrt(g["d2"]), dist[g["dst"][e], g["col"][e]], atol=1e-4)


def test_translation_and_lattice_vector_invariance():
    b = small_mixed_batch(21, n_mol=2, n_cry=2)
    rc = 3.7
    g0 = oracle.radius_graph(b.pos, b.graph_off, b.cell, b.pbc, rc)
    # pairs whose distance is far from the cutoff are unaffected by float32 rounding of a translation
    safe = np.abs(np.sqrt(g0["d2"]) - rc) > 1e-3
    t = np.array([0.25, -1.5, 0.75], dtype=np.float32)
    g1 = oracle.radius_graph(b.pos + t, b.graph_off, b.cell, b.pbc, rc, extra_images=1)
    k0 = {k for k, s in zip(zip(g0["dst"].tolist(), g0["col"].tolist()), safe) if s}
    k1 = set(zip(g1["dst"].tolist(), g1["col"].tolist()))
    assert k0 <= k1 and abs(g1["E"] - g0["E"]) <= np.sum(~safe) + 2
    # add a lattice vector to one atom of a periodic graph: degrees do not change
    gi = int(np.nonzero(b.pbc)[0][0])
    atom = int(b.graph_off[gi])
    pos2 = b.pos.copy()
    pos2[atom] += b.cell[gi][1]
    g2 = oracle.radius_graph(pos2, b.graph_off, b.cell, b.pbc, rc, extra_images=1)
    deg0 = np.diff(g0["row_ptr"])
    deg2 = np.diff(g2["row_ptr"])
    assert np.sum(deg0 != deg2) <= np.sum(~safe)


def test_cfg5_mean_degree_matches_density_estimate():
    """Config 5 (0.1 atoms/A^3, rc 6, 1 A hard core): mean degree ~ rho*4/3*pi*(rc^3 - 1) ~ 90,
    checked on sampled rows of a reduced cell of the same density."""
    from hgnn_inputs.structures import make_cubic_bulk
    rng = np.random.default_rng(0)
    pos, z, cell = make_cubic_bulk(rng, 4000, 0.1, 1.0, 1, 30)
    b = concat_graphs([(pos, z, cell)])
    rows = np.arange(0, 4000, 40)
    per = oracle.radius_graph_rows(b.pos, b.graph_off, b.cell, b.pbc, 6.0, rows)
    deg = np.mean([len(r[0]) for r in per])
    want = 0.1 * 4.0 / 3.0 * np.pi * (6.0 ** 3 - 1.0)
    assert abs(deg - want) / want < 0.05, (deg, want)


def test_config1_shape():
    b, hp = make_config("cfg1")
    assert b.G == 32 and np.all(np.diff(b.graph_off) >= 4) and np.all(np.diff(b.graph_off) <= 20)
    g = oracle.radius_graph(b.pos, b.graph_off, None, None, hp["rc"])
    assert set(np.unique(b.Z)) <= {1, 6, 7, 8}
    assert 2000 < g["E"] < 8000
    assert np.all(g["shift"] == 0)
    assert g["d2"].min() >= 0.81 - 1e-4
