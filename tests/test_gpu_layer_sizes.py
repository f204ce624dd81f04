"""One message-passing layer, forward and reverse, on synthetic destination-sorted edge lists of chosen sizes:
edge counts around the tile / block / launch boundaries of the edge kernels (needs a GPU)."""
import numpy as np
import pytest

import oracle
from hgnn_inputs.weights import init_layer_weights
from parity_util import TOL, relerr

pytestmark = pytest.mark.gpu


def _edges(rng, N, E):
    """E directed edges, sorted by destination, random sources and geometry; some atoms have no edge."""
    dst = np.sort(rng.integers(0, N, size=E)).astype(np.int32)
    col = rng.integers(0, N, size=E).astype(np.int32)
    rvec = (rng.standard_normal((E, 3)) * 1.5).astype(np.float32)
    d2 = (rvec.astype(np.float64) ** 2).sum(1).astype(np.float32)
    row_ptr = np.zeros(N + 1, np.int32)
    row_ptr[1:] = np.cumsum(np.bincount(dst, minlength=N))
    return row_ptr, dst, col, d2, rvec


def _run_layer(N, E, H, dtype, seed, lengths=None):
    import torch
    from paper_2506_21788_amd import binding as B
    rng = np.random.default_rng(seed)
    row_ptr, dst, col, d2, rvec = _edges(rng, N, E)
    if lengths is not None:   # chosen row lengths instead of random destinations
        assert len(lengths) == N and sum(lengths) == E
        dst = np.repeat(np.arange(N, dtype=np.int32), lengths)
        row_ptr = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    colT_ptr, permT = oracle.transpose_plan(col, N)
    W = init_layer_weights(rng, H).astype(np.float32)
    h = rng.standard_normal((N, H)).astype(np.float32)
    v = (rng.standard_normal((N, 3)) * 0.3).astype(np.float32)
    gh = rng.standard_normal((N, H)).astype(np.float32)
    gv = rng.standard_normal((N, 3)).astype(np.float32)
    alpha = 1.0 / max(1.0, E / N)
    dt = {"f32": B.F32, "bf16": B.BF16}[dtype]
    dev = lambda a: torch.as_tensor(a).cuda()
    ws_b, saved_b = B.mp_layer_workspace_bytes(N, E, H, dt)
    ws = torch.empty(ws_b, dtype=torch.uint8, device="cuda")
    saved = torch.empty(saved_b, dtype=torch.uint8, device="cuda")
    t = dict(row_ptr=dev(row_ptr), dst=dev(dst), col=dev(col), d2=dev(d2), rvec=dev(rvec), colT=dev(colT_ptr),
             permT=dev(permT.astype(np.int32)), h=dev(h), v=dev(v), W=dev(W), gh=dev(gh), gv=dev(gv))
    h_out, v_out = torch.empty_like(t["h"]), torch.empty_like(t["v"])
    g_h, g_v, gW = torch.empty_like(t["h"]), torch.empty_like(t["v"]), torch.empty_like(t["W"])
    B.mp_layer_fwd(N, E, H, dt, alpha, t["row_ptr"], t["dst"], t["col"], t["d2"], t["rvec"], t["h"], t["v"], t["W"],
                   h_out, v_out, saved, ws)
    B.mp_layer_bwd(N, E, H, dt, alpha, t["row_ptr"], t["dst"], t["col"], t["d2"], t["rvec"], t["colT"], t["permT"],
                   t["h"], t["W"], saved, t["gh"], t["gv"], g_h, g_v, gW, ws)
    torch.cuda.synchronize()
    ho, vo, cache = oracle.mp_layer_fwd(h, v, dst, col, d2, rvec, W.astype(np.float64), alpha)
    gho, gvo, gWo = oracle.mp_layer_bwd(cache, gh, gv)
    tol = TOL[dtype]
    errs = dict(h=relerr(h_out.cpu().numpy(), ho), v=relerr(v_out.cpu().numpy(), vo),
                g_h=relerr(g_h.cpu().numpy(), gho), g_v=relerr(g_v.cpu().numpy(), gvo))
    got = oracle.unpack_layer(gW.cpu().numpy(), H)
    for k, want in gWo.items():
        errs["gW." + k] = relerr(got[k], want)
    print(f"layer N={N} E={E} H={H} {dtype}", {k: f"{e:.1e}" for k, e in errs.items()}, flush=True)
    for k, e in errs.items():
        assert e <= (tol["fwd"] if k in ("h", "v") else tol["grad"]), (k, e)


@pytest.mark.parametrize("H,dtype,N,E", [(256, "bf16", 700, 40001), (128, "f32", 300, 8191), (64, "bf16", 90, 1000),
                                         (256, "f32", 50, 0)])
def test_layer_without_saved_buffer_recomputes(H, dtype, N, E):
    """saved == NULL in both calls: the reverse pass recomputes what the forward pass would have kept; every output
    equals the saved-buffer calls bit for bit."""
    import torch
    from paper_2506_21788_amd import binding as B
    rng = np.random.default_rng(H + E)
    row_ptr, dst, col, d2, rvec = _edges(rng, N, E)
    colT_ptr, permT = oracle.transpose_plan(col, N)
    dt = {"f32": B.F32, "bf16": B.BF16}[dtype]
    dev = lambda a: torch.as_tensor(a).cuda()
    t = dict(row_ptr=dev(row_ptr), dst=dev(dst), col=dev(col), d2=dev(d2), rvec=dev(rvec), colT=dev(colT_ptr),
             permT=dev(permT.astype(np.int32)), h=dev(rng.standard_normal((N, H)).astype(np.float32)),
             v=dev((rng.standard_normal((N, 3)) * 0.3).astype(np.float32)), W=dev(init_layer_weights(rng, H).astype(np.float32)),
             gh=dev(rng.standard_normal((N, H)).astype(np.float32)), gv=dev(rng.standard_normal((N, 3)).astype(np.float32)))
    alpha = 1.0 / max(1.0, E / N)
    ws_b, saved_b = B.mp_layer_workspace_bytes(N, E, H, dt)
    outs = []
    for keep in (True, False):
        ws = torch.empty(ws_b + (0 if keep else saved_b + 512 + 24 * N), dtype=torch.uint8, device="cuda")
        saved = torch.empty(saved_b, dtype=torch.uint8, device="cuda") if keep else None
        h_out, v_out = torch.full_like(t["h"], float("nan")), torch.full_like(t["v"], float("nan"))
        g_h, g_v, gW = torch.full_like(t["h"], float("nan")), torch.full_like(t["v"], float("nan")), torch.full_like(t["W"], float("nan"))
        B.mp_layer_fwd(N, E, H, dt, alpha, t["row_ptr"], t["dst"], t["col"], t["d2"], t["rvec"], t["h"], t["v"], t["W"],
                       h_out, v_out, saved, ws)
        ws.fill_(0x5a)             # nothing of the forward call survives in the workspace
        B.mp_layer_bwd(N, E, H, dt, alpha, t["row_ptr"], t["dst"], t["col"], t["d2"], t["rvec"], t["colT"], t["permT"],
                       t["h"], t["W"], saved, t["gh"], t["gv"], g_h, g_v, gW, ws)
        torch.cuda.synchronize()
        outs.append([x.cpu().numpy() for x in (h_out, v_out, g_h, g_v, gW)])
    for a, b in zip(*outs):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    # a workspace of the plain size is refused
    ws = torch.empty(ws_b, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.HgnnError) as e:
        B.mp_layer_fwd(N, E, H, dt, alpha, t["row_ptr"], t["dst"], t["col"], t["d2"], t["rvec"], t["h"], t["v"], t["W"],
                       torch.empty_like(t["h"]), torch.empty_like(t["v"]), None, ws)
    assert e.value.code == -6


# With bf16 operands at H = 256 the W2 gradient has a branch-free launch over an even number of whole 32-edge blocks
# per workgroup (needs at least 2 x 256 blocks = 16384 edges) and a checking launch for the rest; the fused edge
# kernels work on 64-edge tiles with a masked last tile.
@pytest.mark.parametrize("E", [0, 1, 31, 32, 33, 63, 64, 65, 16383, 16384, 16385, 16384 + 32, 16384 + 63,
                               2 * 16384 + 97, 3 * 16384 - 1])
def test_layer_bf16_pairs_edge_counts(E):
    _run_layer(N=700, E=E, H=256, dtype="bf16", seed=E + 1)


# With bf16 pairs (H = 256) and with fp32 operands at H = 128 the reverse edge kernel sums g_z1 per destination out of
# its 64-edge tile, in 32-edge units: rows
# inside one unit are written directly, rows that cross units are added from per-unit partials by a second kernel,
# empty rows are zeroed there. Row lengths around the unit and tile sizes, at every alignment, with empty rows between.
@pytest.mark.parametrize("H,dtype", [(256, "bf16"), (128, "f32")])
@pytest.mark.parametrize("pattern", ["mixed", "aligned", "long", "ones", "one_row", "tail_rows_empty"])
def test_layer_row_lengths_with_destination_sums_in_the_edge_kernel(pattern, H, dtype, monkeypatch):
    rng = np.random.default_rng(7)
    if pattern == "mixed":
        lengths = [int(x) for x in rng.choice([0, 0, 1, 2, 5, 30, 31, 32, 33, 63, 64, 65, 96, 127, 129, 200], size=400)]
    elif pattern == "aligned":
        lengths = [32, 32, 64, 0, 32, 96, 0, 0, 64, 128, 32, 1, 31, 32] * 20
    elif pattern == "long":
        lengths = [700, 3, 0, 1025, 64, 5000, 1]
    elif pattern == "ones":
        lengths = [1] * 777
    elif pattern == "one_row":
        lengths = [0, 0, 4321, 0]
    else:
        lengths = [40, 17, 64, 7] + [0] * 50
    N, E = len(lengths), sum(lengths)
    _run_layer(N=N, E=E, H=H, dtype=dtype, seed=11, lengths=lengths)
    # the separate pass over g_z1 (kept for the calls that ask for the gradient with respect to d2) gives the same
    monkeypatch.setenv("HGNN_DSUM_IN_KERNEL", "0")
    _run_layer(N=N, E=E, H=H, dtype=dtype, seed=11, lengths=lengths)


@pytest.mark.parametrize("H,dtype,E", [(64, "f32", 1000), (64, "bf16", 4097), (128, "f32", 8191), (128, "bf16", 8193),
                                       (256, "f32", 4095)])
def test_layer_other_modes_edge_counts(H, dtype, E):
    _run_layer(N=300, E=E, H=H, dtype=dtype, seed=E)


# fp32 operands at H = 128: the W2 gradient recomputes a1 in a kernel of its own (two 16-edge chunks per 32-edge block,
# eight-chunk trips, grids rounded to multiples of eight workgroups, one ragged block at most)
@pytest.mark.parametrize("E", [0, 1, 15, 16, 17, 31, 32, 33, 255, 256, 257, 511, 16385, 3 * 16384 + 45])
def test_layer_f32_128_edge_counts(E):
    _run_layer(N=500, E=E, H=128, dtype="f32", seed=E + 7)


# Atom counts around the split rules of the atom-level weight gradients (about 64 rows per split, at most one round
# of resident workgroups, whole workgroups per compute unit, a grid padded to groups of eight splits) and the row
# tiles of the atom-level products; few edges, so that the atom-level kernels decide the outcome.
@pytest.mark.parametrize("H,dtype,N", [(256, "bf16", 1), (256, "bf16", 255), (256, "bf16", 257), (256, "bf16", 2049),
                                       (256, "bf16", 16385), (256, "bf16", 33001), (128, "f32", 9000),
                                       (128, "bf16", 41000), (64, "f32", 70001), (256, "f32", 12345)])
def test_layer_atom_counts(H, dtype, N):
    _run_layer(N=N, E=3000, H=H, dtype=dtype, seed=N)


# Widths other than 64 / 128 / 256 take the fragment-GEMM path (bf16 operands, width padded to a multiple of 128, rows
# to 256): the paper's 866, widths on both sides of the padding steps, odd and small widths, edge counts around the
# 16 / 32 / 256-row groups.
@pytest.mark.parametrize("H,N,E", [(866, 300, 5000), (384, 200, 3001), (1024, 257, 777), (866, 40, 0), (320, 513, 9000),
                                   (500, 64, 256), (866, 5, 17), (333, 100, 1500), (257, 33, 700), (100, 80, 900), (24, 50, 300),
                                   # enough edges for the 256 x 128 tiles of the per-edge weight gradient: a ragged
                                   # last row tile (Hp = 384: 8 + 4 blocks), a single whole one (Hp = 256 is served
                                   # by the fused kernels, so 200 -> 256), and two whole ones (512)
                                   (320, 2000, 70001), (200, 1500, 66000), (512, 1800, 65536),
                                   # atoms whose edges span many 64-row strips of the forward per-atom sums (whole strips
                                   # in the middle), next to atoms without edges
                                   (384, 3, 1000), (866, 2, 300), (200, 40, 64), (200, 7, 65)])
def test_layer_wide_widths(H, N, E):
    _run_layer(N=N, E=E, H=H, dtype="bf16", seed=H + E)


# ------------------------------------------------------------------------------------------------
# k edge attributes (radial basis of the edge length) in place of d2
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("E,k,rc", [(5000, 8, 5.0), (1, 2, 3.0), (777, 16, 6.0), (0, 4, 5.0)])
def test_edge_rbf_matches_the_oracle(E, k, rc):
    import torch
    from paper_2506_21788_amd import binding as B
    rng = np.random.default_rng(E + k)
    d = rng.uniform(0.0, rc, size=E).astype(np.float32)
    if E > 3:
        d[:3] = (0.0, rc, np.float32(rc) * np.float32(0.999999))
    d2 = (d * d).astype(np.float32)
    attr = torch.full((max(E, 1), k), float("nan"), dtype=torch.float32, device="cuda")
    B.edge_rbf(E, torch.as_tensor(d2).cuda(), k, rc, attr)
    torch.cuda.synchronize()
    if E == 0:
        return
    want = oracle.edge_rbf(d2, k, rc)
    got = attr.cpu().numpy()[:E]
    assert np.all(np.isfinite(got))
    assert relerr(got, want) <= TOL["f32"]["fwd"]      # float32 arithmetic against the float64 definition


def _run_layer_attr(N, E, H, k, seed, rc=5.0):
    import torch
    from paper_2506_21788_amd import binding as B
    rng = np.random.default_rng(seed)
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
    dev = lambda a: torch.as_tensor(np.ascontiguousarray(a)).cuda()
    ws_b, saved_b = B.mp_layer_attr_workspace_bytes(N, E, H, k, B.BF16)
    ws = torch.empty(ws_b, dtype=torch.uint8, device="cuda")
    saved = torch.empty(saved_b, dtype=torch.uint8, device="cuda")
    t = dict(row_ptr=dev(row_ptr), dst=dev(dst), col=dev(col), attr=dev(attr), rvec=dev(rvec), colT=dev(colT_ptr),
             permT=dev(permT.astype(np.int32)), h=dev(h), v=dev(v), W=dev(W), gh=dev(gh), gv=dev(gv))
    h_out, v_out = torch.empty_like(t["h"]), torch.empty_like(t["v"])
    g_h, g_v = torch.empty_like(t["h"]), torch.empty_like(t["v"])
    gW = torch.full_like(t["W"], float("nan"))
    B.mp_layer_attr_fwd(N, E, H, k, B.BF16, alpha, t["row_ptr"], t["dst"], t["col"], t["attr"], t["rvec"], t["h"],
                        t["v"], t["W"], h_out, v_out, saved, ws)
    B.mp_layer_attr_bwd(N, E, H, k, B.BF16, alpha, t["row_ptr"], t["dst"], t["col"], t["attr"], t["rvec"], t["colT"],
                        t["permT"], t["h"], t["W"], saved, t["gh"], t["gv"], g_h, g_v, gW, ws)
    torch.cuda.synchronize()
    ho, vo, cache = oracle.mp_layer_fwd(h, v, dst, col, d2, rvec, W.astype(np.float64), alpha, attr=attr)
    gho, gvo, gWo = oracle.mp_layer_bwd(cache, gh, gv)
    tol = TOL["bf16"]
    errs = dict(h=relerr(h_out.cpu().numpy(), ho), v=relerr(v_out.cpu().numpy(), vo),
                g_h=relerr(g_h.cpu().numpy(), gho), g_v=relerr(g_v.cpu().numpy(), gvo))
    got_flat = gW.cpu().numpy()
    assert np.all(np.isfinite(got_flat)), "a gradient field was left unwritten"
    got = oracle.unpack_layer(got_flat, H, k)
    for name, want in gWo.items():
        errs["gW." + name] = relerr(got[name], want)
    errs["gW.W1[attr rows]"] = relerr(got["W1"][2 * H:], gWo["W1"][2 * H:])
    print(f"layer attr N={N} E={E} H={H} k={k}", {n: f"{e:.1e}" for n, e in errs.items()}, flush=True)
    for n, e in errs.items():
        assert e <= (tol["fwd"] if n in ("h", "v") else tol["grad"]), (n, e)


# H = 64 / 128 / 256 run on the fused kernels (attribute term on the matrix cores): tile boundaries (64 edges), the
# branch-free and the masked tile, every k residue of the four-slot staging, k = 16 (all slots) and k = 2
@pytest.mark.parametrize("N,E,H,k", [(300, 5000, 866, 8), (200, 3001, 256, 16), (100, 1500, 64, 4), (64, 700, 333, 3),
                                     (50, 0, 128, 5), (120, 2000, 300, 1), (700, 40001, 256, 8), (300, 64, 256, 2),
                                     (300, 8193, 128, 13), (90, 1000, 64, 16), (40, 63, 128, 7), (500, 20000, 256, 3)])
def test_layer_with_edge_attributes(N, E, H, k):
    _run_layer_attr(N=N, E=E, H=H, k=k, seed=H + E + k)
