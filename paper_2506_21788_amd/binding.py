"""ctypes binding of libhgnn.so: one Python function per C entry point, same name without the
`hgnn_` prefix. Arguments are torch tensors on the GPU (used as device memory only) or Python
scalars; this module only marshals pointers and checks the status code. Every step of the path runs
inside the library's kernels. There is no fallback: if the library is missing, importing fails."""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhgnn.so")

F32, BF16 = 0, 1
POOL_SUM, POOL_MEAN = 0, 1
ZMAX = 94

EXPORTS = [
    "hgnn_last_error_string", "hgnn_version",
    "hgnn_radius_graph_workspace_bytes", "hgnn_radius_graph_count", "hgnn_radius_graph_fill",
    "hgnn_embed_fwd", "hgnn_embed_bwd", "hgnn_embed_bwd_workspace_bytes", "hgnn_embed_bwd_static",
    "hgnn_set_side_stream", "hgnn_mp_layer_workspace_bytes", "hgnn_mp_layer_fwd", "hgnn_mp_layer_bwd",
    "hgnn_edge_rbf", "hgnn_edge_rbf_bwd", "hgnn_edge_geometry_fwd", "hgnn_edge_geometry_bwd",
    "hgnn_mp_layer_attr_workspace_bytes", "hgnn_mp_layer_attr_fwd", "hgnn_mp_layer_attr_bwd",
    "hgnn_pool_by_graph_fwd", "hgnn_pool_by_graph_bwd",
    "hgnn_multihead_plan_ints", "hgnn_multihead_plan",
    "hgnn_multihead_decode_workspace_bytes", "hgnn_multihead_decode_fwd", "hgnn_multihead_decode_bwd",
    "hgnn_multihead_deep_workspace_bytes", "hgnn_multihead_deep_fwd", "hgnn_multihead_deep_bwd",
    "hgnn_adamw_step",
    "hgnn_profile_begin", "hgnn_profile_end", "hgnn_profile_num_tags", "hgnn_profile_tag_name",
    "hgnn_profile_read",
]


class HgnnError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libhgnn error {code}: {msg}")
        self.code = code


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    lib = C.CDLL(LIB_PATH)
    lib.hgnn_last_error_string.restype = C.c_char_p
    lib.hgnn_multihead_plan_ints.restype = C.c_int64
    lib.hgnn_multihead_plan_ints.argtypes = [C.c_int32] * 3
    return lib


_lib = _load()

vp, i32, i64, f32, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_size_t


def _sig(name, *argtypes):
    fn = getattr(_lib, name)
    fn.restype = C.c_int32
    fn.argtypes = list(argtypes)
    return fn


_rg_ws = _sig("hgnn_radius_graph_workspace_bytes", i32, i32, C.POINTER(sz))
_rg_count = _sig("hgnn_radius_graph_count", vp, i32, i32, vp, vp, vp, vp, f32, vp, sz, vp, C.POINTER(i64))
_rg_fill = _sig("hgnn_radius_graph_fill", vp, i32, i32, vp, vp, vp, vp, f32, vp, sz, vp, sz, vp, i64,
                vp, vp, vp, vp, vp, vp, vp, vp)
_embed_fwd = _sig("hgnn_embed_fwd", vp, i32, i32, vp, vp, vp)
_embed_bwd = _sig("hgnn_embed_bwd", vp, i32, i32, vp, vp, vp, vp, sz)
_embed_bwd_static = _sig("hgnn_embed_bwd_static", vp, i32, i32, vp, vp, vp)
_embed_bwd_ws = _sig("hgnn_embed_bwd_workspace_bytes", i32, i32, C.POINTER(sz))
_mp_ws = _sig("hgnn_mp_layer_workspace_bytes", i32, i64, i32, i32, C.POINTER(sz), C.POINTER(sz))
_mp_fwd = _sig("hgnn_mp_layer_fwd", vp, i32, i64, i32, i32, f32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp,
               vp, sz, vp, sz)
_mp_bwd = _sig("hgnn_mp_layer_bwd", vp, i32, i64, i32, i32, f32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz,
               vp, vp, vp, vp, vp, vp, sz)
_rbf = _sig("hgnn_edge_rbf", vp, i64, vp, i32, f32, vp)
_mpa_ws = _sig("hgnn_mp_layer_attr_workspace_bytes", i32, i64, i32, i32, i32, C.POINTER(sz), C.POINTER(sz))
_mpa_fwd = _sig("hgnn_mp_layer_attr_fwd", vp, i32, i64, i32, i32, i32, f32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                vp, sz, vp, sz)
_mpa_bwd = _sig("hgnn_mp_layer_attr_bwd", vp, i32, i64, i32, i32, i32, f32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz,
                vp, vp, vp, vp, vp, vp, vp, vp, sz)
_rbf_bwd = _sig("hgnn_edge_rbf_bwd", vp, i64, vp, i32, f32, vp, vp)
_geom_fwd = _sig("hgnn_edge_geometry_fwd", vp, i32, i64, vp, vp, vp, vp, vp, vp)
_geom_bwd = _sig("hgnn_edge_geometry_bwd", vp, i32, i64, vp, vp, vp, vp, vp, vp, vp, vp, vp)
_adamw = _sig("hgnn_adamw_step", vp, i64, vp, vp, vp, vp, i32, C.c_double, C.c_double, C.c_double, C.c_double,
              C.c_double)
_pool_fwd = _sig("hgnn_pool_by_graph_fwd", vp, i32, i32, i32, i32, vp, vp, vp)
_pool_bwd = _sig("hgnn_pool_by_graph_bwd", vp, i32, i32, i32, i32, vp, vp, vp, i32)
_plan = _sig("hgnn_multihead_plan", vp, i32, i32, i32, vp, vp, vp)
_dec_ws = _sig("hgnn_multihead_decode_workspace_bytes", i32, i32, i32, i32, i32, i32, C.POINTER(sz), C.POINTER(sz))
_dec_fwd = _sig("hgnn_multihead_decode_fwd", vp, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp,
                vp, sz, vp, sz)
_dec_bwd = _sig("hgnn_multihead_decode_bwd", vp, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, sz,
                vp, vp, vp, vp, vp, vp, vp, sz)
_deep_ws = _sig("hgnn_multihead_deep_workspace_bytes", i32, i32, i32, i32, i32, i32, i32, C.POINTER(sz), C.POINTER(sz))
_deep_fwd = _sig("hgnn_multihead_deep_fwd", vp, i32, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp,
                 vp, sz, vp, sz)
_deep_bwd = _sig("hgnn_multihead_deep_bwd", vp, i32, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, sz,
                 vp, vp, vp, vp, vp, vp, vp, sz)


def last_error_string() -> str:
    return _lib.hgnn_last_error_string().decode()


def version() -> int:
    return int(_lib.hgnn_version())


def set_side_stream(enable):
    """Weight gradients of the layer's reverse pass on the library's side stream (True), on the caller's stream
    (False), or wherever the library chooses per code path (None, the default); returns the previous setting."""
    prev = int(_lib.hgnn_set_side_stream(C.c_int32(-1 if enable is None else (1 if enable else 0))))
    return None if prev < 0 else bool(prev)


def _check(code):
    if code != 0:
        raise HgnnError(code, last_error_string())


def _p(t):
    """Device pointer of a tensor (None -> NULL)."""
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "libhgnn takes contiguous device tensors"
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


# ------------------------------------------------------------------------------------------------
def radius_graph_workspace_bytes(N, G):
    b = sz(0)
    _check(_rg_ws(N, G, C.byref(b)))
    return b.value


def radius_graph_count(N, G, pos, graph_off, cell, pbc, rc, ws, row_ptr):
    E = i64(0)
    _check(_rg_count(_stream(), N, G, _p(pos), _p(graph_off), _p(cell), _p(pbc), rc, _p(ws), _nbytes(ws),
                     _p(row_ptr), C.byref(E)))
    return E.value


def radius_graph_fill(N, G, pos, graph_off, cell, pbc, rc, ws, tmp, row_ptr, E, dst, col, shift, d2, rvec,
                      edge_graph_ptr, colT_ptr, permT):
    _check(_rg_fill(_stream(), N, G, _p(pos), _p(graph_off), _p(cell), _p(pbc), rc, _p(ws), _nbytes(ws),
                    _p(tmp), _nbytes(tmp), _p(row_ptr), E, _p(dst), _p(col), _p(shift), _p(d2), _p(rvec),
                    _p(edge_graph_ptr), _p(colT_ptr), _p(permT)))


def embed_fwd(N, H, Z, emb, h):
    _check(_embed_fwd(_stream(), N, H, _p(Z), _p(emb), _p(h)))


def embed_bwd_workspace_bytes(N, H):
    b = sz(0)
    _check(_embed_bwd_ws(N, H, C.byref(b)))
    return b.value


def embed_bwd(N, H, Z, g_h, g_emb, ws):
    _check(_embed_bwd(_stream(), N, H, _p(Z), _p(g_h), _p(g_emb), _p(ws), _nbytes(ws)))


EMBED_BWD_STATIC_MAX_BYTES = 8 << 20


def embed_bwd_static(N, H, Z, g_h, g_emb):
    _check(_embed_bwd_static(_stream(), N, H, _p(Z), _p(g_h), _p(g_emb)))


def mp_layer_workspace_bytes(N, E, H, dtype):
    a, b = sz(0), sz(0)
    _check(_mp_ws(N, E, H, dtype, C.byref(a), C.byref(b)))
    return a.value, b.value


def edge_rbf(E, d2, k, rc, attr):
    _check(_rbf(_stream(), E, _p(d2), k, rc, _p(attr)))


def mp_layer_attr_workspace_bytes(N, E, H, k, dtype):
    a, b = sz(0), sz(0)
    _check(_mpa_ws(N, E, H, k, dtype, C.byref(a), C.byref(b)))
    return a.value, b.value


def mp_layer_attr_fwd(N, E, H, k, dtype, alpha, row_ptr, dst, col, attr, rvec, h_in, v_in, W, h_out, v_out, saved, ws):
    _check(_mpa_fwd(_stream(), N, E, H, k, dtype, alpha, _p(row_ptr), _p(dst), _p(col), _p(attr), _p(rvec),
                    _p(h_in), _p(v_in), _p(W), _p(h_out), _p(v_out), _p(saved), _nbytes(saved), _p(ws), _nbytes(ws)))


def mp_layer_attr_bwd(N, E, H, k, dtype, alpha, row_ptr, dst, col, attr, rvec, colT_ptr, permT, h_in, W, saved,
                      g_h_out, g_v_out, g_h_in, g_v_in, gW, ws, g_attr=None, g_rvec=None):
    _check(_mpa_bwd(_stream(), N, E, H, k, dtype, alpha, _p(row_ptr), _p(dst), _p(col), _p(attr), _p(rvec),
                    _p(colT_ptr), _p(permT), _p(h_in), _p(W), _p(saved), _nbytes(saved), _p(g_h_out), _p(g_v_out),
                    _p(g_h_in), _p(g_v_in), _p(gW), _p(g_attr), _p(g_rvec), _p(ws), _nbytes(ws)))


def edge_rbf_bwd(E, d2, k, rc, g_attr, g_d2):
    _check(_rbf_bwd(_stream(), E, _p(d2), k, rc, _p(g_attr), _p(g_d2)))


def edge_geometry_fwd(N, E, rvec0, v, dst, col, rvec, d2):
    _check(_geom_fwd(_stream(), N, E, _p(rvec0), _p(v), _p(dst), _p(col), _p(rvec), _p(d2)))


def edge_geometry_bwd(N, E, row_ptr, colT_ptr, permT, rvec, g_rvec, g_d2, g_r, g_r_sum, g_v):
    _check(_geom_bwd(_stream(), N, E, _p(row_ptr), _p(colT_ptr), _p(permT), _p(rvec), _p(g_rvec), _p(g_d2), _p(g_r),
                     _p(g_r_sum), _p(g_v)))


def mp_layer_fwd(N, E, H, dtype, alpha, row_ptr, dst, col, d2, rvec, h_in, v_in, W, h_out, v_out, saved, ws):
    _check(_mp_fwd(_stream(), N, E, H, dtype, alpha, _p(row_ptr), _p(dst), _p(col), _p(d2), _p(rvec),
                   _p(h_in), _p(v_in), _p(W), _p(h_out), _p(v_out), _p(saved), _nbytes(saved), _p(ws), _nbytes(ws)))


def mp_layer_bwd(N, E, H, dtype, alpha, row_ptr, dst, col, d2, rvec, colT_ptr, permT, h_in, W, saved,
                 g_h_out, g_v_out, g_h_in, g_v_in, gW, ws):
    _check(_mp_bwd(_stream(), N, E, H, dtype, alpha, _p(row_ptr), _p(dst), _p(col), _p(d2), _p(rvec),
                   _p(colT_ptr), _p(permT), _p(h_in), _p(W), _p(saved), _nbytes(saved), _p(g_h_out), _p(g_v_out),
                   _p(g_h_in), _p(g_v_in), _p(gW), _p(ws), _nbytes(ws)))


def pool_by_graph_fwd(N, G, H, mode, graph_off, h, p):
    _check(_pool_fwd(_stream(), N, G, H, mode, _p(graph_off), _p(h), _p(p)))


def pool_by_graph_bwd(N, G, H, mode, graph_off, g_p, g_h, accumulate):
    _check(_pool_bwd(_stream(), N, G, H, mode, _p(graph_off), _p(g_p), _p(g_h), int(accumulate)))


def multihead_plan_ints(N, G, S):
    return int(_lib.hgnn_multihead_plan_ints(N, G, S))


def multihead_plan(N, G, S, graph_off, source_id, plan):
    _check(_plan(_stream(), N, G, S, _p(graph_off), _p(source_id), _p(plan)))


def plan_fields(plan, N, G, S):
    """Views of the documented sub-arrays of a plan tensor."""
    o, out = 0, {}
    for name, n in (("grp_graph_ptr", S + 1), ("graph_perm", G), ("grp_atom_ptr", S + 1), ("atom_perm", N),
                    ("atom_graph", N)):
        out[name] = plan[o:o + n]
        o += n
    return out


def multihead_decode_workspace_bytes(N, G, H, Hh, S, dtype):
    a, b = sz(0), sz(0)
    _check(_dec_ws(N, G, H, Hh, S, dtype, C.byref(a), C.byref(b)))
    return a.value, b.value


def multihead_decode_fwd(N, G, H, Hh, S, dtype, plan, p, h, v, Whead, energy, force, saved, ws):
    _check(_dec_fwd(_stream(), N, G, H, Hh, S, dtype, _p(plan), _p(p), _p(h), _p(v), _p(Whead), _p(energy),
                    _p(force), _p(saved), _nbytes(saved), _p(ws), _nbytes(ws)))


def multihead_decode_bwd(N, G, H, Hh, S, dtype, plan, p, h, v, Whead, saved, g_energy, g_force, g_p, g_h, g_v,
                         gWhead, ws):
    _check(_dec_bwd(_stream(), N, G, H, Hh, S, dtype, _p(plan), _p(p), _p(h), _p(v), _p(Whead), _p(saved),
                    _nbytes(saved), _p(g_energy), _p(g_force), _p(g_p), _p(g_h), _p(g_v), _p(gWhead), _p(ws),
                    _nbytes(ws)))


def multihead_deep_workspace_bytes(N, G, H, Hh, D, S, dtype):
    a, b = sz(0), sz(0)
    _check(_deep_ws(N, G, H, Hh, D, S, dtype, C.byref(a), C.byref(b)))
    return a.value, b.value


def multihead_deep_fwd(N, G, H, Hh, D, S, dtype, plan, p, h, v, Whead, energy, force, saved, ws):
    _check(_deep_fwd(_stream(), N, G, H, Hh, D, S, dtype, _p(plan), _p(p), _p(h), _p(v), _p(Whead), _p(energy),
                     _p(force), _p(saved), _nbytes(saved), _p(ws), _nbytes(ws)))


def multihead_deep_bwd(N, G, H, Hh, D, S, dtype, plan, p, h, v, Whead, saved, g_energy, g_force, g_p, g_h, g_v,
                       gWhead, ws):
    _check(_deep_bwd(_stream(), N, G, H, Hh, D, S, dtype, _p(plan), _p(p), _p(h), _p(v), _p(Whead), _p(saved),
                     _nbytes(saved), _p(g_energy), _p(g_force), _p(g_p), _p(g_h), _p(g_v), _p(gWhead), _p(ws),
                     _nbytes(ws)))


# ------------------------------------------------------------------------------------------------
# instrumentation
_prof_begin = _sig("hgnn_profile_begin", C.c_uint64)
_prof_end = _sig("hgnn_profile_end", vp)
_prof_read = _sig("hgnn_profile_read", i32, C.POINTER(i64), C.POINTER(C.c_double))
_lib.hgnn_profile_tag_name.restype = C.c_char_p
_lib.hgnn_profile_tag_name.argtypes = [i32]


def profile_num_tags():
    return int(_lib.hgnn_profile_num_tags())


def profile_tag_name(tag):
    return _lib.hgnn_profile_tag_name(tag).decode()


def adamw_step(w, g, m, v, step, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01):
    """In-place AdamW update of the flat float32 device tensor w (moments m, v; gradient g); step counts from 1."""
    _check(_adamw(_stream(), w.numel(), _p(w), _p(g), _p(m), _p(v), step, lr, beta1, beta2, eps, weight_decay))

def profile_begin(tag_mask):
    _check(_prof_begin(tag_mask))


def profile_end():
    _check(_prof_end(_stream()))


def profile_read(tag):
    n, ms = i64(0), C.c_double(0.0)
    _check(_prof_read(tag, C.byref(n), C.byref(ms)))
    return n.value, ms.value
