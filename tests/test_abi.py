"""The C-ABI library loads and exports every symbol the public header declares (no GPU needed)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "hgnn.h")
LIB = os.path.join(ROOT, "paper_2506_21788_amd", "libhgnn.so")


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hgnn_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_boundary():
    names = declared_symbols()
    for must in ("hgnn_radius_graph_count", "hgnn_radius_graph_fill", "hgnn_mp_layer_fwd", "hgnn_mp_layer_bwd",
                 "hgnn_pool_by_graph_fwd", "hgnn_pool_by_graph_bwd", "hgnn_multihead_decode_fwd",
                 "hgnn_multihead_decode_bwd", "hgnn_multihead_plan", "hgnn_embed_fwd", "hgnn_embed_bwd"):
        assert must in names


def test_library_exports_every_declared_symbol():
    assert os.path.exists(LIB), "build the library first: python -c 'import __graft_entry__ as g; g.build()'"
    lib = ctypes.CDLL(LIB)
    for name in declared_symbols():
        assert hasattr(lib, name), name
    lib.hgnn_version.restype = ctypes.c_int32
    assert lib.hgnn_version() >= 1


def test_binding_names_match_the_header():
    import importlib.util
    spec = importlib.util.find_spec("paper_2506_21788_amd.binding")
    src = open(spec.origin).read()
    for name in declared_symbols():
        assert f'"{name}"' in src, name


def test_host_side_argument_checks_need_no_gpu():
    lib = ctypes.CDLL(LIB)
    lib.hgnn_last_error_string.restype = ctypes.c_char_p
    b = ctypes.c_size_t(0)
    assert lib.hgnn_radius_graph_workspace_bytes(ctypes.c_int32(100), ctypes.c_int32(3), ctypes.byref(b)) == 0
    assert b.value > 0
    assert lib.hgnn_radius_graph_workspace_bytes(ctypes.c_int32(-1), ctypes.c_int32(3), ctypes.byref(b)) == -2
    a, s = ctypes.c_size_t(0), ctypes.c_size_t(0)
    # H outside the supported tile granularity
    rc = lib.hgnn_mp_layer_workspace_bytes(ctypes.c_int32(10), ctypes.c_int64(50), ctypes.c_int32(1025),
                                           ctypes.c_int32(0), ctypes.byref(a), ctypes.byref(s))
    assert rc == -2 and b"1..1024" in lib.hgnn_last_error_string()
    # widths other than 64, 128, 256 exist with bf16 operands only
    unimpl = [l for l in open(HEADER) if "HGNN_ERR_UNIMPLEMENTED" in l and "=" in l]
    code = int(re.search(r"=\s*(-?\d+)", unimpl[0]).group(1))
    rc = lib.hgnn_mp_layer_workspace_bytes(ctypes.c_int32(10), ctypes.c_int64(50), ctypes.c_int32(866),
                                           ctypes.c_int32(0), ctypes.byref(a), ctypes.byref(s))
    assert rc == code and b"bf16" in lib.hgnn_last_error_string()
    rc = lib.hgnn_mp_layer_workspace_bytes(ctypes.c_int32(10), ctypes.c_int64(50), ctypes.c_int32(866),
                                           ctypes.c_int32(1), ctypes.byref(a), ctypes.byref(s))
    assert rc == 0 and a.value > 0 and s.value > 0
    # deep heads: depth range, bf16 only
    f = lib.hgnn_multihead_deep_workspace_bytes
    args = lambda H, Hh, D, dt: [ctypes.c_int32(x) for x in (10, 2, H, Hh, D, 3, dt)] + [ctypes.byref(a), ctypes.byref(s)]
    assert f(*args(866, 889, 3, 1)) == 0 and a.value > 0
    assert f(*args(866, 889, 0, 1)) == -2
    assert f(*args(866, 2000, 3, 1)) == -2
    assert f(*args(866, 889, 3, 0)) == code
    rc = lib.hgnn_mp_layer_workspace_bytes(ctypes.c_int32(10), ctypes.c_int64(50), ctypes.c_int32(128),
                                           ctypes.c_int32(1), ctypes.byref(a), ctypes.byref(s))
    assert rc == 0 and a.value > 0 and s.value >= 50 * 128 * 4
    # edge count that does not fit int32
    rc = lib.hgnn_mp_layer_workspace_bytes(ctypes.c_int32(10), ctypes.c_int64(2 ** 31), ctypes.c_int32(128),
                                           ctypes.c_int32(0), ctypes.byref(a), ctypes.byref(s))
    assert rc == -7
    # gathered node rows are addressed with 32-bit byte offsets: N * 2H * 4 bytes must stay below 4 GiB
    rc = lib.hgnn_mp_layer_workspace_bytes(ctypes.c_int32(3_000_000), ctypes.c_int64(50), ctypes.c_int32(256),
                                           ctypes.c_int32(1), ctypes.byref(a), ctypes.byref(s))
    assert rc == -7 and b"4 GiB" in lib.hgnn_last_error_string()
    rc = lib.hgnn_mp_layer_workspace_bytes(ctypes.c_int32(2_000_000), ctypes.c_int64(50), ctypes.c_int32(256),
                                           ctypes.c_int32(1), ctypes.byref(a), ctypes.byref(s))
    assert rc == 0
    # with bf16 operands at H = 256 the reverse pass recomputes silu(z1): one [E,H] tensor less is saved
    s16, s32 = ctypes.c_size_t(0), ctypes.c_size_t(0)
    assert lib.hgnn_mp_layer_workspace_bytes(ctypes.c_int32(1000), ctypes.c_int64(32000), ctypes.c_int32(256),
                                             ctypes.c_int32(1), ctypes.byref(a), ctypes.byref(s16)) == 0
    assert lib.hgnn_mp_layer_workspace_bytes(ctypes.c_int32(1000), ctypes.c_int64(32000), ctypes.c_int32(256),
                                             ctypes.c_int32(0), ctypes.byref(a), ctypes.byref(s32)) == 0
    assert s16.value < 32000 * 256 * 2 * 2 <= s32.value
    # a head width other than H is served by the one-hidden-layer case of the deep heads: bf16 operands only
    hw = lambda Hh, dt: lib.hgnn_multihead_decode_workspace_bytes(
        ctypes.c_int32(10), ctypes.c_int32(2), ctypes.c_int32(128), ctypes.c_int32(Hh), ctypes.c_int32(2),
        ctypes.c_int32(dt), ctypes.byref(a), ctypes.byref(s))
    assert hw(64, 0) == code and hw(64, 1) == 0 and hw(2000, 1) == -2 and hw(128, 0) == 0
    # layers with edge attributes: one attribute at 64 / 128 / 256 runs on the fused kernels in either operand type
    # (same buffers as the plain layer); several attributes or other widths need bf16 operands
    aw = lambda H, k, dt: lib.hgnn_mp_layer_attr_workspace_bytes(
        ctypes.c_int32(10), ctypes.c_int64(50), ctypes.c_int32(H), ctypes.c_int32(k), ctypes.c_int32(dt),
        ctypes.byref(a), ctypes.byref(s))
    assert aw(128, 1, 0) == 0
    a1, s1 = a.value, s.value
    assert lib.hgnn_mp_layer_workspace_bytes(ctypes.c_int32(10), ctypes.c_int64(50), ctypes.c_int32(128), ctypes.c_int32(0),
                                             ctypes.byref(a), ctypes.byref(s)) == 0 and (a.value, s.value) == (a1, s1)
    assert aw(128, 2, 0) == code and aw(128, 2, 1) == 0 and aw(866, 1, 0) == code and aw(866, 1, 1) == 0
    assert aw(128, 17, 1) == -2 and aw(128, 0, 1) == -2
    lib.hgnn_multihead_plan_ints.restype = ctypes.c_int64
    assert lib.hgnn_multihead_plan_ints(ctypes.c_int32(7), ctypes.c_int32(3), ctypes.c_int32(2)) >= 2 * 3 + 7 + 3 + 3


def test_geometry_entry_points_check_their_arguments_on_the_host():
    lib = ctypes.CDLL(LIB)
    lib.hgnn_last_error_string.restype = ctypes.c_char_p
    nullptr_code = int(re.search(r"HGNN_ERR_NULLPTR\s*=\s*(-?\d+)", open(HEADER).read()).group(1))
    i32, i64, f32, vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_void_p
    fake = lambda n: vp(0x1000 * n)     # never dereferenced: every call below returns before any launch
    # radial basis and its reverse: 2 <= k <= 16, rc > 0
    assert lib.hgnn_edge_rbf_bwd(None, i64(10), fake(1), i32(1), f32(5.0), fake(2), fake(3)) == -2
    assert lib.hgnn_edge_rbf_bwd(None, i64(10), fake(1), i32(17), f32(5.0), fake(2), fake(3)) == -2
    assert lib.hgnn_edge_rbf_bwd(None, i64(10), fake(1), i32(4), f32(0.0), fake(2), fake(3)) == -2
    assert lib.hgnn_edge_rbf_bwd(None, i64(-1), fake(1), i32(4), f32(5.0), fake(2), fake(3)) == -2
    assert lib.hgnn_edge_rbf_bwd(None, i64(0), None, i32(4), f32(5.0), None, None) == 0          # nothing to do
    assert lib.hgnn_edge_rbf_bwd(None, i64(10), fake(1), i32(4), f32(5.0), None, fake(3)) == nullptr_code
    # geometry: forward needs every array, the reverse pass needs rvec only with g_d2 and the index arrays only with g_v
    assert lib.hgnn_edge_geometry_fwd(None, i32(5), i64(0), None, None, None, None, None, None) == 0
    assert lib.hgnn_edge_geometry_fwd(None, i32(5), i64(10), fake(1), None, fake(2), fake(3), fake(4), fake(5)) == nullptr_code
    assert lib.hgnn_edge_geometry_fwd(None, i32(-1), i64(10), fake(1), fake(6), fake(2), fake(3), fake(4), fake(5)) == -2
    bwd = lib.hgnn_edge_geometry_bwd
    assert bwd(None, i32(5), i64(0), None, None, None, None, None, None, None, None, None) == 0
    assert bwd(None, i32(5), i64(10), None, None, None, None, fake(1), fake(2), fake(3), None, None) == nullptr_code  # g_d2 without rvec
    assert bwd(None, i32(5), i64(10), None, None, None, fake(4), fake(1), fake(2), fake(3), None, fake(5)) == nullptr_code  # g_v without index arrays
    assert bwd(None, i32(5), i64(10), None, None, None, fake(4), fake(1), fake(2), fake(3), fake(3), None) == -2     # g_r_sum aliases g_r
    assert b"alias" in lib.hgnn_last_error_string()
    assert bwd(None, i32(5), i64(2 ** 31), None, None, None, fake(4), fake(1), fake(2), fake(3), None, None) == -7   # 3 E overflows
