"""The embedding gradient through the entry point that allocates nothing (its scratch is an array built into the
library) against the entry point that takes a workspace: same kernels, so the results must agree bit for bit. Two calls
in a row, the second on a smaller input, because every call on a GPU shares the one array (needs a GPU)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _both(N, H, seed):
    import torch
    from paper_2506_21788_amd import binding as B
    rng = np.random.default_rng(seed)
    Z = torch.as_tensor(rng.integers(0, B.ZMAX + 1, size=N).astype(np.int32)).cuda()
    g_h = torch.as_tensor(rng.standard_normal((N, H)).astype(np.float32)).cuda()
    ws = torch.empty(max(B.embed_bwd_workspace_bytes(N, H), 16), dtype=torch.uint8, device="cuda")
    want = torch.full((B.ZMAX + 1, H), float("nan"), dtype=torch.float32, device="cuda")
    got = torch.full_like(want, float("nan"))
    B.embed_bwd(N, H, Z, g_h, want, ws)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    B.embed_bwd_static(N, H, Z, g_h, got)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return got.cpu().numpy(), want.cpu().numpy(), Z.cpu().numpy(), g_h.cpu().numpy()


@pytest.mark.parametrize("H", [256, 100])
def test_no_alloc_embedding_gradient_two_calls_in_a_row(H):
    import oracle
    from parity_util import TOL, relerr
    for N, seed in ((70001, 1), (3000, 2), (1, 3), (0, 4)):      # the later calls reuse the array the first one filled
        print("embed_bwd_static", N, H, flush=True)
        got, want, Z, g_h = _both(N, H, seed)
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), (N, H)
        assert relerr(got, oracle.embed_bwd(Z, g_h, got.shape[0])) <= TOL["f32"]["grad"]


def test_no_alloc_embedding_gradient_rejects_sizes_beyond_its_array():
    import torch
    from paper_2506_21788_amd import binding as B
    N, H = 400000, 256
    assert B.embed_bwd_workspace_bytes(N, H) > B.EMBED_BWD_STATIC_MAX_BYTES
    Z = torch.zeros(N, dtype=torch.int32, device="cuda")
    g_h = torch.zeros((16, H), dtype=torch.float32, device="cuda")      # never read: the call must fail on the host
    g_emb = torch.zeros((B.ZMAX + 1, H), dtype=torch.float32, device="cuda")
    with pytest.raises(B.HgnnError) as e:
        B.embed_bwd_static(N, H, Z, g_h, g_emb)
    assert e.value.code == -6 and "scratch" in str(e.value)
    # the largest size it accepts at this width still works
    n_ok = (B.EMBED_BWD_STATIC_MAX_BYTES // ((B.ZMAX + 1) * H * 4)) * 2048
    assert B.embed_bwd_workspace_bytes(n_ok, H) <= B.EMBED_BWD_STATIC_MAX_BYTES
    got, want, _, _ = _both(n_ok, H, 5)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
