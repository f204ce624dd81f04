"""AdamW update: HIP kernel against the float64 oracle, element by element (needs a GPU)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _run(n, steps, seed, **hp):
    import torch
    from oracle.optim import adamw_step
    from paper_2506_21788_amd import binding as B
    rng = np.random.default_rng(seed)
    w0 = rng.standard_normal(n).astype(np.float32)
    w = torch.as_tensor(w0.copy()).cuda()
    m = torch.zeros(n, dtype=torch.float32, device="cuda")
    v = torch.zeros(n, dtype=torch.float32, device="cuda")
    wo, mo, vo = w0.astype(np.float64), np.zeros(n), np.zeros(n)
    mscale = np.zeros(n)   # what m would be if every gradient had the same sign: the scale its rounding errors have
    for t in range(1, steps + 1):
        # gradients over several orders of magnitude, some exactly zero
        g = (rng.standard_normal(n) * 10.0 ** rng.integers(-6, 1, size=n)).astype(np.float32)
        g[rng.random(n) < 0.05] = 0.0
        B.adamw_step(w, torch.as_tensor(g).cuda(), m, v, t, **hp)
        wo, mo, vo = adamw_step(wo, g.astype(np.float64), mo, vo, t, **hp)
        mscale = hp["beta1"] * mscale + (1 - hp["beta1"]) * np.abs(g)
    torch.cuda.synchronize()
    return w.cpu().numpy(), m.cpu().numpy(), v.cpu().numpy(), wo, mo, vo, mscale


def _check(w, m, v, wo, mo, vo, mscale):
    # fp32 arithmetic against fp64: a few ulp per update. m is a signed sum (its terms can cancel), so its error is
    # measured against the sum of the magnitudes; v is a sum of squares and w moves by at most ~lr per update.
    assert np.allclose(w, wo, rtol=2e-6, atol=1e-7)
    assert np.all(np.abs(m - mo) <= 1e-6 * mscale + 1e-30)
    assert np.allclose(v, vo, rtol=1e-5, atol=1e-30)


@pytest.mark.parametrize("n", [1, 3, 4, 5, 1023, 65537])
def test_adamw_matches_the_oracle_small(n):
    print(f"adamw n={n}", flush=True)
    _check(*_run(n, 6, seed=n, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01))


def test_adamw_full_model_size_and_other_constants():
    # all parameters of config 4 in one buffer: 6 layers of 6H^2+6H plus 5 heads of 2(H^2+2H+1), H = 256; ragged tail
    H = 256
    n = 6 * (6 * H * H + 6 * H) + 5 * 2 * (H * H + 2 * H + 1) + 3
    print(f"adamw n={n}", flush=True)
    _check(*_run(n, 3, seed=9, lr=3e-3, beta1=0.8, beta2=0.95, eps=1e-6, weight_decay=0.1))


def test_adamw_empty_and_error_paths():
    import torch
    from paper_2506_21788_amd import binding as B
    e = torch.zeros(0, dtype=torch.float32, device="cuda")
    B.adamw_step(e, e, e, e, 1)   # nothing to do
    w = torch.ones(8, dtype=torch.float32, device="cuda")
    with pytest.raises(RuntimeError):
        B.adamw_step(w, w.clone(), w.clone(), w.clone(), 0)          # updates count from 1
    with pytest.raises(RuntimeError):
        B.adamw_step(w, w.clone(), w.clone(), w.clone(), 1, beta1=1.0)
    torch.cuda.synchronize()
    assert torch.equal(w, torch.ones_like(w))
