"""The gated-norm backward without a workspace (`hstu_gated_norm_bwd_static`, for callers that cannot allocate)
against `hstu_gated_norm_bwd`: same kernels, deterministic, so the outputs must be bit-identical; two calls in a row
on the library's own scratch array, the second on a smaller input (what the first call left there must not matter)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hb():
    assert torch.cuda.is_available(), "GPU tests need a GPU; deselect with -m 'not gpu'"
    from paper_2602_16986_amd import binding
    return binding


def _inputs(T, D, dtype, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    mk = lambda *s: torch.randn(*s, generator=g, dtype=torch.float32)
    a, u, dy = (mk(T, D) * 0.01).to(dtype), mk(T, D).to(dtype), mk(T, D).to(dtype)
    gamma, beta = 1 + 0.1 * mk(D), 0.1 * mk(D)
    return [t.to("cuda:0") for t in (a, u, dy, gamma, beta)]


def _both(hb, T, D, dtype, seed, use_beta):
    a, u, dy, gamma, beta = _inputs(T, D, dtype, seed)
    beta = beta if use_beta else None
    outs = []
    for static in (False, True):
        da, du = torch.full_like(a, float("nan")), torch.full_like(a, float("nan"))
        dg = torch.full((D,), float("nan"), dtype=torch.float32, device="cuda:0")
        db = torch.full((D,), float("nan"), dtype=torch.float32, device="cuda:0")
        if static:
            hb.hstu_gated_norm_bwd_static(dy, a, u, gamma, beta, 1e-5, da, du, dg, db)
        else:
            ws = hb.new_workspace(hb.hstu_gated_norm_bwd_workspace_bytes(T, D), "cuda:0")
            hb.hstu_gated_norm_bwd(dy, a, u, gamma, beta, 1e-5, da, du, dg, db, ws)
        torch.cuda.synchronize()
        outs.append((da, du, dg, db))
    for name, x, y in zip(("dA", "dU", "dgamma", "dbeta"), outs[0], outs[1]):
        assert torch.isfinite(x.float()).all(), name
        assert torch.equal(x, y), f"{name}: static-scratch variant differs from the workspace variant (T={T}, D={D})"


@pytest.mark.parametrize("dtype,D", [(torch.bfloat16, 1024), (torch.bfloat16, 256), (torch.float32, 520), (torch.bfloat16, 8192)])
def test_static_scratch_matches_workspace_variant(hb, dtype, D):
    assert hb.hstu_gated_norm_bwd_workspace_bytes(70000, D) <= hb.hstu_gated_norm_bwd_static_max_bytes()
    print(f"D={D} {dtype}: first call T=5000", flush=True)
    _both(hb, 5000, D, dtype, 1, True)          # many workgroups: fills a large part of the scratch array
    print(f"D={D} {dtype}: second call T=37", flush=True)
    _both(hb, 37, D, dtype, 2, False)           # smaller input right after: stale partial sums must not be read
    print(f"D={D} {dtype}: third call T=0", flush=True)
    _both(hb, 0, D, dtype, 3, True)


def test_static_scratch_rejects_bad_arguments(hb):
    a, u, dy, gamma, beta = _inputs(8, 256, torch.bfloat16, 0)
    with pytest.raises(hb.HstuError):
        hb.hstu_gated_norm_bwd_static(dy, a, u, gamma, None, 1e-5, None, None, None, None)
