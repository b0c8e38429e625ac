"""Parity of the whole-layer entry points (hstu_layer_fwd / hstu_layer_bwd, through the C ABI) against the CPU fp64
layer oracle on the same seeded inputs.  bf16 storage of every activation: tolerance 2e-2 on the max error normalised
by the largest reference magnitude, as for the attention kernels."""
import numpy as np
import pytest
import torch

from oracle import layer as lorc
from paper_2602_16986_amd import workloads as wl

pytestmark = pytest.mark.gpu
TOL = 2e-2


@pytest.fixture(scope="module")
def hb():
    assert torch.cuda.is_available(), "GPU tests need a GPU; deselect with -m 'not gpu'"
    from paper_2602_16986_amd import binding
    return binding


def f64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def check(name, got, ref, tol=TOL):
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    if ref.size == 0:
        return
    assert np.all(np.isfinite(got)), f"{name}: non-finite values"
    err = np.abs(got - ref).max()
    scale = np.abs(ref).max()
    rel = err / scale if scale > 0 else err
    print(f"  {name}: max_abs_err={err:.3e} max|ref|={scale:.3e} normalised={rel:.3e}", flush=True)
    assert rel <= tol, f"{name}: normalised max error {rel:.3e} > {tol}"


def attn_kw(c):
    return dict(num_targets=c.num_targets, K1=c.K1, K2=c.K2, alpha=c.alpha, inv_n=1.0 / c.N, table=c.table, bounds=c.bounds)


def run_case(c):
    from paper_2602_16986_amd.runner import DeviceLayer
    print(f"layer case {c.name}: lengths={c.lengths.tolist()} H={c.H} d={c.d} E={c.E} K1={c.K1} K2={c.K2} "
          f"targets={None if c.num_targets is None else c.num_targets.tolist()}", flush=True)
    dl = DeviceLayer(c)
    for t in (dl.out, dl.u_saved, dl.attn_saved, dl.dz, dl.d_norm_w, dl.d_w1, dl.d_gated_norm_w, dl.d_w2):
        t.fill_(float("nan"))
    dl.fwd()
    torch.cuda.synchronize()
    kw = dict(norm_eps=c.eps, gated_eps=c.eps, **attn_kw(c))
    ref_out, s = lorc.layer_fwd(c.z, c.norm_w, c.w1, c.gated_norm_w, c.w2, c.offsets, c.H, c.d, **kw)
    check("out", f64(dl.out), ref_out)
    check("U (saved)", f64(dl.u_saved), s["u"])
    check("A (saved)", f64(dl.attn_saved), s["a"])
    check("mean", f64(dl.mean), s["mean"], 1e-5)
    check("rstd", f64(dl.rstd), s["rstd"], 1e-5)
    dl.bwd()
    torch.cuda.synchronize()
    g = lorc.layer_bwd(c.z, c.norm_w, c.w1, c.gated_norm_w, c.w2, c.offsets, c.H, c.d, c.dout, **kw)
    check("dZ", f64(dl.dz), g["dz"])
    check("d norm_w", f64(dl.d_norm_w), g["d_norm_w"])
    check("d W1", f64(dl.d_w1), g["d_w1"])
    check("d gated_norm_w", f64(dl.d_gated_norm_w), g["d_gated_norm_w"])
    check("d W2", f64(dl.d_w2), g["d_w2"])
    return dl


@pytest.mark.parametrize("name", wl.LAYER_SMALL)
def test_layer_small(hb, name):
    run_case(wl.layer_case(name))


def test_layer_mid(hb):
    """Four sequences of 1024..2048 tokens, H=4, d=128, E=512: the layer shape of the benchmark at a size the oracle
    finishes in seconds."""
    run_case(wl.layer_case("layer-mid"))


def test_layer_backward_twice_is_identical(hb):
    """The backward rebuilds its intermediates from (Z, U, A, statistics) alone: a second call after unrelated work in
    the same workspace returns bit-identical gradients (attention and norms are deterministic, the GEMM plans are fixed)."""
    from paper_2602_16986_amd.runner import DeviceLayer
    dl = DeviceLayer(wl.layer_case("layer-small-sparse-targets"))
    dl.fwd()
    dl.bwd()
    first = [t.clone() for t in (dl.dz, dl.d_norm_w, dl.d_w1, dl.d_gated_norm_w, dl.d_w2)]
    dl.ws_bwd.fill_(0x5A)
    dl.bwd()
    torch.cuda.synchronize()
    for a, b in zip(first, (dl.dz, dl.d_norm_w, dl.d_w1, dl.d_gated_norm_w, dl.d_w2)):
        assert torch.equal(a, b)


def test_layer_empty_batch(hb):
    from paper_2602_16986_amd.runner import DeviceLayer
    dl = DeviceLayer(wl.build_layer("empty", [0, 0], 2, 64, 96))
    for t in (dl.d_norm_w, dl.d_w1, dl.d_gated_norm_w, dl.d_w2):
        t.fill_(float("nan"))
    dl.fwd()
    dl.bwd()
    torch.cuda.synchronize()
    for t in (dl.d_norm_w, dl.d_w1, dl.d_gated_norm_w, dl.d_w2):
        assert not t.any()


def test_layer_rejects_fp32_and_small_workspace(hb):
    from paper_2602_16986_amd.runner import DeviceLayer
    dl = DeviceLayer(wl.layer_case("layer-small-dense"))
    with pytest.raises(hb.HstuError):
        hb.hstu_layer_fwd(dl.problem, dl.z, dl.out, dl.u_saved, dl.attn_saved, dl.mean, dl.rstd, dl.ws_fwd[:4096])
    dl.problem.params.attn.dtype = hb.HSTU_FP32
    with pytest.raises(hb.HstuError):
        dl.fwd()
