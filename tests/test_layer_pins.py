"""Pins of the whole-layer oracle (paper Eq. 1-5 and the layer pseudocode of the appendix) against torch on the CPU in
fp64: the forward against a formulation built from torch.nn.functional.layer_norm / silu / matmul and the dense
masked-attention formulation of the attention pins, every gradient against torch autograd through that formulation,
and a directional central difference through the oracle's own forward.  No GPU."""
import numpy as np
import pytest
import torch

from oracle import layer as lorc
from paper_2602_16986_amd import workloads as wl
from tests.test_oracle_pins import dense_attention_torch

F = torch.nn.functional


def tiny_layer(seed, lengths, H=2, d=8, E=12, **kw):
    c = wl.build_layer("tiny", lengths, H, d, E, "fp32", seed=seed, **kw)
    return c


def attn_kw(c):
    return dict(num_targets=c.num_targets, K1=c.K1, K2=c.K2, alpha=c.alpha, inv_n=1.0 / c.N, table=c.table, bounds=c.bounds)


class _AttnView:
    """What dense_attention_torch reads from a workload."""
    def __init__(self, c):
        self.B, self.offsets, self.num_targets, self.H, self.d = c.B, c.offsets, c.num_targets, c.H, c.d
        self.K1, self.K2, self.alpha, self.N, self.table, self.bounds = c.K1, c.K2, c.alpha, c.N, c.table, c.bounds


def torch_layer(c, z, norm_w, w1, gw, w2):
    T, HD = z.shape[0], c.H * c.d
    x = F.layer_norm(z, (c.E,), weight=norm_w, bias=None, eps=c.eps)
    act = F.silu(x @ w1.T)
    u, v, q, k = act.split(HD, dim=1)
    shp = (T, c.H, c.d)
    a = dense_attention_torch(_AttnView(c), q.reshape(shp), k.reshape(shp), v.reshape(shp)).reshape(T, HD)
    y = F.layer_norm(a, (HD,), weight=gw, bias=None, eps=c.eps) * u
    return y @ w2.T + z


CASES = [
    dict(lengths=[7, 0, 13, 1]),
    dict(lengths=[19, 5], K1=4, K2=3),
    dict(lengths=[12, 9, 30], K1=5, K2=2, num_targets=[4, 9, 7]),
    dict(lengths=[23], K1=0, K2=5, bias=False),
]


@pytest.mark.parametrize("i", range(len(CASES)))
def test_layer_forward_and_gradients_match_torch_autograd(i):
    c = tiny_layer(i, **CASES[i])
    f64 = lambda a: torch.tensor(np.asarray(a, dtype=np.float64), requires_grad=True)
    z, nw, w1, gw, w2 = f64(c.z), f64(c.norm_w), f64(c.w1), f64(c.gated_norm_w), f64(c.w2)
    out_t = torch_layer(c, z, nw, w1, gw, w2)
    out_t.backward(torch.tensor(c.dout.astype(np.float64)))
    out, _ = lorc.layer_fwd(c.z, c.norm_w, c.w1, c.gated_norm_w, c.w2, c.offsets, c.H, c.d, norm_eps=c.eps, gated_eps=c.eps,
                            **attn_kw(c))
    np.testing.assert_allclose(out, out_t.detach().numpy(), rtol=1e-10, atol=1e-11)
    g = lorc.layer_bwd(c.z, c.norm_w, c.w1, c.gated_norm_w, c.w2, c.offsets, c.H, c.d, c.dout, norm_eps=c.eps,
                       gated_eps=c.eps, **attn_kw(c))
    for name, ref in (("dz", z.grad), ("d_norm_w", nw.grad), ("d_w1", w1.grad), ("d_gated_norm_w", gw.grad), ("d_w2", w2.grad)):
        np.testing.assert_allclose(g[name], ref.numpy(), rtol=1e-9, atol=1e-10, err_msg=name)


def test_layer_gradient_by_central_differences():
    """<grad, direction> against (f(p + h dir) - f(p - h dir)) / 2h of the scalar <out, dout>, for every parameter."""
    c = tiny_layer(9, lengths=[11, 6], K1=3, K2=2)
    kw = dict(norm_eps=c.eps, gated_eps=c.eps, **attn_kw(c))
    params = dict(dz=c.z.astype(np.float64), d_norm_w=c.norm_w.astype(np.float64), d_w1=c.w1.astype(np.float64),
                  d_gated_norm_w=c.gated_norm_w.astype(np.float64), d_w2=c.w2.astype(np.float64))
    order = ["dz", "d_norm_w", "d_w1", "d_gated_norm_w", "d_w2"]

    def scalar(p):
        out, _ = lorc.layer_fwd(p["dz"], p["d_norm_w"], p["d_w1"], p["d_gated_norm_w"], p["d_w2"], c.offsets, c.H, c.d, **kw)
        return float((out * c.dout).sum())

    g = lorc.layer_bwd(*(params[n] for n in order), c.offsets, c.H, c.d, c.dout, **kw)
    rng = np.random.default_rng(0)
    for name in order:
        direction = rng.standard_normal(params[name].shape)
        h = 1e-5
        plus, minus = dict(params), dict(params)
        plus[name] = params[name] + h * direction
        minus[name] = params[name] - h * direction
        fd = (scalar(plus) - scalar(minus)) / (2 * h)
        an = float((g[name] * direction).sum())
        assert an == pytest.approx(fd, rel=2e-6, abs=1e-8), name


def test_layer_output_column_order_is_u_v_q_k():
    """Swapping the Q and K blocks of W1 transposes the score matrix: with a causal mask the output changes, so the
    order of the four blocks is observable; swapping them back in the reference restores agreement."""
    c = tiny_layer(3, lengths=[9, 4])
    HD = c.H * c.d
    swapped = np.concatenate([c.w1[:2 * HD], c.w1[3 * HD:], c.w1[2 * HD:3 * HD]])
    kw = dict(norm_eps=c.eps, gated_eps=c.eps, **attn_kw(c))
    a, _ = lorc.layer_fwd(c.z, c.norm_w, c.w1, c.gated_norm_w, c.w2, c.offsets, c.H, c.d, **kw)
    b, s = lorc.layer_fwd(c.z, c.norm_w, swapped, c.gated_norm_w, c.w2, c.offsets, c.H, c.d, **kw)
    assert np.abs(a - b).max() > 1e-3
    t64 = lambda t: torch.tensor(np.asarray(t, dtype=np.float64))
    ref = torch_layer(c, t64(c.z), t64(c.norm_w), t64(swapped), t64(c.gated_norm_w), t64(c.w2)).numpy()
    np.testing.assert_allclose(b, ref, rtol=1e-10, atol=1e-11)
    # the rows of W1 that produce U gate the output: zeroing them zeroes Y, leaving the residual
    no_gate = c.w1.copy()
    no_gate[:HD] = 0
    r, _ = lorc.layer_fwd(c.z, c.norm_w, no_gate, c.gated_norm_w, c.w2, c.offsets, c.H, c.d, **kw)
    np.testing.assert_allclose(r, c.z, atol=1e-12)


def test_empty_batch():
    c = wl.build_layer("empty", [0, 0], 2, 8, 12, "fp32")
    kw = dict(norm_eps=c.eps, gated_eps=c.eps, **attn_kw(c))
    out, _ = lorc.layer_fwd(c.z, c.norm_w, c.w1, c.gated_norm_w, c.w2, c.offsets, c.H, c.d, **kw)
    assert out.shape == (0, 12)


def torch_fp8_rows(t):
    """Row-wise E4M3 fake quantisation with torch's own float8 conversion: dequantised rows (fp64)."""
    t32 = t.to(torch.float32)
    amax = t32.abs().amax(dim=1, keepdim=True)
    safe = torch.where(amax > 0, amax, torch.full_like(amax, 448.0))
    q = (t32 * (torch.tensor(448.0) / safe)).to(torch.float8_e4m3fn).to(torch.float64)
    return q * (safe / torch.tensor(448.0)).to(torch.float64)


@pytest.mark.parametrize("i", [0, 2])
def test_fp8_forward_matches_torch_fake_quantisation(i):
    """The FP8 forward against the same layer written with torch ops, the quantised operands produced by torch's
    float8_e4m3fn conversion (dequantised, then an ordinary fp64 matmul)."""
    c = tiny_layer(i, E=16, **CASES[i])
    t64 = lambda a: torch.tensor(np.asarray(a, dtype=np.float64))
    z, nw, w1, gw, w2 = t64(c.z), t64(c.norm_w), t64(c.w1), t64(c.gated_norm_w), t64(c.w2)
    T, HD = z.shape[0], c.H * c.d
    x = F.layer_norm(z, (c.E,), weight=nw, eps=c.eps)
    act = F.silu(torch_fp8_rows(x) @ torch_fp8_rows(w1).T)
    u, v, q, k = act.split(HD, dim=1)
    shp = (T, c.H, c.d)
    a = dense_attention_torch(_AttnView(c), q.reshape(shp), k.reshape(shp), v.reshape(shp)).reshape(T, HD)
    y = F.layer_norm(a, (HD,), weight=gw, eps=c.eps) * u
    ref = torch_fp8_rows(y) @ torch_fp8_rows(w2).T + z
    out, _ = lorc.layer_fwd_fp8(c.z, c.norm_w, c.w1, c.gated_norm_w, c.w2, c.offsets, c.H, c.d, norm_eps=c.eps, gated_eps=c.eps,
                                **attn_kw(c))
    np.testing.assert_allclose(out, ref.numpy(), rtol=1e-9, atol=1e-10)
    # and it stays within the format's error of the unquantised layer
    exact, _ = lorc.layer_fwd(c.z, c.norm_w, c.w1, c.gated_norm_w, c.w2, c.offsets, c.H, c.d, norm_eps=c.eps, gated_eps=c.eps,
                              **attn_kw(c))
    assert np.abs(out - exact).max() < 0.15 * np.abs(exact - c.z).max()
    assert np.abs(out - exact).max() > 0


def test_backward_at_the_fp8_forward_activations():
    """Backward of the FP8 forward with the quantisation treated as the identity: torch autograd through the unquantised
    layer whose first projection is overridden in value (x W1^T + (pre_fp8 - x W1^T).detach()) gives the same gradients."""
    c = tiny_layer(2, E=16, **CASES[2])
    kw = dict(norm_eps=c.eps, gated_eps=c.eps, **attn_kw(c))
    _, sf = lorc.layer_fwd_fp8(c.z, c.norm_w, c.w1, c.gated_norm_w, c.w2, c.offsets, c.H, c.d, **kw)
    g = lorc.layer_bwd(c.z, c.norm_w, c.w1, c.gated_norm_w, c.w2, c.offsets, c.H, c.d, c.dout, pre_override=sf["pre"], **kw)
    f64 = lambda a: torch.tensor(np.asarray(a, dtype=np.float64), requires_grad=True)
    z, nw, w1, gw, w2 = f64(c.z), f64(c.norm_w), f64(c.w1), f64(c.gated_norm_w), f64(c.w2)
    T, HD = z.shape[0], c.H * c.d
    x = F.layer_norm(z, (c.E,), weight=nw, eps=c.eps)
    plain = x @ w1.T
    pre = plain + (torch.tensor(sf["pre"]) - plain).detach()
    act = F.silu(pre)
    u, v, q, k = act.split(HD, dim=1)
    shp = (T, c.H, c.d)
    a = dense_attention_torch(_AttnView(c), q.reshape(shp), k.reshape(shp), v.reshape(shp)).reshape(T, HD)
    out = (F.layer_norm(a, (HD,), weight=gw, eps=c.eps) * u) @ w2.T + z
    out.backward(torch.tensor(c.dout.astype(np.float64)))
    for name, ref in (("dz", z.grad), ("d_norm_w", nw.grad), ("d_w1", w1.grad), ("d_gated_norm_w", gw.grad), ("d_w2", w2.grad)):
        np.testing.assert_allclose(g[name], ref.numpy(), rtol=1e-9, atol=1e-10, err_msg=name)
