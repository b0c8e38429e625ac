"""CPU fp64 oracle of one whole HSTU layer and its backward (paper Eq. 1-5 of the Background section and the
layer pseudocode of the appendix, "ULTRA-HSTU pseudocode with activation rematerialisation").

TEST INFRASTRUCTURE ONLY: imported by the tests and the smoke check, never by the product path.

Forward, for token rows Z [T, E] of a jagged batch:
    X      = LayerNorm_E(Z) * norm_w                                 (Eq. 1; weight only, as in the pseudocode)
    U,V,Q,K = SiLU(X W1^T), W1 [4 H d, E], output columns in the order U, V, Q, K     (Eq. 2; f1 one linear map)
    A      = attention(Q, K, V)                                      (Eq. 3, the attention oracle)
    Y      = LayerNorm_{Hd}(A) * gated_norm_w  (.)  U                (Eq. 4 before f2, the gated-norm oracle)
    out    = Y W2^T + Z, W2 [E, H d]                                 (f2 one linear map, Eq. 5 residual)
The backward is the chain rule taken step by step in the order of the pseudocode.  Rematerialisation changes what is
stored, not what is computed, so the oracle simply keeps every intermediate.  Weights follow the [out, in] layout.
The mathematics is the definition written out with numpy matmuls; the attention and the gated norm are the C oracle's.
"""
from __future__ import annotations

import numpy as np

from . import hstu_oracle as orc


def layer_norm_fwd(z, w, eps):
    """Row-wise layer norm with a weight and no bias: biased variance, eps inside the square root."""
    z = np.asarray(z, dtype=np.float64)
    mean = z.mean(axis=1)
    var = ((z - mean[:, None]) ** 2).mean(axis=1)
    rstd = 1.0 / np.sqrt(var + eps)
    return (z - mean[:, None]) * rstd[:, None] * np.asarray(w, dtype=np.float64)[None, :], mean, rstd


def layer_norm_bwd(dx, z, w, eps):
    """Gradient of layer_norm_fwd with respect to its input and its weight."""
    z, dx, w = (np.asarray(t, dtype=np.float64) for t in (z, dx, w))
    _, mean, rstd = layer_norm_fwd(z, w, eps)
    zhat = (z - mean[:, None]) * rstd[:, None]
    dzhat = dx * w[None, :]
    dz = rstd[:, None] * (dzhat - dzhat.mean(axis=1, keepdims=True) - zhat * (dzhat * zhat).mean(axis=1, keepdims=True))
    return dz, (dx * zhat).sum(axis=0)


def sigmoid(t):
    return 1.0 / (1.0 + np.exp(-t))


def layer_fwd(z, norm_w, w1, gated_norm_w, w2, offsets, H, d, *, norm_eps=1e-5, gated_eps=1e-5, pre_override=None, **attn):
    """Returns (out [T, E], intermediates dict).  ``attn``: keyword arguments of the attention oracle
    (num_targets, K1, K2, alpha, inv_n, table, bounds).  ``pre_override``: pre-activations [T, 4 H d] to use in place of
    X W1^T (the FP8 forward's, when the backward is to be taken at its activations)."""
    z = np.asarray(z, dtype=np.float64)
    w1, w2 = np.asarray(w1, dtype=np.float64), np.asarray(w2, dtype=np.float64)
    T = z.shape[0]
    HD = H * d
    assert w1.shape == (4 * HD, z.shape[1]) and w2.shape == (z.shape[1], HD)
    x, mean, rstd = layer_norm_fwd(z, norm_w, norm_eps)
    pre = x @ w1.T if pre_override is None else np.asarray(pre_override, dtype=np.float64)      # [T, 4 H d]
    act = pre * sigmoid(pre)
    u, v, q, k = (act[:, i * HD:(i + 1) * HD] for i in range(4))
    a = orc.attn_fwd(q.reshape(T, H, d), k.reshape(T, H, d), v.reshape(T, H, d), offsets, **attn).reshape(T, HD)
    y, _, _ = orc.gated_norm_fwd(a, u, gated_norm_w, None, gated_eps)
    out = y @ w2.T + z
    return out, dict(x=x, mean=mean, rstd=rstd, pre=pre, u=u, v=v, q=q, k=k, a=a, y=y)


def layer_bwd(z, norm_w, w1, gated_norm_w, w2, offsets, H, d, dout, *, norm_eps=1e-5, gated_eps=1e-5, pre_override=None, **attn):
    """Returns dict(dz, d_norm_w, d_w1, d_gated_norm_w, d_w2) for upstream gradient dout [T, E].  With ``pre_override`` the
    chain rule of the unquantised layer is evaluated at those pre-activations (backward of the FP8 forward with the
    quantisation treated as the identity)."""
    dout = np.asarray(dout, dtype=np.float64)
    w1, w2 = np.asarray(w1, dtype=np.float64), np.asarray(w2, dtype=np.float64)
    T = dout.shape[0]
    HD = H * d
    _, s = layer_fwd(z, norm_w, w1, gated_norm_w, w2, offsets, H, d, norm_eps=norm_eps, gated_eps=gated_eps,
                     pre_override=pre_override, **attn)
    dy = dout @ w2                                   # out = Y W2^T + Z
    d_w2 = dout.T @ s["y"]
    da, du, d_gw, _ = orc.gated_norm_bwd(dy, s["a"], s["u"], gated_norm_w, None, gated_eps)
    shp = (T, H, d)
    dq, dk, dv = orc.attn_bwd(s["q"].reshape(shp), s["k"].reshape(shp), s["v"].reshape(shp), da.reshape(shp), offsets, **attn)
    dact = np.concatenate([du, dv.reshape(T, HD), dq.reshape(T, HD), dk.reshape(T, HD)], axis=1)
    sg = sigmoid(s["pre"])
    dpre = dact * (sg * (1.0 + s["pre"] * (1.0 - sg)))     # d/dt [t sigmoid(t)]
    dx = dpre @ w1
    d_w1 = dpre.T @ s["x"]
    dz_norm, d_nw = layer_norm_bwd(dx, z, norm_w, norm_eps)
    return dict(dz=dz_norm + dout, d_norm_w=d_nw, d_w1=d_w1, d_gated_norm_w=d_gw, d_w2=d_w2)


def layer_fwd_fp8(z, norm_w, w1, gated_norm_w, w2, offsets, H, d, *, norm_eps=1e-5, gated_eps=1e-5, **attn):
    """The forward with both projections on row-wise quantised E4M3 operands (paper Section 4.2.2): X and Y are quantised
    per token row as they leave their norms, W1 and W2 per output feature, the products are taken on the decoded codes and
    rescaled, the residual Z enters the second projection as its two-dimensional additive operand.  Everything else as
    layer_fwd.  Returns (out, intermediates)."""
    from . import fp8
    z = np.asarray(z, dtype=np.float64)
    T, HD = z.shape[0], H * d
    x, mean, rstd = layer_norm_fwd(z, norm_w, norm_eps)
    xq, xs = fp8.rowwise_quant(x.astype(np.float32))
    w1q, w1s = fp8.rowwise_quant(np.asarray(w1, dtype=np.float32))
    pre = fp8.gemm_bias2d(xq, xs, w1q, w1s, None)
    act = pre * sigmoid(pre)
    u, v, q, k = (act[:, i * HD:(i + 1) * HD] for i in range(4))
    a = orc.attn_fwd(q.reshape(T, H, d), k.reshape(T, H, d), v.reshape(T, H, d), offsets, **attn).reshape(T, HD)
    y, _, _ = orc.gated_norm_fwd(a, u, gated_norm_w, None, gated_eps)
    yq, ys = fp8.rowwise_quant(y.astype(np.float32))
    w2q, w2s = fp8.rowwise_quant(np.asarray(w2, dtype=np.float32))
    out = fp8.gemm_bias2d(yq, ys, w2q, w2s, z)
    return out, dict(mean=mean, rstd=rstd, pre=pre, u=u, a=a, y=y)
