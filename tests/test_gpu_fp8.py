"""Parity of the FP8 entry points (row-wise E4M3 quantisation, alone and fused behind the norms; projection on quantised
operands with a two-dimensional additive operand) against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import fp8 as orc
from paper_2602_16986_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def hb():
    assert torch.cuda.is_available(), "GPU tests need a GPU; deselect with -m 'not gpu'"
    from paper_2602_16986_amd import binding
    return binding


def bf16_dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).to(DEV).to(torch.bfloat16)


def gpu_quant(hb, x, u=None, gamma=None, eps=1e-5, dtype=torch.bfloat16):
    xt = torch.from_numpy(np.ascontiguousarray(x)).to(DEV).to(dtype)
    ut = None if u is None else torch.from_numpy(np.ascontiguousarray(u)).to(DEV).to(dtype)
    gt = None if gamma is None else torch.from_numpy(gamma.astype(np.float32)).to(DEV)
    q = torch.full(x.shape, 0x7F, dtype=torch.uint8, device=DEV)
    s = torch.full((x.shape[0],), float("nan"), dtype=torch.float32, device=DEV)
    hb.hstu_norm_quant_fp8(xt, ut, gt, None, eps, q, s)
    torch.cuda.synchronize()
    return q.cpu().numpy(), s.cpu().numpy()


@pytest.mark.parametrize("shape", [(1000, 512), (37, 64), (513, 1024), (64, 8), (5, 2056)])
def test_rowwise_quant_bit_exact(hb, shape):
    """bf16 rows in, codes and scales out: the inputs are exact in fp32, so are amax, the two divisions and the product;
    every code and every scale must equal the oracle's bit for bit."""
    rng = np.random.default_rng(shape[0])
    x = wl.round_to_bf16((rng.standard_normal(shape) * rng.uniform(1e-3, 50, (shape[0], 1))).astype(np.float32))
    x[shape[0] // 2] = 0.0                                   # a row of zeros
    x[0, : min(8, shape[1])] = [448, -448, 1e-4, 0, 3, 2.5, -0.0, 100][: min(8, shape[1])]
    x = wl.round_to_bf16(x)
    print(f"row-wise quantisation {shape}", flush=True)
    codes, scale = gpu_quant(hb, x)
    ref_codes, ref_scale = orc.rowwise_quant(x)
    assert np.array_equal(scale.view(np.uint32), ref_scale.view(np.uint32)), "scales"
    same = codes == ref_codes
    both_zero = (orc.e4m3_decode(codes) == 0) & (orc.e4m3_decode(ref_codes) == 0)      # sign of an exact zero
    assert np.all(same | both_zero), f"{np.count_nonzero(~(same | both_zero))} codes differ"


def test_rowwise_quant_fp32_input_bit_exact(hb):
    rng = np.random.default_rng(5)
    x = (rng.standard_normal((300, 256)) * 7).astype(np.float32)
    codes, scale = gpu_quant(hb, x, dtype=torch.float32)
    ref_codes, ref_scale = orc.rowwise_quant(x)
    assert np.array_equal(scale, ref_scale) and np.array_equal(codes, ref_codes)


@pytest.mark.parametrize("gated", [False, True])
def test_norm_quant_fused(hb, gated):
    """Quantisation fused behind the (gated) norm.  The norm's fp32 result differs from the oracle's fp64 one in the last
    bits, so a code may fall on the other side of a rounding boundary: scales agree to fp32 accuracy, the dequantised rows
    are within one E4M3 step of the oracle's, almost all codes are equal, and both are within the format's error of y."""
    rng = np.random.default_rng(11)
    T, D = 777, 512
    a = wl.round_to_bf16(rng.standard_normal((T, D)).astype(np.float32) * 0.3 + 0.1)
    u = wl.round_to_bf16(rng.standard_normal((T, D)).astype(np.float32)) if gated else None
    g = (1 + 0.1 * rng.standard_normal(D)).astype(np.float32)
    codes, scale = gpu_quant(hb, a, u, g)
    y, ref_codes, ref_scale = orc.norm_quant(a, u, g, None, 1e-5)
    assert np.allclose(scale, ref_scale, rtol=2e-6, atol=0)
    deq, ref_deq = orc.dequant(codes, scale), orc.dequant(ref_codes, ref_scale)
    step = np.maximum(np.abs(ref_deq) * 2.0 ** -3, ref_scale[:, None].astype(np.float64) * 2.0 ** -9)   # spacing at that value
    assert np.all(np.abs(deq - ref_deq) <= step * 1.001)
    frac = np.mean(codes == ref_codes)
    print(f"  fused norm + quantisation (gated={gated}): {100 * frac:.3f} % of the codes equal the oracle's", flush=True)
    assert frac > 0.995
    assert np.all(np.abs(deq - y) <= np.maximum(np.abs(y) * 2.0 ** -4, scale[:, None] * 2.0 ** -10) * 1.01 + 1e-6)


def run_gemm(hb, M, N, K, with_c=True, in_place=False, rows=None):
    a, b, c = wl.fp8_gemm_inputs(M, N, K, seed=M % 97 + N + K, with_c=with_c)
    print(f"fp8 gemm M={M} N={N} K={K} c={'yes' if with_c else 'no'} in_place={in_place}", flush=True)
    qa = torch.empty((M, K), dtype=torch.uint8, device=DEV)
    sa = torch.empty(M, dtype=torch.float32, device=DEV)
    qb = torch.empty((N, K), dtype=torch.uint8, device=DEV)
    sb = torch.empty(N, dtype=torch.float32, device=DEV)
    hb.hstu_norm_quant_fp8(bf16_dev(a), None, None, None, 0.0, qa, sa)
    hb.hstu_norm_quant_fp8(bf16_dev(b), None, None, None, 0.0, qb, sb)
    ct = None if c is None else bf16_dev(c)
    d = ct if in_place else torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
    hb.hstu_fp8_gemm_bias2d(qa, sa, qb, sb, ct, d)
    torch.cuda.synchronize()
    sel = slice(None) if rows is None else rows
    idx = slice(None) if rows is None else torch.from_numpy(rows).to(DEV)
    ref = orc.gemm_bias2d(qa[idx].cpu().numpy(), sa[idx].cpu().numpy(), qb.cpu().numpy(), sb.cpu().numpy(), None if c is None else c[sel])
    got = d[idx].float().cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got))
    err = np.abs(got - ref).max() / np.abs(ref).max()
    print(f"  normalised max error {err:.3e}", flush=True)
    assert err <= 1e-2                                        # one bf16 rounding of the result (2^-9 of its magnitude)
    # the quantised operands themselves are the oracle's (bit-exact test above), so this also bounds the whole op
    return err


@pytest.mark.parametrize("M,N,K", [(1000, 512, 512), (129, 64, 128), (4097, 192, 256), (300, 1024, 1024), (1, 128, 512)])
def test_fp8_gemm_bias2d(hb, M, N, K):
    run_gemm(hb, M, N, K)


def test_fp8_gemm_without_c_and_in_place(hb):
    run_gemm(hb, 700, 256, 512, with_c=False)
    run_gemm(hb, 700, 256, 512, in_place=True)


def test_fp8_gemm_rejects_unsupported_shapes(hb):
    qa = torch.zeros((8, 96), dtype=torch.uint8, device=DEV)
    with pytest.raises(hb.HstuError):
        hb.hstu_fp8_gemm_bias2d(qa, torch.ones(8, device=DEV), torch.zeros((64, 96), dtype=torch.uint8, device=DEV),
                                torch.ones(64, device=DEV), None, torch.zeros((8, 64), dtype=torch.bfloat16, device=DEV))


def test_fp8_gemm_paper_shape_sampled_rows(hb):
    """(m, k = n) = (250K, 512), one of the paper's table rows: sampled output rows against the oracle."""
    rng = np.random.default_rng(0)
    M = 250_000
    rows = np.sort(np.concatenate([rng.choice(M, size=2000, replace=False), [0, M - 1, M - 2]]))
    run_gemm(hb, M, 512, 512, rows=np.unique(rows))
