"""Pins of the FP8 oracle (row-wise E4M3 quantisation and the projection with a two-dimensional additive operand,
paper Section 4.2.2 and its FP8 benchmark appendix) against the format's definition, brute force over all 256 codes,
torch's own float8_e4m3fn conversion on the CPU, and error bounds.  No GPU."""
import numpy as np
import pytest
import torch

from oracle import fp8


def test_decode_table_known_values():
    """Values fixed by the OCP FP8 E4M3 definition (bias 7, no infinities, S.1111.111 = NaN)."""
    v = fp8.e4m3_values()
    assert v[0x00] == 0.0 and v[0x80] == 0.0
    assert v[0x38] == 1.0 and v[0xB8] == -1.0           # 0.0111.000
    assert v[0x40] == 2.0 and v[0x3C] == 1.5
    assert v[0x01] == 2.0 ** -9 and v[0x07] == 7 * 2.0 ** -9
    assert v[0x08] == 2.0 ** -6                         # smallest normal
    assert v[0x7E] == 448.0 and v[0xFE] == -448.0       # largest finite
    assert np.isnan(v[0x7F]) and np.isnan(v[0xFF])
    assert np.count_nonzero(np.isnan(v)) == 2
    finite = np.sort(v[:0x7F])
    assert np.all(np.diff(finite) > 0)                  # positive codes are ordered


def test_encode_inverts_decode():
    codes = np.array([c for c in range(256) if c not in (0x7F, 0xFF)], dtype=np.uint8)
    back = fp8.e4m3_encode(fp8.e4m3_decode(codes).astype(np.float32))
    keep = codes != 0x80                                # -0 decodes to 0.0: the sign of zero is kept by signbit
    assert np.array_equal(back[keep], codes[keep])
    assert back[~keep][0] == 0x80


def brute_force_encode(x):
    vals = fp8.e4m3_values()
    pos = vals[:0x7F]                                   # codes 0..0x7E ascending
    out = np.empty(x.shape, dtype=np.uint8)
    for i, xv in enumerate(x):
        mag = min(abs(float(xv)), 448.0)
        d = np.abs(pos - mag)
        best = np.flatnonzero(d == d.min())
        code = best[0] if len(best) == 1 else [c for c in best if c % 2 == 0][0]     # tie: even mantissa
        out[i] = code | (0x80 if np.signbit(xv) else 0)
    return out


def test_encode_is_nearest_with_ties_to_even():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(3000) * 3, rng.standard_normal(2000) * 200, rng.standard_normal(2000) * 0.01,
                        rng.uniform(-2.0 ** -6, 2.0 ** -6, 1000)]).astype(np.float32)
    vals = fp8.e4m3_values()[:0x7F]
    mids = ((vals[:-1] + vals[1:]) / 2).astype(np.float32)          # exact ties (representable in fp32)
    x = np.concatenate([x, mids, -mids, np.array([448.0, 449.0, 1e6, -1e6, 463.9, 0.0], dtype=np.float32)])
    assert np.array_equal(fp8.e4m3_encode(x), brute_force_encode(x))


def test_encode_matches_torch_float8():
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(20000) * 50, rng.standard_normal(5000) * 0.02]).astype(np.float32)
    x = x[np.abs(x) <= 448.0]
    ref = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = fp8.e4m3_encode(x)
    same = got == ref
    zero = (fp8.e4m3_decode(got) == 0) & (fp8.e4m3_decode(ref) == 0)   # the sign of a rounded-to-zero value may differ
    assert np.all(same | zero)


def test_rowwise_quant_properties():
    rng = np.random.default_rng(2)
    x = (rng.standard_normal((64, 96)) * rng.uniform(0.01, 30, (64, 1))).astype(np.float32)
    x[5] = 0.0
    codes, scale = fp8.rowwise_quant(x)
    assert scale.dtype == np.float32 and scale[5] == 1.0 and not codes[5].any()
    deq = fp8.dequant(codes, scale)
    amax = np.abs(x).max(axis=1)
    # the largest element of a row lands on +-448; every element is within half a step of its value
    hit = np.abs(fp8.e4m3_decode(codes)).max(axis=1)
    assert np.all(hit[amax > 0] == 448.0)
    bound = np.maximum(np.abs(x) * 2.0 ** -4, scale[:, None] * 2.0 ** -10) * (1 + 1e-6)
    assert np.all(np.abs(deq - x) <= bound)
    # scaling a row by a power of two changes its scale and nothing else
    c2, s2 = fp8.rowwise_quant(x * np.float32(4.0))
    assert np.array_equal(c2, codes) and np.allclose(s2[amax > 0], 4 * scale[amax > 0], rtol=0)


def test_gemm_bias2d_exact_small_integers():
    """Operands whose quantisation is exact: the product must be the integer matrix product plus C."""
    a = np.array([[1, 2, 0, -4], [8, 0, 1, 2]], dtype=np.float32)
    b = np.array([[1, 1, 1, 1], [0, 2, -2, 0.5], [4, 0, 0, 0]], dtype=np.float32)
    c = np.array([[10, 20, 30], [-1, -2, -3]], dtype=np.float64)
    qa, sa = fp8.rowwise_quant(a)
    qb, sb = fp8.rowwise_quant(b)
    assert np.allclose(fp8.dequant(qa, sa), a, rtol=1e-7) and np.allclose(fp8.dequant(qb, sb), b, rtol=1e-7)
    d = fp8.gemm_bias2d(qa, sa, qb, sb, c)
    np.testing.assert_allclose(d, a.astype(np.float64) @ b.astype(np.float64).T + c, rtol=1e-6)


def test_gemm_bias2d_equals_product_of_dequantised_operands():
    rng = np.random.default_rng(3)
    a = rng.standard_normal((37, 64)).astype(np.float32)
    b = (rng.standard_normal((24, 64)) * 0.1).astype(np.float32)
    c = rng.standard_normal((37, 24))
    qa, sa = fp8.rowwise_quant(a)
    qb, sb = fp8.rowwise_quant(b)
    d = fp8.gemm_bias2d(qa, sa, qb, sb, c)
    ref = fp8.dequant(qa, sa) @ fp8.dequant(qb, sb).T + c
    np.testing.assert_allclose(d, ref, rtol=1e-12, atol=1e-12)
    # and it is close to the unquantised product: error of a K=64 dot product of 2^-4-accurate terms
    exact = a.astype(np.float64) @ b.astype(np.float64).T + c
    assert np.abs(d - exact).max() < 0.1 * np.abs(exact - c).max()
    assert np.array_equal(fp8.gemm_bias2d(qa, sa, qb, sb, None), d - c) or np.allclose(fp8.gemm_bias2d(qa, sa, qb, sb, None), d - c)


def test_norm_quant_matches_torch_layer_norm():
    rng = np.random.default_rng(4)
    a = rng.standard_normal((17, 40))
    u = rng.standard_normal((17, 40))
    g = 1 + 0.1 * rng.standard_normal(40)
    y, codes, scale = fp8.norm_quant(a, u, g, None, 1e-5)
    ref = torch.nn.functional.layer_norm(torch.tensor(a), (40,), weight=torch.tensor(g), eps=1e-5).numpy() * u
    np.testing.assert_allclose(y, ref, rtol=1e-10, atol=1e-12)
    c2, s2 = fp8.rowwise_quant(ref.astype(np.float32))
    assert np.array_equal(c2, codes) and np.array_equal(s2, scale)
