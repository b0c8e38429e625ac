"""CPU oracle of the FP8 path around the layer's two projections (paper Section 4.2.2, "Mixed-Precision Training and
Inference", and the FP8 benchmarks of the appendix): row-wise scaling and quantisation of activations and weights to
8-bit floats, and the projection D = A B^T + C evaluated on the quantised operands with a two-dimensional additive
operand C (the residual).

TEST INFRASTRUCTURE ONLY: imported by the tests and the smoke check, never by the product path.

Format: OCP FP8 E4M3 ("e4m3fn"): 1 sign, 4 exponent bits (bias 7), 3 mantissa bits, no infinities, largest finite
value 448, subnormals in steps of 2^-9; the paper names H100's FP8 and states no format for the GEMM inputs; E4M3 is the
one with the precision that forward activations and weights need and the one gfx950's matrix cores take natively.
Row-wise scaling: one fp32 scale per row, scale = amax / 448 (a row of zeros gets scale 1), code = nearest E4M3 value
(ties to even) of x * (448 / amax).  Where floating point decides a code, the decision is taken in fp32 in exactly this
order of operations (one division per row, one multiplication per element), which is what the kernel does too; every
other quantity is fp64.
"""
from __future__ import annotations

import numpy as np

E4M3_MAX = 448.0


def e4m3_values() -> np.ndarray:
    """All 256 codes decoded (fp64); codes 0x7F and 0xFF are NaN."""
    out = np.empty(256, dtype=np.float64)
    for code in range(256):
        sign = -1.0 if code & 0x80 else 1.0
        e, m = (code >> 3) & 0xF, code & 0x7
        if e == 0xF and m == 0x7:
            out[code] = np.nan
        elif e == 0:
            out[code] = sign * m * 2.0 ** -9                    # subnormal: m/8 * 2^-6
        else:
            out[code] = sign * (1.0 + m / 8.0) * 2.0 ** (e - 7)
    return out


_DECODE = e4m3_values()


def e4m3_decode(codes) -> np.ndarray:
    return _DECODE[np.asarray(codes, dtype=np.uint8)]


def e4m3_encode(x) -> np.ndarray:
    """Nearest E4M3 code of each fp32 value, ties to the even mantissa, magnitudes beyond 448 saturate to 448.
    Written from the format's definition: pick the exponent bucket, round the scaled mantissa with numpy's rint
    (ties to even), carry into the next bucket when the mantissa overflows."""
    x = np.asarray(x, dtype=np.float32).astype(np.float64)
    sign = np.signbit(x)
    mag = np.minimum(np.abs(x), E4M3_MAX)
    # exponent of the bucket: normal numbers start at 2^-6; below that the step is that of the subnormals
    with np.errstate(divide="ignore"):
        e = np.floor(np.log2(np.where(mag > 0, mag, 1.0)))
    e = np.clip(e, -6, 8)
    step = 2.0 ** (e - 3)                                       # spacing of representable values in the bucket
    k = np.rint(mag / step)                                     # integer multiple of the step (8..16 for normals, 0..8 below)
    val = k * step
    # encode val (exactly representable now, possibly the first value of the next bucket)
    with np.errstate(divide="ignore"):
        e2 = np.floor(np.log2(np.where(val > 0, val, 1.0)))
    normal = val >= 2.0 ** -6
    e2 = np.where(normal, e2, -6)
    mant = np.where(normal, val / 2.0 ** e2 * 8.0 - 8.0, val / 2.0 ** -9)
    code = np.where(normal, ((e2 + 7).astype(np.int64) << 3) | mant.astype(np.int64), mant.astype(np.int64))
    code = code | (sign.astype(np.int64) << 7)
    return code.astype(np.uint8)


def rowwise_quant(x):
    """x [R, C] (values exactly representable in fp32) -> (codes uint8 [R, C], scale fp32 [R])."""
    x = np.asarray(x, dtype=np.float32)
    amax = np.abs(x).max(axis=1) if x.shape[1] else np.zeros(x.shape[0], dtype=np.float32)
    amax = amax.astype(np.float32)
    safe = np.where(amax > 0, amax, np.float32(E4M3_MAX)).astype(np.float32)
    scale = (safe / np.float32(E4M3_MAX)).astype(np.float32)            # fp32 division
    inv = (np.float32(E4M3_MAX) / safe).astype(np.float32)              # fp32 division
    scaled = (x * inv[:, None]).astype(np.float32)                      # fp32 multiplication
    return e4m3_encode(scaled), scale


def dequant(codes, scale):
    return e4m3_decode(codes) * np.asarray(scale, dtype=np.float64)[:, None]


def gemm_bias2d(a_codes, a_scale, b_codes, b_scale, c=None):
    """D [M, N] = (A_q B_q^T) * a_scale[m] * b_scale[n] + C, A_q [M, K], B_q [N, K] E4M3 codes, everything in fp64."""
    a = e4m3_decode(a_codes)
    b = e4m3_decode(b_codes)
    d = (a @ b.T) * np.asarray(a_scale, dtype=np.float64)[:, None] * np.asarray(b_scale, dtype=np.float64)[None, :]
    return d if c is None else d + np.asarray(c, dtype=np.float64)


def norm_quant(a, u, gamma, beta=None, eps=1e-5):
    """Row-wise quantisation fused behind the (optionally gated) layer norm of Eq. 1 / Eq. 4: returns the fp64 norm
    output y, and the codes and scales of y taken through fp32 as rowwise_quant does."""
    a = np.asarray(a, dtype=np.float64)
    mean = a.mean(axis=1, keepdims=True)
    var = ((a - mean) ** 2).mean(axis=1, keepdims=True)
    y = (a - mean) / np.sqrt(var + eps) * np.asarray(gamma, dtype=np.float64)[None, :]
    if beta is not None:
        y = y + np.asarray(beta, dtype=np.float64)[None, :]
    if u is not None:
        y = y * np.asarray(u, dtype=np.float64)
    codes, scale = rowwise_quant(y.astype(np.float32))
    return y, codes, scale
