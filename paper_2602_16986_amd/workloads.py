"""Seeded synthetic jagged batches shaped like the paper's long user histories.

This module holds input generation only: sequence lengths, random tensors,
bucket lower bounds and the rounding of inputs to the storage type.  None of
the layer's arithmetic lives here, so the CPU oracle's tests and the HIP path's
tests can both draw their inputs from it without sharing any method code.

The paper's workload is a private industrial one (user interaction histories
of 3,072 to 16,384 events, Section 5.1; 16k x 18 layers in production,
Section 1); these batches stand in for it.  One ``numpy.random.default_rng``
stream per workload, draw order: lengths, Q, K, V, U, bias table, gamma, dO, dY.
"""
from __future__ import annotations

import dataclasses
from typing import Optional

import numpy as np

NUM_BUCKETS = 128
MAX_DISTANCE = 65536


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def fp32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Upper 16 bits of already bf16-representable fp32 values, as uint16."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_fp32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def log_bucket_bounds(num_buckets: int = NUM_BUCKETS, max_distance: int = MAX_DISTANCE) -> np.ndarray:
    """Integer lower bounds of log-spaced distance buckets.

    bounds[0] = 0 and bounds[b] = max(b, floor(max_distance**(b/num_buckets))),
    strictly increasing.  Distances at or beyond the last bound share the last
    bucket.  The bounds are data handed to both implementations, so neither
    evaluates a logarithm.
    """
    b = np.arange(num_buckets, dtype=np.float64)
    geo = np.floor(np.exp(b * np.log(float(max_distance)) / num_buckets)).astype(np.int64)
    bounds = np.maximum(np.arange(num_buckets, dtype=np.int64), geo)
    bounds[0] = 0
    for i in range(1, num_buckets):  # enforce strict monotonicity
        if bounds[i] <= bounds[i - 1]:
            bounds[i] = bounds[i - 1] + 1
    return bounds.astype(np.int32)


@dataclasses.dataclass
class Workload:
    name: str
    dtype: str                      # "bf16" or "fp32": storage type of q,k,v,u,out,grads
    lengths: np.ndarray             # int32[B]
    offsets: np.ndarray             # int32[B+1]
    num_targets: Optional[np.ndarray]  # int32[B] or None
    H: int
    d: int
    K1: int                         # local window; <0 = dense causal, 0 = no local keys
    K2: int                         # global prefix
    alpha: float
    N: float                        # normaliser; kernels take 1/N
    q: np.ndarray                   # fp32 [T,H,d], already rounded to dtype
    k: np.ndarray
    v: np.ndarray
    u: np.ndarray
    table: Optional[np.ndarray]     # fp32 [H,NUM_BUCKETS] or None
    bounds: Optional[np.ndarray]    # int32 [NUM_BUCKETS] or None
    gamma: np.ndarray               # fp32 [H*d]
    dout: np.ndarray                # fp32 [T,H,d], gradient w.r.t. attention output
    dy: np.ndarray                  # fp32 [T,H,d], gradient w.r.t. gated-norm output
    eps: float = 1e-5
    backward: bool = False

    @property
    def B(self) -> int:
        return int(self.lengths.shape[0])

    @property
    def T(self) -> int:
        return int(self.offsets[-1])

    @property
    def max_seqlen(self) -> int:
        return int(self.lengths.max()) if self.B else 0

    def with_mask(self, K1: int, K2: int, name: Optional[str] = None) -> "Workload":
        return dataclasses.replace(self, K1=K1, K2=K2, name=name or self.name)


def _normal(rng, shape, scale, dtype):
    x = rng.standard_normal(shape, dtype=np.float32) * np.float32(scale)
    return round_to_bf16(x) if dtype == "bf16" else x


def build(name, lengths, H, d, dtype, *, seed=0, rng=None, bias=True, K1=-1, K2=0,
          num_targets=None, N=None, alpha=1.0, backward=False) -> Workload:
    """Draw all tensors of one jagged batch.  ``lengths`` may be given or drawn by the caller."""
    rng = rng if rng is not None else np.random.default_rng(seed)
    lengths = np.asarray(lengths, dtype=np.int32)
    offsets = np.zeros(lengths.shape[0] + 1, dtype=np.int32)
    np.cumsum(lengths, out=offsets[1:])
    T = int(offsets[-1])
    s = 1.0 / np.sqrt(d)
    q = _normal(rng, (T, H, d), s, dtype)
    k = _normal(rng, (T, H, d), s, dtype)
    v = _normal(rng, (T, H, d), s, dtype)
    u = _normal(rng, (T, H, d), s, dtype)
    if bias:
        table = (rng.standard_normal((H, NUM_BUCKETS), dtype=np.float32) * np.float32(0.1))
        bounds = log_bucket_bounds()
    else:
        table, bounds = None, None
    gamma = (1.0 + 0.1 * rng.standard_normal(H * d, dtype=np.float32)).astype(np.float32)
    dout = _normal(rng, (T, H, d), 1.0, dtype)
    dy = _normal(rng, (T, H, d), 1.0, dtype)
    if N is None:
        N = float(max(int(lengths.max()), 1)) if lengths.size else 1.0
    nt = None if num_targets is None else np.asarray(num_targets, dtype=np.int32)
    return Workload(name=name, dtype=dtype, lengths=lengths, offsets=offsets, num_targets=nt,
                    H=H, d=d, K1=K1, K2=K2, alpha=alpha, N=float(N), q=q, k=k, v=v, u=u,
                    table=table, bounds=bounds, gamma=gamma, dout=dout, dy=dy, backward=backward)


def config(name: str, seed: int = 0) -> Workload:
    """The five benchmark configurations (C1..C5); C3 comes in a dense and a sparse flavour
    over identical tensors (same seed, same draw order)."""
    rng = np.random.default_rng(seed)
    if name == "C1":
        return build("C1", [37, 128, 200, 64], 2, 32, "fp32", rng=rng, bias=False, N=200.0)
    if name == "C2":
        L = rng.integers(512, 2049, size=32)
        return build("C2", L, 4, 128, "bf16", rng=rng)
    if name in ("C3", "C3-dense", "C3-sparse"):
        L = rng.integers(8192, 16385, size=8)
        w = build("C3-dense", L, 4, 128, "bf16", rng=rng, backward=True)
        return w.with_mask(1024, 256, "C3-sparse") if name == "C3-sparse" else w
    if name == "C4":
        L = rng.integers(32768, 65537, size=2)
        return build("C4", L, 4, 128, "bf16", rng=rng, K1=2048, K2=512, backward=True)
    if name == "C5":
        L = np.full(16, 4096 + 256)
        return build("C5", L, 8, 128, "bf16", rng=rng, num_targets=np.full(16, 256), backward=True)
    raise ValueError(f"unknown config {name!r}")


def small(name: str, seed: int = 0) -> Workload:
    """Reduced cases the CPU oracle finishes in seconds; they still span several
    128-row tiles, ragged tails, empty sequences and every mask family."""
    rng = np.random.default_rng(seed)
    if name == "bf16-dense":
        return build(name, [300, 0, 1, 129, 517, 64], 2, 128, "bf16", rng=rng, backward=True)
    if name == "bf16-sparse":
        return build(name, [700, 5, 0, 257, 1100], 2, 128, "bf16", rng=rng, K1=200, K2=70, backward=True)
    if name == "bf16-sparse-aligned":
        return build(name, [1024, 640, 128], 2, 128, "bf16", rng=rng, K1=256, K2=128, backward=True)
    if name == "bf16-local-only":
        return build(name, [600, 333], 1, 128, "bf16", rng=rng, K1=130, K2=0, backward=True)
    if name == "bf16-global-only":
        return build(name, [600, 333], 1, 128, "bf16", rng=rng, K1=0, K2=100, backward=True)
    if name == "bf16-targets":
        return build(name, [400, 90, 260, 31], 2, 128, "bf16", rng=rng,
                     num_targets=[100, 0, 260, 30], backward=True)
    if name == "bf16-targets-sparse":
        return build(name, [500, 300], 2, 128, "bf16", rng=rng, K1=96, K2=40,
                     num_targets=[130, 17], backward=True)
    if name == "bf16-d64":
        return build(name, [200, 77, 310], 3, 64, "bf16", rng=rng, K1=100, K2=20, backward=True)
    if name == "fp32-sparse":
        return build(name, [150, 0, 260, 33], 2, 32, "fp32", rng=rng, K1=64, K2=16,
                     num_targets=[10, 0, 0, 5], backward=True)
    if name == "fp32-d128":
        return build(name, [130, 65], 2, 128, "fp32", rng=rng, backward=True)
    raise ValueError(f"unknown small case {name!r}")


SMALL_CASES = ["bf16-dense", "bf16-sparse", "bf16-sparse-aligned", "bf16-local-only",
               "bf16-global-only", "bf16-targets", "bf16-targets-sparse", "bf16-d64",
               "fp32-sparse", "fp32-d128"]


# ----------------------------------------------------------------------------------------------
# attention truncation (Section 4.3): jagged batches of opaque token rows
# ----------------------------------------------------------------------------------------------
@dataclasses.dataclass
class TruncationCase:
    name: str
    lengths: np.ndarray          # int32 [B], history + candidates
    offsets: np.ndarray          # int32 [B+1]
    num_targets: Optional[np.ndarray]
    keep: int                    # most recent history rows that survive
    width: int                   # elements per row
    dtype: str                   # "bf16" (stored as uint16 bit patterns), "fp32"
    x: np.ndarray                # [T, width] rows (uint16 bits or float32)


def truncation_case(name: str, seed: int = 0) -> TruncationCase:
    """Seeded batches for the row selection.  "AT-3072-512" has the shape the paper reports for
    attention truncation (sequences up to 3072 cut to their latest 512 tokens) at the batch size and
    embedding width of its memory figures (256 sequences, 512 features, bf16); the others are small
    cases with empty sequences, candidates, odd widths and more sequences than one scan chunk."""
    rng = np.random.default_rng(1000 + seed)
    nt = None
    if name == "AT-3072-512":
        lengths, keep, width, dtype = rng.integers(1024, 3073, 256), 512, 512, "bf16"
    elif name == "small":
        lengths, keep, width, dtype = np.array([5, 0, 1, 40, 17, 3, 64, 0]), 6, 8, "bf16"
    elif name == "small-targets":
        lengths, keep, width, dtype = np.array([50, 9, 0, 33, 21, 128]), 16, 520, "bf16"
        nt = np.array([10, 9, 0, 0, 5, 1])
    elif name == "small-fp32":
        lengths, keep, width, dtype = rng.integers(0, 90, 37), 31, 12, "fp32"
        nt = np.minimum(rng.integers(0, 8, 37), lengths)
    elif name == "many-sequences":
        lengths, keep, width, dtype = rng.integers(0, 24, 3001), 7, 16, "bf16"
        nt = np.minimum(rng.integers(0, 3, 3001), lengths)
    elif name == "empty":
        lengths, keep, width, dtype = np.zeros(3, dtype=np.int64), 4, 8, "bf16"
    elif name == "keep-all":
        lengths, keep, width, dtype = rng.integers(1, 70, 12), 1 << 20, 64, "bf16"
    elif name == "keep-none":
        lengths, keep, width, dtype = rng.integers(1, 70, 12), 0, 64, "bf16"
        nt = np.minimum(rng.integers(0, 4, 12), lengths)
    else:
        raise ValueError(f"unknown truncation case {name!r}")
    lengths = np.asarray(lengths, dtype=np.int32)
    offsets = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    T = int(offsets[-1])
    if dtype == "bf16":
        x = rng.integers(0, 1 << 16, size=(T, width), dtype=np.uint16)      # arbitrary bit patterns: rows are opaque
    else:
        x = rng.standard_normal((T, width)).astype(np.float32)
    return TruncationCase(name, lengths, offsets, None if nt is None else np.asarray(nt, dtype=np.int32), keep, width, dtype, x)


TRUNCATION_SMALL = ["small", "empty", "small-targets", "small-fp32", "many-sequences", "keep-all", "keep-none"]


# ----------------------------------------------------------------------------------------------
# whole HSTU layer (Eq. 1-5 and the layer pseudocode of the appendix): token rows and weights
# ----------------------------------------------------------------------------------------------
@dataclasses.dataclass
class LayerCase:
    name: str
    dtype: str                         # storage type of z, w1, w2, dout and every activation
    lengths: np.ndarray
    offsets: np.ndarray
    num_targets: Optional[np.ndarray]
    H: int
    d: int
    E: int                             # embedding width of the token rows
    K1: int
    K2: int
    alpha: float
    N: float
    table: Optional[np.ndarray]
    bounds: Optional[np.ndarray]
    z: np.ndarray                      # fp32 [T, E] layer input (rounded to dtype)
    norm_w: np.ndarray                 # fp32 [E]
    w1: np.ndarray                     # fp32 [4 H d, E] (rounded to dtype), output order U, V, Q, K
    gated_norm_w: np.ndarray           # fp32 [H d]
    w2: np.ndarray                     # fp32 [E, H d] (rounded to dtype)
    dout: np.ndarray                   # fp32 [T, E] gradient of the layer output (rounded to dtype)
    eps: float = 1e-5

    @property
    def B(self) -> int:
        return int(self.lengths.shape[0])

    @property
    def T(self) -> int:
        return int(self.offsets[-1])

    @property
    def max_seqlen(self) -> int:
        return int(self.lengths.max()) if self.B else 0


def build_layer(name, lengths, H, d, E, dtype="bf16", *, seed=0, K1=-1, K2=0, num_targets=None, bias=True) -> LayerCase:
    """Draw order: z, norm_w, w1, gated_norm_w, w2, table, dout.  Token rows ~ N(0, 1); weights ~ N(0, 1/fan_in) so that
    the pre-activations are O(1); norm weights 1 + 0.1 N(0, 1); alpha = 1/sqrt(d) keeps the scores O(1)."""
    rng = np.random.default_rng(2000 + seed)
    lengths = np.asarray(lengths, dtype=np.int32)
    offsets = np.zeros(lengths.shape[0] + 1, dtype=np.int32)
    np.cumsum(lengths, out=offsets[1:])
    T, HD = int(offsets[-1]), H * d
    z = _normal(rng, (T, E), 1.0, dtype)
    norm_w = (1.0 + 0.1 * rng.standard_normal(E, dtype=np.float32)).astype(np.float32)
    w1 = _normal(rng, (4 * HD, E), 1.0 / np.sqrt(E), dtype)
    gated_norm_w = (1.0 + 0.1 * rng.standard_normal(HD, dtype=np.float32)).astype(np.float32)
    w2 = _normal(rng, (E, HD), 1.0 / np.sqrt(HD), dtype)
    table = rng.standard_normal((H, NUM_BUCKETS), dtype=np.float32) * np.float32(0.1) if bias else None
    bounds = log_bucket_bounds() if bias else None
    dout = _normal(rng, (T, E), 1.0, dtype)
    N = float(max(int(lengths.max()), 1)) if lengths.size else 1.0
    nt = None if num_targets is None else np.asarray(num_targets, dtype=np.int32)
    return LayerCase(name, dtype, lengths, offsets, nt, H, d, E, K1, K2, 1.0 / float(np.sqrt(d)), N, table, bounds, z, norm_w,
                     w1, gated_norm_w, w2, dout)


def layer_case(name: str, seed: int = 0) -> LayerCase:
    """"layer-C3": the 8k-16k attention configuration inside a layer of embedding width 512 (the width of the paper's
    memory figures, Section 4.2.2).  The others are cases the CPU oracle finishes in seconds."""
    if name == "layer-C3":
        L = np.random.default_rng(seed).integers(8192, 16385, size=8)      # the lengths of C3-dense
        return build_layer(name, L, 4, 128, 512, seed=seed)
    if name == "layer-mid":
        L = np.random.default_rng(seed + 1).integers(1024, 2049, size=4)
        return build_layer(name, L, 4, 128, 512, seed=seed)
    if name == "layer-long":      # sequences of the benchmark's length range, as many as the oracle affords
        return build_layer(name, [8192, 4200], 4, 128, 512, seed=seed)
    if name == "layer-long-sparse":
        return build_layer(name, [8192, 4200], 4, 128, 512, seed=seed, K1=1024, K2=256)
    if name == "layer-small-dense":
        return build_layer(name, [70, 0, 33, 129], 2, 64, 96, seed=seed)
    if name == "layer-small-sparse-targets":
        return build_layer(name, [200, 90, 31], 2, 128, 256, seed=seed, K1=64, K2=16, num_targets=[20, 0, 30])
    if name == "layer-small-nobias":
        return build_layer(name, [150, 1, 300], 1, 128, 128, seed=seed, K1=100, K2=0, bias=False)
    raise ValueError(f"unknown layer case {name!r}")


LAYER_SMALL = ["layer-small-dense", "layer-small-sparse-targets", "layer-small-nobias"]


# ----------------------------------------------------------------------------------------------
# FP8 projection with a two-dimensional additive operand (Section 4.2.2 and the FP8 GEMM table of the appendix)
# ----------------------------------------------------------------------------------------------
FP8_GEMM_SHAPES = {                      # (m, k = n) of the paper's table: "1M" and "250K" token rows, widths 512 and 1K
    "1M-512": (1 << 20, 512), "1M-1K": (1 << 20, 1024), "250K-512": (250_000, 512), "250K-1K": (250_000, 1024),
}


def fp8_gemm_inputs(M: int, N: int, K: int, seed: int = 0, with_c: bool = True):
    """Unquantised operands of D = A B^T + C: activations a [M, K] like gated-norm outputs (N(0,1) with a per-row spread of
    magnitudes), weights b [N, K] ~ N(0, 1/K), residual c [M, N] ~ N(0,1); bf16-representable fp32 arrays."""
    rng = np.random.default_rng(3000 + seed)
    a = rng.standard_normal((M, K), dtype=np.float32) * rng.uniform(0.2, 3.0, (M, 1)).astype(np.float32)
    b = rng.standard_normal((N, K), dtype=np.float32) * np.float32(1.0 / np.sqrt(K))
    c = rng.standard_normal((M, N), dtype=np.float32) if with_c else None
    return round_to_bf16(a), round_to_bf16(b), None if c is None else round_to_bf16(c)
