"""FLOP and byte accounting for the benchmark (closed forms over the mask; no kernel arithmetic).

Conventions: per unmasked (query, key) pair and head the forward costs 4*d FLOPs (two products),
the backward 10*d (five products, the score recompute included, the FlashAttention convention)
or 8*d counted strictly.  SiLU, mask and bias work is never counted, and neither are masked
elements computed inside partially masked tiles.
"""
from __future__ import annotations

import numpy as np


def visible_pairs_one(L: int, M: int, K1: int, K2: int) -> int:
    """Visible (query, key) pairs of one sequence with M trailing candidates (per head)."""
    n = L - M
    i = np.arange(n, dtype=np.int64)
    if K1 < 0:
        hist = int((i + 1).sum())
        cand = n
    else:
        hist = int((np.minimum(i + 1, K1) + np.minimum(K2, np.maximum(0, i - K1 + 1))).sum())
        in_window = min(n, max(K1 - 1, 0))                      # keys with n - j < K1
        cand = in_window + min(K2, max(0, n - max(K1, 1) + 1)) if K1 >= 1 else min(K2, n)
    return hist + M * (cand + 1)


def visible_pairs(lengths, num_targets, K1: int, K2: int) -> int:
    nt = np.zeros(len(lengths), dtype=np.int64) if num_targets is None else num_targets
    return sum(visible_pairs_one(int(L), int(M), K1, K2) for L, M in zip(lengths, nt))


def visible_pairs_tail(lengths, num_targets, K1: int, K2: int, tail: int) -> int:
    """Pairs of the last min(n, tail) history rows and the candidates of every sequence: all pairs minus those of the
    leading history rows (which see exactly what they would see in a sequence that ends with them)."""
    nt = np.zeros(len(lengths), dtype=np.int64) if num_targets is None else num_targets
    total = 0
    for L, M in zip(lengths, nt):
        n = int(L) - int(M)
        total += visible_pairs_one(int(L), int(M), K1, K2) - visible_pairs_one(max(n - tail, 0), 0, K1, K2)
    return total


def attention_flops(w, pairs_per_head=None):
    p = visible_pairs(w.lengths, w.num_targets, w.K1, w.K2) if pairs_per_head is None else pairs_per_head
    pairs = p * w.H
    return {"pairs": pairs, "fwd": 4.0 * w.d * pairs, "bwd": 10.0 * w.d * pairs, "bwd_strict": 8.0 * w.d * pairs}


def bytes_per_elem(dtype: str) -> int:
    return 2 if dtype == "bf16" else 4


def epilogue_bytes(w):
    e = bytes_per_elem(w.dtype) * w.T * w.H * w.d
    return {"fwd": 3 * e + 8 * w.T, "bwd": 5 * e}


def expand_bytes(w, kernel: str) -> float:
    """Bytes the expansion kernel in front of an attention pass writes: the distance-indexed seed tables of the pipelined
    forward (bf16, 128 features per head: two variants of max_seqlen + 128 + 1 + 192 entries per head, rounded up to 64), or
    the plain per-distance bias table (max_seqlen + 1 entries per head)."""
    if kernel == "bias_expand_fwd" and w.dtype == "bf16" and w.d == 128:
        seed_len = (w.max_seqlen + 128 + 1 + 192 + 63) // 64 * 64
        return 2.0 * w.H * seed_len * 4
    return float(w.H) * (w.max_seqlen + 1) * 4
