"""CPU oracle of attention truncation (paper Section 4.3, "Attention Truncation").

TEST INFRASTRUCTURE ONLY: imported by the tests and the smoke check, never by the product path.

After the first group of layers has seen every token, the remaining layers run on a segment of each
user's history; the paper finds that the most recent ``keep`` history tokens work best.  On a jagged
batch that is: of sequence b with n_b history rows followed by M_b candidate rows, the kept rows are the
last min(n_b, keep) history rows and all M_b candidates, in their order, packed sequence after sequence.
The backward of this selection hands each kept row its gradient and every dropped row zero.
Plain loops over sequences; integer work is exact, data rows are moved, never changed.
"""
from __future__ import annotations

import numpy as np


def kept_rows(length: int, keep: int, targets: int = 0) -> int:
    """Rows of one sequence that survive: min(history, keep) + candidates."""
    history = length - targets
    assert history >= 0 and keep >= 0
    return min(history, keep) + targets


def tail_offsets(offsets, keep, num_targets=None):
    """Offsets [B+1] of the truncated batch."""
    offsets = np.asarray(offsets, dtype=np.int64)
    B = offsets.shape[0] - 1
    out = np.zeros(B + 1, dtype=np.int64)
    for b in range(B):
        m = 0 if num_targets is None else int(num_targets[b])
        out[b + 1] = out[b] + kept_rows(int(offsets[b + 1] - offsets[b]), keep, m)
    return out


def tail_slice(x, offsets, keep, num_targets=None):
    """Returns (rows of x that survive [T', ...], new offsets [B+1])."""
    x = np.asarray(x)
    offsets = np.asarray(offsets, dtype=np.int64)
    new = tail_offsets(offsets, keep, num_targets)
    out = np.zeros((int(new[-1]),) + x.shape[1:], dtype=x.dtype)
    for b in range(offsets.shape[0] - 1):
        kept = int(new[b + 1] - new[b])
        end = int(offsets[b + 1])
        out[new[b]:new[b + 1]] = x[end - kept:end]
    return out, new


def tail_slice_bwd(dy, offsets, keep, num_targets=None):
    """Gradient with respect to the untruncated rows [T, ...]: dy on the kept rows, zero elsewhere."""
    dy = np.asarray(dy)
    offsets = np.asarray(offsets, dtype=np.int64)
    new = tail_offsets(offsets, keep, num_targets)
    assert dy.shape[0] == new[-1]
    dx = np.zeros((int(offsets[-1]),) + dy.shape[1:], dtype=dy.dtype)
    for b in range(offsets.shape[0] - 1):
        kept = int(new[b + 1] - new[b])
        end = int(offsets[b + 1])
        dx[end - kept:end] = dy[new[b]:new[b + 1]]
    return dx
