"""Pins of the attention-truncation oracle (paper Section 4.3) against a hand-worked example, a
per-row predicate written independently of the per-sequence slicing, and the algebra the operation
must obey (identity, composition, adjointness of its backward).  No GPU."""
import os

import numpy as np
import pytest

from oracle import truncation as tr

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def read_golden(name):
    vals = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, *rest = line.split()
            vals[key] = np.array([int(v) for v in rest], dtype=np.int64)
    return vals


def random_batch(seed, B, max_len, max_targets, width=3):
    rng = np.random.default_rng(seed)
    targets = rng.integers(0, max_targets + 1, B)
    lengths = targets + rng.integers(0, max_len + 1, B)
    offsets = np.concatenate([[0], np.cumsum(lengths)])
    x = rng.standard_normal((int(offsets[-1]), width))
    return x, offsets, targets


@pytest.mark.parametrize("case", ["A", "B"])
def test_hand_worked_example(case):
    g = read_golden("truncation_B3_keep2.txt")
    offsets = np.concatenate([[0], np.cumsum(g["lengths"])])
    ids = np.arange(offsets[-1])
    rows, new = tr.tail_slice(ids, offsets, int(g["keep"][0]), g["targets_" + case])
    assert rows.tolist() == g["rows_" + case].tolist()
    assert new.tolist() == g["offsets_" + case].tolist()


@pytest.mark.parametrize("seed", range(6))
def test_per_row_predicate(seed):
    """A row at position p of a sequence with n history rows survives iff it is a candidate (p >= n)
    or one of the last `keep` history rows (p >= n - keep): select with a boolean mask over all rows."""
    x, offsets, targets = random_batch(seed, B=9, max_len=20, max_targets=3)
    keep = [0, 1, 4, 7, 19, 25][seed]
    mask = np.zeros(x.shape[0], dtype=bool)
    counts = []
    for b in range(len(targets)):
        n = offsets[b + 1] - offsets[b] - targets[b]
        for p in range(offsets[b + 1] - offsets[b]):
            mask[offsets[b] + p] = p >= n - keep
        counts.append(int(mask[offsets[b]:offsets[b + 1]].sum()))
    y, new = tr.tail_slice(x, offsets, keep, targets)
    assert np.array_equal(y, x[mask])
    assert np.diff(new).tolist() == counts
    # backward: gradient rows land where the mask is set, zero elsewhere
    dy = np.arange(y.size, dtype=np.float64).reshape(y.shape) + 1.0
    dx = tr.tail_slice_bwd(dy, offsets, keep, targets)
    assert np.array_equal(dx[mask], dy) and not dx[~mask].any()


def test_identity_and_empty():
    x, offsets, targets = random_batch(11, B=7, max_len=12, max_targets=2)
    y, new = tr.tail_slice(x, offsets, 12, targets)          # keep >= every history: nothing dropped
    assert np.array_equal(y, x) and np.array_equal(new, offsets)
    y, new = tr.tail_slice(x, offsets, 0, None)              # nothing kept
    assert y.shape == (0, 3) and not new.any()
    y, new = tr.tail_slice(x, offsets, 0, targets)           # only the candidates stay
    assert np.diff(new).tolist() == targets.tolist()
    for b in range(7):
        assert np.array_equal(y[new[b]:new[b + 1]], x[offsets[b + 1] - targets[b]:offsets[b + 1]])


@pytest.mark.parametrize("seed", range(4))
def test_composition(seed):
    """Truncating to a and then to b <= a is truncating to b."""
    x, offsets, targets = random_batch(20 + seed, B=8, max_len=30, max_targets=2)
    a, b = 17, 5
    ya, offa = tr.tail_slice(x, offsets, a, targets)
    yab, offab = tr.tail_slice(ya, offa, b, targets)
    yb, offb = tr.tail_slice(x, offsets, b, targets)
    assert np.array_equal(yab, yb) and np.array_equal(offab, offb)


@pytest.mark.parametrize("seed", range(4))
def test_backward_is_the_adjoint(seed):
    """<slice(x), g> == <x, slice_bwd(g)> for every x, g: the backward is the transpose of a selection."""
    x, offsets, targets = random_batch(40 + seed, B=6, max_len=25, max_targets=3)
    keep = 6
    y, new = tr.tail_slice(x, offsets, keep, targets)
    g = np.random.default_rng(seed).standard_normal(y.shape)
    lhs = float((y * g).sum())
    rhs = float((x * tr.tail_slice_bwd(g, offsets, keep, targets)).sum())
    assert lhs == pytest.approx(rhs, rel=1e-13)
