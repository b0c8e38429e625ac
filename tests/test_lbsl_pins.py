"""Pins of the Load-Balanced Stochastic Length oracle (paper Section 4.1 and Alg. 1 of the appendix) against the numbers the
paper prints, closed forms, a hand-worked example, the exact law of a weighted draw without replacement, and the properties
the paper states for the method.  No GPU."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import lbsl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def read_golden(name):
    vals = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, *rest = line.split()
            vals[key] = [float(v) for v in rest]
    return vals


def test_weight_is_the_keep_probability_of_stochastic_length():
    """SL keeps a sequence of n > L^(alpha/2) whole with probability L^alpha / n^2.  L = 65536, alpha = 1.5: l_SL = 4096."""
    L, alpha = 65536, 1.5
    sl_len = round(L ** (alpha / 2))
    assert sl_len == 4096
    for n in (4097, 5000, 30000, 65536):
        assert lbsl.sl_weight(n, sl_len) == pytest.approx(L ** alpha / n ** 2, rel=1e-12)
    assert lbsl.sl_weight(65536, sl_len) == pytest.approx(1.0 / 256.0, rel=1e-12)
    for n in (1, 100, 4096):
        assert lbsl.sl_weight(n, sl_len) == 1.0
    # the bias the paper asks to preserve: shorter sequences are more likely to stay unsampled
    ws = [lbsl.sl_weight(n, sl_len) for n in range(4096, 65536, 997)]
    assert all(a >= b for a, b in zip(ws, ws[1:]))


def test_average_training_length_matches_the_papers_table():
    """Users with a full raw history of L items, alpha = 1.7 (one value for all three rows): the expected length after SL,
    w L + (1 - w) l_SL, reproduces the paper's 'around' figures within 3 %."""
    g = read_golden("lbsl_training_lengths.txt")
    alpha = 1.7
    for L, want in zip(g["raw"], g["train"]):
        sl_len = int(round(L ** (alpha / 2)))
        w = lbsl.sl_weight(int(L), sl_len)
        got = w * L + (1.0 - w) * sl_len
        assert abs(got - want) / want < 0.03, (L, got, want)
        # the same through the load function at gamma = 1 (load = length)
        assert lbsl.standard_sl_load(int(L), sl_len, 1.0) == pytest.approx(got, rel=1e-12)


def test_standard_sl_decides_by_the_uniform():
    lens = [5, 10, 11, 40, 1000]
    new, keep = lbsl.standard_sl(lens, [1e-9] * 5, 10)          # a tiny uniform keeps everything whole
    assert new == lens and all(keep)
    new, keep = lbsl.standard_sl(lens, [1 - 1e-9] * 5, 10)      # a uniform next to 1 samples every long sequence
    assert new == [5, 10, 10, 10, 10] and keep == [True, True, False, False, False]
    new, keep = lbsl.standard_sl([20], [0.2499], 10)            # weight of n = 20 is exactly 1/4
    assert keep == [True]
    new, keep = lbsl.standard_sl([20], [0.2501], 10)
    assert keep == [False] and new == [10]


def test_expected_load_is_the_mean_of_the_sampled_load():
    """standard_sl_load is the expectation of the realised load: average standard_sl over a fine grid of uniforms."""
    sl_len, gamma = 64, 1.6
    grid = (np.arange(20000) + 0.5) / 20000
    for n in (10, 64, 65, 200, 640):
        mean = np.mean([lbsl.seq_load(lbsl.standard_sl([n], [u], sl_len)[0][0], gamma) for u in grid])
        assert mean == pytest.approx(lbsl.standard_sl_load(n, sl_len, gamma), rel=1e-3)


def test_weighted_permutation_two_items_exact():
    """P(a before b) = p_a / (p_a + p_b): integrate the indicator over a fine grid of the two uniforms."""
    pa, pb = 0.7, 0.2
    m = 400
    grid = (np.arange(m) + 0.5) / m
    first_a = sum(lbsl.weighted_permutation([pa, pb], [ua, ub])[0] == 0 for ua in grid for ub in grid)
    assert first_a / m ** 2 == pytest.approx(pa / (pa + pb), abs(2.0 / m))


def test_weighted_permutation_follows_sequential_sampling_without_replacement():
    """Every ordering of three items has probability prod_i p_(i) / (sum of the weights not yet drawn)."""
    p = [0.5, 0.3, 0.05]
    rng = np.random.default_rng(7)
    draws = 60000
    counts = {perm: 0 for perm in itertools.permutations(range(3))}
    for _ in range(draws):
        counts[tuple(lbsl.weighted_permutation(p, rng.uniform(1e-12, 1.0, 3)))] += 1
    for perm, c in counts.items():
        left, prob = sum(p), 1.0
        for i in perm:
            prob *= p[i] / left
            left -= p[i]
        assert c / draws == pytest.approx(prob, abs=4 * math.sqrt(prob * (1 - prob) / draws) + 1e-3), perm


def test_weighted_permutation_degenerate_cases():
    assert lbsl.weighted_permutation([], []) == []
    assert lbsl.weighted_permutation([1.0], [0.3]) == [0]
    assert lbsl.weighted_permutation([1.0, 1.0, 1.0], [0.5, 0.5, 0.5]) == [0, 1, 2]      # ties by index
    assert lbsl.weighted_permutation([1.0, 0.0], [0.9, 0.1])[-1] == 1                   # weight 0 goes last


def test_constrained_fill_hand_worked():
    g = read_golden("lbsl_fill_worked.txt")
    lengths = [int(v) for v in g["lengths"]]
    order = [int(v) for v in g["order"]]
    sl_len, gamma = int(g["sl_len"][0]), g["gamma"][0]
    chosen = lbsl.constrained_fill(lengths, order, g["target"][0], sl_len, gamma)
    assert [int(c) for c in chosen] == [int(v) for v in g["chosen"]]
    new = [n if c else min(n, sl_len) for n, c in zip(lengths, chosen)]
    assert new == [int(v) for v in g["new_lengths"]]
    assert sum(lbsl.seq_load(n, gamma) for n in new) == g["realised"][0]


def test_constrained_fill_respects_the_budget_and_is_greedy():
    rng = np.random.default_rng(3)
    for trial in range(50):
        b = int(rng.integers(1, 40))
        lengths = [int(v) for v in rng.integers(1, 3000, b)]
        sl_len, gamma = int(rng.integers(50, 800)), float(rng.uniform(1.05, 1.95))
        order = [int(i) for i in rng.permutation(b)]
        floor = sum(lbsl.seq_load(min(n, sl_len), gamma) for n in lengths)     # load with every long sequence cut
        target = float(rng.uniform(0.8, 3.0)) * floor
        chosen = lbsl.constrained_fill(lengths, order, target, sl_len, gamma)
        s = 0.0
        for u in order:                                        # replay: every refusal was forced, every admission fitted
            extra = lbsl.seq_load(lengths[u], gamma) - lbsl.seq_load(min(lengths[u], sl_len), gamma)
            fits = s + extra <= target - floor
            assert chosen[u] == fits
            if fits:
                s += extra
        realised = sum(lbsl.seq_load(n if c else min(n, sl_len), gamma) for n, c in zip(lengths, chosen))
        assert realised == pytest.approx(floor + s, rel=1e-12)
        assert realised <= max(target, floor) * (1 + 1e-12)    # never above the target (unless the floor already is)


def test_constrained_fill_is_the_listings_condition_when_no_sequence_is_short():
    """Every n_u >= l_SL: admit u iff s + (n_u^gamma - l_SL^gamma) <= target - b l_SL^gamma, the condition as printed."""
    rng = np.random.default_rng(5)
    for trial in range(30):
        b = int(rng.integers(1, 30))
        sl_len, gamma = int(rng.integers(50, 500)), float(rng.uniform(1.05, 1.95))
        lengths = [int(v) for v in rng.integers(sl_len, 20 * sl_len, b)]
        order = [int(i) for i in rng.permutation(b)]
        base = lbsl.seq_load(sl_len, gamma)
        target = float(rng.uniform(1.0, 6.0)) * b * base
        want, s = [False] * b, 0.0
        for u in order:
            if s + (lbsl.seq_load(lengths[u], gamma) - base) <= target - b * base:
                want[u] = True
                s += lbsl.seq_load(lengths[u], gamma) - base
        assert lbsl.constrained_fill(lengths, order, target, sl_len, gamma) == want


def test_everything_short_is_left_alone():
    sim = lbsl.Lbsl(2, 1, 1, 100, 1.5)
    batches = [[5, 50, 100], [1, 99]]
    us = [[0.5, 0.5, 0.5], [0.5, 0.5]]
    for _ in range(3):
        new, keep, realised = sim.step(batches, us)
        assert new == batches
        assert realised[0] == pytest.approx(sum(n ** 1.5 for n in batches[0]))


def test_target_after_warmup_is_the_mean_expected_load():
    """Two ranks, two warm-up steps, gamma = 2, l_SL = 10: expected load of n = 20 is 1/4 * 400 + 3/4 * 100 = 175."""
    sim = lbsl.Lbsl(2, 2, 3, 10, 2.0)
    sim.step([[20, 5], [20]], [[0.9, 0.9], [0.1]])            # rank loads 175 + 25 = 200 and 175
    assert sim.target == 0.0 and sim.rank_load == [200.0, 175.0]
    sim.step([[10], [20, 20]], [[0.5], [0.5, 0.5]])           # + 100 and + 350
    assert sim.target == pytest.approx((300.0 + 525.0) / (2 * 2))
    assert sim.rank_load == [0.0, 0.0]
    sim.step([[20], [20]], [[0.5], [0.5]])                    # step 3: multiple of T_recal = 3 -> mean of one step's loads / 3
    assert sim.target == pytest.approx((175.0 + 175.0) / (2 * 3))


def lengths_like_production(rng, b):
    """Heavy-tailed raw lengths up to 16384 with a different mean per draw (the cross-rank imbalance the method targets)."""
    scale = rng.uniform(1500, 9000)
    return [int(v) for v in np.clip(rng.gamma(1.2, scale, b), 16, 16384)]


def test_balance_improves_and_mean_load_is_preserved():
    """The paper's claim for recalibration every batch: the average load matches standard SL's, the spread across ranks
    shrinks (max / min rank load)."""
    R, b, sl_len, gamma = 16, 64, 3822, 1.5
    rng = np.random.default_rng(11)
    sim = lbsl.Lbsl(R, 4, 1, sl_len, gamma)
    ratios_lbsl, ratios_sl, mean_lbsl, mean_sl = [], [], [], []
    for t in range(60):
        batches = [lengths_like_production(rng, b) for _ in range(R)]
        us = [list(rng.uniform(1e-12, 1.0, b)) for _ in range(R)]
        new, keep, realised = sim.step(batches, us)
        if t >= 8:
            sl_real = [sum(lbsl.seq_load(n, gamma) for n in lbsl.standard_sl(batches[r], us[r], sl_len)[0]) for r in range(R)]
            ratios_lbsl.append(max(realised) / min(realised))
            ratios_sl.append(max(sl_real) / min(sl_real))
            mean_lbsl.append(np.mean(realised))
            mean_sl.append(np.mean(sl_real))
    print("max/min rank load: LBSL", np.mean(ratios_lbsl), "standard SL", np.mean(ratios_sl),
          "mean load LBSL / SL", np.mean(mean_lbsl) / np.mean(mean_sl))
    assert np.mean(ratios_lbsl) < 0.8 * np.mean(ratios_sl), (np.mean(ratios_lbsl), np.mean(ratios_sl))
    assert np.mean(mean_lbsl) == pytest.approx(np.mean(mean_sl), rel=0.1)


def test_fit_gamma_recovers_a_power_law():
    ns = [512, 1024, 2048, 4096, 8192]
    assert lbsl.fit_gamma(ns, [3e-7 * n ** 1.73 for n in ns]) == pytest.approx(1.73, abs=1e-9)
    assert lbsl.fit_gamma(ns, [5.0 * n for n in ns]) == pytest.approx(1.0, abs=1e-9)
