"""The library's Load-Balanced Stochastic Length (hstu_lbsl_*, host code behind the C ABI) against the CPU oracle on the same
seeded lengths and uniforms: decisions and new lengths identical, loads and target to 1e-12.  Host-only entry points: these
run without a GPU."""
import numpy as np
import pytest

from oracle import lbsl as orc


@pytest.fixture(scope="module")
def hb():
    from paper_2602_16986_amd import binding
    return binding


def draw_step(rng, R, max_b, max_len, short_frac):
    sizes = rng.integers(0, max_b + 1, R)
    offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    total = int(offsets[-1])
    lengths = np.where(rng.uniform(size=total) < short_frac, rng.integers(0, 64, total), rng.integers(1, max_len + 1, total)).astype(np.int32)
    uniforms = rng.uniform(1e-12, 1.0, total)
    return offsets, lengths, uniforms


@pytest.mark.parametrize("R,t_warm,t_recal,sl_len,gamma,max_b,max_len,short_frac,seed", [
    (1, 1, 1, 100, 1.5, 40, 2000, 0.2, 0),
    (4, 3, 2, 918, 1.3, 64, 3072, 0.1, 1),
    (8, 2, 5, 3822, 1.7, 128, 16384, 0.3, 2),
    (3, 4, 3, 10, 1.999, 17, 50, 0.5, 3),          # warm-up longer than the recalibration interval
    (5, 1, 1, 2120, 1.05, 33, 8192, 0.0, 4),       # no short sequence: the listing's condition verbatim
    (2, 2, 2, 1, 1.5, 9, 5, 0.5, 5),               # sampling length 1, zero-length sequences
])
def test_steps_match_the_oracle(hb, R, t_warm, t_recal, sl_len, gamma, max_b, max_len, short_frac, seed):
    rng = np.random.default_rng(100 + seed)
    lib = hb.Lbsl(R, t_warm, t_recal, sl_len, gamma)
    ref = orc.Lbsl(R, t_warm, t_recal, sl_len, gamma)
    for t in range(14):
        offsets, lengths, uniforms = draw_step(rng, R, max_b, max_len, short_frac)
        new, keep, real = lib.step(offsets, lengths, uniforms)
        batches = [lengths[offsets[r]:offsets[r + 1]].tolist() for r in range(R)]
        us = [uniforms[offsets[r]:offsets[r + 1]].tolist() for r in range(R)]
        rnew, rkeep, rreal = ref.step(batches, us)
        assert new.tolist() == [n for b in rnew for n in b], f"step {t}: new lengths"
        assert keep.astype(bool).tolist() == [k for b in rkeep for k in b], f"step {t}: unsampled set"
        np.testing.assert_allclose(real, rreal, rtol=1e-12, atol=0)
        assert lib.target == pytest.approx(ref.target, rel=1e-12)
        np.testing.assert_allclose(lib.rank_load, ref.rank_load, rtol=1e-12, atol=0)
        assert lib.step_no == ref.step_no == t + 1


def test_weight_and_expected_load(hb):
    for n, sl_len, gamma in [(0, 5, 1.5), (5, 5, 1.5), (6, 5, 1.5), (16384, 3822, 1.7), (65536, 4096, 1.2)]:
        assert hb.hstu_lbsl_weight(n, sl_len) == pytest.approx(orc.sl_weight(n, sl_len), rel=1e-15)
        assert hb.hstu_lbsl_expected_load(n, sl_len, gamma) == pytest.approx(orc.standard_sl_load(n, sl_len, gamma), rel=1e-14)


def test_empty_ranks_and_empty_step(hb):
    lib = hb.Lbsl(3, 1, 1, 10, 1.5)
    new, keep, real = lib.step([0, 0, 0, 0], [], [])
    assert new.size == 0 and real.tolist() == [0.0, 0.0, 0.0] and lib.target == 0.0
    # target 0 after a warm-up without data: the budget is negative, nobody enters the untruncated set, long sequences are cut
    new, keep, real = lib.step([0, 2, 2, 3], [50, 3, 20], [0.5, 0.5, 0.5])
    assert new.tolist() == [10, 3, 10] and keep.tolist() == [0, 0, 0]


def test_bad_arguments_are_rejected(hb):
    for bad in [(0, 1, 1, 10, 1.5), (2, 0, 1, 10, 1.5), (2, 1, 0, 10, 1.5), (2, 1, 1, 0, 1.5), (2, 1, 1, 10, 0.0), (2, 1, 1, 10, float("nan"))]:
        with pytest.raises(hb.HstuError):
            hb.Lbsl(*bad)
    lib = hb.Lbsl(2, 1, 1, 10, 1.5)
    with pytest.raises(hb.HstuError):
        lib.step([0, 2, 1], [5], [0.5])                      # offsets decrease
    with pytest.raises(hb.HstuError):
        lib.step([0, 1, 2], [5, -1], [0.5, 0.5])             # negative length
    with pytest.raises(hb.HstuError):
        lib.step([0, 1, 2], [5, 7], [0.5, 0.0])              # uniform outside (0, 1]
    with pytest.raises(hb.HstuError):
        lib.step([1, 1, 2], [5], [0.5])                      # offsets do not start at 0
    assert lib.step_no == 0                                   # a rejected step changes nothing


def test_fit_gamma(hb):
    ns = [512, 1024, 2048, 4096, 8192]
    ts = [3e-7 * n ** 1.73 * (1 + 0.01 * (-1) ** i) for i, n in enumerate(ns)]
    assert hb.hstu_lbsl_fit_gamma(ns, ts) == pytest.approx(orc.fit_gamma(ns, ts), rel=1e-12)
    with pytest.raises(hb.HstuError):
        hb.hstu_lbsl_fit_gamma([5.0], [1.0])
    with pytest.raises(hb.HstuError):
        hb.hstu_lbsl_fit_gamma([5.0, 5.0], [1.0, 2.0])
