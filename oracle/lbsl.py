"""CPU oracle of Load-Balanced Stochastic Length (paper Section 4.1, "Load-Balanced Stochastic Length", and Alg. 1 of
the appendix "Algorithm of Load Balanced Stochastic Length").

TEST INFRASTRUCTURE: plain Python loops in double precision, written from the paper's description, independent of the
library's implementation (no shared code).  Only tests/, the smoke check and the benchmark's CPU baseline may import it.

What the paper fixes and what is a reading of it:
  * load of a sequence of length n: n ** gamma; load of a rank: the sum over its batch (Section 4.1).
  * Stochastic Length (SL), which the paper takes from the HSTU paper: with sampling length l_SL = L ** (alpha / 2), a
    sequence with n <= l_SL is left alone; a longer one is left alone with probability L ** alpha / n ** 2 =
    (l_SL / n) ** 2 and cut to l_SL items otherwise.  READING: SLWeight(n; alpha) is that probability of staying unsampled
    (the text says the weights keep SL's bias toward leaving shorter sequences unsampled).
  * READING: StandardSL_Loads is the EXPECTED load of the rank's batch under standard SL, computed from the raw lengths
    (the listing calls it a pre-truncation proxy): sum of  w n^gamma + (1 - w) l_SL^gamma.
  * READING: "apply the same sampling rule as StandardSL" to a sequence outside the untruncated set means: it is cut to
    l_SL items if it is longer (which items SL picks is not this module's business: it deals in lengths).
  * The weighted random permutation without replacement is drawn with exponential clocks: item u gets the key
    -ln(U_u) / p_u from a uniform U_u in (0, 1) that the CALLER passes in, and the items are taken by ascending key (ties by
    index).  That is sequential sampling without replacement with probabilities proportional to p_u.
  * The mean over ranks that the listing obtains with an all-reduce is a plain mean over the simulated ranks.
  * READING: the listing prices the all-sampled batch at b * l_SL^gamma and admitting u at n_u^gamma - l_SL^gamma, which
    presumes every raw sequence is at least l_SL long (the paper's production regime).  A sequence shorter than l_SL
    is not touched by SL and weighs n_u^gamma either way; priced the listing's way, a batch with many short sequences
    gets a negative budget, admits nobody and lands far below the target, against the text's "matches l as closely as
    possible".  So the sampled weight of a sequence is min(n_u, l_SL)^gamma here: the baseline is the sum of those, and
    admitting u costs n_u^gamma - min(n_u, l_SL)^gamma.  When every n_u >= l_SL this is the listing's condition verbatim.
  * READING: the periodic recalibration runs after the warm-up only.  The listing's "else if t mod T_recal = 0" would
    also fire inside a warm-up longer than T_recal and clear the accumulators that the warm-up mean (divided by T_warm)
    is about to use.
  * The first window after warm-up may hold fewer than T_recal steps; the listing divides by T_recal all the same, and so
    does this.
"""
import math


def sl_weight(n, sl_len):
    """Probability that standard SL leaves a sequence of n items unsampled."""
    return 1.0 if n <= sl_len else (float(sl_len) / float(n)) ** 2


def seq_load(n, gamma):
    return math.pow(float(n), gamma) if n > 0 else 0.0


def standard_sl_load(n, sl_len, gamma):
    """Expected load of one sequence under standard SL."""
    w = sl_weight(n, sl_len)
    return w * seq_load(n, gamma) + (1.0 - w) * seq_load(min(n, sl_len), gamma)


def standard_sl(lengths, uniforms, sl_len):
    """Standard SL on one batch: (new lengths, unsampled flags).  Sequence u stays whole iff uniforms[u] < SLWeight."""
    out, keep = [], []
    for n, u in zip(lengths, uniforms):
        whole = u < sl_weight(n, sl_len)
        keep.append(bool(whole))
        out.append(int(n) if whole else min(int(n), sl_len))
    return out, keep


def weighted_permutation(weights, uniforms):
    """Indices in the order of a weighted draw without replacement (exponential clocks, see the module header)."""
    keys = []
    for i, (w, u) in enumerate(zip(weights, uniforms)):
        keys.append((-math.log(u) / w if w > 0.0 else math.inf, i))
    keys.sort()
    return [i for _, i in keys]


def constrained_fill(lengths, order, target, sl_len, gamma):
    """The untruncated set of Alg. 1: walk `order`, admit u while the extra load over an all-sampled batch stays within
    target - (load of the all-sampled batch)."""
    sampled = [seq_load(min(n, sl_len), gamma) for n in lengths]
    budget = target - sum(sampled)
    s = 0.0
    chosen = [False] * len(lengths)
    for u in order:
        extra = seq_load(lengths[u], gamma) - sampled[u]
        if s + extra <= budget:
            chosen[u] = True
            s += extra
    return chosen


class Lbsl:
    """Alg. 1 over `world_size` simulated ranks."""

    def __init__(self, world_size, warmup_steps, recal_interval, sl_len, gamma):
        self.R, self.t_warm, self.t_recal, self.sl_len, self.gamma = world_size, warmup_steps, recal_interval, sl_len, gamma
        self.step_no = 0
        self.target = 0.0
        self.rank_load = [0.0] * world_size

    def step(self, batches, uniforms):
        """batches[r]: raw lengths of rank r; uniforms[r]: one number in (0, 1) per sequence.
        Returns (new lengths per rank, unsampled flags per rank, realised load per rank)."""
        self.step_no += 1
        t = self.step_no
        out_len, out_keep, realised = [], [], []
        for r in range(self.R):
            lens, us = list(batches[r]), list(uniforms[r])
            self.rank_load[r] += sum(standard_sl_load(n, self.sl_len, self.gamma) for n in lens)
            if t <= self.t_warm:
                new, keep = standard_sl(lens, us, self.sl_len)
            else:
                w = [sl_weight(n, self.sl_len) for n in lens]
                order = weighted_permutation(w, us)
                keep = constrained_fill(lens, order, self.target, self.sl_len, self.gamma)
                new = [int(n) if k else min(int(n), self.sl_len) for n, k in zip(lens, keep)]
            out_len.append(new)
            out_keep.append(keep)
            realised.append(sum(seq_load(n, self.gamma) for n in new))
        if t == self.t_warm:
            self.target = sum(self.rank_load) / (self.R * self.t_warm)
            self.rank_load = [0.0] * self.R
        elif t > self.t_warm and t % self.t_recal == 0:
            self.target = sum(self.rank_load) / (self.R * self.t_recal)
            self.rank_load = [0.0] * self.R
        return out_len, out_keep, realised


def fit_gamma(lengths, times):
    """Least-squares slope of log(time) against log(length): the load exponent that a measured cost curve implies."""
    xs = [math.log(float(n)) for n in lengths]
    ys = [math.log(float(t)) for t in times]
    mx, my = sum(xs) / len(xs), sum(ys) / len(ys)
    return sum((x - mx) * (y - my) for x, y in zip(xs, ys)) / sum((x - mx) ** 2 for x in xs)
