"""Randomised (but seeded) sweep of shapes, masks and options through the whole attention path
(forward + backward through the C ABI) against the oracle: a net for index arithmetic that the
hand-picked cases miss (ragged tails at every tile size, windows that straddle tile edges,
empty and one-token sequences in any position, prefix lengths around block boundaries)."""
import numpy as np
import pytest
import torch

from paper_2602_16986_amd import workloads as wl
from tests.test_gpu_parity import run_case

pytestmark = pytest.mark.gpu


def draw_case(seed):
    rng = np.random.default_rng(10_000 + seed)
    B = int(rng.integers(1, 7))
    hi = int(rng.choice([70, 200, 450, 900]))
    L = rng.integers(0, hi + 1, size=B)
    if rng.random() < 0.3:
        L[rng.integers(0, B)] = 1
    if L.sum() == 0:
        L[0] = 33
    H = int(rng.integers(1, 4))
    d = int(rng.choice([32, 64, 128, 128]))
    dtype = "fp32" if rng.random() < 0.2 else "bf16"
    K1 = int(rng.choice([-1, -1, 0, 1, 17, 64, 129, 300]))
    K2 = int(rng.choice([0, 0, 5, 64, 130, 257])) if K1 >= 0 else 0
    targets = None
    if rng.random() < 0.4:
        targets = np.array([int(rng.integers(0, min(l, 40) + 1)) for l in L], dtype=np.int32)
    alpha = 1.0 if rng.random() < 0.7 else float(rng.choice([0.5, 0.125]))
    bias = bool(rng.random() < 0.8)
    return wl.build(f"rand{seed}", L, H, d, dtype, rng=rng, bias=bias, K1=K1, K2=K2, num_targets=targets,
                    alpha=alpha, backward=True)


@pytest.mark.parametrize("seed", range(32))
def test_random_config(seed):
    assert torch.cuda.is_available()
    run_case(draw_case(seed))
