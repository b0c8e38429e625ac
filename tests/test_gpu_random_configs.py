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


def draw_many_heads(seed):
    """More heads and longer sequences: the scheduler sorts (sequence, block) pairs and writes every entry once per head,
    and key blocks of a global prefix are cut into pieces whose partial-sum slots are laid out per head."""
    rng = np.random.default_rng(77_000 + seed)
    B = int(rng.integers(1, 6))
    L = rng.integers(0, int(rng.choice([200, 900, 1500, 2600])) + 1, size=B)
    if L.sum() == 0:
        L[0] = 33
    H = int(rng.choice([1, 2, 4, 5, 8]))
    d = int(rng.choice([32, 64, 128, 128]))
    K1 = int(rng.choice([-1, 0, 1, 64, 129, 300, 700]))
    K2 = int(rng.choice([0, 5, 64, 130, 257, 600])) if K1 >= 0 else 0
    targets = None
    if rng.random() < 0.4:
        targets = np.array([int(rng.integers(0, min(l, 40) + 1)) for l in L], dtype=np.int32)
    return wl.build(f"heads{seed}", L, H, d, "bf16", rng=rng, bias=bool(rng.random() < 0.8), K1=K1, K2=K2, num_targets=targets,
                    backward=True)


@pytest.mark.parametrize("seed", range(10))
def test_random_config_many_heads(seed):
    run_case(draw_many_heads(seed))


def draw_pipelined(seed):
    """bf16 with 128 features and sequences of up to 3,000 tokens: the software-pipelined kernels with tile lists long enough
    for their steady state, lists that jump between the global prefix and the local band, prefixes that end inside a
    32-key sub-block (patched seeds), candidate suffixes, and blocks cut into pieces."""
    rng = np.random.default_rng(55_000 + seed)
    B = int(rng.integers(1, 5))
    L = rng.integers(1, int(rng.choice([700, 1600, 3000])) + 1, size=B)
    H = int(rng.choice([1, 2, 3]))
    K1 = int(rng.choice([-1, -1, 40, 250, 1000, 1024]))
    K2 = int(rng.choice([0, 32, 33, 100, 513])) if K1 >= 0 else 0
    targets = None
    if rng.random() < 0.4:
        targets = np.array([int(rng.integers(0, min(l, 150) + 1)) for l in L], dtype=np.int32)
    alpha = 1.0 if rng.random() < 0.5 else float(rng.choice([0.5, 0.0884]))
    return wl.build(f"pipe{seed}", L, H, 128, "bf16", rng=rng, bias=bool(rng.random() < 0.8), K1=K1, K2=K2, num_targets=targets,
                    alpha=alpha, backward=True)


@pytest.mark.parametrize("seed", range(16))
def test_random_config_pipelined_kernels(seed):
    run_case(draw_pipelined(seed))


# ----------------------------------------------------------------------------------------------
# the entry points around the attention: whole layer (bf16 and FP8 forward), FP8 GEMM, truncation, query tail
# ----------------------------------------------------------------------------------------------
def draw_layer(seed):
    rng = np.random.default_rng(20_000 + seed)
    B = int(rng.integers(1, 5))
    L = rng.integers(0, int(rng.choice([60, 200, 500])) + 1, size=B)
    if L.sum() == 0:
        L[0] = 40
    H, d = [(1, 128), (2, 64), (4, 32), (2, 128), (4, 64), (1, 64)][int(rng.integers(0, 6))]
    E = int(rng.choice([64, 128, 256, 512, 136]))
    K1 = int(rng.choice([-1, -1, 0, 33, 130]))
    K2 = int(rng.choice([0, 8, 70])) if K1 >= 0 else 0
    targets = None
    if rng.random() < 0.4:
        targets = np.array([int(rng.integers(0, min(l, 20) + 1)) for l in L], dtype=np.int32)
    return wl.build_layer(f"rand-layer{seed}", L, H, d, E, seed=seed, K1=K1, K2=K2, num_targets=targets, bias=bool(rng.random() < 0.8))


@pytest.mark.parametrize("seed", range(8))
def test_random_layer(seed):
    from tests.test_gpu_layer import run_case as run_layer
    run_layer(draw_layer(seed))


@pytest.mark.parametrize("seed", range(10))
def test_random_fp8_gemm(seed):
    from paper_2602_16986_amd import binding as hb
    from tests.test_gpu_fp8 import run_gemm
    rng = np.random.default_rng(30_000 + seed)
    M = int(rng.choice([1, 31, 127, 128, 129, 1000, 5000]))
    N = 64 * int(rng.integers(1, 17))
    K = int(rng.choice([128, 256, 512, 1024]))
    run_gemm(hb, M, N, K, with_c=bool(rng.random() < 0.7))


@pytest.mark.parametrize("seed", range(8))
def test_random_truncation_and_query_tail(seed):
    """One random jagged batch through both halves of an attention truncation: the row selection (bit-exact) and the
    forward over the rows that survive it (query tail)."""
    from oracle import hstu_oracle as orc
    from oracle import truncation as trunc
    from paper_2602_16986_amd import binding as hb
    from paper_2602_16986_amd.runner import DeviceWorkload
    w = draw_case(100 + seed)
    if w.dtype != "bf16":
        w = wl.build(w.name, w.lengths, w.H, w.d, "bf16", seed=seed, K1=w.K1, K2=w.K2, num_targets=w.num_targets, alpha=w.alpha)
    keep = int(np.random.default_rng(seed).choice([1, 16, 100, 400]))
    dw = DeviceWorkload(w)
    # row selection of Q (any tensor would do): offsets and rows bit-exact
    new_off = torch.empty(w.B + 1, dtype=torch.int32, device=dw.device)
    hb.hstu_truncate_offsets(dw.offsets, keep, dw.num_targets, new_off)
    ref_rows, ref_off = trunc.tail_slice(np.arange(w.T), w.offsets, keep, w.num_targets)
    assert np.array_equal(new_off.cpu().numpy(), ref_off)
    qs = torch.zeros(len(ref_rows) + 1, w.H, w.d, dtype=torch.bfloat16, device=dw.device)
    hb.hstu_truncate_fwd(dw.offsets, new_off, dw.q, qs[:len(ref_rows)] if len(ref_rows) else qs[:0])
    torch.cuda.synchronize()
    assert torch.equal(qs[:len(ref_rows)], dw.q[torch.from_numpy(ref_rows).to(dw.device)])
    # forward over exactly those rows
    prob = hb.AttnProblem(dw.q, dw.k, dw.v, dw.out, dw.offsets, max_seqlen=w.max_seqlen, num_targets=dw.num_targets,
                          local_window=w.K1, global_prefix=w.K2, alpha=w.alpha, inv_n=1.0 / w.N, rab_table=dw.table,
                          rab_bounds=dw.bounds, query_tail=keep)
    ws = hb.new_workspace(hb.hstu_attn_workspace_bytes(prob, False), dw.device)
    dw.out.fill_(-3.0)
    hb.hstu_attn_fwd(prob, dw.q, dw.k, dw.v, dw.out, ws)
    torch.cuda.synchronize()
    got = dw.out.float().cpu().numpy().astype(np.float64)
    if len(ref_rows):
        ref = orc.attn_fwd(w.q, w.k, w.v, w.offsets, rows=ref_rows, num_targets=w.num_targets, K1=w.K1, K2=w.K2, alpha=w.alpha,
                           inv_n=1.0 / w.N, table=w.table, bounds=w.bounds)
        scale = max(np.abs(ref).max(), 1e-30)
        assert np.abs(got[ref_rows] - ref).max() / scale <= 2e-2
    other = np.ones(w.T, dtype=bool)
    other[ref_rows] = False
    assert np.all(got[other] == -3.0)
