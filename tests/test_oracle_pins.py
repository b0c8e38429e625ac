"""Pins of the CPU oracle against things other than itself: a dense numpy
formulation with an explicitly built mask, closed forms, invariants, library
routines (torch layer_norm / silu / autograd on the CPU, fp64) and finite
differences.  None of these tests needs a GPU."""
import os

import numpy as np
import pytest
import torch

from oracle import hstu_oracle as orc
from paper_2602_16986_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------------------------
# independent dense formulation (different code shape from the streaming C oracle)
# ----------------------------------------------------------------------------------------------
def paper_mask_history(n, K1, K2):
    """Mask of n history tokens built in the paper's flipped-index form (Section 4.2.1) and
    flipped back.  Paper: M[i', j] = 1 if L-K1 <= i'+j <= L, or j <= K2 and j <= L-i'.  With
    0-based inclusive indices the constants become L := n-1, K1 := K1-1, K2 := K2-1."""
    Lp, K1p, K2p = n - 1, K1 - 1, K2 - 1
    ip, j = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
    causal = ip + j <= Lp
    if K1 < 0:
        flipped = causal
    else:
        local = (Lp - K1p <= ip + j) & causal
        glob = (j <= K2p) & causal
        flipped = local | glob
    return flipped[::-1].copy()          # row t = query time


def dense_mask_and_dist(L, M, K1, K2):
    """Full mask/distances of a sequence with M trailing candidates, built from
    paper_mask_history: candidate rows are the last row of the (n+1)-token history mask
    restricted to the n history keys, plus the candidate's own diagonal entry."""
    n = L - M
    mask = np.zeros((L, L), dtype=bool)
    dist = np.zeros((L, L), dtype=np.int64)
    mask[:n, :n] = paper_mask_history(n, K1, K2)
    i, j = np.meshgrid(np.arange(L), np.arange(L), indexing="ij")
    dist[:n, :n] = (i - j)[:n, :n]
    if M > 0:
        ext = paper_mask_history(n + 1, K1, K2)[n, :n]      # position n looking at the history
        mask[n:, :n] = ext[None, :]
        dist[n:, :n] = (n - np.arange(n))[None, :]
        for c in range(n, L):
            mask[c, c] = True
            dist[c, c] = 0
    return mask, np.where(mask, dist, 0)


def dense_attention_numpy(w: wl.Workload, q=None, k=None, v=None):
    q = w.q if q is None else q
    k = w.k if k is None else k
    v = w.v if v is None else v
    out = np.zeros(q.shape, dtype=np.float64)
    for b in range(w.B):
        s0, s1 = int(w.offsets[b]), int(w.offsets[b + 1])
        L = s1 - s0
        if L == 0:
            continue
        M = 0 if w.num_targets is None else int(w.num_targets[b])
        mask, dist = dense_mask_and_dist(L, M, w.K1, w.K2)
        for h in range(w.H):
            S = w.alpha * q[s0:s1, h].astype(np.float64) @ k[s0:s1, h].astype(np.float64).T
            if w.table is not None:
                bucket = np.searchsorted(w.bounds, dist, side="right") - 1
                S = S + w.table[h].astype(np.float64)[bucket]
            P = S / (1.0 + np.exp(-S)) / w.N * mask
            out[s0:s1, h] = P @ v[s0:s1, h].astype(np.float64)
    return out


def dense_attention_torch(w: wl.Workload, q, k, v, table=None):
    """Same dense formulation in torch fp64 so autograd supplies reference gradients (``table``: the
    bias table as a torch tensor, when its gradient is wanted too)."""
    outs = []
    for b in range(w.B):
        s0, s1 = int(w.offsets[b]), int(w.offsets[b + 1])
        L = s1 - s0
        M = 0 if w.num_targets is None else int(w.num_targets[b])
        o = torch.zeros((L, w.H, w.d), dtype=torch.float64)
        if L:
            mask, dist = dense_mask_and_dist(L, M, w.K1, w.K2)
            mask_t = torch.from_numpy(mask)
            heads = []
            for h in range(w.H):
                S = w.alpha * q[s0:s1, h] @ k[s0:s1, h].T
                if w.table is not None:
                    bucket = np.searchsorted(w.bounds, dist, side="right") - 1
                    row = torch.from_numpy(w.table[h].astype(np.float64)) if table is None else table[h]
                    S = S + row[torch.from_numpy(bucket)]
                P = torch.nn.functional.silu(S) / w.N * mask_t
                heads.append(P @ v[s0:s1, h])
            o = torch.stack(heads, dim=1)
        outs.append(o)
    return torch.cat(outs, dim=0)


def oracle_fwd(w: wl.Workload, q=None, k=None, v=None, **kw):
    args = dict(num_targets=w.num_targets, K1=w.K1, K2=w.K2, alpha=w.alpha, inv_n=1.0 / w.N,
                table=w.table, bounds=w.bounds)
    args.update(kw)
    return orc.attn_fwd(w.q if q is None else q, w.k if k is None else k, w.v if v is None else v, w.offsets, **args)


def oracle_bwd(w: wl.Workload, dout=None, **kw):
    args = dict(num_targets=w.num_targets, K1=w.K1, K2=w.K2, alpha=w.alpha, inv_n=1.0 / w.N,
                table=w.table, bounds=w.bounds)
    args.update(kw)
    return orc.attn_bwd(w.q, w.k, w.v, w.dout if dout is None else dout, w.offsets, **args)


def tiny(seed, lengths, H=2, d=8, **kw):
    return wl.build("tiny", lengths, H, d, "fp32", seed=seed, **kw)


TINY_CASES = [
    dict(lengths=[7, 0, 13, 1], K1=-1, K2=0),
    dict(lengths=[19, 5], K1=4, K2=3),
    dict(lengths=[19, 5], K1=1, K2=0),
    dict(lengths=[23], K1=0, K2=5),
    dict(lengths=[23], K1=0, K2=0),
    dict(lengths=[12, 9, 30], K1=-1, K2=0, num_targets=[4, 0, 30]),
    dict(lengths=[12, 9, 30], K1=5, K2=2, num_targets=[4, 9, 7]),
    dict(lengths=[40], K1=100, K2=3),
]


# ----------------------------------------------------------------------------------------------
# P0: the mask against the hand-worked table and the paper's flipped-index formula
# ----------------------------------------------------------------------------------------------
def test_mask_matches_hand_worked_table():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "sla_mask_L8_K1_3_K2_2.txt")) if l[0] in "01"]
    golden = np.array(rows, dtype=int).astype(bool)
    m, dist = orc.mask(8, 0, 3, 2)
    assert np.array_equal(m, golden)
    assert np.array_equal(paper_mask_history(8, 3, 2), golden)
    i, j = np.nonzero(golden)
    assert np.array_equal(dist[i, j], i - j)


@pytest.mark.parametrize("L,M,K1,K2", [(17, 0, -1, 0), (17, 0, 5, 3), (17, 0, 1, 0), (17, 0, 0, 4), (17, 0, 0, 0),
                                       (17, 6, -1, 0), (17, 6, 4, 2), (17, 17, 3, 1), (33, 1, 40, 0), (1, 0, 2, 2),
                                       (64, 10, 8, 60), (50, 0, 7, 7)])
def test_mask_matches_flipped_index_formula(L, M, K1, K2):
    m, dist = orc.mask(L, M, K1, K2)
    m_ref, d_ref = dense_mask_and_dist(L, M, K1, K2)
    assert np.array_equal(m, m_ref)
    assert np.array_equal(np.where(m, dist, 0), d_ref)
    assert orc.count_pairs([L], [M], K1, K2) == int(m_ref.sum())


# ----------------------------------------------------------------------------------------------
# P1: brute force, dense formulation
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("case", range(len(TINY_CASES)))
@pytest.mark.parametrize("bias", [False, True])
def test_forward_matches_dense_formulation(case, bias):
    w = tiny(100 + case, bias=bias, alpha=0.7, N=11.0, **TINY_CASES[case])
    if bias:   # small bounds so that tiny distances span several buckets
        w.bounds = np.array([0, 1, 2, 3, 5, 8, 13, 21], dtype=np.int32)
        w.table = np.random.default_rng(5).standard_normal((w.H, 8)).astype(np.float32)
    got = oracle_fwd(w)
    ref = dense_attention_numpy(w)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-14)
    assert np.abs(ref).max() > 0 or w.K1 == 0


def test_forward_matches_dense_formulation_c1_shape():
    w = wl.config("C1")
    np.testing.assert_allclose(oracle_fwd(w), dense_attention_numpy(w), rtol=1e-11, atol=1e-14)
    assert orc.count_pairs(w.lengths) * w.H == 62278


def test_rows_subset_equals_full():
    w = tiny(3, [19, 0, 33], K1=6, K2=2, num_targets=[3, 0, 5])
    full = oracle_fwd(w)
    rows = np.array([0, 18, 19, 40, 51])
    assert np.array_equal(oracle_fwd(w, rows=rows), full[rows])
    dq, dk, dv = oracle_bwd(w)
    rq, rk, rv = oracle_bwd(w, rows=rows)
    assert np.array_equal(rq, dq[rows]) and np.array_equal(rk, dk[rows]) and np.array_equal(rv, dv[rows])


# ----------------------------------------------------------------------------------------------
# P2-P4: closed forms
# ----------------------------------------------------------------------------------------------
def test_row0_closed_form():
    w = tiny(7, [9, 4], bias=True, alpha=1.3, N=5.0)
    out = oracle_fwd(w)
    for b in range(2):
        t = int(w.offsets[b])
        for h in range(w.H):
            s = 1.3 * float(w.q[t, h].astype(np.float64) @ w.k[t, h].astype(np.float64)) + float(w.table[h, 0])
            expect = s / (1.0 + np.exp(-s)) / 5.0 * w.v[t, h].astype(np.float64)
            np.testing.assert_allclose(out[t, h], expect, rtol=1e-13)


def closed_form_count(p, K1, K2):
    """history keys visible from position p (row p itself included when it is a history row)"""
    if K1 < 0:
        return p + 1
    return min(p + 1, K1) + min(K2, max(0, p - K1 + 1))


@pytest.mark.parametrize("K1,K2", [(-1, 0), (5, 3), (1, 0), (0, 4), (3, 0), (0, 0), (9, 50), (50, 2)])
def test_zero_query_counts_visible_keys(K1, K2):
    # Q = 0 and a constant bias table c give A_i = silu(c)/N * sum of visible v_j; with V = 1 the
    # row counts its visible keys, which has a closed form.
    L, M, c, N = 31, 6, 0.75, 3.0      # c exactly representable in fp32
    n = L - M
    w = tiny(1, [L], H=1, d=4, bias=True, K1=K1, K2=K2, num_targets=[M], N=N)
    w.table = np.full_like(w.table, c)
    q = np.zeros_like(w.q)
    v = np.ones_like(w.v)
    out = oracle_fwd(w, q=q, v=v)
    silu_c = c / (1.0 + np.exp(-c))
    counts = out[:, 0, 0] * N / silu_c
    for i in range(n):
        assert abs(counts[i] - closed_form_count(i, K1, K2)) < 1e-9
    for i in range(n, L):
        # a candidate is row n of [history; itself]: the closed form at p = n counts the
        # candidate's own slot when the window reaches it (K1 != 0); with K1 = 0 only the
        # prefix rule applies and the self pair is added on top.
        expect = closed_form_count(n, K1, K2) if K1 != 0 else min(K2, n) + 1
        assert abs(counts[i] - expect) < 1e-9
    # no bias and Q = 0: silu(0) = 0, the output vanishes
    w0 = tiny(1, [L], H=1, d=4, bias=False, K1=K1, K2=K2)
    assert np.all(oracle_fwd(w0, q=np.zeros_like(w0.q)) == 0.0)


def test_complexity_bound_of_semi_local_mask():
    # Section 4.2.1: cost O((K1 + K2) L): every row sees at most K1 + K2 keys, exactly that many
    # once the row index is at least K1 + K2.
    m, _ = orc.mask(200, 0, 17, 9)
    per_row = m.sum(axis=1)
    assert per_row.max() == 26 and np.all(per_row[26:] == 26)


# ----------------------------------------------------------------------------------------------
# P5: invariants
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("K1,K2", [(-1, 0), (6, 2)])
def test_causality_under_perturbation_of_later_tokens(K1, K2):
    w = tiny(11, [25, 14], bias=True, K1=K1, K2=K2)
    base = oracle_fwd(w)
    cut = 10
    q2, k2, v2 = w.q.copy(), w.k.copy(), w.v.copy()
    rng = np.random.default_rng(0)
    for arr in (q2, k2, v2):
        arr[cut + 1:25] += rng.standard_normal(arr[cut + 1:25].shape).astype(np.float32)
    pert = oracle_fwd(w, q=q2, k=k2, v=v2)
    assert np.array_equal(pert[:cut + 1], base[:cut + 1])      # bit-identical up to the cut
    assert np.array_equal(pert[25:], base[25:])                # the other sequence untouched
    assert not np.array_equal(pert[cut + 1:25], base[cut + 1:25])


def test_window_at_least_length_equals_dense():
    w = tiny(12, [21, 8, 30], bias=True)
    dense = oracle_fwd(w)
    assert np.array_equal(oracle_fwd(w, K1=30, K2=0), dense)
    assert np.array_equal(oracle_fwd(w, K1=1000, K2=7), dense)
    assert np.array_equal(oracle_fwd(w, K1=0, K2=30), dense)
    assert np.array_equal(oracle_fwd(w, K1=3, K2=30), dense)
    assert not np.array_equal(oracle_fwd(w, K1=29, K2=0), dense)


def test_zero_length_sequences_produce_no_output():
    w = tiny(13, [0, 9, 0, 0, 6, 0], bias=True)
    out = oracle_fwd(w)
    assert out.shape[0] == 15
    w2 = tiny(13, [9, 6], bias=True)
    w2.q, w2.k, w2.v, w2.table = w.q, w.k, w.v, w.table
    assert np.array_equal(oracle_fwd(w2), out)
    empty = tiny(13, [0, 0])
    assert oracle_fwd(empty).shape == (0, 2, 8)
    dq, dk, dv = oracle_bwd(empty)
    assert dq.shape == (0, 2, 8)


# ----------------------------------------------------------------------------------------------
# P6: structure
# ----------------------------------------------------------------------------------------------
def test_linear_in_v_and_inverse_in_n():
    w = tiny(14, [17, 6], bias=True, K1=5, K2=2)
    a = oracle_fwd(w)
    np.testing.assert_allclose(oracle_fwd(w, v=2.5 * w.v.astype(np.float64)), 2.5 * a, rtol=1e-13)
    np.testing.assert_allclose(oracle_fwd(w, inv_n=1.0 / (4 * w.N)), a / 4, rtol=1e-13)


def test_batch_and_head_independence():
    w = tiny(15, [11, 7, 16], H=3, bias=True, K1=4, K2=1, num_targets=[2, 0, 5])
    full = oracle_fwd(w)
    for b in range(3):
        s0, s1 = int(w.offsets[b]), int(w.offsets[b + 1])
        alone = orc.attn_fwd(w.q[s0:s1], w.k[s0:s1], w.v[s0:s1], [0, s1 - s0], num_targets=[w.num_targets[b]],
                             K1=4, K2=1, alpha=w.alpha, inv_n=1.0 / w.N, table=w.table, bounds=w.bounds)
        assert np.array_equal(alone, full[s0:s1])
    for h in range(3):
        alone = orc.attn_fwd(w.q[:, h:h + 1], w.k[:, h:h + 1], w.v[:, h:h + 1], w.offsets, num_targets=w.num_targets,
                             K1=4, K2=1, alpha=w.alpha, inv_n=1.0 / w.N, table=w.table[h:h + 1], bounds=w.bounds)
        assert np.array_equal(alone[:, 0], full[:, h])
    # permuting the sequences permutes the output blocks
    perm = [2, 0, 1]
    seg = [slice(int(w.offsets[b]), int(w.offsets[b + 1])) for b in range(3)]
    qp, kp, vp = (np.concatenate([x[seg[b]] for b in perm]) for x in (w.q, w.k, w.v))
    op = orc.attn_fwd(qp, kp, vp, np.concatenate([[0], np.cumsum(w.lengths[perm])]), num_targets=w.num_targets[perm],
                      K1=4, K2=1, alpha=w.alpha, inv_n=1.0 / w.N, table=w.table, bounds=w.bounds)
    assert np.array_equal(op, np.concatenate([full[seg[b]] for b in perm]))


# ----------------------------------------------------------------------------------------------
# P7: target-aware rows reduce to plain causal runs
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("K1,K2", [(-1, 0), (7, 3)])
def test_candidates_equal_separate_single_candidate_runs(K1, K2):
    n, M = 20, 5
    w = tiny(16, [n + M], bias=True, K1=K1, K2=K2, num_targets=[M], N=9.0)
    full = oracle_fwd(w)
    for c in range(M):
        idx = list(range(n)) + [n + c]
        single = orc.attn_fwd(w.q[idx], w.k[idx], w.v[idx], [0, n + 1], K1=K1, K2=K2, alpha=w.alpha,
                              inv_n=1.0 / 9.0, table=w.table, bounds=w.bounds)     # no targets: plain mask
        np.testing.assert_allclose(full[n + c], single[n], rtol=1e-13, atol=1e-16)
        np.testing.assert_allclose(full[:n], single[:n], rtol=1e-13, atol=1e-16)


# ----------------------------------------------------------------------------------------------
# P8: library special cases for the epilogue
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("with_beta", [False, True])
def test_gated_norm_forward_is_layer_norm_times_u(with_beta):
    rng = np.random.default_rng(2)
    T, H, d = 13, 2, 8
    a, u = rng.standard_normal((T, H, d)), rng.standard_normal((T, H, d))
    gamma, beta = rng.standard_normal(H * d), rng.standard_normal(H * d) if with_beta else None
    y, mean, rstd = orc.gated_norm_fwd(a, u, gamma, beta, eps=1e-5)
    ta = torch.from_numpy(a.reshape(T, -1))
    ref = torch.nn.functional.layer_norm(ta, (H * d,), torch.from_numpy(gamma),
                                         None if beta is None else torch.from_numpy(beta), 1e-5)
    ref = ref * torch.from_numpy(u.reshape(T, -1))
    np.testing.assert_allclose(y.reshape(T, -1), ref.numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(mean, a.reshape(T, -1).mean(1), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(rstd, 1 / np.sqrt(a.reshape(T, -1).var(1) + 1e-5), rtol=1e-12)


@pytest.mark.parametrize("with_beta", [False, True])
def test_gated_norm_backward_matches_autograd(with_beta):
    rng = np.random.default_rng(3)
    T, D = 11, 24
    a, u, dy = rng.standard_normal((T, D)), rng.standard_normal((T, D)), rng.standard_normal((T, D))
    gamma, beta = rng.standard_normal(D), rng.standard_normal(D) if with_beta else None
    ta, tu, tg = (torch.from_numpy(x).requires_grad_() for x in (a, u, gamma))
    tb = None if beta is None else torch.from_numpy(beta).requires_grad_()
    y = torch.nn.functional.layer_norm(ta, (D,), tg, tb, 1e-5) * tu
    y.backward(torch.from_numpy(dy))
    da, du, dgamma, dbeta = orc.gated_norm_bwd(dy, a, u, gamma, beta, eps=1e-5)
    np.testing.assert_allclose(da, ta.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(du, tu.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dgamma, tg.grad.numpy(), rtol=1e-10, atol=1e-12)
    if with_beta:
        np.testing.assert_allclose(dbeta, tb.grad.numpy(), rtol=1e-10, atol=1e-12)
    else:
        np.testing.assert_allclose(dbeta, (dy * u).sum(0), rtol=1e-12)


def test_silu_matches_library():
    # one key, one feature: A = silu(q k)/N * v
    x = np.linspace(-6, 6, 25)
    for s in x:
        out = orc.attn_fwd(np.array([[[s]]]), np.array([[[1.0]]]), np.array([[[1.0]]]), [0, 1])
        assert abs(out[0, 0, 0] - float(torch.nn.functional.silu(torch.tensor(s, dtype=torch.float64)))) < 1e-14


# ----------------------------------------------------------------------------------------------
# P9: gradients
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("case", range(len(TINY_CASES)))
def test_backward_matches_autograd_of_dense_formulation(case):
    w = tiny(200 + case, bias=True, alpha=0.9, N=7.0, **TINY_CASES[case])
    w.bounds = np.array([0, 1, 2, 4, 7, 12], dtype=np.int32)
    w.table = np.random.default_rng(6).standard_normal((w.H, 6)).astype(np.float32)
    q, k, v = (torch.from_numpy(x.astype(np.float64)).requires_grad_() for x in (w.q, w.k, w.v))
    out = dense_attention_torch(w, q, k, v)
    out.backward(torch.from_numpy(w.dout.astype(np.float64)))
    dq, dk, dv = oracle_bwd(w)
    np.testing.assert_allclose(dq, q.grad.numpy(), rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(dk, k.grad.numpy(), rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(dv, v.grad.numpy(), rtol=1e-10, atol=1e-13)


def test_backward_matches_central_differences():
    w = tiny(31, [9, 6], H=1, d=4, bias=True, K1=4, K2=2, num_targets=[2, 0], alpha=1.1, N=3.0)
    w.bounds = np.array([0, 1, 3], dtype=np.int32)
    w.table = np.random.default_rng(8).standard_normal((1, 3)).astype(np.float32)
    q, k, v, g = (x.astype(np.float64) for x in (w.q, w.k, w.v, w.dout))
    dq, dk, dv = orc.attn_bwd(q, k, v, g, w.offsets, num_targets=w.num_targets, K1=4, K2=2, alpha=1.1,
                              inv_n=1 / 3.0, table=w.table, bounds=w.bounds)

    def loss(q_, k_, v_):
        return float((oracle_fwd(w, q=q_, k=k_, v=v_) * g).sum())

    h = 1e-6
    rng = np.random.default_rng(9)
    for name, arr, grad in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        for _ in range(12):
            idx = tuple(int(rng.integers(0, s)) for s in arr.shape)
            plus, minus = arr.copy(), arr.copy()
            plus[idx] += h
            minus[idx] -= h
            args = {"q": (plus, k, v), "k": (q, plus, v), "v": (q, k, plus)}[name]
            argsm = {"q": (minus, k, v), "k": (q, minus, v), "v": (q, k, minus)}[name]
            fd = (loss(*args) - loss(*argsm)) / (2 * h)
            assert abs(fd - grad[idx]) < 1e-7 * max(1.0, abs(fd)), (name, idx, fd, grad[idx])


@pytest.mark.parametrize("case", range(len(TINY_CASES)))
def test_bias_table_gradient_matches_autograd_of_dense_formulation(case):
    w = tiny(300 + case, bias=True, alpha=0.8, N=5.0, **TINY_CASES[case])
    w.bounds = np.array([0, 1, 2, 4, 7, 12], dtype=np.int32)
    w.table = np.random.default_rng(16).standard_normal((w.H, 6)).astype(np.float32)
    q, k, v = (torch.from_numpy(x.astype(np.float64)) for x in (w.q, w.k, w.v))
    table = torch.from_numpy(w.table.astype(np.float64)).requires_grad_()
    out = dense_attention_torch(w, q, k, v, table=table)
    out.backward(torch.from_numpy(w.dout.astype(np.float64)))
    got = orc.attn_bwd_bias(w.q, w.k, w.v, w.dout, w.offsets, num_targets=w.num_targets, K1=w.K1, K2=w.K2,
                            alpha=w.alpha, inv_n=1.0 / w.N, table=w.table, bounds=w.bounds)
    np.testing.assert_allclose(got, table.grad.numpy(), rtol=1e-10, atol=1e-13)


def test_bias_table_gradient_matches_central_differences():
    w = tiny(33, [11, 7], H=2, d=4, bias=True, K1=5, K2=2, num_targets=[3, 0], alpha=1.2, N=4.0)
    w.bounds = np.array([0, 1, 3, 6], dtype=np.int32)
    w.table = np.random.default_rng(18).standard_normal((2, 4)).astype(np.float32)
    g = w.dout.astype(np.float64)
    kw = dict(num_targets=w.num_targets, K1=5, K2=2, alpha=1.2, inv_n=0.25, bounds=w.bounds)
    got = orc.attn_bwd_bias(w.q, w.k, w.v, g, w.offsets, table=w.table, **kw)
    h = 1e-6
    for hh in range(2):
        for c in range(4):
            plus, minus = w.table.astype(np.float64), w.table.astype(np.float64)
            plus[hh, c] += h
            minus[hh, c] -= h
            fd = (float((orc.attn_fwd(w.q, w.k, w.v, w.offsets, table=plus, **kw) * g).sum()) -
                  float((orc.attn_fwd(w.q, w.k, w.v, w.offsets, table=minus, **kw) * g).sum())) / (2 * h)
            assert abs(fd - got[hh, c]) < 1e-7 * max(1.0, abs(fd)), (hh, c, fd, got[hh, c])


def test_bias_table_gradient_single_pair_closed_form():
    # one token: the only pair is (0, 0) at distance 0 -> bucket 0;  dL/dtable = (dO . v) silu'(s) / N
    w = tiny(35, [1], H=1, d=3, bias=True, N=2.0)
    w.bounds = np.array([0, 5], dtype=np.int32)
    w.table = np.array([[0.3, -0.7]], dtype=np.float32)
    got = orc.attn_bwd_bias(w.q, w.k, w.v, w.dout, w.offsets, inv_n=0.5, table=w.table, bounds=w.bounds)
    s = float(w.q[0, 0].astype(np.float64) @ w.k[0, 0].astype(np.float64)) + float(w.table[0, 0])
    sg = 1.0 / (1.0 + np.exp(-s))
    expect = float(w.dout[0, 0].astype(np.float64) @ w.v[0, 0].astype(np.float64)) * sg * (1 + s * (1 - sg)) * 0.5
    assert abs(got[0, 0] - expect) < 1e-14 and got[0, 1] == 0.0


def test_bucket_lookup_edges():
    # distances at, just below and beyond each bound; beyond the last bound shares the last bucket
    bounds = wl.log_bucket_bounds()
    assert bounds[0] == 0 and np.all(np.diff(bounds) > 0) and bounds.shape == (128,)
    L = 300
    w = tiny(40, [L], H=1, d=2, bias=True)
    w.bounds = np.array([0, 1, 2, 10, 100, 250], dtype=np.int32)
    w.table = np.arange(1, 7, dtype=np.float32).reshape(1, 6)
    q = np.zeros_like(w.q)
    v = np.zeros_like(w.v)
    for j, expect_bucket in ((L - 1, 0), (L - 2, 1), (L - 3, 2), (L - 10, 2), (L - 11, 3), (L - 100, 3),
                             (L - 101, 4), (L - 250, 4), (L - 251, 5), (0, 5)):
        v[:] = 0
        v[j] = 1.0
        out = orc.attn_fwd(q, w.k, v, w.offsets, table=w.table, bounds=w.bounds)
        c = float(w.table[0, expect_bucket])
        assert abs(out[L - 1, 0, 0] - c / (1 + np.exp(-c))) < 1e-14
