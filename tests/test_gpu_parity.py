"""Parity of the HIP path (through the C ABI) against the CPU fp64 oracle, element by element,
on the same seeded inputs.  Tolerance tol = 2e-2 for bf16 storage, 1e-5 for fp32, applied to the
max error normalised by the largest reference magnitude and to the max-abs error (the latter
against tol * max(1, max|ref|): a bf16 output of magnitude 10 cannot be closer than 0.03)."""
import numpy as np
import pytest
import torch

from oracle import hstu_oracle as orc
from paper_2602_16986_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL = {"bf16": 2e-2, "fp32": 1e-5}


@pytest.fixture(scope="module")
def hb():
    assert torch.cuda.is_available(), "GPU tests need a GPU; deselect with -m 'not gpu'"
    from paper_2602_16986_amd import binding
    return binding


def to_np(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def check(name, got, ref, tol):
    got = np.asarray(got, dtype=np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    if ref.size == 0:
        return
    assert np.all(np.isfinite(got)), f"{name}: non-finite values"
    err = np.abs(got - ref).max()
    scale = np.abs(ref).max()
    rel = err / scale if scale > 0 else err
    print(f"  {name}: max_abs_err={err:.3e} max|ref|={scale:.3e} normalised={rel:.3e}", flush=True)
    assert err <= tol * max(1.0, scale), f"{name}: max abs error {err:.3e} > {tol * max(1.0, scale):.3e}"
    assert rel <= tol, f"{name}: normalised max error {rel:.3e} > {tol}"


def oracle_args(w):
    return dict(num_targets=w.num_targets, K1=w.K1, K2=w.K2, alpha=w.alpha, inv_n=1.0 / w.N, table=w.table,
                bounds=w.bounds)


def run_case(w, fused=False):
    from paper_2602_16986_amd.runner import DeviceWorkload
    print(f"case {w.name}: lengths={w.lengths.tolist()} H={w.H} d={w.d} {w.dtype} K1={w.K1} K2={w.K2} "
          f"targets={None if w.num_targets is None else w.num_targets.tolist()}", flush=True)
    tol = TOL[w.dtype]
    dw = DeviceWorkload(w, fused_qkvu=fused)
    dw.out.fill_(float("nan"))
    out = to_np(dw.attn_fwd())
    torch.cuda.synchronize()
    ref = orc.attn_fwd(w.q, w.k, w.v, w.offsets, **oracle_args(w))
    check("A", out, ref, tol)
    for t in (dw.dq, dw.dk, dw.dv):
        t.fill_(float("nan"))
    dq, dk, dv = (to_np(t) for t in dw.attn_bwd())
    torch.cuda.synchronize()
    rq, rk, rv = orc.attn_bwd(w.q, w.k, w.v, w.dout, w.offsets, **oracle_args(w))
    check("dQ", dq, rq, tol)
    check("dK", dk, rk, tol)
    check("dV", dv, rv, tol)
    return dw


@pytest.mark.parametrize("name", wl.SMALL_CASES)
def test_small_cases(hb, name):
    run_case(wl.small(name))


def test_config1_fp32_forward(hb):
    w = wl.config("C1")
    from paper_2602_16986_amd.runner import DeviceWorkload
    dw = DeviceWorkload(w)
    out = to_np(dw.attn_fwd())
    ref = orc.attn_fwd(w.q, w.k, w.v, w.offsets, **oracle_args(w))
    check("A", out, ref, 1e-5)


def test_fused_strided_views(hb):
    # Q, K, V, U as column slices of one [T, 4*H*d] buffer: row strides differ from H*d
    run_case(wl.small("bf16-sparse"), fused=True)


def test_general_alpha(hb):
    w = wl.small("bf16-targets-sparse")
    w.alpha = 0.37
    run_case(w)


def test_empty_batch_and_errors(hb):
    from paper_2602_16986_amd.runner import DeviceWorkload
    w = wl.build("empty", [0, 0], 2, 128, "bf16", seed=0)
    dw = DeviceWorkload(w)
    dw.attn_fwd()
    dw.attn_bwd()
    torch.cuda.synchronize()
    # too-small workspace and bad head_dim are reported, not launched
    w2 = wl.small("bf16-dense")
    dw2 = DeviceWorkload(w2)
    with pytest.raises(hb.HstuError) as e:
        hb.hstu_attn_fwd(dw2.problem, dw2.q, dw2.k, dw2.v, dw2.out, dw2.ws_fwd[:256])
    assert e.value.status == -4
    dw2.problem.params.head_dim = 48
    with pytest.raises(hb.HstuError) as e:
        hb.hstu_attn_fwd(dw2.problem, dw2.q, dw2.k, dw2.v, dw2.out, dw2.ws_fwd)
    assert e.value.status == -3
    dw2.problem.params.head_dim = 128
    bad = w2.offsets.copy()
    bad[2] = bad[1] - 1
    dw2.problem._host[:] = bad
    with pytest.raises(hb.HstuError) as e:
        hb.hstu_attn_fwd(dw2.problem, dw2.q, dw2.k, dw2.v, dw2.out, dw2.ws_fwd)
    assert e.value.status == -2


@pytest.mark.parametrize("dtype,D", [("bf16", 256), ("bf16", 1024), ("fp32", 64), ("bf16", 520), ("bf16", 4096),
                                      ("bf16", 1536), ("bf16", 2048), ("fp32", 1032), ("bf16", 8192), ("fp32", 4104)])
def test_gated_norm(hb, dtype, D):
    rng = np.random.default_rng(1)
    T = 301
    rnd = (lambda *s: wl.round_to_bf16(rng.standard_normal(s, dtype=np.float32))) if dtype == "bf16" else \
          (lambda *s: rng.standard_normal(s, dtype=np.float32))
    a, u, dy = rnd(T, D) * np.float32(0.01), rnd(T, D), rnd(T, D)
    a = wl.round_to_bf16(a) if dtype == "bf16" else a
    gamma = (1 + 0.1 * rng.standard_normal(D)).astype(np.float32)
    beta = (0.1 * rng.standard_normal(D)).astype(np.float32)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    dev = "cuda:0"
    ta, tu, tdy = (torch.from_numpy(x).to(dev, tdt) for x in (a, u, dy))
    tg, tb = torch.from_numpy(gamma).to(dev), torch.from_numpy(beta).to(dev)
    tol = TOL[dtype]
    for use_beta in (False, True):
        y = torch.full_like(ta, float("nan"))
        mean = torch.empty(T, dtype=torch.float32, device=dev)
        rstd = torch.empty(T, dtype=torch.float32, device=dev)
        hb.hstu_gated_norm_fwd(ta, tu, tg, tb if use_beta else None, 1e-5, y, mean, rstd)
        ry, rmean, rrstd = orc.gated_norm_fwd(a, u, gamma, beta if use_beta else None, 1e-5)
        check(f"Y(beta={use_beta})", to_np(y), ry, tol)
        check("mean", to_np(mean), rmean, 1e-5)
        np.testing.assert_allclose(to_np(rstd), rrstd, rtol=1e-4)
        da, du = torch.full_like(ta, float("nan")), torch.full_like(ta, float("nan"))
        dg = torch.empty(D, dtype=torch.float32, device=dev)
        db = torch.empty(D, dtype=torch.float32, device=dev)
        ws = hb.new_workspace(hb.hstu_gated_norm_bwd_workspace_bytes(T, D), dev)
        hb.hstu_gated_norm_bwd(tdy, ta, tu, tg, tb if use_beta else None, 1e-5, da, du, dg, db, ws)
        rda, rdu, rdg, rdb = orc.gated_norm_bwd(dy, a, u, gamma, beta if use_beta else None, 1e-5)
        check("dA", to_np(da), rda, tol)
        check("dU", to_np(du), rdu, tol)
        check("dgamma", to_np(dg), rdg, 1e-3 if dtype == "bf16" else 1e-5)
        check("dbeta", to_np(db), rdb, 1e-3 if dtype == "bf16" else 1e-5)


def test_layer_chain_small(hb):
    """attention fwd -> gated norm fwd -> gated norm bwd -> attention bwd on one small batch,
    each stage checked against the oracle fed with the GPU's own (rounded) input to that stage."""
    from paper_2602_16986_amd.runner import DeviceWorkload
    w = wl.small("bf16-targets")
    dw = DeviceWorkload(w)
    dw.layer_step()
    torch.cuda.synchronize()
    a_gpu = to_np(dw.out)
    ry, _, _ = orc.gated_norm_fwd(a_gpu, w.u, w.gamma, None, w.eps)
    check("Y", to_np(dw.y), ry, 2e-2)
    rda, rdu, rdg, _ = orc.gated_norm_bwd(w.dy, a_gpu, w.u, w.gamma, None, w.eps)
    check("dA", to_np(dw.dattn), rda, 2e-2)
    check("dU", to_np(dw.du), rdu, 2e-2)
    check("dgamma", to_np(dw.dgamma), rdg, 2e-2)
    rq, rk, rv = orc.attn_bwd(w.q, w.k, w.v, to_np(dw.dattn), w.offsets, **oracle_args(w))
    check("dQ", to_np(dw.dq), rq, 2e-2)
    check("dK", to_np(dw.dk), rk, 2e-2)
    check("dV", to_np(dw.dv), rv, 2e-2)


@pytest.mark.parametrize("B,lo,hi,K1,K2", [
    (24, 500, 1100, 64, 128),     # a few hundred global-prefix key blocks, each cut into 3-4 pieces
    (96, 520, 700, 32, 128),      # more cut candidates than partial-sum slots: the piece size grows until they fit
    (3, 2500, 4000, 96, 300),     # long pieces, ragged prefix (300 keys = 2.3 key blocks)
])
def test_backward_with_cut_key_blocks(hb, B, lo, hi, K1, K2):
    """dK/dV of key blocks that the scheduler cuts along the query axis (keys of the global prefix are seen by
    every query): pieces leave fp32 partial sums that a combine kernel adds up; compared with the oracle."""
    rng = np.random.default_rng(B * 1000 + K2)
    L = rng.integers(lo, hi + 1, size=B)
    L[1] = 0                                              # an empty sequence in the middle of the list
    w = wl.build(f"cut-B{B}", L, 2, 128, "bf16", rng=rng, K1=K1, K2=K2, backward=True)
    run_case(w)


def test_backward_cut_key_blocks_d64_and_fp32(hb):
    rng = np.random.default_rng(77)
    w = wl.build("cut-d64", rng.integers(900, 1500, size=4), 2, 64, "bf16", rng=rng, K1=40, K2=100, backward=True)
    run_case(w)
    w = wl.build("cut-fp32", rng.integers(600, 900, size=3), 2, 32, "fp32", rng=rng, K1=40, K2=100, backward=True)
    run_case(w)


def bias_gradient_case(w):
    """d table of hstu_attn_bwd (p->d_rab_table) against the oracle; dq, dk, dv must not change with it."""
    from paper_2602_16986_amd.runner import DeviceWorkload
    tol = TOL[w.dtype]
    dw = DeviceWorkload(w, bias_grad=True)
    dw.dtable.fill_(float("nan"))
    dq, dk, dv = (to_np(t) for t in dw.attn_bwd())
    torch.cuda.synchronize()
    ref = orc.attn_bwd_bias(w.q, w.k, w.v, w.dout, w.offsets, **oracle_args(w))
    check("dtable", to_np(dw.dtable), ref, tol)
    plain = DeviceWorkload(w)
    pq, pk, pv = (to_np(t) for t in plain.attn_bwd())
    torch.cuda.synchronize()
    assert np.array_equal(dq, pq) and np.array_equal(dk, pk) and np.array_equal(dv, pv)


@pytest.mark.parametrize("name", wl.SMALL_CASES)
def test_bias_table_gradient_small_cases(hb, name):
    w = wl.small(name)
    if w.table is None:
        pytest.skip("case without a bias table")
    bias_gradient_case(w)


def test_bias_table_gradient_general_alpha_and_targets(hb):
    rng = np.random.default_rng(91)
    L = rng.integers(100, 700, size=5)
    w = wl.build("dbias-alpha", L, 2, 128, "bf16", rng=rng, K1=150, K2=40, alpha=0.5, backward=True,
                 num_targets=np.array([17, 0, 33, 5, 64], dtype=np.int32))
    bias_gradient_case(w)
    w = wl.build("dbias-fp32", rng.integers(50, 300, size=3), 2, 64, "fp32", rng=rng, backward=True,
                 num_targets=np.array([3, 0, 9], dtype=np.int32))
    bias_gradient_case(w)


def test_bias_table_gradient_long_sequences(hb):
    """Sequences long enough that whole 128 x 64 tiles fall inside one bucket of the log-spaced table (distances beyond about
    2,200): those tiles add a plain sum instead of diagonal sums.  bf16 / 128 features (pipelined tiles), and fp32 / 32
    features (general path), dense and with a local window wider than the single-bucket distance."""
    rng = np.random.default_rng(92)
    bias_gradient_case(wl.build("dbias-long", [6000, 3100], 2, 128, "bf16", rng=rng, backward=True))
    bias_gradient_case(wl.build("dbias-long-window", [7000], 1, 128, "bf16", rng=rng, K1=4000, K2=300, backward=True))
    bias_gradient_case(wl.build("dbias-long-fp32", [4200], 1, 32, "fp32", rng=rng, backward=True))


# ----------------------------------------------------------------------------------------------
# forward restricted to the last rows of every sequence (hstu_attn_params.query_tail)
# ----------------------------------------------------------------------------------------------
def tail_rows(w, tail):
    """Global indices of the rows a query tail computes: the last min(n, tail) history rows and the candidates."""
    rows = []
    for b in range(w.B):
        s0, s1 = int(w.offsets[b]), int(w.offsets[b + 1])
        M = 0 if w.num_targets is None else int(w.num_targets[b])
        n = s1 - s0 - M
        rows.extend(range(s0 + max(n - tail, 0), s1))
    return np.array(rows, dtype=np.int64)


@pytest.mark.parametrize("name,tail", [("bf16-dense", 1), ("bf16-dense", 100), ("bf16-dense", 10000), ("bf16-sparse", 130),
                                       ("bf16-targets", 64), ("bf16-targets-sparse", 7), ("bf16-d64", 33), ("fp32-sparse", 40)])
def test_forward_query_tail(hb, name, tail):
    """Only the tail rows are computed (against the oracle's rows, one by one) and every other output row keeps its old
    contents; the scheduler visits fewer tiles than for the whole batch."""
    from paper_2602_16986_amd.runner import DeviceWorkload
    w = wl.small(name)
    dw = DeviceWorkload(w)
    dw.attn_fwd()
    torch.cuda.synchronize()
    all_tiles = hb.hstu_attn_schedule_stats(dw.problem, dw.ws_fwd, False)["tiles"]
    prob = hb.AttnProblem(dw.q, dw.k, dw.v, dw.out, dw.offsets, max_seqlen=w.max_seqlen, seq_offsets_host=w.offsets,
                          num_targets=dw.num_targets, local_window=w.K1, global_prefix=w.K2, alpha=w.alpha, inv_n=1.0 / w.N,
                          rab_table=dw.table, rab_bounds=dw.bounds, query_tail=tail)
    ws = hb.new_workspace(hb.hstu_attn_workspace_bytes(prob, False), dw.device)
    sentinel = 12288.0
    dw.out.fill_(sentinel)
    hb.hstu_attn_fwd(prob, dw.q, dw.k, dw.v, dw.out, ws)
    torch.cuda.synchronize()
    rows = tail_rows(w, tail)
    print(f"query tail {tail} on {name}: {len(rows)} of {w.T} rows", flush=True)
    got = to_np(dw.out)
    ref = orc.attn_fwd(w.q, w.k, w.v, w.offsets, rows=rows, **oracle_args(w))
    check("A (tail rows)", got[rows], ref, TOL[w.dtype])
    other = np.ones(w.T, dtype=bool)
    other[rows] = False
    assert np.all(got[other] == np.float64(torch.tensor(sentinel, dtype=dw.out.dtype).item())), "rows outside the tail were written"
    tiles = hb.hstu_attn_schedule_stats(prob, ws, False)["tiles"]
    assert tiles <= all_tiles
    if len(rows) < w.T // 2:
        assert tiles < all_tiles
    with pytest.raises(hb.HstuError):                          # forward only
        hb.hstu_attn_bwd(prob, dw.q, dw.k, dw.v, dw.dout, dw.dq, dw.dk, dw.dv, dw.ws_bwd)


def test_schedule_is_a_longest_first_permutation(hb):
    """The forward work list of a dense batch, read back from the workspace.  Every (sequence, row block, head) appears
    either once (whole) or as pieces [t0, t1) that tile its list of column tiles exactly, each piece with a partial-sum slot
    of its own.  The list is made of groups of 4 entries, each group written once per head (4 consecutive items share a
    head); the entries come with non-increasing cost (tiles of the entry; a whole block of a dense causal batch without
    candidates has last row / 32 + 1), equal costs in natural order (sequence, block descending, piece)."""
    from paper_2602_16986_amd.runner import DeviceWorkload
    rng = np.random.default_rng(4)
    G = 4
    some_cut = False
    for lengths in ([300, 0, 1, 129, 517, 64], rng.integers(1, 3000, size=23).tolist(), [4000]):
        w = wl.build("sched", lengths, 3, 128, "bf16", seed=1)
        dw = DeviceWorkload(w)
        dw.attn_fwd()
        torch.cuda.synchronize()
        st = hb.hstu_attn_schedule_stats(dw.problem, dw.ws_fwd, False)
        n = st["items"]
        items = dw.ws_fwd[256:256 + 32 * n].cpu().numpy().view(np.int32).reshape(n, 8)
        BM = 128
        full = lambda b, rb: (min((rb + 1) * BM, lengths[b]) - 1) // 32 + 1
        got = [(int(b), int(rbh) >> 8, int(rbh) & 255, int(t0), int(t1), int(slot)) for b, rbh, t0, t1, slot, *_ in items]
        assert n % w.H == 0
        # every block covered exactly once
        cover = {}
        for b, rb, h, t0, t1, slot in got:
            cover.setdefault((b, rb, h), []).append((t0, min(t1, full(b, rb)), slot))
        assert set(cover) == {(b, rb, h) for b, L in enumerate(lengths) for rb in range((L + BM - 1) // BM) for h in range(w.H)}
        slots = [slot for v in cover.values() for _, _, slot in v if slot >= 0]
        assert len(slots) == len(set(slots))
        for (b, rb, h), v in cover.items():
            v.sort()
            if len(v) == 1:
                assert v[0] == (0, full(b, rb), -1)
            else:
                some_cut = True
                assert v[0][0] == 0 and v[-1][1] == full(b, rb) and all(x[1] == y[0] for x, y in zip(v, v[1:]))
                assert [x[2] for x in v] == list(range(v[0][2], v[0][2] + len(v)))      # consecutive slots in piece order
        # run structure and order
        entries = []
        for g0 in range(0, n, G * w.H):
            grp = got[g0:g0 + G * w.H]
            size = len(grp) // w.H
            first = [(b, rb, t0, t1) for b, rb, h, t0, t1, slot in grp[:size]]
            for h in range(w.H):
                assert [(b, rb, hh, t0, t1) for b, rb, hh, t0, t1, slot in grp[h * size:(h + 1) * size]] == \
                       [(b, rb, h, t0, t1) for b, rb, t0, t1 in first]
            entries += first
        cost = [min(t1, full(b, rb)) - t0 for b, rb, t0, t1 in entries]
        for (a, ca), (b_, cb) in zip(zip(entries, cost), zip(entries[1:], cost[1:])):
            assert ca > cb or (ca == cb and (a[0], -a[1], a[2]) < (b_[0], -b_[1], b_[2])), "not longest-first with natural ties"
    assert some_cut, "the single long sequence should have had its last blocks cut"


def test_reuse_schedule_gives_identical_results(hb):
    """A second forward (backward) that reuses the work lists of the first in the same workspace, on new tensors of the
    same batch (the next layer of a model): bit-identical to a call that builds its own lists; a value other than 0/1 is
    rejected."""
    from paper_2602_16986_amd.runner import DeviceWorkload
    for name in ("bf16-sparse", "bf16-targets"):
        w = wl.small(name)
        dw = DeviceWorkload(w)
        dw.attn_fwd()
        dw.attn_bwd()
        torch.cuda.synchronize()
        # "next layer": other values, same geometry
        q2, k2, v2 = (t.flip(0).contiguous() for t in (dw.q, dw.k, dw.v))
        outs = []
        for reuse in (0, 1):
            out = torch.full_like(dw.out, float("nan"))
            dw.attn_fwd()                                   # leaves this problem's forward lists in ws_fwd
            dw.problem.params.reuse_schedule = reuse
            hb.hstu_attn_fwd(dw.problem, q2, k2, v2, out, dw.ws_fwd)
            dq, dk, dv = (torch.full_like(t, float("nan")) for t in (dw.q, dw.k, dw.v))
            dw.problem.params.reuse_schedule = 0
            dw.attn_bwd()                                   # this problem's backward lists in ws_bwd
            dw.problem.params.reuse_schedule = reuse
            hb.hstu_attn_bwd(dw.problem, q2, k2, v2, dw.dout, dq, dk, dv, dw.ws_bwd)
            torch.cuda.synchronize()
            dw.problem.params.reuse_schedule = 0
            outs.append((out, dq, dk, dv))
        for a, b in zip(*outs):
            assert not torch.isnan(a.float()).any()
            assert torch.equal(a, b)
    dw.problem.params.reuse_schedule = 2
    with pytest.raises(hb.HstuError) as e:
        hb.hstu_attn_fwd(dw.problem, dw.q, dw.k, dw.v, dw.out, dw.ws_fwd)
    assert e.value.status == -2
    dw.problem.params.reuse_schedule = 0


@pytest.mark.parametrize("lengths,H,K1,K2", [([3000], 2, -1, 0), ([1500, 40], 1, -1, 0), ([2500], 2, 700, 300)])
def test_small_batch_blocks_are_cut_in_every_pass(hb, lengths, H, K1, K2):
    """One or two long sequences: fewer blocks than the chip has workgroup slots, so the forward and the dQ pass cut their
    query blocks along the key axis and the dK/dV pass its key blocks along the query axis (partial sums + combine); parity
    as for any other case, and the lists do hold pieces."""
    from paper_2602_16986_amd.runner import DeviceWorkload
    w = wl.build("small-batch", lengths, H, 128, "bf16", seed=5, K1=K1, K2=K2, backward=True)
    run_case(w)
    dw = DeviceWorkload(w)
    dw.attn_fwd()
    dw.attn_bwd()
    torch.cuda.synchronize()
    blocks = sum((L + 127) // 128 for L in lengths) * H
    assert hb.hstu_attn_schedule_stats(dw.problem, dw.ws_fwd, False)["items"] > blocks
    assert hb.hstu_attn_schedule_stats(dw.problem, dw.ws_bwd, True)["items"] > blocks      # the dQ list


def test_huge_window_and_prefix_equal_dense(hb):
    """local_window / global_prefix near INT32_MAX (the index sums of the kernels must not wrap): same results, bit for bit,
    as the dense causal mask, forward and backward, with a ragged last tile and candidates."""
    from paper_2602_16986_amd.runner import DeviceWorkload
    lengths = [333, 97, 1000]
    targets = np.array([5, 0, 40], dtype=np.int32)
    outs = []
    for K1, K2 in ((-1, 0), (2 ** 31 - 1, 0), (2 ** 31 - 1, 2 ** 31 - 1), (0, 2 ** 31 - 1)):
        w = wl.build("huge-window", lengths, 2, 128, "bf16", seed=9, K1=K1, K2=K2, num_targets=targets, backward=True)
        dw = DeviceWorkload(w)
        dw.attn_fwd()
        dw.attn_bwd()
        torch.cuda.synchronize()
        outs.append([t.clone() for t in (dw.out, dw.dq, dw.dk, dw.dv)])
    for other in outs[1:]:
        for a, b in zip(outs[0], other):
            assert torch.equal(a, b)


def test_inconsistent_device_offsets_compute_nothing(hb):
    """Offsets that live on the device only (no host copy to validate) and contradict the description: the scheduler writes an
    empty work list, no output row is touched, and the statistics call reports the batch; a consistent batch in the same
    workspace afterwards works as usual."""
    from paper_2602_16986_amd.runner import DeviceWorkload
    w = wl.small("bf16-targets")
    dw = DeviceWorkload(w)
    good = dw.offsets.clone()
    cases = []
    bad = good.clone(); bad[2] = bad[1] - 3; cases.append(("decreasing", bad, None))
    bad = good.clone(); bad[-1] = w.T + 5; cases.append(("past the end", bad, None))
    bad = good.clone(); bad[0] = 1; cases.append(("not from zero", bad, None))
    tg = dw.num_targets.clone(); tg[0] = 10 ** 6; cases.append(("candidates > length", good.clone(), tg))
    for what, off, targets in cases:
        prob = hb.AttnProblem(dw.q, dw.k, dw.v, dw.out, off, max_seqlen=w.max_seqlen, num_targets=dw.num_targets if targets is None else targets,
                              local_window=w.K1, global_prefix=w.K2, alpha=w.alpha, inv_n=1.0 / w.N, rab_table=dw.table,
                              rab_bounds=dw.bounds)
        dw.out.fill_(3.0)
        dq, dk, dv = (torch.full_like(dw.q, 5.0) for _ in range(3))
        hb.hstu_attn_fwd(prob, dw.q, dw.k, dw.v, dw.out, dw.ws_fwd)
        hb.hstu_attn_bwd(prob, dw.q, dw.k, dw.v, dw.dout, dq, dk, dv, dw.ws_bwd)
        torch.cuda.synchronize()
        assert torch.all(dw.out == 3.0) and all(torch.all(t == 5.0) for t in (dq, dk, dv)), what
        for ws, bwd in ((dw.ws_fwd, False), (dw.ws_bwd, True)):
            with pytest.raises(hb.HstuError) as e:
                hb.hstu_attn_schedule_stats(prob, ws, bwd)
            assert e.value.status == -2, what
    dw.attn_fwd()
    torch.cuda.synchronize()
    assert hb.hstu_attn_schedule_stats(dw.problem, dw.ws_fwd, False)["items"] > 0
    ref = orc.attn_fwd(w.q, w.k, w.v, w.offsets, **oracle_args(w))
    check("A after a rejected batch", to_np(dw.out), ref, TOL[w.dtype])
