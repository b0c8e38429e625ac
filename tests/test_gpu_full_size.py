"""Parity at the benchmark's full sizes, in the launch configuration bench.py times: the HIP path runs
the whole configuration, the CPU oracle recomputes a sample of token rows (all heads) one by one.
Sampled rows: a seeded random set plus the rows where the tiling and the mask change behaviour
(sequence starts and ends, workgroup block edges, window and prefix edges, first candidates)."""
import numpy as np
import pytest
import torch

from oracle import hstu_oracle as orc
from paper_2602_16986_amd import workloads as wl

pytestmark = pytest.mark.gpu
TOL = 2e-2


def sample_rows(w, n_random=40, seed=7):
    rng = np.random.default_rng(seed)
    rows = set(rng.integers(0, w.T, size=n_random).tolist())
    # stratified: one random row of every (sequence, 128-row block), so that every work item of the forward and of both
    # backward passes (query blocks and key blocks of 128 rows) has an output row compared with the oracle
    for b in range(w.B):
        s0, L = int(w.offsets[b]), int(w.lengths[b])
        for r0 in range(0, L, 128):
            rows.add(s0 + int(rng.integers(r0, min(r0 + 128, L))))
    for b in range(w.B):
        s0, L = int(w.offsets[b]), int(w.lengths[b])
        M = 0 if w.num_targets is None else int(w.num_targets[b])
        local = [0, 1, 31, 32, 63, 64, 255, 256, 257, L - 1, L - 2, L // 2, (L // 256) * 256 - 1, (L // 256) * 256]
        if w.K1 >= 0:
            local += [w.K1 - 1, w.K1, w.K1 + 1, w.K2 - 1, w.K2, w.K2 + w.K1, L - w.K1]
        if M:
            local += [L - M - 1, L - M, L - M + 1, L - 1]
        if b < 2 or b == w.B - 1:
            rows.update(s0 + i for i in local if 0 <= i < L)
    return np.array(sorted(rows), dtype=np.int64)


def check(name, got, ref):
    err = np.abs(got - ref).max()
    scale = np.abs(ref).max()
    print(f"  {name}: rows={ref.shape[0]} max_abs_err={err:.3e} max|ref|={scale:.3e} normalised={err / scale:.3e}", flush=True)
    assert np.isfinite(got).all()
    assert err <= TOL * max(1.0, scale) and err / scale <= TOL, name


@pytest.mark.parametrize("name", ["C2", "C3-dense", "C3-sparse", "C4", "C5"])
def test_full_size_sampled(name):
    assert torch.cuda.is_available()
    from paper_2602_16986_amd.runner import DeviceWorkload
    w = wl.config(name)
    print(f"config {name}: B={w.B} T={w.T} H={w.H} d={w.d} K1={w.K1} K2={w.K2}", flush=True)
    dw = DeviceWorkload(w)
    rows = sample_rows(w)
    kw = dict(num_targets=w.num_targets, K1=w.K1, K2=w.K2, alpha=w.alpha, inv_n=1.0 / w.N, table=w.table,
              bounds=w.bounds)
    idx = torch.from_numpy(rows).to(dw.device)
    f64 = lambda t: t.index_select(0, idx).float().cpu().numpy().astype(np.float64)
    q, k, v, do = (x.astype(np.float64) for x in (w.q, w.k, w.v, w.dout))
    dw.out.fill_(float("nan"))
    dw.attn_fwd()
    torch.cuda.synchronize()
    print("  forward done on GPU", flush=True)
    check("A", f64(dw.out), orc.attn_fwd(q, k, v, w.offsets, rows=rows, **kw))
    assert torch.isfinite(dw.out.float()).all()
    if w.backward:
        for t in (dw.dq, dw.dk, dw.dv):
            t.fill_(float("nan"))
        dw.attn_bwd()
        torch.cuda.synchronize()
        print("  backward done on GPU", flush=True)
        rq, rk, rv = orc.attn_bwd(q, k, v, do, w.offsets, rows=rows, **kw)
        check("dQ", f64(dw.dq), rq)
        check("dK", f64(dw.dk), rk)
        check("dV", f64(dw.dv), rv)
        for t in (dw.dq, dw.dk, dw.dv):
            assert torch.isfinite(t.float()).all()
    if name == "C5":
        # the epilogue over every token, fed with the GPU's own attention output
        dw.norm_fwd()
        dw.norm_bwd()
        torch.cuda.synchronize()
        a_gpu = dw.out.float().cpu().numpy().astype(np.float64)
        ry, _, _ = orc.gated_norm_fwd(a_gpu, w.u, w.gamma, None, w.eps)
        got = dw.y.float().cpu().numpy().astype(np.float64)
        check("Y", got.reshape(w.T, -1), ry.reshape(w.T, -1))
        rda, rdu, rdg, _ = orc.gated_norm_bwd(w.dy, a_gpu, w.u, w.gamma, None, w.eps)
        check("dA", dw.dattn.float().cpu().numpy().astype(np.float64).reshape(w.T, -1), rda.reshape(w.T, -1))
        check("dU", dw.du.float().cpu().numpy().astype(np.float64).reshape(w.T, -1), rdu.reshape(w.T, -1))
        check("dgamma", dw.dgamma.cpu().numpy().astype(np.float64), rdg)


def test_c2_forward_every_row():
    """The 512-2048 configuration, forward: every output row against the oracle."""
    from paper_2602_16986_amd.runner import DeviceWorkload
    w = wl.config("C2")
    dw = DeviceWorkload(w)
    dw.out.fill_(float("nan"))
    dw.attn_fwd()
    torch.cuda.synchronize()
    ref = orc.attn_fwd(w.q.astype(np.float64), w.k.astype(np.float64), w.v.astype(np.float64), w.offsets, num_targets=w.num_targets,
                       K1=w.K1, K2=w.K2, alpha=w.alpha, inv_n=1.0 / w.N, table=w.table, bounds=w.bounds)
    check("A (all rows of C2)", dw.out.float().cpu().numpy().astype(np.float64), ref)


def _visible_tiles(L, M, K1, K2, r0, r1, BN):
    """Column tiles of width BN with a visible pair for rows [r0, r1] of a sequence (brute force over the tiles, from the
    mask's definition: history key j seen from position p iff j <= p and (dense or p - j < K1 or j < K2); a candidate
    stands at position n and also sees itself)."""
    n = L - M
    tiles = []
    for t in range((L + BN - 1) // BN):
        j0, j1 = t * BN, min(t * BN + BN, L) - 1
        vis = False
        # history keys of the tile seen from positions [p_lo, p_hi]
        p_lo, p_hi = min(r0, n), min(r1, n)
        jh1 = min(j1, n - 1, p_hi)
        if j0 <= jh1:
            if K1 < 0 or j0 < K2:
                vis = True
            else:                                    # band: some p in [p_lo, p_hi], j in [j0, jh1] with j <= p < j + K1
                vis = max(p_lo, j0) <= min(p_hi, jh1 + K1 - 1) and K1 > 0
        if not vis and r1 >= n:                      # candidates' own keys
            vis = max(r0, n, j0) <= min(r1, j1)
        if vis:
            tiles.append(t)
    return tiles


@pytest.mark.parametrize("name", ["C3-dense", "C4"])
def test_full_size_work_lists(name):
    """The forward work list of a full-size configuration, read back from the workspace: every (sequence, 128-row block,
    head) is there exactly once, whole or as pieces that tile its list of visible 32-key tiles exactly (the tile count is
    recomputed here from the mask's definition), pieces own distinct partial-sum slots, and the entries come longest
    first."""
    from paper_2602_16986_amd import binding as hb
    from paper_2602_16986_amd.runner import DeviceWorkload
    w = wl.config(name)
    dw = DeviceWorkload(w)
    dw.attn_fwd()
    torch.cuda.synchronize()
    st = hb.hstu_attn_schedule_stats(dw.problem, dw.ws_fwd, False)
    n = st["items"]
    items = dw.ws_fwd[256:256 + 32 * n].cpu().numpy().view(np.int32).reshape(n, 8)
    BM, BN = 128, 32
    count = {}
    for b, L in enumerate(w.lengths.tolist()):
        M = 0 if w.num_targets is None else int(w.num_targets[b])
        for rb in range((L + BM - 1) // BM):
            count[(b, rb)] = len(_visible_tiles(L, M, w.K1, w.K2, rb * BM, min(rb * BM + BM, L) - 1, BN))
    assert st["tiles"] == sum(count.values()) * w.H
    cover = {}
    for b, rbh, t0, t1, slot, seq0, length, hist in items.tolist():
        # every entry carries its sequence's first row, length and history length
        M = 0 if w.num_targets is None else int(w.num_targets[b])
        assert (seq0, length, hist) == (int(w.offsets[b]), int(w.lengths[b]), int(w.lengths[b]) - M)
        cover.setdefault((b, rbh >> 8, rbh & 255), []).append((t0, min(t1, count[(b, rbh >> 8)]), slot))
    assert set(cover) == {(b, rb, h) for (b, rb) in count for h in range(w.H)}
    slots = [x[2] for v in cover.values() for x in v if x[2] >= 0]
    assert len(slots) == len(set(slots))
    for (b, rb, h), v in cover.items():
        v.sort()
        assert v[0][0] == 0 and v[-1][1] == count[(b, rb)] and all(x[1] == y[0] for x, y in zip(v, v[1:])), (b, rb, h, v)
        assert (len(v) == 1) == (v[0][2] < 0)
    # longest first: the cost of the list's entries (one per group of 4 x H items) never increases
    cost = [min(t1, count[(b, rbh >> 8)]) - t0 for b, rbh, t0, t1, slot, *_ in items.tolist()]
    G = 4 * w.H
    firsts = [max(cost[i:i + G]) for i in range(0, n, G)]
    lasts = [min(cost[i:i + G]) for i in range(0, n, G)]
    assert all(a >= b for a, b in zip(lasts, firsts[1:])), "entries are not in longest-first order"
    print(f"{name}: {n} items, {st['tiles']} tiles, longest {max(cost)}, shortest {min(cost)}", flush=True)


def test_more_blocks_than_the_scheduler_sorts():
    """A batch with more (sequence, block) pairs than the scheduler sorts in LDS (8192) and more sequences than it
    caches (1024): the list falls back to natural order without cuts.  Forward and backward against the oracle on sampled
    rows, and the list is still a full permutation."""
    from paper_2602_16986_amd import binding as hb
    from paper_2602_16986_amd.runner import DeviceWorkload
    rng = np.random.default_rng(11)
    lengths = rng.integers(700, 1100, size=1100).tolist()               # 1100 sequences x 6-9 blocks of 128 rows = 8.6 k pairs
    w = wl.build("many-blocks", lengths, 1, 128, "bf16", seed=5, K1=300, K2=40, backward=True)
    assert sum((L + 127) // 128 for L in lengths) > 8192 and len(lengths) > 1024
    dw = DeviceWorkload(w)
    dw.out.fill_(float("nan"))
    dw.attn_fwd()
    torch.cuda.synchronize()
    st = hb.hstu_attn_schedule_stats(dw.problem, dw.ws_fwd, False)
    items = dw.ws_fwd[256:256 + 32 * st["items"]].cpu().numpy().view(np.int32).reshape(-1, 8)
    seen = sorted((int(b), int(rbh) >> 8, int(rbh) & 255) for b, rbh, *_ in items)
    assert seen == sorted((b, rb, 0) for b, L in enumerate(lengths) for rb in range((L + 127) // 128))
    assert (items[:, 4] < 0).all(), "no cuts expected on the unsorted path"
    rows = np.unique(np.concatenate([rng.integers(0, w.T, size=300), w.offsets[:-1], w.offsets[1:] - 1]))
    kw = dict(num_targets=w.num_targets, K1=w.K1, K2=w.K2, alpha=w.alpha, inv_n=1.0 / w.N, table=w.table, bounds=w.bounds)
    idx = torch.from_numpy(rows).to(dw.device)
    f64 = lambda t: t.index_select(0, idx).float().cpu().numpy().astype(np.float64)
    q, k, v, do = (x.astype(np.float64) for x in (w.q, w.k, w.v, w.dout))
    check("A", f64(dw.out), orc.attn_fwd(q, k, v, w.offsets, rows=rows, **kw))
    assert torch.isfinite(dw.out.float()).all()
    for t in (dw.dq, dw.dk, dw.dv):
        t.fill_(float("nan"))
    dw.attn_bwd()
    torch.cuda.synchronize()
    rq, rk, rv = orc.attn_bwd(q, k, v, do, w.offsets, rows=rows, **kw)
    check("dQ", f64(dw.dq), rq)
    check("dK", f64(dw.dk), rk)
    check("dV", f64(dw.dv), rv)
    for t in (dw.dq, dw.dk, dw.dv):
        assert torch.isfinite(t.float()).all()


def test_causality_and_empty_sequences_on_gpu():
    """Properties that hold at any size: perturbing later tokens leaves earlier rows bit-identical,
    and zero-length sequences neither produce nor disturb output."""
    from paper_2602_16986_amd.runner import DeviceWorkload
    w = wl.build("prop", [700, 0, 300], 2, 128, "bf16", seed=3, K1=150, K2=40)
    dw = DeviceWorkload(w)
    base = dw.attn_fwd().clone()
    torch.cuda.synchronize()
    cut = 333
    for t in (dw.q, dw.k, dw.v):
        t[cut + 1:700] += 1.0
    pert = dw.attn_fwd().clone()
    torch.cuda.synchronize()
    assert torch.equal(pert[:cut + 1], base[:cut + 1])
    assert torch.equal(pert[700:], base[700:])
    assert not torch.equal(pert[cut + 1:700], base[cut + 1:700])
    # same batch without the empty sequence gives the same rows
    w2 = wl.build("prop2", [700, 300], 2, 128, "bf16", seed=3, K1=150, K2=40)
    w2.q, w2.k, w2.v, w2.table = w.q, w.k, w.v, w.table
    out2 = DeviceWorkload(w2).attn_fwd()
    torch.cuda.synchronize()
    dw = DeviceWorkload(w)
    assert torch.equal(out2, dw.attn_fwd())
    # a window at least as long as the sequence equals dense causal
    wd = wl.build("dense", [700, 0, 300], 2, 128, "bf16", seed=3)
    ww = wl.build("wide", [700, 0, 300], 2, 128, "bf16", seed=3, K1=700, K2=0)
    assert torch.equal(DeviceWorkload(wd).attn_fwd(), DeviceWorkload(ww).attn_fwd())


def test_bias_table_gradient_at_c2_scale():
    """Gradient of the bias table on the 512-2048 configuration (42 k tokens, 1.3e8 pairs per head set): every
    bucket against the oracle."""
    import torch
    from oracle import hstu_oracle as orc
    from paper_2602_16986_amd import workloads as wl
    from paper_2602_16986_amd.runner import DeviceWorkload
    w = wl.config("C2")
    dw = DeviceWorkload(w, bias_grad=True)
    dw.attn_bwd()
    torch.cuda.synchronize()
    got = dw.dtable.float().cpu().numpy().astype(np.float64)
    ref = orc.attn_bwd_bias(w.q, w.k, w.v, w.dout, w.offsets, K1=w.K1, K2=w.K2, alpha=w.alpha, inv_n=1.0 / w.N,
                            table=w.table, bounds=w.bounds)
    err = np.abs(got - ref).max()
    scale = np.abs(ref).max()
    print(f"  dtable C2: max_abs_err={err:.3e} max|ref|={scale:.3e}", flush=True)
    assert err <= 2e-2 * max(1.0, scale) and err / scale <= 2e-2


@pytest.mark.parametrize("name,tail", [("C3-dense", 512), ("C5", 1)])
def test_full_size_query_tail(name, tail):
    """The forward restricted to the last rows of every sequence at full size (the 16k -> 512 shape of an attention
    truncation in front; candidates plus one history row on C5): sampled tail rows against the oracle, rows outside untouched."""
    from paper_2602_16986_amd import binding as hb
    from paper_2602_16986_amd.runner import DeviceWorkload
    w = wl.config(name)
    dw = DeviceWorkload(w)
    prob = hb.AttnProblem(dw.q, dw.k, dw.v, dw.out, dw.offsets, max_seqlen=w.max_seqlen, seq_offsets_host=w.offsets,
                          num_targets=dw.num_targets, local_window=w.K1, global_prefix=w.K2, alpha=w.alpha, inv_n=1.0 / w.N,
                          rab_table=dw.table, rab_bounds=dw.bounds, query_tail=tail)
    ws = hb.new_workspace(hb.hstu_attn_workspace_bytes(prob, False), dw.device)
    dw.out.fill_(768.0)
    hb.hstu_attn_fwd(prob, dw.q, dw.k, dw.v, dw.out, ws)
    torch.cuda.synchronize()
    rng = np.random.default_rng(3)
    rows, outside = [], []
    for b in range(w.B):
        s0, s1 = int(w.offsets[b]), int(w.offsets[b + 1])
        M = 0 if w.num_targets is None else int(w.num_targets[b])
        q0 = s0 + max(s1 - s0 - M - tail, 0)
        rows += [q0, s1 - 1] + rng.integers(q0, s1, size=6).tolist()
        if q0 > s0:
            outside += [s0, q0 - 1] + rng.integers(s0, q0, size=4).tolist()
    rows = np.unique(np.array(rows, dtype=np.int64))
    kw = dict(num_targets=w.num_targets, K1=w.K1, K2=w.K2, alpha=w.alpha, inv_n=1.0 / w.N, table=w.table, bounds=w.bounds)
    q, k, v = (x.astype(np.float64) for x in (w.q, w.k, w.v))
    got = dw.out.index_select(0, torch.from_numpy(rows).to(dw.device)).float().cpu().numpy().astype(np.float64)
    print(f"query tail {tail} on {name}", flush=True)
    check("A (tail rows)", got, orc.attn_fwd(q, k, v, w.offsets, rows=rows, **kw))
    untouched = dw.out.index_select(0, torch.tensor(sorted(set(outside)), device=dw.device)).float()
    assert torch.all(untouched == 768.0)
