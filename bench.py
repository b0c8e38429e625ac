#!/usr/bin/env python3
"""Benchmark of the jagged HSTU attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C3-dense]

One step = one pass of the whole hot path over one synthetic jagged batch already resident in HBM:
tile scheduling + bias expansion + attention forward, gated-norm forward, gated-norm backward,
attention backward (dQ pass and dK/dV pass).  Prints ONE JSON line.  `value` is useful attention
TFLOP/s (forward 4*d + backward 10*d FLOPs per unmasked pair and head) over the whole step time.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA peak
PEAK_FP32_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0
# Bytes behind the L2 per launch (read + written) come from rocprofv3 FETCH_SIZE / WRITE_SIZE runs whose summaries sit under
# profiles/; profiles/traffic.json holds the figures together with a hash of the kernel sources they were measured with.
# When the sources have changed since, the figure is stale and `traffic` is reported as null.
ROOT = os.path.dirname(os.path.abspath(__file__))


TRAFFIC_SOURCES = ("attn_core.hip", "attn_fwd_pipe.hip", "gated_norm.hip", "schedule.hip", "api.hip", "hstu_common.h", "hstu_geometry.h",
                   "hstu_kernels.h")


def kernel_sources_hash():
    """Hash of the sources of the kernels whose traffic profiles/traffic.json holds (attention, gated norm, scheduler and the
    entry points that launch them)."""
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2602_16986_amd", "csrc")
    for name in TRAFFIC_SOURCES:
        h.update(name.encode())
        h.update(open(os.path.join(d, name), "rb").read())
    return h.hexdigest()


def measured_traffic(workload, kernel):
    try:
        t = json.load(open(os.path.join(ROOT, "profiles", "traffic.json")))
    except (OSError, ValueError):
        return None
    if t.get("kernel_sources_sha256") != kernel_sources_hash():
        return None
    return t.get("bytes_per_launch", {}).get(workload, {}).get(kernel)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C3-dense",
                    help="C1, C2, C3-dense, C3-sparse, C4, C5 (default: the 8k-16k config the metric is quoted on)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle baseline sample")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--fwd-only", action="store_true", help="time the forward attention only (profiling aid)")
    ap.add_argument("--bias-grad", action="store_true",
                    help="also compute the gradient of the relative-bias table in the attention backward")
    ap.add_argument("--op", default="attention", choices=["attention", "truncate", "layer", "fp8gemm"],
                    help="attention: the hot path (default).  truncate: the row selection of attention truncation "
                         "(Section 4.3) on the AT-3072-512 batch, forward + backward, in GB/s against the HBM roofline.  "
                         "layer: one whole HSTU layer with rematerialisation (hstu_layer_fwd + hstu_layer_bwd) on layer-C3")
    ap.add_argument("--fp8-shape", default="1M-512", help="--op fp8gemm: 1M-512, 1M-1K, 250K-512, 250K-1K (the paper's table)")
    ap.add_argument("--fp8", action="store_true", help="--op layer: forward with both projections in FP8 (Section 4.2.2)")
    ap.add_argument("--layer-case", default="layer-C3", help="layer workload for --op layer (layer-C3, layer-mid, ...)")
    ap.add_argument("--query-tail", type=int, default=0,
                    help="attention op, forward only: compute only the last N history rows (and the candidates) of every sequence")
    ap.add_argument("--fused-qkvu", action="store_true",
                    help="attention op: Q, K, V, U as column blocks of one [T, 4*H*d] buffer (row stride 4x) instead of four tensors")
    ap.add_argument("--reuse-schedule", action="store_true",
                    help="attention op: after the warm-up the steps reuse the work lists in the workspaces (the layers of one model "
                         "after the first); reported next to the headline, never as it: `value` of the default run includes the scheduler")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="default run (C3-dense): skip the short timed steps of the other configurations (C3-sparse, C4, C5, C2)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (profiling aid: calibrates the HBM byte counters)")
    return ap.parse_args()


def time_loop(fn, steps, torch):
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def cpu_baseline(w, fl, target_seconds):
    """The oracle as it stands, timed on this host's cores on a bounded row sample of the same batch."""
    from oracle import hstu_oracle as orc
    rng = np.random.default_rng(123)
    kw = dict(num_targets=w.num_targets, K1=w.K1, K2=w.K2, alpha=w.alpha, inv_n=1.0 / w.N, table=w.table,
              bounds=w.bounds)
    threads = orc.num_threads()
    # pilot on a few rows to size the sample
    pilot = np.sort(rng.choice(w.T, size=min(w.T, 8 * threads), replace=False))
    q, k, v, do = (x.astype(np.float64) for x in (w.q, w.k, w.v, w.dout))
    t0 = time.time()
    orc.attn_fwd(q, k, v, w.offsets, rows=pilot, **kw)
    if w.backward:
        orc.attn_bwd(q, k, v, do, w.offsets, rows=pilot, **kw)
    per_row = (time.time() - t0) / len(pilot)
    n = int(max(len(pilot), min(w.T, target_seconds / max(per_row, 1e-9))))
    rows = np.sort(rng.choice(w.T, size=n, replace=False))
    t0 = time.time()
    orc.attn_fwd(q, k, v, w.offsets, rows=rows, **kw)
    if w.backward:
        orc.attn_bwd(q, k, v, do, w.offsets, rows=rows, **kw)
    dt = time.time() - t0
    flops_total = fl["fwd"] + (fl["bwd"] if w.backward else 0.0)
    # a uniform row sample carries the same fraction of the pairs in expectation
    sample_flops = flops_total * n / w.T
    return {"value": sample_flops / dt / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "sample": f"{n} of {w.T} token rows drawn uniformly (all heads): oracle forward"
                      f"{' + backward (dQ, dK, dV rows)' if w.backward else ''}, fp64, {dt:.1f} s"}


def calibrate_copy(torch, device):
    """One plain 1 GiB device-to-device copy: the known-size kernel the HBM byte counters are scaled by."""
    src = torch.empty(1 << 30, dtype=torch.uint8, device=device)
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst


def bench_truncate(args):
    """Row selection of attention truncation: offsets + gather (forward), scatter with zero fill (backward).
    Algorithmic bytes: forward reads and writes the kept rows (2 x T' x row bytes); backward reads the kept
    rows' gradient and writes every row of the untruncated gradient ((T' + T) x row bytes)."""
    import torch
    from paper_2602_16986_amd import binding as hb
    from paper_2602_16986_amd import workloads
    c = workloads.truncation_case("AT-3072-512")
    dev = torch.device("cuda:0")
    off = torch.from_numpy(c.offsets).to(dev)
    x = torch.from_numpy(c.x.view(np.int16)).to(dev)
    new_off = torch.empty(len(c.lengths) + 1, dtype=torch.int32, device=dev)
    cap = min(x.shape[0], len(c.lengths) * c.keep)
    y = torch.empty(cap, c.width, dtype=x.dtype, device=dev)
    dx = torch.empty_like(x)

    def step():
        hb.hstu_truncate_offsets(off, c.keep, None, new_off)
        hb.hstu_truncate_fwd(off, new_off, x, y)
        hb.hstu_truncate_bwd(off, new_off, y, dx)

    if args.calibrate_copy:
        calibrate_copy(torch, dev)
    for _ in range(args.warmup):
        step()
    ms_step = time_loop(step, args.steps, torch)
    hb.hstu_profile_enable(True)
    kern = {}
    for _ in range(args.steps):
        step()
        for name, ms in hb.hstu_profile_read():
            kern.setdefault(name, []).append(ms)
    hb.hstu_profile_enable(False)
    kern = {k: float(np.mean(v)) for k, v in kern.items()}
    kept = int(new_off[-1].item())
    row = c.width * 2
    algo = {"truncate_fwd": 2.0 * kept * row, "truncate_bwd": float(kept + x.shape[0]) * row}
    dom = max(algo, key=lambda k: kern[k])
    achieved = algo[dom] / (kern[dom] * 1e-3) / 1e9
    out = {"metric": "GB/s, jagged row selection of attention truncation (forward + backward)",
           "value": sum(algo.values()) / (ms_step * 1e-3) / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "u8", "data": "synthetic",
           "config": {"workload": c.name, "B": len(c.lengths), "T": int(x.shape[0]), "kept_rows": kept, "keep": c.keep,
                      "row_bytes": row},
           "roofline": {"kernel": dom, "bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                        "frac": achieved / PEAK_HBM_GBS, "traffic": measured_traffic(c.name, dom)},
           "kernel_ms": kern,
           "kernel_gbs": {k: algo[k] / (kern[k] * 1e-3) / 1e9 for k in algo}}
    if not args.no_cpu_baseline:
        from oracle import truncation as orc
        t0 = time.time()
        yy, _ = orc.tail_slice(c.x, c.offsets, c.keep, None)
        orc.tail_slice_bwd(yy, c.offsets, c.keep, None)
        dt = time.time() - t0
        out["cpu_baseline"] = {"value": sum(algo.values()) / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                               "sample": f"the whole batch, forward + backward, numpy row copies, {dt:.2f} s"}
    print(json.dumps(out))


# FP8 GEMM with fused 2-D bias on H100, TFLOP/s (the paper's appendix table, "Bias-Fused FP8"); same metric, other hardware
PAPER_FP8_GEMM_TFLOPS = {"1M-512": 414.0, "1M-1K": 734.0, "250K-512": 414.0, "250K-1K": 721.0}


def bench_fp8_gemm(args):
    """D = A B^T + C on row-wise quantised E4M3 operands, C and D bf16 (hstu_fp8_gemm_bias2d), at the (m, k = n) shapes of
    the paper's FP8 GEMM table.  FLOPs 2 m n k; algorithmic bytes m (k + 4 n) + n k (A once, C once, D once, weights once)."""
    import torch
    from paper_2602_16986_amd import binding as hb
    from paper_2602_16986_amd import workloads
    M, KN = workloads.FP8_GEMM_SHAPES[args.fp8_shape]
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev).manual_seed(0)
    # device-side synthetic operands with the recipe of workloads.fp8_gemm_inputs (drawn on the GPU: 1M x 1K on the host takes minutes)
    a = (torch.randn(M, KN, generator=g, device=dev) * (0.2 + 2.8 * torch.rand(M, 1, generator=g, device=dev))).to(torch.bfloat16)
    b = (torch.randn(KN, KN, generator=g, device=dev) / KN ** 0.5).to(torch.bfloat16)
    c = torch.randn(M, KN, generator=g, device=dev).to(torch.bfloat16)
    qa = torch.empty((M, KN), dtype=torch.uint8, device=dev)
    sa = torch.empty(M, dtype=torch.float32, device=dev)
    qb = torch.empty((KN, KN), dtype=torch.uint8, device=dev)
    sb = torch.empty(KN, dtype=torch.float32, device=dev)
    hb.hstu_norm_quant_fp8(a, None, None, None, 0.0, qa, sa)
    hb.hstu_norm_quant_fp8(b, None, None, None, 0.0, qb, sb)
    d = torch.empty_like(c)
    step = lambda: hb.hstu_fp8_gemm_bias2d(qa, sa, qb, sb, c, d)
    quant = lambda: hb.hstu_norm_quant_fp8(a, None, None, None, 0.0, qa, sa)
    if args.calibrate_copy:
        calibrate_copy(torch, dev)
    for _ in range(args.warmup):
        step()
    ms = time_loop(step, args.steps, torch)
    ms_quant = time_loop(quant, args.steps, torch)
    hb.hstu_profile_enable(True)
    kt = []
    for _ in range(args.steps):
        step()
        kt += [t for _, t in hb.hstu_profile_read()]
    hb.hstu_profile_enable(False)
    kms = float(np.mean(kt))
    flops = 2.0 * M * KN * KN
    algo_bytes = float(M) * (KN + 4 * KN) + KN * KN
    achieved = algo_bytes / (kms * 1e-3) / 1e9
    out = {"metric": "TFLOP/s, FP8 GEMM with fused 2-D bias D = A B + C (m, k = n)", "value": flops / (ms * 1e-3) / 1e12,
           "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": flops / (ms * 1e-3) / 1e12 / PAPER_FP8_GEMM_TFLOPS[args.fp8_shape], "dtype": "fp8-e4m3",
           "data": "synthetic", "config": {"workload": f"fp8-gemm-{args.fp8_shape}", "m": M, "k": KN, "n": KN},
           "paper_h100_tflops": PAPER_FP8_GEMM_TFLOPS[args.fp8_shape],
           "roofline": {"kernel": "fp8_gemm_bias2d", "bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                        "frac": achieved / PEAK_HBM_GBS, "traffic": measured_traffic(args.fp8_shape, "fp8_gemm_bias2d")},
           "kernel_ms": {"fp8_gemm_bias2d": kms, "rowwise_quant_of_A": ms_quant},
           "mfma_frac_of_fp8_peak": flops / (kms * 1e-3) / 1e12 / 5000.0,
           "quant_gbs": float(M) * KN * 3 / (ms_quant * 1e-3) / 1e9}
    if not args.no_cpu_baseline:
        from oracle import fp8 as orc
        rows = min(M, 1 << 18)
        qa_h, sa_h, qb_h, sb_h = qa[:rows].cpu().numpy(), sa[:rows].cpu().numpy(), qb.cpu().numpy(), sb.cpu().numpy()
        c_h = c[:rows].float().cpu().numpy()
        t0 = time.time()
        orc.gemm_bias2d(qa_h, sa_h, qb_h, sb_h, c_h)
        dt = time.time() - t0
        out["cpu_baseline"] = {"value": 2.0 * rows * KN * KN / dt / 1e12, "unit": "TFLOP/s", "cores": os.cpu_count(), "kind": "oracle",
                               "sample": f"the first {rows} rows: decode + fp64 matmul + scales + C, {dt:.2f} s"}
    print(json.dumps(out))


def bench_layer(args):
    """One whole layer, forward + backward with rematerialisation.  Useful FLOPs: attention 4 d + 10 d per unmasked
    pair and head, projections 2 M N K each forward and twice that backward (the rematerialised U/V/Q/K GEMM of the
    backward is executed but not counted)."""
    import torch
    from paper_2602_16986_amd import binding as hb
    from paper_2602_16986_amd import flops, workloads
    from paper_2602_16986_amd.runner import DeviceLayer
    c = workloads.layer_case(args.layer_case)
    dl = DeviceLayer(c, fp8=args.fp8)
    HD = c.H * c.d
    fl = flops.attention_flops(c)
    gemm_fwd = 2.0 * c.T * c.E * 4 * HD + 2.0 * c.T * HD * c.E
    useful = fl["fwd"] + fl["bwd"] + 3.0 * gemm_fwd
    for _ in range(args.warmup):
        dl.step()
    ms_step = time_loop(dl.step, args.steps, torch)
    parts = {"layer_fwd": time_loop(dl.fwd, args.steps, torch), "layer_bwd": time_loop(dl.bwd, args.steps, torch)}
    hb.hstu_profile_enable(True)
    kern = {}
    for _ in range(args.steps):
        for tag, fn in (("fwd", dl.fwd), ("bwd", dl.bwd)):
            fn()
            for name, ms in hb.hstu_profile_read():
                kern.setdefault(f"{tag}:{name}", []).append(ms)
    hb.hstu_profile_enable(False)
    kern = {k: float(np.mean(v)) for k, v in kern.items()}
    algo = {"fwd:attn_fwd": 4.0, "bwd:attn_bwd_dq": 6.0, "bwd:attn_bwd_dkdv": 8.0}
    dom = max(algo, key=lambda k: kern[k])
    achieved = algo[dom] * c.d * fl["pairs"] / (kern[dom] * 1e-3) / 1e12
    e = 2 * c.T
    out = {"metric": "useful TFLOP/s, one HSTU layer forward + backward with activation rematerialisation",
           "value": useful / (ms_step * 1e-3) / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
           "data": "synthetic",
           "config": {"workload": c.name, "B": c.B, "T": c.T, "H": c.H, "d": c.d, "E": c.E, "K1": c.K1, "K2": c.K2,
                      "unmasked_pairs": fl["pairs"], "forward_projections": "fp8-e4m3" if args.fp8 else "bf16"},
           "frac_of_peak": useful / (ms_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
           "roofline": {"kernel": dom, "bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                        "frac": achieved / PEAK_BF16_TFLOPS, "traffic": None},
           "entry_ms": parts, "kernel_ms": kern,
           # the forward's two projection blocks, each with the norm in front of it (and the SiLU behind the first)
           "pre_attention_ms": sum(v for k, v in kern.items() if k in ("fwd:layer_norm_fwd", "fwd:gemm_uvqk", "fwd:silu_fwd",
                                                                       "fwd:layer_norm_quant", "fwd:fp8_gemm_uvqk")),
           "post_attention_ms": sum(v for k, v in kern.items() if k in ("fwd:gated_norm_fwd", "fwd:gemm_out", "fwd:gated_norm_quant",
                                                                        "fwd:fp8_gemm_out")),
           "attention_share_of_step": (kern["fwd:attn_fwd"] + kern["bwd:attn_bwd_dq"] + kern["bwd:attn_bwd_dkdv"]) / ms_step,
           # activations that live from the forward to the backward, with and without rematerialisation (Section 4.2.2):
           # kept: Z, U, A and two statistics per row; otherwise also X, V, Q, K, Y and the pre-activations
           "saved_bytes": {"rematerialised": e * (c.E + 2 * HD) + 8 * c.T,
                           "everything_kept": e * (2 * c.E + 4 * HD + 4 * HD + 2 * HD) + 8 * c.T}}
    print(json.dumps(out))


def other_configs(args, torch, hb, flops, workloads, DeviceWorkload, peak):
    """Short timed steps of the configurations the headline is not quoted on: the same step loop, 10 warm-up and 30 timed steps."""
    res = {}
    for name in ("C3-sparse", "C4", "C5", "C2"):
        w = workloads.config(name)
        fl = flops.attention_flops(w)
        dw = DeviceWorkload(w)
        step = dw.layer_step if w.backward else dw.attn_fwd
        for _ in range(10):                       # (the chip idles while the host builds the inputs: let its clocks settle)
            step()
        ms = time_loop(step, 30, torch)
        hb.hstu_profile_enable(True)
        kern = {}
        for _ in range(5):
            step()
            for kname, t in hb.hstu_profile_read():
                kern.setdefault(kname, []).append(t)
        hb.hstu_profile_enable(False)
        kern = {k: float(np.mean(v)) for k, v in kern.items()}
        useful = fl["fwd"] + (fl["bwd"] if w.backward else 0.0)
        r = {"pass": "fwd+bwd+epilogue" if w.backward else "fwd", "ms_per_step": ms, "tflops": useful / (ms * 1e-3) / 1e12,
             "frac_of_peak": useful / (ms * 1e-3) / 1e12 / peak, "unmasked_pairs": fl["pairs"],
             "fwd_tflops": fl["fwd"] / (kern["attn_fwd"] * 1e-3) / 1e12, "kernel_ms": kern}
        if w.backward:
            r["bwd_tflops"] = fl["bwd"] / ((kern["attn_bwd_dq"] + kern["attn_bwd_dkdv"]) * 1e-3) / 1e12
        res[name] = r
        del dw
        torch.cuda.empty_cache()
    return res


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus must be 1 (sequences shard across GPUs "
              "with no exchange in the attention path)", file=sys.stderr)
        sys.exit(2)
    if args.op == "truncate":
        return bench_truncate(args)
    if args.op == "layer":
        return bench_layer(args)
    if args.op == "fp8gemm":
        return bench_fp8_gemm(args)
    import torch
    from paper_2602_16986_amd import binding as hb
    from paper_2602_16986_amd import flops, workloads
    from paper_2602_16986_amd.runner import DeviceWorkload

    w = workloads.config(args.workload)
    fl = flops.attention_flops(w)
    dw = DeviceWorkload(w, bias_grad=args.bias_grad, fused_qkvu=args.fused_qkvu)
    do_bwd = w.backward and not args.fwd_only
    if args.query_tail > 0:                                  # forward over the last rows only: count only their pairs
        do_bwd = False
        fl = flops.attention_flops(w, pairs_per_head=flops.visible_pairs_tail(w.lengths, w.num_targets, w.K1, w.K2, args.query_tail))
        dw.problem = hb.AttnProblem(dw.q, dw.k, dw.v, dw.out, dw.offsets, max_seqlen=w.max_seqlen, seq_offsets_host=w.offsets,
                                    num_targets=dw.num_targets, local_window=w.K1, global_prefix=w.K2, alpha=w.alpha,
                                    inv_n=1.0 / w.N, rab_table=dw.table, rab_bounds=dw.bounds, query_tail=args.query_tail)
        dw.ws_fwd = hb.new_workspace(hb.hstu_attn_workspace_bytes(dw.problem, False), dw.device)

    def step():
        if do_bwd:
            dw.layer_step()
        else:
            dw.attn_fwd()

    if args.calibrate_copy:
        calibrate_copy(torch, dw.device)
    for _ in range(args.warmup):
        step()
    ms_step = time_loop(step, args.steps, torch)
    ms_reuse = None
    if args.reuse_schedule:                                  # the lists of this batch are in both workspaces now
        dw.problem.params.reuse_schedule = 1
        ms_reuse = time_loop(step, args.steps, torch)
        dw.problem.params.reuse_schedule = 0

    # per-entry-point and per-kernel times (separate loops, HIP events inside the library)
    parts = {"attn_fwd": time_loop(dw.attn_fwd, args.steps, torch)}
    if do_bwd:
        parts["gated_norm_fwd"] = time_loop(dw.norm_fwd, args.steps, torch)
        parts["gated_norm_bwd"] = time_loop(dw.norm_bwd, args.steps, torch)
        parts["attn_bwd"] = time_loop(lambda: dw.attn_bwd(dout=dw.dattn), args.steps, torch)
    hb.hstu_profile_enable(True)
    kern = {}
    for _ in range(args.steps):
        step()
        for name, ms in hb.hstu_profile_read():
            kern.setdefault(name, []).append(ms)
    hb.hstu_profile_enable(False)
    kern = {k: float(np.mean(v)) for k, v in kern.items()}

    useful = fl["fwd"] + (fl["bwd"] if do_bwd else 0.0)
    value = useful / (ms_step * 1e-3) / 1e12
    peak = PEAK_BF16_TFLOPS if w.dtype == "bf16" else PEAK_FP32_TFLOPS

    # Roofline of the dominant kernel, in USEFUL FLOPs: of the 10 d the backward owes per unmasked pair (S, dP, dV, dK,
    # dQ) the dK/dV pass is credited with dV, dK and half of the S and dP that both passes compute (6 d), the dQ pass with dQ
    # and the other half (4 d); the forward with its 4 d.  What the passes execute (4 d, 6 d, 8 d) is reported beside it.
    useful_d = {"attn_fwd": 4.0, "attn_bwd_dq": 4.0, "attn_bwd_dkdv": 6.0}
    executed_d = {"attn_fwd": 4.0, "attn_bwd_dq": 6.0, "attn_bwd_dkdv": 8.0}
    dom = max((k for k in kern if k in useful_d), key=lambda k: kern[k])
    achieved = useful_d[dom] * w.d * fl["pairs"] / (kern[dom] * 1e-3) / 1e12
    roofline = {"kernel": dom, "bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                "frac": achieved / peak, "traffic": measured_traffic(w.name, dom),
                "flops_basis": "useful: %g d per unmasked pair and head" % useful_d[dom]}
    executed = {k: executed_d[k] * w.d * fl["pairs"] / (kern[k] * 1e-3) / 1e12 / peak for k in kern if k in executed_d}

    sched = hb.hstu_attn_schedule_stats(dw.problem, dw.ws_fwd, False)
    eb = flops.epilogue_bytes(w)
    out = {
        "metric": "useful TFLOP/s (fwd, fwd+bwd) & % bf16 MFMA peak, jagged HSTU attention",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "pass": ("fwd+bwd+epilogue" if do_bwd else "fwd") + ("+dbias" if args.bias_grad else "") +
                           (f", last {args.query_tail} rows" if args.query_tail > 0 else ""), "B": w.B, "T": w.T, "H": w.H,
                   "d": w.d, "K1": w.K1, "K2": w.K2, "min_len": int(w.lengths.min()), "max_len": int(w.lengths.max()),
                   "unmasked_pairs": fl["pairs"]},
        "frac_of_peak": value / peak,
        "fwd_tflops": fl["fwd"] / (kern["attn_fwd"] * 1e-3) / 1e12,
        "fwd_frac_of_peak": fl["fwd"] / (kern["attn_fwd"] * 1e-3) / 1e12 / peak,
        "roofline": roofline, "mfma_executed_frac": executed,
        "entry_ms": parts, "kernel_ms": kern,
        "schedule": {**sched, "skipped_tile_frac": 1.0 - sched["tiles"] / max(sched["dense_tiles"], 1)},
    }
    if do_bwd:
        bwd_ms = kern["attn_bwd_dq"] + kern["attn_bwd_dkdv"]
        out["bwd_tflops"] = fl["bwd"] / (bwd_ms * 1e-3) / 1e12
        out["bwd_tflops_strict"] = fl["bwd_strict"] / (bwd_ms * 1e-3) / 1e12
        out["bwd_frac_of_peak"] = out["bwd_tflops"] / peak
        out["epilogue_gbs"] = {"fwd": eb["fwd"] / (kern["gated_norm_fwd"] * 1e-3) / 1e9,
                               "bwd": eb["bwd"] / (kern["gated_norm_bwd"] * 1e-3) / 1e9, "peak": PEAK_HBM_GBS}
    # the bias / seed expansion kernels (latency-bound: tens of KB to a few MB per launch)
    from paper_2602_16986_amd.flops import expand_bytes
    out["bias_expand_gbs"] = {k: expand_bytes(w, k) / (kern[k] * 1e-3) / 1e9 for k in ("bias_expand_fwd", "bias_expand_bwd") if k in kern}
    if w.name == "C3-dense" and do_bwd and not args.no_other_configs and args.query_tail == 0 and not args.bias_grad:
        out["other_configs"] = other_configs(args, torch, hb, flops, workloads, DeviceWorkload, peak)
    if ms_reuse is not None:
        useful = fl["fwd"] + (fl["bwd"] if do_bwd else 0.0)
        out["with_reused_schedule"] = {"ms_per_step": ms_reuse, "tflops": useful / (ms_reuse * 1e-3) / 1e12}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, fl, args.cpu_seconds)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
