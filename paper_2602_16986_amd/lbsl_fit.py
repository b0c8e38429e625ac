"""Fit the load exponent gamma of Load-Balanced Stochastic Length (paper Section 4.1: load of a sequence = n^gamma) to
this library's own cost curve on the GPU at hand.

For every length n the whole hot path (attention forward, gated norm forward and backward, attention backward) runs on a
batch of equal sequences that holds about `--tokens` tokens, so that the chip is full at every length; time per
sequence against n, fitted by hstu_lbsl_fit_gamma.  Usage:  python -m paper_2602_16986_amd.lbsl_fit [--K1 1024 --K2 256]
"""
from __future__ import annotations

import argparse
import json

import torch

from . import binding as hb
from . import workloads as wl
from .runner import DeviceWorkload


def time_per_sequence(n: int, tokens: int, K1: int, K2: int, H: int, d: int, steps: int) -> float:
    B = max(1, tokens // n)
    w = wl.build(f"fit-{n}", [n] * B, H, d, "bf16", seed=n, K1=K1, K2=K2, alpha=1.0 / d ** 0.5, backward=True)
    dw = DeviceWorkload(w)
    for _ in range(3):
        dw.layer_step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        dw.layer_step()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps / B


def main():
    ap = argparse.ArgumentParser(description=__doc__)
    ap.add_argument("--lengths", type=int, nargs="+", default=[1024, 2048, 4096, 8192, 16384])
    ap.add_argument("--tokens", type=int, default=65536)
    ap.add_argument("--K1", type=int, default=-1, help="local window (-1: dense causal mask)")
    ap.add_argument("--K2", type=int, default=0, help="global prefix")
    ap.add_argument("--heads", type=int, default=4)
    ap.add_argument("--head-dim", type=int, default=128)
    ap.add_argument("--steps", type=int, default=10)
    a = ap.parse_args()
    ms = [time_per_sequence(n, a.tokens, a.K1, a.K2, a.heads, a.head_dim, a.steps) for n in a.lengths]
    gamma = hb.hstu_lbsl_fit_gamma(a.lengths, ms)
    print(json.dumps({"K1": a.K1, "K2": a.K2, "lengths": a.lengths, "ms_per_sequence": [round(x, 5) for x in ms], "gamma": round(gamma, 4)}))


if __name__ == "__main__":
    main()
