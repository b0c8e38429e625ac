"""Where the attention kernels' workgroups spend their time: prologue, tile loop, epilogue, and how many are resident.

Needs a measurement build of the library that records the wall clock per work item:

    python -m paper_2602_16986_amd.build --define HSTU_FWD_TIMELINE=1 --define HSTU_BWD_TIMELINE=1 --output /tmp/libhstu_timeline.so
    HSTU_ATTN_LIB=/tmp/libhstu_timeline.so python -m paper_2602_16986_amd.attn_timeline C3-sparse C3-dense C4

For every workload: forward and backward launches, then for each of the three passes, per work item the time from the
workgroup's start to the barrier that ends its prologue, to the end of its tile loop and to the completion of its stores (100 MHz clock, 10 ns ticks), the number of
workgroups alive and inside their tile loop over 20 slices of the launch, and the loop time by quartile of start time.
"""
import ctypes
import os
import sys

import numpy as np
import torch

from . import workloads as wl
from .runner import DeviceWorkload

MAX_ITEMS = 16384


def timeline(name: str) -> None:
    lib = ctypes.CDLL(os.environ["HSTU_ATTN_LIB"])
    if not hasattr(lib, "hstu_debug_fwd_timeline"):
        raise SystemExit("this library was not built with HSTU_FWD_TIMELINE=1")
    lib.hstu_debug_fwd_timeline.argtypes = [ctypes.c_void_p, ctypes.c_int]
    w = wl.config(name)
    dw = DeviceWorkload(w)
    backward = hasattr(lib, "hstu_debug_bwd_timeline") and w.dout is not None
    for _ in range(20):
        dw.attn_fwd()
        if backward:
            dw.attn_bwd()
    torch.cuda.synchronize()
    buf = np.zeros(5 * MAX_ITEMS, dtype=np.uint64)
    if lib.hstu_debug_fwd_timeline(buf.ctypes.data, MAX_ITEMS) < 0:
        raise SystemExit("reading the timeline failed")
    report(name + " forward", buf.reshape(MAX_ITEMS, 5).copy())
    if backward:
        lib.hstu_debug_bwd_timeline.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int]
        for which, label in ((0, "dQ pass"), (1, "dK/dV pass")):
            buf[:] = 0
            if lib.hstu_debug_bwd_timeline(buf.ctypes.data, MAX_ITEMS, which) < 0:
                raise SystemExit("reading the timeline failed")
            report(f"{name} {label}", buf.reshape(MAX_ITEMS, 5).copy())


def report(name: str, t: np.ndarray) -> None:
    t = t[t[:, 0] > 0]
    t = t[t[:, 0] + 1_000_000 > t[:, 0].max()]           # drop what an earlier workload left beyond this list's length (10 ms window)
    base = int(t[:, 0].min())
    start, loop0, loop1, end = [(t[:, i].astype(np.int64) - base) / 100.0 for i in range(4)]      # microseconds
    span = end.max()
    life = end - start
    print(f"{name}: {len(t)} work items, launch {span:.1f} us, last workgroup starts at {start.max():.1f} us")
    for label, v in (("prologue", loop0 - start), ("tile loop", loop1 - loop0), ("epilogue", end - loop1), ("lifetime", life)):
        print(f"  {label:9s} mean {v.mean():7.2f}  p10 {np.percentile(v, 10):7.2f}  median {np.percentile(v, 50):7.2f}  "
              f"p90 {np.percentile(v, 90):7.2f}  max {v.max():7.2f} us   {100 * v.sum() / life.sum():5.1f} % of lifetime")
    print(f"  resident workgroups, mean over the launch: {life.sum() / span:.1f}; inside the tile loop: {(loop1 - loop0).sum() / span:.1f}")
    mids = (np.arange(20) + 0.5) * span / 20
    print("  alive   per twentieth of the launch:", [int(((start <= m) & (end > m)).sum()) for m in mids])
    print("  in loop per twentieth of the launch:", [int(((loop0 <= m) & (loop1 > m)).sum()) for m in mids])
    order = np.argsort(start)
    q = len(order) // 4
    for k in range(4):
        sel = order[k * q:(k + 1) * q]
        print(f"  start quartile {k}: started {start[sel].min():.1f}..{start[sel].max():.1f} us, tile loop mean "
              f"{(loop1 - loop0)[sel].mean():.2f} us, prologue mean {(loop0 - start)[sel].mean():.2f} us")


if __name__ == "__main__":
    for workload in sys.argv[1:] or ["C3-sparse"]:
        timeline(workload)
