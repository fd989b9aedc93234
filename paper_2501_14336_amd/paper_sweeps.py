#!/usr/bin/env python3
"""Sweeps shaped like the paper's evaluation, on synthetic inputs, for laying results beside the SHAPES of its figures
(the figures' numbers are for another GPU and are not reproduced here):

  non-batch   uniform [0,1), n = 2^21 .. 2^29, k = 2^4 .. 2^12                      (Section 5.3.1)
  batch       16 tasks, n = 2^16 .. 2^24, same k                                     (Section 5.3.2)
  ablation    16 tasks of 2^20, the first one element shorter (ragged batch), k = 2048; and this library's own
              switches: sampled prefilter on/off, digit width 8 / 11 / 12             (Section 5.3.3)
  quantile    k = n/100, n/4, n/2                                                     (Section 5.4)
  robustness  uniform [0.6,0.7], uniform [128.6,128.7], Zipf(1.1), k = 512, adaptive scaling off/on (Section 5.5)

Run on a machine with the GPU:   python -m paper_2501_14336_amd.paper_sweeps [--quick] > sweeps.md
Prints markdown tables of median microseconds per call (HIP events around the call, input resident, workspace and
outputs allocated beforehand; 3 warm-up calls, 10 timed).
"""
from __future__ import annotations

import argparse
import sys

import numpy as np


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--quick", action="store_true", help="smaller maximum sizes (2^26 instead of 2^29)")
    args = ap.parse_args()
    import torch
    from . import binding as B
    from . import workloads as W

    if not torch.cuda.is_available():
        print("paper_sweeps: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream(dev)

    def timed(call, reps=10):
        for _ in range(3):
            call()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        torch.cuda.synchronize()
        for a, b in evs:
            a.record(stream)
            call()
            b.record(stream)
        torch.cuda.synchronize()
        ms = sorted(a.elapsed_time(b) for a, b in evs)
        return ms[len(ms) // 2] * 1e3

    def us(x, k, largest=True, scaling=False, tuning=None, sorted_out=False):
        batch, n = x.shape
        flags = (B.RTOPK_FLAG_SCALING if scaling else 0) | (B.RTOPK_FLAG_SORTED if sorted_out else 0)
        ws = torch.empty(B.rtopk_workspace_bytes(batch, n, k, B.RTOPK_F32, flags, tuning), dtype=torch.uint8, device=dev)
        out = (torch.empty((batch, k), dtype=x.dtype, device=dev), torch.empty((batch, k), dtype=torch.int64, device=dev))
        t = timed(lambda: B.topk(x, k, largest, scaling=scaling, seed=1, tuning=tuning, workspace=ws, out=out, sorted=sorted_out))
        tr = B.read_trace(ws, batch)
        assert all(r.error == 0 and r.done for r in tr)
        del ws, out
        return t

    def table(title, head, rows):
        print("\n### " + title + "\n")
        print("| " + " | ".join(head) + " |")
        print("|" + "|".join("---" for _ in head) + "|")
        for r in rows:
            print("| " + " | ".join(r) + " |")
        sys.stdout.flush()

    top = 26 if args.quick else 29
    ks = [1 << e for e in (4, 6, 8, 10, 12)]
    print("# Paper-shaped sweeps on one MI355X (median microseconds per call)\n")
    print("Synthetic inputs from the seeded generators of `paper_2501_14336_amd/workloads.py`; fp32 keys, largest, "
          "unsorted output unless stated.  keys/s = batch * n / time.")

    # ---- non-batch, uniform [0, 1)
    base = W.uniform01(1 << top, 9001)
    xd = torch.from_numpy(base).to(dev)
    rows = []
    for e in range(21, top + 1, 2):
        x = xd[None, : 1 << e]
        cells = [us(x, k) for k in ks]
        rows.append(["2^%d" % e] + ["%.0f" % c for c in cells] + ["%.2e" % ((1 << e) / (cells[2] * 1e-6))])
    table("Non-batch queries, uniform [0,1) (paper Section 5.3.1)", ["n"] + ["k=%d" % k for k in ks] + ["keys/s at k=256"], rows)

    # ---- sorted output on the same shapes (the paper's timings include its sort of the k results, Section 5.2)
    rows = []
    for e in (21, 25, top):
        x = xd[None, : 1 << e]
        rows.append(["2^%d" % e] + ["%.0f / %.0f" % (us(x, k), us(x, k, sorted_out=True)) for k in (16, 256, 4096)])
    table("Unsorted / sorted output (Section 5.2 counts the sort in)", ["n"] + ["k=%d" % k for k in (16, 256, 4096)], rows)

    # ---- batch of 16
    rows = []
    for e in range(16, min(24, top - 4) + 1, 2):
        x = xd[: 16 << e].view(16, 1 << e)
        cells = [us(x, k) for k in ks]
        rows.append(["2^%d" % e] + ["%.0f" % c for c in cells] + ["%.2e" % ((16 << e) / (cells[2] * 1e-6))])
    table("Batch of 16 queries, uniform [0,1) (Section 5.3.2)", ["n per task"] + ["k=%d" % k for k in ks] + ["keys/s at k=256"], rows)

    # ---- ablation: ragged batch, and this library's own switches
    n = 1 << 20
    x16 = xd[: 16 * n].view(16, n)
    flat = xd[1: 16 * n]                                                        # the first task one element shorter
    offs = torch.tensor([0] + [n - 1 + r * n for r in range(16)], dtype=torch.int64, device=dev)
    rk = torch.full((16,), 2048, dtype=torch.int64, device=dev)
    ragged = timed(lambda: B.topk_ragged(flat, offs, rk, n, 2048))
    rows = [["16 x 2^20, equal lengths (every row 16-byte aligned)", "%.0f" % us(x16, 2048)],
            ["first task 2^20 - 1: rows start off the 16-byte grid (ragged entry point, allocates per call)", "%.0f" % ragged]]
    table("Ragged batch: on-demand offset padding (Section 5.3.3), k = 2048", ["input", "us"], rows)
    x = xd[None, : 1 << min(26, top)]
    rows = []
    for k in (256, 1 << 16):
        rows.append(["2^%d, k=%d" % (min(26, top), k)] +
                    ["%.0f" % us(x, k, tuning=t) for t in (dict(prefilter=-1), dict(prefilter=1), dict(prefilter=-1, digit_bits=8),
                                                           dict(prefilter=-1, digit_bits=11), dict(prefilter=-1, digit_bits=12))])
    table("This library's own switches", ["input", "two sweeps over X", "sample + one sweep", "d = 8", "d = 11", "d = 12"], rows)

    # ---- quantiles
    rows = []
    for e in (24, 26, top):
        x = xd[None, : 1 << e]
        rows.append(["2^%d" % e] + ["%.0f" % us(x, max(1, (1 << e) // d)) for d in (100, 4, 2)])
    table("Quantile selection, k = O(n) (Section 5.4)", ["n", "k = n/100", "k = n/4", "k = n/2"], rows)
    del xd, x16, flat

    # ---- robustness
    rows = []
    e = min(26, top)
    for name, gen in (("uniform [0,1)", lambda: W.uniform01(1 << e, 9002)),
                      ("uniform [0.6,0.7]", lambda: W.uniform_range(1 << e, 9003, 0.6, 0.7)),
                      ("uniform [128.6,128.7]", lambda: W.uniform_range(1 << e, 9004, 128.6, 128.7)),
                      ("Zipf(1.1)", lambda: W.zipf(1 << e, 9005))):
        x = torch.from_numpy(gen()).to(dev)[None, :]
        rows.append([name, "%.0f" % us(x, 512), "%.0f" % us(x, 512, scaling=True)])
        del x
    table("Robustness, n = 2^%d, k = 512 (Section 5.5)" % e, ["distribution", "scaling off", "adaptive scaling on"], rows)
    return 0


if __name__ == "__main__":
    sys.exit(main())
