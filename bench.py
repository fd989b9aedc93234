#!/usr/bin/env python3
"""Benchmark of the radix top-k hot path on one MI355X.

A "step" is one complete selection (every kernel of the path: sample histogram, the sweep over X, later digit
passes, single-workgroup finish) over one batch of synthetic input that is already resident in HBM.  The
workload is the benchmark's headline case that fits one GPU:

    config 4: single query, n = 2^28 fp32 keys i.i.d. uniform in [-1e6, 1e6), k = 2^20, largest

Prints ONE JSON line: keys/sec over the timed region, the roofline of the dominant kernel (measured live with HIP
events recorded by the library on the launch stream), the CPU oracle timed on a bounded sample, and -- after the
timed region of the headline, so that it is not disturbed -- one row per (config, k, direction, scaling) of
the benchmark's other configurations (`configs`), each with its time, keys/s, the bytes its passes moved and the
fraction of HBM peak that is.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth


def bytes_moved(tr, n, es, k):
    """Bytes one row's passes read and wrote, from the row's own pass records (the algorithmic-bytes model of
    the design notes, evaluated with the run's real candidate counts).  Returns (bytes, description)."""
    ps = tr.passes
    out = (es + 8) * k
    if not ps:
        return 0, "skipped"
    if ps[0].where == 4:                                   # one-sweep row kernel: X once (+ its first part again, cached)
        return es * n + out, "one sweep"
    def pass_bytes(i):
        """read of pass i's source + write of its candidates (an in-place pass writes none; after in-place passes
        that began over X the source is still X)"""
        p = ps[i]
        if p.source == 3:
            return 0
        src_in_x = i > 0 and (ps[i - 1].window >> 26) & 1
        rd = es * n if src_in_x else 8 * p.cand_before
        if src_in_x and p.source == 2:
            # an index digit read from X: only the positions its winners and its bin can have are read -- from the row's
            # start up to the last position whose inverted index, taken from this digit up, is not below the chosen bin
            # (with the bins of the index digits before it, all left in place, above it)
            wide, q = p.bin, i - 1
            while q >= 0 and ps[q].source == 2:
                wide |= ps[q].bin << (ps[q].shift - p.shift)
                q -= 1
            idx_max = (1 << max(1, (n - 1).bit_length())) - 1
            rd = es * max(0, min(n, idx_max - (wide << p.shift) + 1))
        if i > 0 and (ps[i - 1].window >> 25) & 1 and not src_in_x:
            q = i - 1                                      # the array the in-place chain reads is as long as when it was written
            while q > 0 and (ps[q - 1].window >> 25) & 1 and not (ps[q - 1].window >> 26) & 1:
                q -= 1
            rd = 8 * ps[q].cand_before
        wr = 0 if (p.window >> 25) & 1 else 8 * p.cand_after
        return rd + wr

    later = sum(pass_bytes(i) for i in range(1, len(ps)))
    first_wr = 0 if (ps[0].window >> 25) & 1 else 8 * ps[0].cand_after
    if ps[0].where == 3:                                   # one workgroup per row
        if n * es <= 256 * 1024:
            return es * n + first_wr + later + out, "row in registers"
        return 2 * es * n + first_wr + later + out, "one workgroup, two sweeps"
    if tr.pre_elems:                                       # sample + one sweep that counts and keeps
        b = es * tr.pre_elems + es * n + 8 * tr.pre_kept
        if tr.pre_missed and tr.pre_merged:               # the sweep declined and counted two digits of the crowded bin:
            return b + later + out, "sample + counting sweep, two-digit pass over X"   # pass 0 has no sweep of its own
        if tr.pre_missed:
            b += es * n + first_wr
            return b + later + out, "sample + counting sweep + second sweep"
        if tr.pre_merged:                                  # pass 0 has no sweep; pass 1 reads all that was kept
            rest = sum(pass_bytes(i) for i in range(2, len(ps)))
            return b + 8 * tr.pre_kept + 8 * ps[1].cand_after + rest + out, "sample + one sweep, two-digit pass"
        return b + 8 * tr.pre_kept + first_wr + later + out, "sample + one sweep"
    return 2 * es * n + first_wr + later + out, "two sweeps"


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--log2n", type=int, default=28, help="row length 2^log2n (default: the headline 2^28)")
    ap.add_argument("--log2k", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="only the headline workload")
    ap.add_argument("--only-config", default="", help="of the configs rows, run only those whose name starts with this")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain device copy of the input (n*4 bytes read, n*4 written), so that a "
                         "counter run contains a kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2501_14336_amd import binding as B
    from paper_2501_14336_amd import workloads as W
    from tests import verify

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 2
    B.load()
    dev = torch.device("cuda:0")
    n, k = 1 << args.log2n, 1 << args.log2k
    steps, warmup = args.steps, args.warmup

    # ---- workload: config 4, generated on the host by the seeded generator, then made resident
    x_host = W.config4(n)
    x = torch.from_numpy(x_host).to(dev)[None, :]
    vals = torch.empty((1, k), dtype=torch.float32, device=dev)
    idx = torch.empty((1, k), dtype=torch.int64, device=dev)
    ws = torch.empty(B.rtopk_workspace_bytes(1, n, k, B.RTOPK_F32), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream(dev)

    def make_events(count):
        evs = []
        for _ in range(count):
            e = torch.cuda.Event(enable_timing=True)
            e.record(stream)  # instantiates the underlying hipEvent_t
            evs.append(e)
        return evs

    if args.calibration_copy:
        y = torch.empty_like(x)
        y.copy_(x)
        torch.cuda.synchronize()
        del y

    for _ in range(warmup):
        B.topk(x, k, True, workspace=ws, out=(vals, idx))
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` steps.  On every 10th step the library records 5 HIP events on the
    # launch stream around the two big kernels (an event costs a few microseconds of stream time, so not on all).
    sampled = [i for i in range(steps) if i % 10 == 0]
    per_step = {i: make_events(B.RTOPK_NUM_EVENTS) for i in sampled}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        evs = per_step.get(i)
        B.topk(x, k, True, workspace=ws, out=(vals, idx), events=[e.cuda_event for e in evs] if evs else None)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    per_step = list(per_step.values())
    wall_ms = (t1 - t0) * 1e3
    ms_per_step = wall_ms / steps
    keys_per_s = n * steps / (t1 - t0)

    hist_ms = float(np.mean([evs[1].elapsed_time(evs[2]) for evs in per_step]))
    classify_ms = float(np.mean([evs[2].elapsed_time(evs[3]) for evs in per_step]))
    call_ms = float(np.mean([evs[0].elapsed_time(evs[4]) for evs in per_step]))

    # ---- algorithmic bytes from the run's own pass records
    tr = B.read_trace(ws, 1)[0]
    assert tr.error == 0 and tr.done, "device reported an inconsistent state"

    # ---- parity of the LAST TIMED step's output: the definition check (O(n), independent of the method) decides
    # whether it is the top-k of the row
    verify.check_topk_properties(x_host.view(np.uint32), verify.F32, k, True,
                                 vals[0].view(torch.int32).cpu().numpy().view(np.uint32), idx[0].cpu().numpy())

    es = 4
    prefilter = tr.pre_elems != 0
    path_bytes, path_kind = bytes_moved(tr, n, es, k)
    if prefilter:
        hist_bytes = es * tr.pre_elems                 # the sample
        sweep_bytes = es * n + 8 * tr.pre_kept         # X once, what is kept written once
        names = ("hist_keys_sample", "prefilter_keys")
    else:
        p0 = tr.passes[0]
        hist_bytes = es * n
        sweep_bytes = es * n + 8 * p0.cand_after + (es + 8) * p0.winners
        names = ("hist_keys", "classify_keys")
    floor_bytes = 2 * es * n + (es + 8) * k            # two sweeps + the output
    floor1_bytes = es * n + (es + 8) * k               # X read once + the output
    dominant = (names[1], classify_ms, sweep_bytes) if classify_ms >= hist_ms else (names[0], hist_ms, hist_bytes)
    achieved = dominant[2] / (dominant[1] * 1e-3) / 1e9

    # traffic: not measured in this run -- the figure recorded from the rocprofv3 counter runs kept under profiles/
    traffic, traffic_src = None, None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic_config4.json")
    if os.path.exists(tpath) and args.log2n == 28 and args.log2k == 20:
        try:
            rec = json.load(open(tpath))
            traffic = rec.get(dominant[0] + "_bytes_per_launch")
            traffic_src = ("profiles/hbm_traffic_config4.json: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this "
                           "command, recorded at commit %s" % rec.get("commit", "?"))
        except Exception:
            traffic = None

    # the whole call: the timed region's own time per step (calls back to back on one stream; the steps that carry
    # the library's five event markers run about 10 us longer, see gpu_ms_per_marked_call)
    whole_frac = path_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS
    out = {
        "metric": "top-k keys/sec (single query n=2^28 fp32, k=2^20) and % of HBM peak BW",
        "value": keys_per_s,
        "unit": "keys/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "parity_checked": True,
        "config": {"workload": "config4: 1 x 2^%d fp32 U[-1e6,1e6) seed 4000, k=2^%d, largest, int64 indices"
                               % (args.log2n, args.log2k),
                   "batch": 1, "n": n, "k": k},
        "roofline": {"bound": "hbm", "kernel": dominant[0], "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_src,
                     "kernel_ms": dominant[1], "algorithmic_bytes": dominant[2],
                     "whole_call_frac": whole_frac, "whole_call_target_0.60_met": bool(whole_frac >= 0.60)},
        "whole_path": {"ms_per_call": ms_per_step, "gpu_ms_per_marked_call": call_ms, names[0] + "_ms": hist_ms,
                       names[1] + "_ms": classify_ms,
                       "structure": path_kind, "elements_counted_before_the_sweep": tr.pre_elems if prefilter else n,
                       "bytes_moved_by_all_passes": path_bytes,
                       "achieved_frac_of_hbm_peak": whole_frac,
                       "sample_misled": bool(tr.pre_missed) if prefilter else None,
                       "one_read_floor_bytes": floor1_bytes,
                       "one_read_floor_frac_of_hbm_peak": floor1_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                       "two_sweep_floor_bytes": floor_bytes,
                       "two_sweep_floor_frac_of_hbm_peak": floor_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                       "passes": [[p.where, p.cand_before, p.cand_after, p.winners] for p in tr.passes]},
    }

    # ---- every other (config, k, direction, scaling) of the benchmark spec, after the headline's timed region
    def time_rows(xd, kk, largest, scaling, code, batch, nn, reps=10, sorted_out=False, wsb=None):
        vb = torch.empty((batch, kk), dtype=xd.dtype, device=dev)
        ib = torch.empty((batch, kk), dtype=torch.int64, device=dev)
        flags = (B.RTOPK_FLAG_SCALING if scaling else 0) | (B.RTOPK_FLAG_SORTED if sorted_out else 0)
        need = B.rtopk_workspace_bytes(batch, nn, kk, code, flags)
        if wsb is None or wsb.numel() < need:
            wsb = None
            torch.cuda.empty_cache()
            wsb = torch.empty(need, dtype=torch.uint8, device=dev)
        for _ in range(3):
            B.topk(xd, kk, largest, scaling=scaling, seed=77, workspace=wsb, out=(vb, ib), sorted=sorted_out)
        evs = [make_events(2) for _ in range(reps)]
        torch.cuda.synchronize()
        for a, b in evs:
            a.record(stream)
            B.topk(xd, kk, largest, scaling=scaling, seed=77, workspace=wsb, out=(vb, ib), sorted=sorted_out)
            b.record(stream)
        torch.cuda.synchronize()
        ms = sorted(a.elapsed_time(b) for a, b in evs)
        trs = B.read_trace(wsb, batch)
        assert all(t.error == 0 and t.done for t in trs), "device reported an inconsistent state"
        return ms[len(ms) // 2], ms[0], trs, wsb, vb, ib

    def row(name, xd, bits_host, kk, largest, scaling, code, batch, nn, esz, check_rows=(0,), wsb=None):
        med, best, trs, wsb, vb, ib = time_rows(xd, kk, largest, scaling, code, batch, nn, wsb=wsb)
        moved = 0
        kind = ""
        for t in trs:
            b, kind = bytes_moved(t, nn, esz, kk)
            moved += b
        floor1 = batch * (esz * nn + (esz + 8) * kk)
        # parity of the timed output on some rows (definition check)
        vw = vb.view(torch.int32 if esz == 4 else torch.int16).cpu().numpy().view(np.uint32 if esz == 4 else np.uint16)
        iw = ib.cpu().numpy()
        b2 = bits_host.reshape(batch, nn)
        for r in check_rows:
            verify.check_topk_properties(b2[r], code, kk, largest, vw[r], iw[r])
        entry = {"config": name, "batch": batch, "n": nn, "k": kk, "dtype": ("f32", "f16", "bf16")[code],
                 "largest": bool(largest), "scaling": bool(scaling), "ms": med, "ms_min": best,
                 "keys_per_s": batch * nn / (med * 1e-3), "structure": kind, "bytes_moved": moved,
                 "frac_of_hbm_peak_on_bytes_moved": moved / (med * 1e-3) / 1e9 / HBM_PEAK_GBS,
                 "one_read_floor_bytes": floor1,
                 "frac_of_hbm_peak_on_one_read_floor": floor1 / (med * 1e-3) / 1e9 / HBM_PEAK_GBS,
                 "passes": len(trs[0].passes), "parity_checked_rows": len(check_rows)}
        return entry, wsb

    if not args.no_configs:
        rows = []
        want = args.only_config

        def wanted(name):                       # a block ("C3") runs if the prefix lies inside it or it inside the prefix;
            return name.startswith(want) or want.startswith(name)

        def row_wanted(name):                   # a row of a block only if its own name starts with the prefix
            return name.startswith(want) or (want.startswith(name) and " " not in name)

        def ms_of(name):
            for r in rows:
                if r["config"] == name:
                    return r["ms"]
            return None

        # config 4, the other k (same resident input)
        wsb = ws
        for lk in (20, 24, 27):
            name = "C4 k=2^%d" % lk
            if lk == args.log2k:
                rows.append({"config": name, "batch": 1, "n": n, "k": k, "dtype": "f32", "largest": True, "scaling": False,
                             "ms": ms_per_step, "keys_per_s": n / (ms_per_step * 1e-3), "structure": path_kind,
                             "bytes_moved": path_bytes, "frac_of_hbm_peak_on_bytes_moved": whole_frac,
                             "note": "the headline, from the timed region above"})
            elif wanted(name) and args.log2n == 28:
                e, wsb = row(name, x, x_host.view(np.uint32), 1 << lk, True, False, B.RTOPK_F32, 1, n, 4, wsb=wsb)
                rows.append(e)
        if wanted("C4 sorted") and args.log2n == 28:
            med, best, _, wsb, _, _ = time_rows(x, k, True, False, B.RTOPK_F32, 1, n, reps=5, sorted_out=True, wsb=wsb)
            rows.append({"config": "C4 sorted k=2^%d" % args.log2k, "ms": med, "sort_share_of_call": 1.0 - ms_per_step / med,
                         "note": "radix sort of the k pairs on the grid after the selection"})
        del wsb, x, ws, vals, idx
        torch.cuda.empty_cache()

        if wanted("C1"):
            b1 = W.config1().view(np.uint32)
            e, _ = row("C1", torch.from_numpy(b1.view(np.float32)).to(dev)[None, :], b1, 32, True, False, B.RTOPK_F32, 1,
                       1 << 16, 4)
            rows.append(e)
        if wanted("C2"):
            b2 = W.config2().view(np.uint32)
            x2 = torch.from_numpy(b2.view(np.float32)).to(dev)[None, :]
            w2 = None
            for kk in (16, 256, 4096, 65536, 1 << 20):
                for largest in (True, False):
                    if not row_wanted("C2 k=%d %s" % (kk, "largest" if largest else "smallest")):
                        continue
                    e, w2 = row("C2 k=%d %s" % (kk, "largest" if largest else "smallest"), x2, b2, kk, largest, False,
                                B.RTOPK_F32, 1, 1 << 24, 4, wsb=w2)
                    rows.append(e)
            if row_wanted("C2 sorted k=4096") and ms_of("C2 k=4096 largest") is not None:
                med, best, _, w2, _, _ = time_rows(x2, 4096, True, False, B.RTOPK_F32, 1, 1 << 24, sorted_out=True, wsb=w2)
                rows.append({"config": "C2 sorted k=4096", "ms": med,
                             "sort_share_of_call": 1.0 - ms_of("C2 k=4096 largest") / med,
                             "note": "bitonic sort of the k pairs in LDS after the selection (the paper counts 0.1-0.6 % "
                                     "for its sort, Section 5.2)"})
            del x2, w2
        if wanted("C3"):
            b3 = W.config3()
            x3 = torch.from_numpy(b3.view(np.int16)).to(dev).view(torch.bfloat16)
            w3 = None
            for kk in (50, 1024, 8192):
                if not row_wanted("C3 k=%d" % kk):
                    continue
                e, w3 = row("C3 k=%d" % kk, x3, b3, kk, True, False, B.RTOPK_BF16, 1024, 131072, 2,
                            check_rows=tuple(range(0, 1024, 97)), wsb=w3)
                rows.append(e)
            for kk in (50, 8192):
                if not row_wanted("C3 sorted k=%d" % kk) or ms_of("C3 k=%d" % kk) is None:
                    continue
                med, best, _, w3, _, _ = time_rows(x3, kk, True, False, B.RTOPK_BF16, 1024, 131072, sorted_out=True, wsb=w3)
                rows.append({"config": "C3 sorted k=%d" % kk, "ms": med, "sort_share_of_call": 1.0 - ms_of("C3 k=%d" % kk) / med})
            if ms_of("C3 k=50") is not None:
                out["batch_case"] = {"workload": "config3: 1024 x 131072 bf16 logits N(0,9)+8 spikes, k=50, largest",
                                     "keys_per_s": 1024 * 131072 / (ms_of("C3 k=50") * 1e-3), "ms_per_step": ms_of("C3 k=50")}
            del x3, w3
        torch.cuda.empty_cache()
        if wanted("C5"):
            for case in "abc":
                for npdt, code, esz in ((np.float32, B.RTOPK_F32, 4), (np.float16, B.RTOPK_F16, 2)):
                    if not wanted("C5%s %s" % (case, ("f32", "f16")[code])):
                        continue
                    h = W.config5(case, dtype=npdt)
                    bits = verify.as_bits(h, code)
                    xd = torch.from_numpy(h).to(dev)[None, :]
                    w5 = None
                    for largest in ((True, False) if case != "a" else (True,)):
                        for scaling in ((False, True) if code == B.RTOPK_F32 else (False,)):
                            if not row_wanted("C5%s %s %s%s" % (case, ("f32", "f16")[code], "largest" if largest else "smallest",
                                                                " scaled" if scaling else "")):
                                continue
                            e, w5 = row("C5%s %s %s%s" % (case, ("f32", "f16")[code], "largest" if largest else "smallest",
                                                          " scaled" if scaling else ""), xd, bits, 1 << 16, largest, scaling,
                                        code, 1, 1 << 26, esz, wsb=w5)
                            rows.append(e)
                    del xd, w5
                    torch.cuda.empty_cache()
        out["configs"] = rows

    # ---- CPU baseline: the oracle as it stands, on a bounded sample of the same workload (about 10-15 s)
    if not args.no_cpu_baseline:
        import oracle
        ns = min(n, 1 << 26)
        ks = max(1, ns * k // n)
        sample = x_host[:ns]
        c0 = time.perf_counter()
        oracle.topk(sample, oracle.F32, ks, True)
        cs = time.perf_counter() - c0
        out["cpu_baseline"] = {"value": ns / cs, "unit": "keys/s", "cores": 1, "kind": "oracle",
                               "sample": "first 2^%d keys of the same dataset, k=%d (same k/n), full sort of "
                                         "(value, index) pairs, single thread, %.1f s" % (ns.bit_length() - 1, ks, cs)}
        # a stronger CPU selection for scale (a library's introselect: values only, no indices, no tie rule)
        c0 = time.perf_counter()
        np.partition(sample, ns - ks)
        cp = time.perf_counter() - c0
        out["cpu_partition"] = {"value": ns / cp, "unit": "keys/s", "cores": 1,
                                "kind": "numpy.partition (introselect) on the same sample, values only, %.2f s" % cp}

    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
