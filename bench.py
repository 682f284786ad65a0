#!/usr/bin/env python3
"""Benchmark of the retention step (score -> greedy selection -> compaction)
on one MI355X.  Prints one JSON line.

A step is one kvr_retain call over all heads of the workload, with K, V and
Q (or s) already resident in HBM.  value = heads / second.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def cpu_baseline(w, data, b, lam, budget_s=12.0):
    """The fp64 oracle, as it stands, on a bounded sample of the same heads."""
    import numpy as np
    from oracle import alpha_oracle as O
    from paper_2605_14292_amd import workloads as W
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = 1
    rng = np.random.default_rng(11)
    heads = rng.permutation(w.heads)
    done, t_used = 0, 0.0
    for h in heads:
        K64, V64 = W.to_f64(data["K"][h]), W.to_f64(data["V"][h])
        Q64 = W.to_f64(data["Q"][h]) if "Q" in data else None
        s64 = W.to_f64(data["s"][h]) if "s" in data else None
        t0 = time.perf_counter()
        r = O.retain(K64, V64, b, lam, 1e-6, Q=Q64, s=s64)
        O.compact(K64, r["sorted"])
        O.compact(V64, r["sorted"])
        t_used += time.perf_counter() - t0
        done += 1
        if t_used >= budget_s:
            break
    return {"value": done / t_used, "unit": "head-events/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{done} of {w.heads} heads of {w.name} (fp64 numpy oracle, {t_used:.1f} s, "
                      "rate extrapolates linearly over heads)"}


def cpu_baseline_flat(w, data, s, group, b, lam, budget_s=12.0):
    """The fp64 oracle's flat-mode event on a bounded sample of sequences."""
    from oracle import alpha_oracle as O
    from paper_2605_14292_amd import workloads as W
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = 1
    done, t_used = 0, 0.0
    for q in range(w.seqs):
        sl = slice(q * group, (q + 1) * group)
        K64, V64, s64 = W.to_f64(data["K"][sl]), W.to_f64(data["V"][sl]), W.to_f64(s[q])
        t0 = time.perf_counter()
        O.retain_flat(K64, V64, s64, b, lam, 1e-6)
        t_used += time.perf_counter() - t0
        done += 1
        if t_used >= budget_s:
            break
    return {"value": done * group / t_used, "unit": "head-events/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{done} of {w.seqs} sequences ({group} heads each) of {w.name}, flat-signature mode "
                      f"(fp64 numpy oracle, {t_used:.1f} s, rate extrapolates linearly over sequences)"}


def cpu_baseline_budgeted(w, data, b_h, keep, lam, budget_s=12.0):
    """The fp64 oracle's budgeted selection + compaction on a bounded sample of heads."""
    import numpy as np
    from oracle import alpha_oracle as O
    from paper_2605_14292_amd import workloads as W
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = 1
    rng = np.random.default_rng(11)
    bh, kp = b_h.cpu().numpy(), keep.cpu().numpy().astype(bool)
    done, t_used = 0, 0.0
    for h in rng.permutation(w.heads):
        K64, V64 = W.to_f64(data["K"][h]), W.to_f64(data["V"][h])
        t0 = time.perf_counter()
        s64 = O.score_softmax_mean(K64, W.to_f64(data["Q"][h])) if "Q" in data else W.to_f64(data["s"][h])
        r = O.select_budgeted(s64, V64, w.n, int(bh[h]), kp[h], lam, 1e-6)
        O.compact(K64, r["sorted"]); O.compact(V64, r["sorted"])
        t_used += time.perf_counter() - t0
        done += 1
        if t_used >= budget_s:
            break
    return {"value": done / t_used, "unit": "head-events/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{done} of {w.heads} heads of {w.name}, budget-allocator frame (fp64 numpy oracle, "
                      f"{t_used:.1f} s, rate extrapolates linearly over heads)"}


def time_other(name, steps=5, warmup=2, seed=0, lam=None, flat=False, cold=False, budgeted=False):
    """A short run of another benchmark configuration at its full size, for the
    `other_configs` object: the default workload carries the headline figures, the others are
    reported beside it from the same process.  `cold`: the small configurations (c1, c2) fit the
    256 MiB memory-side cache, so a loop over one set of buffers times cache hits; with `cold` every
    step takes the next of enough copies of the inputs to exceed that cache several times over, and
    the hot figure (one set of buffers) is reported beside it."""
    import torch
    from paper_2605_14292_amd import binding as B
    from paper_2605_14292_amd import workloads as W
    w = W.WORKLOADS[name]
    lam = w.lam if lam is None else lam
    data = W.generate(w, seed=seed, device="cuda:0")
    Q, s = data.get("Q"), data.get("s")
    group = w.layers * w.kv_heads
    if flat:
        s = s.view(w.seqs, group, w.n)[:, 0].contiguous()
        out = B.FlatBuffers(w.heads, group, w.n, w.b, w.d, w.torch_dtype, "cuda:0", want_trace=False)
        step = lambda: B.kvr_retain_flat(data["K"], data["V"], s, group, w.b, lam, 1e-6, out=out)
    elif budgeted:      # the frame of main()'s --budgeted: b_h in [b/2, b], 4 sinks + 16 recent protected, position ids
        g = torch.Generator(device="cuda:0").manual_seed(seed + 17)
        b_h = torch.randint(w.b // 2, w.b + 1, (w.heads,), generator=g, device="cuda:0", dtype=torch.int32)
        keep = torch.zeros((w.heads, w.n), dtype=torch.uint8, device="cuda:0")
        keep[:, :4] = 1
        keep[:, w.n - 16:] = 1
        pos = torch.arange(w.n, dtype=torch.int32, device="cuda:0").repeat(w.heads, 1).contiguous()
        out = B.BudgetBuffers(w.heads, w.n, w.b, w.d, w.torch_dtype, "cuda:0", with_pos=True)
        step = lambda: B.kvr_retain_budgeted(data["K"], data["V"], w.b, lam, 1e-6, Q=Q, s=s, b_h=b_h, keep=keep,
                                             pos=pos, out=out)
    else:
        out = B.RetainBuffers(w.heads, w.n, w.b, w.d, w.torch_dtype, "cuda:0", "Q" in data, want_trace=False)
        step = lambda: B.kvr_retain(data["K"], data["V"], w.b, lam, 1e-6, Q=Q, s=s, out=out)

    def timed(fn, k):
        a, z = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(k):
            fn(i)
        z.record()
        torch.cuda.synchronize()
        return a.elapsed_time(z) / k

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    ms = timed(lambda i: step(), steps)
    cold_ms, copies = None, 0
    if cold and not flat:
        set_bytes = sum(v.numel() * v.element_size() for v in data.values())
        copies = int(min(4096, max(16, -(-1_000_000_000 // set_bytes))))
        sets = [data] + [{k: v.clone() for k, v in data.items()} for _ in range(copies - 1)]
        cstep = lambda i: B.kvr_retain(sets[i % copies]["K"], sets[i % copies]["V"], w.b, lam, 1e-6,
                                       Q=sets[i % copies].get("Q"), s=sets[i % copies].get("s"), out=out)
        torch.cuda.synchronize()
        cold_ms = timed(cstep, copies)          # every set once: none of it is in a cache
        del sets
    bytes_step = w.algorithmic_bytes_per_head(w.b, lam) * w.heads
    if flat:
        bytes_step -= (4 * w.n + 4 * w.b) * (w.heads - w.seqs)
    if budgeted:
        rows = (3 if w.scores == "given" else 2) * w.d * w.elem_bytes
        bytes_step += int((float(b_h.float().mean().item()) - w.b) * rows * w.heads) + (w.n + 4 * w.n + 4 * w.b) * w.heads
    del data, out
    torch.cuda.empty_cache()
    res = {"ms_per_step": ms, "head_events_per_s": w.heads / (ms * 1e-3), "steps": steps,
           "algorithmic_GBps": bytes_step / (ms * 1e-3) / 1e9,
           "frac_of_hbm_peak": bytes_step / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
           "heads": w.heads, "n": w.n, "b": w.b, "lambda": lam}
    if cold_ms is not None:
        res.update({"inputs": "hot: one set of buffers, served by the memory-side cache",
                    "ms_per_step_cold": cold_ms, "cold_input_sets": copies,
                    "head_events_per_s_cold": w.heads / (cold_ms * 1e-3)})
    return res


def kernel_name(w, b, lam, has_q):
    """The kernels one kvr_retain call launches for this shape (the roofline
    object prices the whole step against the step's algorithmic bytes)."""
    if w.dtype == "bf16" and 128 < w.n <= 256 and not has_q and 1 < b <= 128 and lam > 0:
        return ("kvr::retain_pruned_kernel (the whole step; kvr::retain_dense_kernel follows for the heads "
                "it marks, a few microseconds when there are none)")
    if w.dtype == "bf16" and w.n <= 256:
        if w.n > 128 and w.heads <= 256:
            return "kvr::retain_dense16_kernel (the whole step is this one launch; one head per CU, sixteen waves each)"
        return "kvr::retain_dense_kernel (the whole step is this one launch)"
    if w.dtype == "bf16" and w.n <= 8192 and b <= 1024:
        tail = ["kvr::select_pool_kernel (selection + compaction)"]
    else:
        tail = ["kvr::select_generic_kernel", "kvr::compact_kernel"]
    fits_lds = w.G <= 32 and w.G * w.n <= (24576 if w.G <= 8 else 31488)
    score = ("kvr::score_kernel" if w.dtype != "bf16" else
             "kvr::score_mfma_kernel" if fits_lds else "kvr::score_wide_kernel")
    if w.dtype != "bf16" and w.n <= 256 and w.G <= 16:
        return "kvr::select_dense_f32_kernel (scores, selection and kept rows: the whole step is this one launch)"
    parts = ([score] if has_q else []) + tail
    return " + ".join(parts) + " (whole step; the select kernel dominates)"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c3", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--b", type=int, default=None)
    ap.add_argument("--lam", type=float, default=None)
    ap.add_argument("--flat", action="store_true",
                    help="flat-signature mode (Eq. 1 over all layers and heads of a sequence): one "
                         "selection per sequence, every head keeps the same tokens; needs a workload "
                         "with given scores (c3)")
    ap.add_argument("--budgeted", action="store_true",
                    help="budget-allocator frame: per-head budgets b_h in [b/2, b], 4 sink tokens and a "
                         "recent window of 16 protected per head, position ids carried along")
    ap.add_argument("--window", type=int, default=1,
                    help="observation window: the scores are computed from WINDOW positions x the workload's "
                         "grouped queries (G * WINDOW <= 256 queries per head; workloads with computed scores)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the short runs of the other benchmark configurations")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run a plain 1 GiB device copy a few times and exit (reference point for "
                         "the FETCH_SIZE / WRITE_SIZE counters of rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (heads shard with no exchange; "
                 "each GPU would run these kernels on its own slice); --gpus must be 1")

    import torch
    from paper_2605_14292_amd import binding as B
    from paper_2605_14292_amd import workloads as W

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    dev = "cuda:0"
    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": src.numel() * 4, "bytes_written": src.numel() * 4}))
        return
    w = W.WORKLOADS[args.workload]
    if args.window != 1:
        import dataclasses
        if w.scores != "computed" or args.window < 1 or w.G * args.window > 256:
            sys.exit("bench.py: --window needs a workload with computed scores and G * WINDOW <= 256")
        w = dataclasses.replace(w, G=w.G * args.window,
                                what=w.what + f", observation window of {args.window} positions")
    b = w.b if args.b is None else args.b
    lam = w.lam if args.lam is None else args.lam
    data = W.generate(w, seed=args.seed, device=dev)
    Q, s = data.get("Q"), data.get("s")
    group = w.layers * w.kv_heads
    if args.flat:
        if s is None:
            sys.exit("bench.py: --flat needs a workload whose scores are given (c3)")
        s = s.view(w.seqs, group, w.n)[:, 0].contiguous()     # one score vector per sequence
        out = B.FlatBuffers(w.heads, group, w.n, b, w.d, w.torch_dtype, dev, want_trace=False)

        def step():
            B.kvr_retain_flat(data["K"], data["V"], s, group, b, lam, 1e-6, out=out)
    elif args.budgeted:
        g = torch.Generator(device=dev).manual_seed(args.seed + 17)
        b_h = torch.randint(b // 2, b + 1, (w.heads,), generator=g, device=dev, dtype=torch.int32)
        keep = torch.zeros((w.heads, w.n), dtype=torch.uint8, device=dev)
        keep[:, :4] = 1
        keep[:, w.n - 16:] = 1
        pos = torch.arange(w.n, dtype=torch.int32, device=dev).repeat(w.heads, 1).contiguous()
        out = B.BudgetBuffers(w.heads, w.n, b, w.d, w.torch_dtype, dev, with_pos=True)
        mean_bh = float(b_h.float().mean().item())

        def step():
            B.kvr_retain_budgeted(data["K"], data["V"], b, lam, 1e-6, Q=Q, s=s, b_h=b_h, keep=keep, pos=pos, out=out)
    else:
        out = B.RetainBuffers(w.heads, w.n, b, w.d, w.torch_dtype, dev, "Q" in data, want_trace=False)

        def step():
            B.kvr_retain(data["K"], data["V"], b, lam, 1e-6, Q=Q, s=s, out=out)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # HIP events on the stream the kernels are launched on (torch's current stream), one pair
    # around the K steps: nothing but the steps' own launches sits between them
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(args.steps):
        step()
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    dev_avg_ms = ev0.elapsed_time(ev1) / args.steps

    # a plain device copy of 1 GiB, for the fraction of what a streaming kernel reaches on this machine
    csrc = torch.empty(1 << 28, dtype=torch.float32, device=dev)
    cdst = torch.empty_like(csrc)
    cdst.copy_(csrc)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(5):
        cdst.copy_(csrc)
    c1.record()
    torch.cuda.synchronize()
    copy_gbps = 2 * csrc.numel() * 4 * 5 / (c0.elapsed_time(c1) * 1e-3) / 1e9
    del csrc, cdst

    bytes_step = w.algorithmic_bytes_per_head(b, lam) * w.heads
    if args.flat:       # scores and indices are per sequence, not per head
        bytes_step -= (4 * w.n + 4 * b) * (w.heads - w.seqs)
    if args.budgeted:   # kept rows follow the per-head budgets; the keep mask and position ids are read
        e = w.elem_bytes
        rows = (3 if w.scores == "given" else 2) * w.d * e       # K in (given scores only), K out, V out
        bytes_step += int((mean_bh - b) * rows * w.heads) + (w.n + 4 * w.n + 4 * b) * w.heads
    achieved = bytes_step / (dev_avg_ms * 1e-3) / 1e9
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get(f"{w.name}{'flat' if args.flat else ''}{'budgeted' if args.budgeted else ''}"
                                               f"{'window%d' % args.window if args.window != 1 else ''}:b{b}:lam{lam}")
    line = {
        "metric": "retention events/sec (heads*events)",
        "value": w.heads / (wall / args.steps),
        "unit": "head-events/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.what}" + (", flat-signature mode (one selection per sequence)"
                                                        if args.flat else "")
                                + (", budget-allocator frame (b_h in [b/2, b], 20 protected tokens per head)"
                                   if args.budgeted else ""), "heads": w.heads, "n": w.n, "b": b,
                   "d": w.d, "lambda": lam, "scores": w.scores, "G": w.G if w.scores == "computed" else 0},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "device_copy_GBps": copy_gbps, "frac_of_device_copy": achieved / copy_gbps,
                     "kernel": ("kvr::signature_flat_kernel + kvr::select_dense_f32_kernel + kvr::compact_kernel (whole step)"
                                if args.flat else
                                "kvr::budget_prepare_kernel + selection kernels of the shape + kvr::budget_finalize_kernel (whole step)"
                                if args.budgeted else kernel_name(w, b, lam, Q is not None)), "device_ms_avg": dev_avg_ms,
                     "algorithmic_bytes_per_step": bytes_step},
    }
    if not args.no_cpu_baseline:
        if args.flat:
            line["cpu_baseline"] = cpu_baseline_flat(w, data, s, group, b, lam)
        elif args.budgeted:
            line["cpu_baseline"] = cpu_baseline_budgeted(w, data, b_h, keep, lam)
        else:
            line["cpu_baseline"] = cpu_baseline(w, data, b, lam)
    default_run = (args.workload == "c3" and not args.flat and not args.budgeted and args.b is None
                   and args.lam is None)
    if default_run and not args.no_other_configs:
        del data, out
        torch.cuda.empty_cache()
        line["other_configs"] = {
            "c1": time_other("c1", steps=20, warmup=5, seed=args.seed, cold=True),
            "c2": time_other("c2", steps=20, warmup=5, seed=args.seed, cold=True),
            "c3 flat-signature mode": time_other("c3", seed=args.seed, flat=True),
            "c3 budget-allocator frame": time_other("c3", seed=args.seed, budgeted=True),
            "c5": time_other("c5", seed=args.seed),
            "c5 lambda=0": time_other("c5", seed=args.seed, lam=0.0),
            "c4": time_other("c4", seed=args.seed),
        }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
