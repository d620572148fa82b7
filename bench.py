#!/usr/bin/env python3
"""Benchmark of libtw's hot path on one MI355X.

Headline (`value`): algorithmic GB/s of the fused reduce + residual-add + RMSNorm
(TokenWeave, arXiv 2505.11329, Appendix A Listing 1) on the 70B-class one-GPU
shard (N=1024 rows, H=8192, P=8 partial buffers) inside a 32-CU budget, inputs
resident in HBM, four rotating buffer sets (738 MB) so that no step re-reads
data left in the 256 MB Infinity Cache. A step is one call of
tw_reduce_add_rmsnorm. Algorithmic bytes per step = (P + 3) * 2 * H * N.

The same JSON line carries: `roofline` (HBM, against the 8 TB/s vendor peak,
from HIP events around every launch of the timed region), `cpu_baseline` (the
fp64 oracle timed on this machine's host cores), `budgets` (GB/s per CU budget next
to what a plain streaming kernel reaches with the same budget), `split` (two-
stream token split vs one launch) and `overlap` (fused kernel next to the bf16
MFMA GEMM vs the two run back to back).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X vendor figure
MFMA_BF16_PEAK_TFLOPS = 2500.0
WORKLOAD = "c3_70b_shard_tp8"
HEADLINE_BUDGET = 32
# HBM bytes per launch of the headline kernel from hardware counters (FETCH_SIZE and
# WRITE_SIZE, each scaled by what the same counter reads for a 192 MiB copy); the
# figures and commands are in profiles/fused_kernel_c3_70b_shard_tp8_budget32.md.
MEASURED_TRAFFIC_BYTES = {(WORKLOAD, 32): (147653 + 32768) * 1024}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--budget", type=int, default=HEADLINE_BUDGET, help="CU budget of the timed steps")
    ap.add_argument("--no-extras", action="store_true", help="only the timed region (for profilers)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the benchmark line: token sweep 32..64K of the fused kernel at H=8192 (P=8, "
                         "P=4) and H=4096 (P=2), whole device / shared / 32 CUs (the analogue of the paper's "
                         "Tables 1-2), and a sweep over hidden sizes 1024..16384 at a fixed volume, one JSON "
                         "object")
    ap.add_argument("--split-sweep", action="store_true",
                    help="instead of the benchmark line: for a range of token counts, the woven layer boundary "
                         "timed at the equal split and at the offsets {0,64,128,192,256,512} past it (the sweep "
                         "of Algorithm 1), next to the row tw_smart_split_point picks without timing anything")
    ap.add_argument("--counters-run", choices=("fused", "gemm", "weave"), default=None,
                    help="for rocprofv3 --pmc. fused: a few fused launches plus plain copy launches of known "
                         "size (tw_hbm_probe, 192 MiB read + 192 MiB written each) to scale the byte counters "
                         "by. gemm: a few launches of the bf16 GEMM on the overlap demo's shape. weave (for "
                         "rocprofv3 --kernel-trace): the T=4096 layer boundary unsplit, then woven in the "
                         "ordered schedule, then as one chain per split, five calls each with a device "
                         "synchronisation after every call, so that the trace shows which kernels overlap")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus %d is not "
              "supported. `value` is the one GPU's throughput." % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2505_11329_amd as tw
    import tw_workloads as W

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    stream = torch.cuda.Stream()

    def gpu(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(dev)

    def fused_sets(name, nsets, N=None):
        sets = []
        for k in range(nsets):
            d = W.make_fused_inputs(name, N=N, seed=k)
            s = dict(partials=[gpu(p) for p in d["partials"]], residual=gpu(d["residual"]),
                     weight=gpu(d["weight"]), eps=d["eps"], N=d["N"], H=d["H"], P=d["P"])
            s["out"] = torch.empty_like(s["residual"])
            s["res_out"] = torch.empty_like(s["residual"])
            sets.append(s)
        return sets

    def algo_bytes(s, rows=None):
        return (s["P"] + 3) * 2 * s["H"] * (s["N"] if rows is None else rows)

    def event_times(fns, iters, warm, on_stream):
        """Per-launch durations (us) from HIP event pairs recorded on the launch stream."""
        for i in range(warm):
            fns[i % len(fns)]()
        on_stream.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
        for i in range(iters):
            evs[i][0].record(on_stream)
            fns[i % len(fns)]()
            evs[i][1].record(on_stream)
        on_stream.synchronize()
        return np.array([a.elapsed_time(b) for a, b in evs]) * 1e3

    def interleaved_medians(cands, rounds=4, iters=8, warm=2):
        """Median launch time (µs) of each candidate {key: fn or list of fns}. The candidates take turns in
        short bursts so that clock and temperature drift hits all of them alike (the GEMMs are power-limited),
        and the order rotates from round to round: what ran just before a burst moves its times by a few
        percent, so no candidate keeps the same predecessor."""
        keys = list(cands)
        acc = {k: [] for k in keys}
        step = max(1, len(keys) // rounds)
        for r in range(rounds):
            shift = (r * step) % len(keys)
            for k in keys[shift:] + keys[:shift]:
                fns = cands[k] if isinstance(cands[k], (list, tuple)) else [cands[k]]
                acc[k].append(event_times(fns, iters, warm, stream))
        return {k: round(float(np.median(np.concatenate(v))), 1) for k, v in acc.items()}

    if args.sweep:
        def sweep_point(H, P, N, cfgname):
            per_set = (P + 3) * 2 * H * N
            nsets = max(2, min(6, int((600 << 20) // per_set) + 1))
            if nsets * per_set > (12 << 30):
                nsets = 2
            ss = []
            for k in range(nsets):
                # large batches are drawn on the GPU (same distributions): the host generator is slow
                gen = torch.Generator(device=dev)
                gen.manual_seed(1000 * k + N)
                cfg = W.CONFIGS[cfgname]
                parts = [torch.empty((N, H), dtype=torch.bfloat16, device=dev).normal_(0.0, cfg["partial_std"],
                                                                                        generator=gen)
                         for _ in range(P)]
                resid = torch.empty((N, H), dtype=torch.bfloat16, device=dev).normal_(0.0, 1.0, generator=gen)
                s_ = dict(partials=parts, residual=resid, weight=gpu(W.uniform_bf16((H,), 0.5, 1.5, 0,
                                                                                   W.STREAM_WEIGHT)),
                          eps=cfg["eps"], N=N, H=H, P=P, out=torch.empty_like(resid),
                          res_out=torch.empty_like(resid))
                ss.append(s_)
            torch.cuda.synchronize()   # the inputs were drawn on torch's stream, the launches go to ours
            row = {"H": H, "P": P, "N": N, "algorithmic_MB": round(per_set / 1e6, 2)}
            for label, b in (("whole_device", 0), ("shared", tw.CU_SHARED), ("budget32", 32)):
                fns = [tw.prepare_reduce_add_rmsnorm(x["partials"], x["residual"], x["weight"], x["eps"],
                                                     cu_budget=b, out=x["out"], residual_out=x["res_out"],
                                                     stream=stream)[0] for x in ss]
                iters = 40 if N <= 8192 else 12
                t = event_times(fns, iters, 4, stream)
                row[label + "_us"] = round(float(np.median(t)), 2)
                row[label + "_GBps"] = round(per_set / np.median(t) / 1e3, 1)
            del ss
            torch.cuda.empty_cache()
            return row
        rows = []
        for (H, P, cfgname) in ((8192, 8, "c3_70b_shard_tp8"), (8192, 4, "c4_split_sweep_tp4"), (4096, 2, "c2_8b_tp2")):
            for N in (32, 64, 128, 256, 512, 1024, 2048, 4096, 8192, 16384, 32768, 65536):
                rows.append(sweep_point(H, P, N, cfgname))
        # hidden sizes between and beyond the paper's two, at ~180 MB of algorithmic bytes each
        hidden = []
        for (P, cfgname) in ((8, "c3_70b_shard_tp8"), (2, "c2_8b_tp2")):
            for H in (1024, 2048, 2560, 3072, 3584, 4096, 5120, 6144, 7168, 8192, 10240, 12288, 16384):
                hidden.append(sweep_point(H, P, int(180e6 / ((P + 3) * 2 * H)) // 64 * 64, cfgname))
        print(json.dumps({"sweep": rows, "hidden_size_sweep": hidden,
                          "note": "median of HIP-event timed launches, rotating buffer sets, bf16"}))
        return
    if args.split_sweep:
        K1, H, P, N2 = 1024, 8192, 8, 3584
        comm = torch.cuda.Stream()
        cus = tw.device_cu_count()
        gen = torch.Generator(device=dev)
        gen.manual_seed(7)

        def rnd(shape, std):
            return torch.empty(shape, dtype=torch.bfloat16, device=dev).normal_(0.0, std, generator=gen)
        W1, W2 = rnd((H, K1), 0.02), rnd((N2, H), 0.02)
        weight = gpu(W.uniform_bf16((H,), 0.5, 1.5, 0, W.STREAM_WEIGHT))
        rows = []
        for T in range(4096, 8192 + 1, 256):
            X1, resid = rnd((T, K1), 0.02), rnd((T, H), 1.0)
            parts = [rnd((T, H), 0.25) for _ in range(P)]
            out, res_out = torch.empty_like(resid), torch.empty_like(resid)
            Y = torch.empty((T, N2), dtype=torch.bfloat16, device=dev)
            torch.cuda.synchronize()   # inputs drawn on torch's stream, launches on ours

            def layer_fn(split_row, schedule=tw.WEAVE_AUTO):
                def f():
                    with torch.cuda.stream(stream):
                        tw.weave_layer(X1, W1, parts, resid, weight, 1e-5, W2, split_row, stream, comm,
                                       fused_cu_budget=tw.CU_SHARED, gemm_cu_budget=0, out=out,
                                       residual_out=res_out, Y=Y, parent=stream, use_parent=True, join=True,
                                       schedule=schedule)
                return f
            half = (T // 2 + 63) // 64 * 64
            k_smart, ws, wu = tw.smart_split_point(T, 64, [H, N2], cus, gemm_k=[K1, H])
            ks = sorted({half + off for off in (0, 64, 128, 192, 256, 512) if half + off < T} | {k_smart})
            cands = {k: layer_fn(k) for k in [0] + ks}
            for k in sorted({half, k_smart}):      # the same two cuts under the other schedule
                cands["ordered_%d" % k] = layer_fn(k, tw.WEAVE_ORDERED)
            timed = interleaved_medians(cands)
            unsplit_us = timed.pop(0)
            ordered = {int(k[8:]): timed.pop(k) for k in list(timed) if isinstance(k, str)}
            k_best = min(timed, key=timed.get)
            rows.append({"T": T, "equal_split_row": half, "equal_us": timed[half],
                         "measured_best_row": k_best, "measured_best_us": timed[k_best],
                         "smart_row": k_smart, "smart_us": timed[k_smart],
                         "model_cost_split": ws, "model_cost_unsplit": wu, "unsplit_us": unsplit_us,
                         "ordered_equal_us": ordered[half], "ordered_smart_us": ordered[k_smart],
                         "all_us": {str(k): v for k, v in sorted(timed.items())}})
            del X1, resid, parts, out, res_out, Y
            torch.cuda.empty_cache()

        # where splitting starts to pay: the plain chain (three launches on one stream, no events)
        # against the woven layer in shared mode and with a 32-CU budget, over batch sizes, for the
        # attention-side boundary of the sweep above and for the MLP-side boundary of the same model
        def threshold_sweep(K1, N2, W1, W2):
            thr = []
            for T in (256, 512, 1024, 2048, 4096, 6144, 8192, 16384):
                X1, resid = rnd((T, K1), 0.02), rnd((T, H), 1.0)
                parts = [rnd((T, H), 0.25) for _ in range(P)]
                out, res_out = torch.empty_like(resid), torch.empty_like(resid)
                Y = torch.empty((T, N2), dtype=torch.bfloat16, device=dev)
                torch.cuda.synchronize()

                def plain():
                    tw.gemm_bf16(X1, W1, C=parts[0], stream=stream)
                    tw.reduce_add_rmsnorm(parts, resid, weight, 1e-5, cu_budget=0, out=out, residual_out=res_out,
                                          stream=stream)
                    tw.gemm_bf16(out, W2, C=Y, stream=stream)

                def woven(split_row, fb, gb, schedule=tw.WEAVE_AUTO):
                    def f():
                        with torch.cuda.stream(stream):
                            tw.weave_layer(X1, W1, parts, resid, weight, 1e-5, W2, split_row, stream, comm,
                                           fused_cu_budget=fb, gemm_cu_budget=gb, out=out, residual_out=res_out,
                                           Y=Y, parent=stream, use_parent=True, join=True, schedule=schedule)
                    return f
                cands = {"plain_us": plain}
                row = {"T": T}
                k, _, _ = tw.smart_split_point(T, 64, [H, N2], cus, gemm_k=[K1, H])
                if k < T:
                    row["split_row"] = k
                    cands["woven_shared_us"] = woven(k, tw.CU_SHARED, 0)
                    cands["woven_shared_ordered_us"] = woven(k, tw.CU_SHARED, 0, tw.WEAVE_ORDERED)
                    cands["woven_shared_chains_us"] = woven(k, tw.CU_SHARED, 0, tw.WEAVE_CHAINS)
                k32, _, _ = tw.smart_split_point(T, 64, [H, N2], cus - 32, gemm_k=[K1, H])
                if k32 < T:
                    cands["woven_budget32_us"] = woven(k32, 32, cus - 32)
                row.update(interleaved_medians(cands))
                thr.append(row)
                del X1, resid, parts, out, res_out, Y
                torch.cuda.empty_cache()
            return thr
        thr = threshold_sweep(K1, N2, W1, W2)
        K1m, N2m = 3584, 1280
        thr_mlp = threshold_sweep(K1m, N2m, rnd((H, K1m), 0.02), rnd((N2m, H), 0.02))

        def spread(key):
            rate = np.array([r["T"] / r[key] for r in rows])
            return round(float(rate.std() / rate.mean()), 4)
        print(json.dumps({"split_sweep": rows, "threshold_sweep": thr, "threshold_sweep_mlp_side": thr_mlp,
                          "tokens_per_us_relative_spread": {"equal": spread("equal_us"), "smart": spread("smart_us"),
                                                            "measured_best": spread("measured_best_us"),
                                                            "ordered_equal": spread("ordered_equal_us"),
                                                            "ordered_smart": spread("ordered_smart_us")},
                          "note": "layer boundary [Tx1024]x[1024x8192] -> fused H=8192 P=8 (shared mode) -> "
                                  "[Tx8192]x[8192x3584]; medians of HIP-event timed calls of tw_weave_layer, the "
                                  "candidates of one T taking turns in bursts of 8; smart_row comes from tile "
                                  "counts alone; the schedule is the library's choice (TW_WEAVE_AUTO) except "
                                  "in the threshold sweeps' _ordered and _chains columns; threshold_sweep_mlp_side is the "
                                  "boundary [Tx3584]x[3584x8192] -> fused -> [Tx8192]x[8192x1280]"}))
        return
    if args.counters_run == "weave":
        T, K1, H, P, N2 = 4096, 1024, 8192, 8, 3584
        gen = torch.Generator(device=dev)
        gen.manual_seed(0)

        def rnd(shape, std):
            return torch.empty(shape, dtype=torch.bfloat16, device=dev).normal_(0.0, std, generator=gen)
        X1, W1, W2 = rnd((T, K1), 0.02), rnd((H, K1), 0.02), rnd((N2, H), 0.02)
        parts, resid = [rnd((T, H), 0.25) for _ in range(P)], rnd((T, H), 1.0)
        weight = gpu(W.uniform_bf16((H,), 0.5, 1.5, 0, W.STREAM_WEIGHT))
        comm = torch.cuda.Stream()
        torch.cuda.synchronize()
        k, _, _ = tw.smart_split_point(T, 128, [H, N2], tw.device_cu_count(), gemm_k=[K1, H])
        order = [("unsplit", 0, tw.WEAVE_ORDERED), ("ordered", k, tw.WEAVE_ORDERED), ("chains", k, tw.WEAVE_CHAINS)]
        for name, split_row, schedule in order:
            for i in range(5):
                with torch.cuda.stream(stream):
                    tw.weave_layer(X1, W1, parts, resid, weight, 1e-5, W2, split_row, stream, comm,
                                   fused_cu_budget=tw.CU_SHARED, gemm_cu_budget=0, parent=stream, use_parent=True,
                                   join=True, schedule=schedule)
                torch.cuda.synchronize()
        print(json.dumps({"counters_run": "weave", "T": T, "split_row": k, "calls_per_schedule": 5,
                          "order": [o[0] for o in order]}))
        return
    if args.counters_run == "gemm":
        gc = W.CONFIGS["c5_overlap_tp8"]["gemm"]
        g = W.make_gemm_inputs(gc["M"], gc["K"], gc["N"], gc["std"], 0, "nk")
        A, B = gpu(g["A"]), gpu(g["B"])
        C = torch.empty((gc["M"], gc["N"]), dtype=torch.bfloat16, device=dev)
        for i in range(12):
            tw.gemm_bf16(A, B, C=C, cu_budget=0, stream=stream)
        torch.cuda.synchronize()
        print(json.dumps({"counters_run": "gemm", "flops_per_launch": 2.0 * gc["M"] * gc["K"] * gc["N"]}))
        return
    if args.counters_run == "fused":
        sets = fused_sets(WORKLOAD, 4)
        pb = 192 << 20
        src = torch.empty(pb, dtype=torch.uint8, device=dev).random_()
        dst = torch.empty(pb, dtype=torch.uint8, device=dev)
        torch.cuda.synchronize()
        for i in range(12):
            s = sets[i % 4]
            tw.reduce_add_rmsnorm(s["partials"], s["residual"], s["weight"], s["eps"], cu_budget=args.budget,
                                  out=s["out"], residual_out=s["res_out"], stream=stream)
            tw.hbm_probe(src, dst, pb, tw.PROBE_COPY, cu_budget=args.budget, stream=stream)
        torch.cuda.synchronize()
        print(json.dumps({"counters_run": True, "fused_algorithmic_bytes": algo_bytes(sets[0]),
                          "copy_bytes_read": pb, "copy_bytes_written": pb, "cu_budget": args.budget}))
        return

    # ---------------- timed region: K steps of the headline workload ----------------
    sets = fused_sets(WORKLOAD, 4)
    nbytes = algo_bytes(sets[0])
    launches = [tw.prepare_reduce_add_rmsnorm(s["partials"], s["residual"], s["weight"], s["eps"],
                                              cu_budget=args.budget, out=s["out"], residual_out=s["res_out"],
                                              stream=stream)[0] for s in sets]
    for i in range(args.warmup):
        launches[i % 4]()
    stream.synchronize()
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        evs[i][0].record(stream)
        launches[i % 4]()
        evs[i][1].record(stream)
    stream.synchronize()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    kern_us = np.array([a.elapsed_time(b) for a, b in evs]) * 1e3
    avg_us = float(kern_us.mean())
    value = nbytes / (ms_per_step * 1e-3) / 1e9
    achieved = nbytes / (avg_us * 1e-6) / 1e9

    result = {
        "metric": "fused reduce+add+RMSNorm GB/s & % HBM peak at fixed CU budget; overlap makespan",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: N=1024 rows (1/8 of 8192 tokens), H=8192, P=8" % WORKLOAD,
                   "storage": "bf16 tensors in HBM, fp32 arithmetic, one rounding per stored value",
                   "cu_budget": args.budget, "eps": sets[0]["eps"],
                   "buffer_sets_rotated": 4, "algorithmic_bytes_per_step": nbytes,
                   "clocks": "not locked (non-root)"},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": (round(MEASURED_TRAFFIC_BYTES[(WORKLOAD, args.budget)] / (avg_us * 1e-6) / 1e9, 1)
                                 if (WORKLOAD, args.budget) in MEASURED_TRAFFIC_BYTES else None),
                     "traffic_bytes_per_launch": MEASURED_TRAFFIC_BYTES.get((WORKLOAD, args.budget)),
                     "kernel": "tw::fused_kernel<8,1,false>", "avg_launch_us": round(avg_us, 2),
                     "p10_us": round(float(np.percentile(kern_us, 10)), 2),
                     "p50_us": round(float(np.percentile(kern_us, 50)), 2),
                     "p90_us": round(float(np.percentile(kern_us, 90)), 2)},
    }

    if not args.no_extras:
        extras(result, tw, W, torch, np, stream, sets, fused_sets, algo_bytes, event_times, interleaved_medians, gpu)
    del sets, launches
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(W, np)
    print(json.dumps(result))


def extras(result, tw, W, torch, np, stream, sets, fused_sets, algo_bytes, event_times, interleaved_medians, gpu):
    """Per-budget table, probe ceilings, split sweep, overlap demo. All outside the timed region."""
    nbytes = algo_bytes(sets[0])

    def fused_fns(ss, budget, st=stream):
        return [tw.prepare_reduce_add_rmsnorm(s["partials"], s["residual"], s["weight"], s["eps"], cu_budget=budget,
                                              out=s["out"], residual_out=s["res_out"], stream=st)[0] for s in ss]

    # what a budget can stream: read-only and copy probes over 192 MiB buffers, rotated
    pb = 192 << 20
    srcs = [torch.empty(pb, dtype=torch.uint8, device="cuda:0").random_() for _ in range(4)]
    dsts = [torch.empty(pb, dtype=torch.uint8, device="cuda:0") for _ in range(4)]
    budgets = {}
    for b in (8, 16, 32, 64, 128, 256):
        t = event_times(fused_fns(sets, b), 60, 8, stream)
        row = {"us": round(float(np.median(t)), 1), "GBps": round(nbytes / np.median(t) / 1e3, 1),
               "frac_hbm_peak": round(nbytes / np.median(t) / 1e3 / HBM_PEAK_GBS, 4)}
        fns = [(lambda i=i: tw.hbm_probe(srcs[i], dsts[i], pb, tw.PROBE_READ, cu_budget=b, stream=stream))
               for i in range(4)]
        tp = event_times(fns, 20, 4, stream)
        row["probe_read_GBps"] = round(pb / np.median(tp) / 1e3, 1)
        # the fused kernel's own mix: P+1 streams read, 2 written, 16 MiB each, no arithmetic
        sb = pb // 12
        sb -= sb % 16384
        fns = [(lambda i=i: tw.hbm_probe_mixed(srcs[i], dsts[i], sb, 9, 2, cu_budget=b, stream=stream))
               for i in range(4)]
        tp = event_times(fns, 20, 4, stream)
        row["probe_mix_9r2w_GBps"] = round(11 * sb / np.median(tp) / 1e3, 1)
        row["frac_of_mix_probe"] = round(row["GBps"] / row["probe_mix_9r2w_GBps"], 3)
        # where the workgroups ran: distinct (XCC, SE, SH, CU) places decoded from the hardware id registers
        x = sets[0]
        _, _, hw = tw.reduce_add_rmsnorm_traced(x["partials"], x["residual"], x["weight"], x["eps"], cu_budget=b,
                                                out=x["out"], residual_out=x["res_out"], stream=stream)
        stream.synchronize()
        hw = hw.cpu().numpy().astype(np.int64) & 0xFFFFFFFF
        places = set(zip((hw[:, 1] & 0xF).tolist(), ((hw[:, 0] >> 13) & 0x7).tolist(),
                         ((hw[:, 0] >> 12) & 0x1).tolist(), ((hw[:, 0] >> 8) & 0xF).tolist()))
        row["workgroups"] = int(hw.shape[0])
        row["cus_occupied"] = len(places)
        budgets[str(b)] = row
    # context only: the same launch when its inputs are still in the 256 MB Infinity Cache (as they
    # would be right after the kernels that produce them); one buffer set, no rotation
    for b in (32, 256):
        t = event_times(fused_fns(sets[:1], b), 40, 8, stream)
        budgets[str(b)]["inputs_in_infinity_cache_GBps"] = round(nbytes / np.median(t) / 1e3, 1)
    t = event_times(fused_fns(sets, tw.CU_SHARED), 60, 8, stream)
    budgets["shared"] = {"us": round(float(np.median(t)), 1), "GBps": round(nbytes / np.median(t) / 1e3, 1),
                         "frac_hbm_peak": round(nbytes / np.median(t) / 1e3 / HBM_PEAK_GBS, 4),
                         "note": "cu_budget=TW_CU_SHARED run alone: 256-thread workgroups on every CU"}
    result["budgets"] = {"workload": WORKLOAD, "per_budget": budgets,
                         "note": "probe_read = one stream read; probe_mix_9r2w = 9 streams read + 2 written with "
                                 "the fused kernel's launch shape and access pattern but no arithmetic: the "
                                 "ceiling that this many compute units allow"}
    del srcs, dsts
    torch.cuda.empty_cache()

    # 8B-class shape (config 2) per budget
    s2 = fused_sets("c2_8b_tp2", 6)
    nb2 = algo_bytes(s2[0])
    c2 = {}
    for b in (8, 16, 32, 256):
        t = event_times(fused_fns(s2, b), 60, 8, stream)
        c2[str(b)] = {"us": round(float(np.median(t)), 1), "GBps": round(nb2 / np.median(t) / 1e3, 1)}
    result["config2_8b_tp2"] = c2

    # what the single pass saves: the same step as "all-reduce to bf16, then residual add + RMSNorm
    # re-reading what it stored" (two launches, three passes), both on the whole device
    abl = {}
    for name, ss in ((WORKLOAD.split(":")[0], sets), ("c2_8b_tp2", s2)):
        scr = [torch.empty_like(x["residual"]) for x in ss]
        unf = [(lambda x=x, sc=sc: tw.reduce_add_rmsnorm_unfused(x["partials"], x["residual"], x["weight"], x["eps"],
                                                                 out=x["out"], residual_out=x["res_out"],
                                                                 sum_scratch=sc, stream=stream))
               for x, sc in zip(ss, scr)]
        t_u = float(np.median(event_times(unf, 60, 8, stream)))
        t_f = float(np.median(event_times(fused_fns(ss, 0), 60, 8, stream)))
        P_, H_, N_ = ss[0]["P"], ss[0]["H"], ss[0]["N"]
        abl[name] = {"fused_us": round(t_f, 1), "unfused_us": round(t_u, 1), "speedup": round(t_u / t_f, 3),
                     "bytes_ratio_unfused_over_fused": round((P_ + 6) / (P_ + 3), 3),
                     "unfused_GBps_of_its_own_bytes": round((P_ + 6) * 2 * H_ * N_ / t_u / 1e3, 1)}
        del scr, unf
    result["ablation_unfused"] = {
        "per_config": abl,
        "note": "tw_reduce_add_rmsnorm_unfused: (P+6)*2H bytes per row in two launches against the fused "
                "kernel's (P+3)*2H in one; whole device, rotating buffer sets"}
    del s2
    torch.cuda.empty_cache()

    # token split (config 4): one launch vs two halves on two streams, makespan on the parent
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    split = {}
    cfg4 = W.CONFIGS["c4_split_sweep_tp4"]
    for N in (1024, 4096):
        nsets = 4 if N <= 1024 else 2
        s4 = fused_sets("c4_split_sweep_tp4", nsets, N=N)
        nb4 = algo_bytes(s4[0])
        k = tw.split_point(N, cfg4["split_multiple"])
        for b in cfg4["cu_budgets"]:
            t1 = event_times(fused_fns(s4, b), 40, 6, stream)

            def split_fn(s, b=b, k=k):
                def f():
                    with torch.cuda.stream(stream):
                        tw.split_launch(s["partials"], s["residual"], s["weight"], s["eps"], k, sa, sb, cu_budget=b,
                                        out=s["out"], residual_out=s["res_out"], parent=stream, use_parent=True,
                                        join=True)
                return f
            t2 = event_times([split_fn(s) for s in s4], 40, 6, stream)
            split["N%d_b%d" % (N, b)] = {"unsplit_us": round(float(np.median(t1)), 1),
                                         "split_us": round(float(np.median(t2)), 1),
                                         "unsplit_GBps": round(nb4 / np.median(t1) / 1e3, 1),
                                         "split_GBps": round(nb4 / np.median(t2) / 1e3, 1)}
        del s4
        torch.cuda.empty_cache()
    result["split"] = {"workload": "c4_split_sweep_tp4 (H=8192, P=4, k=N/2)", "per_case": split,
                       "note": "each half gets the budget, so the split run occupies 2x the CUs"}

    # overlap demo (config 5): fused(A, 32 CUs) next to GEMM(B) vs back to back
    cfg5 = W.CONFIGS["c5_overlap_tp8"]
    gc = cfg5["gemm"]
    half = cfg5["N"] // 2
    s5 = fused_sets("c5_overlap_tp8", 2, N=half)
    nb5 = algo_bytes(s5[0])
    g = W.make_gemm_inputs(gc["M"], gc["K"], gc["N"], gc["std"], 0, "nk")
    A, B = gpu(g["A"]), gpu(g["B"])
    C = torch.empty((gc["M"], gc["N"]), dtype=torch.bfloat16, device="cuda:0")
    flops = 2.0 * gc["M"] * gc["K"] * gc["N"]
    comm, comp = torch.cuda.Stream(), torch.cuda.Stream()
    cus_total = tw.device_cu_count()
    tf = event_times(fused_fns(s5, 32), 30, 5, stream)
    tg = event_times([lambda: tw.gemm_bf16(A, B, C=C, cu_budget=0, stream=stream)], 30, 5, stream)

    def serial_fn(s):
        def f():
            tw.reduce_add_rmsnorm(s["partials"], s["residual"], s["weight"], s["eps"], cu_budget=32,
                                  out=s["out"], residual_out=s["res_out"], stream=stream)
            tw.gemm_bf16(A, B, C=C, cu_budget=0, stream=stream)
        return f

    def overlap_fn(s, fused_budget, gemm_budget):
        # the caller's stream is the compute stream (as in the paper: a compute stream and a
        # communication stream), so only the comm stream is forked from and joined into it
        def f():
            with torch.cuda.stream(stream):
                tw.overlap_launch(dict(partials=s["partials"], residual=s["residual"], weight=s["weight"],
                                       eps=s["eps"], cu_budget=fused_budget, out=s["out"],
                                       residual_out=s["res_out"]),
                                  dict(A=A, B=B, C=C, cu_budget=gemm_budget), comm, stream, parent=stream,
                                  use_parent=True, join=True)
        return f
    # the best schedule without overlap on one GPU: no partition, each kernel gets every CU in turn
    def serial_whole_fn(s):
        def f():
            tw.reduce_add_rmsnorm(s["partials"], s["residual"], s["weight"], s["eps"], cu_budget=0,
                                  out=s["out"], residual_out=s["res_out"], stream=stream)
            tw.gemm_bf16(A, B, C=C, cu_budget=0, stream=stream)
        return f
    # the schedules take turns, in rotating order
    ov = interleaved_medians({
        "serial32": [serial_fn(s) for s in s5], "serial_whole": [serial_whole_fn(s) for s in s5],
        "budget32": [overlap_fn(s, 32, cus_total - 32) for s in s5],
        "shared": [overlap_fn(s, tw.CU_SHARED, 0) for s in s5]}, rounds=8, iters=10, warm=2)

    # each kernel's own duration while the other runs: event pairs on the two streams
    def contended(fused_budget, gemm_budget, gemm_first):
        f_us, g_us = [], []
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        for rep in range(16):
            s = s5[rep % 2]
            torch.cuda.synchronize()

            def launch_gemm():
                ev[0].record(comp)
                tw.gemm_bf16(A, B, C=C, cu_budget=gemm_budget, stream=comp)
                ev[1].record(comp)

            def launch_fused():
                ev[2].record(comm)
                tw.reduce_add_rmsnorm(s["partials"], s["residual"], s["weight"], s["eps"], cu_budget=fused_budget,
                                      out=s["out"], residual_out=s["res_out"], stream=comm)
                ev[3].record(comm)
            if gemm_first:
                launch_gemm()
                launch_fused()
            else:
                launch_fused()
                launch_gemm()
            torch.cuda.synchronize()
            if rep >= 2:
                g_us.append(ev[0].elapsed_time(ev[1]) * 1e3)
                f_us.append(ev[2].elapsed_time(ev[3]) * 1e3)
        return float(np.median(f_us)), float(np.median(g_us))
    cont_f32, cont_g32 = contended(32, cus_total - 32, False)
    cont_fsh, cont_gsh = contended(tw.CU_SHARED, 0, True)
    result["overlap"] = {
        "workload": "c5_overlap_tp8: fused N=2048,H=8192,P=8 @32 CUs || GEMM [2048x8192]x[8192x3584] bf16",
        "fused_alone_us": round(float(np.median(tf)), 1), "gemm_alone_us": round(float(np.median(tg)), 1),
        "gemm_alone_TFLOPs": round(flops / np.median(tg) / 1e6, 1),
        "gemm_frac_mfma_peak": round(flops / np.median(tg) / 1e6 / MFMA_BF16_PEAK_TFLOPS, 4),
        "serial_budget32_us": ov["serial32"],
        "serial_whole_device_us": ov["serial_whole"],
        "overlapped_budget32_us": ov["budget32"],
        "overlapped_shared_us": ov["shared"],
        "gain_budget32_vs_serial_budget32": round(ov["serial32"] / ov["budget32"], 3),
        "gain_budget32_vs_serial_whole_device": round(ov["serial_whole"] / ov["budget32"], 3),
        "gain_shared_vs_serial_whole_device": round(ov["serial_whole"] / ov["shared"], 3),
        "under_contention_budget32": {"fused_us": round(cont_f32, 1), "fused_GBps": round(nb5 / cont_f32 / 1e3, 1),
                                      "gemm_us": round(cont_g32, 1)},
        "under_contention_shared": {"fused_us": round(cont_fsh, 1), "fused_GBps": round(nb5 / cont_fsh / 1e3, 1),
                                    "gemm_us": round(cont_gsh, 1)},
        "note": "serial_budget32 = fused at 32 CUs then GEMM on one stream; serial_whole_device = fused on all CUs "
                "then GEMM on all CUs (the best schedule without overlap); overlapped_budget32 = tw_overlap_launch, "
                "fused confined to 32 CUs, GEMM on the other 224; overlapped_shared = tw_overlap_launch with "
                "cu_budget=TW_CU_SHARED: small fused workgroups co-resident with the GEMM's on every CU. The "
                "caller's stream is the compute stream; the schedules take turns in bursts, in rotating order; makespans include fork and join",
    }
    del s5
    torch.cuda.empty_cache()

    # one woven layer boundary (G1 -> fused -> G2), T = 4096 tokens, attention-side shapes of a 70B-class
    # TP=8 model: G1 [T x 1024] x [1024 x 8192], fused H=8192 P=8, G2 [T x 8192] x [8192 x 3584]
    T, K1, H, P, N2 = 4096, 1024, 8192, 8, 3584
    d = W.make_fused_inputs("c5_overlap_tp8", N=T)
    g1 = W.make_gemm_inputs(T, K1, H, 0.02, 1, "nk")
    X1, W1 = gpu(g1["A"]), gpu(g1["B"])
    W2 = gpu(W.normal_bf16((N2, H), 0.02, 2, W.STREAM_GEMM_B))
    parts = [torch.empty((T, H), dtype=torch.bfloat16, device="cuda:0")] + [gpu(p) for p in d["partials"][1:]]
    resid, weight = gpu(d["residual"]), gpu(d["weight"])
    out, res_out = torch.empty_like(resid), torch.empty_like(resid)
    Y = torch.empty((T, N2), dtype=torch.bfloat16, device="cuda:0")
    cus = tw.device_cu_count()

    def layer_fn(split_row, fb, gb, schedule=tw.WEAVE_AUTO):
        def f():
            with torch.cuda.stream(stream):
                tw.weave_layer(X1, W1, parts, resid, weight, d["eps"], W2, split_row, stream, comm,
                               fused_cu_budget=fb, gemm_cu_budget=gb, out=out, residual_out=res_out, Y=Y,
                               parent=stream, use_parent=True, join=True, schedule=schedule)
        return f
    # the schedules take turns in bursts of 8 calls, in rotating order
    cands = {"unsplit": layer_fn(0, 0, 0)}
    plan = {}
    for fb in (32, 64, 96):
        k, ws, wu = tw.smart_split_point(T, 128, [H, N2], cus - fb, gemm_k=[K1, H])
        plan[fb] = (k, ws, wu)
        cands["woven_%d" % fb] = layer_fn(k, fb, cus - fb)
        cands["unsplit_%d" % fb] = layer_fn(0, fb, cus - fb)
    k, ws, wu = tw.smart_split_point(T, 128, [H, N2], cus, gemm_k=[K1, H])
    plan["shared"] = (k, ws, wu)
    cands["woven_shared"] = layer_fn(k, tw.CU_SHARED, 0)
    cands["woven_shared_ordered"] = layer_fn(k, tw.CU_SHARED, 0, tw.WEAVE_ORDERED)
    cands["woven_shared_chains"] = layer_fn(k, tw.CU_SHARED, 0, tw.WEAVE_CHAINS)
    med = interleaved_medians(cands, rounds=5, iters=8, warm=2)
    weave = {"unsplit_whole_device_us": med["unsplit"]}
    for fb in (32, 64, 96):
        k, ws, wu = plan[fb]
        weave["fused_budget_%d" % fb] = {"split_row": k, "model_cost_split": ws, "model_cost_unsplit": wu,
                                         "woven_us": med["woven_%d" % fb],
                                         "unsplit_same_budgets_us": med["unsplit_%d" % fb]}
    k, ws, wu = plan["shared"]
    weave["fused_shared"] = {"split_row": k, "model_cost_split": ws, "model_cost_unsplit": wu,
                             "woven_us": med["woven_shared"], "woven_ordered_us": med["woven_shared_ordered"],
                             "woven_chains_us": med["woven_shared_chains"]}
    result["weave_layer"] = {
        "workload": "T=4096: G1 [Tx1024]x[1024x8192] -> fused H=8192 P=8 -> G2 [Tx8192]x[8192x3584], bf16",
        "cases": weave,
        "note": "woven = tw_weave_layer at the wave-aware split row, fused kernel confined to its budget and the "
                "GEMMs to the other CUs (fused_shared: co-resident; woven_us with the schedule the library "
                "picks, then each schedule forced); unsplit_same_budgets = same budgets, no split; unsplit_whole_device = "
                "each kernel on all CUs in turn, one stream, no events; the schedules take turns in bursts",
    }


def cpu_baseline(W, np):
    """The fp64 oracle, as it stands, timed on this machine's host cores on the headline
    workload (all 1024 rows), single-threaded and row-parallel."""
    import oracle
    d = W.make_fused_inputs(WORKLOAD)
    nbytes = (d["P"] + 3) * 2 * d["H"] * d["N"]
    threads = max(1, min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "0") or 0) or 64))

    def timed(nt, budget_s):
        times = []
        t_end = time.perf_counter() + budget_s
        while len(times) < 3 or time.perf_counter() < t_end:
            t = time.perf_counter()
            oracle.fused_mt(d["partials"], d["residual"], d["weight"], d["eps"], nt)
            times.append(time.perf_counter() - t)
        return float(np.median(times)), len(times)

    t1, n1 = timed(1, 6.0)
    tn, nn = timed(threads, 6.0)
    return {"value": round(nbytes / tn / 1e9, 3), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": "all 1024 rows of %s, median of %d runs (row-parallel pthreads, output allocation included)"
                      % (WORKLOAD, nn),
            "single_thread_GBps": round(nbytes / t1 / 1e9, 3), "single_thread_runs": n1}


if __name__ == "__main__":
    main()
