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
# WRITE_SIZE, each scaled by what the same counter reads for a 192 MiB copy). They are
# not measured in this run (counters need the profiler): they are the figures of the
# named profile, valid for the kernel source whose hash is recorded beside them. A
# kernel edit changes the hash; the line then reports traffic as null until the
# profile is taken again (tests/test_bench_contract.py fails on the mismatch too).
TRAFFIC_FROM_PROFILE = {
    (WORKLOAD, 32): {
        "profile": "profiles/fused_kernel_c3_70b_shard_tp8_budget32.md",
        "kernel": "tw::fused_kernel<8, 1, false, false>",
        "fetched_KiB": 147648, "written_KiB": 32768,
        "kernel_source_sha256_12": "ec6e1d1ac6d8",
    },
    (WORKLOAD, 0): {
        "profile": "profiles/fused_kernel_c3_whole_device_and_shared.md",
        "kernel": "tw::fused_thin_kernel<8, 4, false, false>",
        "fetched_KiB": 147686, "written_KiB": 32745,
        "kernel_source_sha256_12": "ec6e1d1ac6d8",
    },
}
KERNEL_SOURCES = ("paper_2505_11329_amd/csrc/tw_fused.hip", "paper_2505_11329_amd/csrc/tw_device.h")


_streams_tried = [0]


def overlapping_stream(tw, torch, others, tries=12):
    """A new torch stream whose kernels run side by side with those of every stream in `others`. The HIP
    runtime maps a process's streams onto few hardware queues (4 here) and two streams on one queue
    never overlap, whatever the events between them say: about every fourth stream torch hands out
    shares the first one's queue. tw_streams_overlap tells; streams that fail stay in torch's pool."""
    for _ in range(tries):
        cand = torch.cuda.Stream()
        _streams_tried[0] += 1
        if all(tw.streams_overlap(o, cand) for o in others):
            return cand
    raise RuntimeError("no stream found that overlaps with the given ones after %d tries" % tries)


def kernel_source_hash():
    """First 12 hex digits of the SHA-256 over the fused kernel's source files."""
    import hashlib
    h = hashlib.sha256()
    for rel in KERNEL_SOURCES:
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:12]

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
    ap.add_argument("--ceiling", action="store_true",
                    help="instead of the benchmark line: GB/s per compute unit of plain streaming kernels "
                         "(tw_hbm_probe_shaped / tw_hbm_probe_mixed_shaped) for budgets 1..32 x workgroup size x "
                         "accesses in flight x read / copy / 9-read-2-write: the per-CU HBM ceiling the fused "
                         "kernel is measured against")
    ap.add_argument("--gemm-phases", action="store_true",
                    help="where the clocks of the 256x256 GEMM tile's K loop go (tw_gemm_bf16_traced), as JSON")
    ap.add_argument("--counters-run", choices=("fused", "gemm", "weave", "probe", "train"), default=None,
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

    def train_times(fns, trains, length, warm, on_stream):
        """Per-launch durations (us) from trains of `length` back-to-back launches between ONE pair of HIP
        events on the launch stream (elapsed / length, one figure per train). A pair of events around a
        single launch reads about 2 us more than the kernel takes (an empty pair reads 4 us); a train
        amortises that and agrees with the profiler's kernel trace, at the price of including the gaps
        between consecutive kernels."""
        for i in range(warm):
            fns[i % len(fns)]()
        on_stream.synchronize()
        out, k = [], 0
        for _ in range(trains):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(on_stream)
            for _ in range(length):
                fns[k % len(fns)]()
                k += 1
            e1.record(on_stream)
            on_stream.synchronize()
            out.append(e0.elapsed_time(e1) * 1e3 / length)
        return np.array(out)

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

    if args.ceiling:
        ceiling_sweep(tw, torch, np, stream, train_times)
        return
    if args.gemm_phases:
        gemm_phases(tw, torch, np, stream, train_times)
        return
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
                length = 10 if N <= 8192 else 4
                t = train_times(fns, 6 if N <= 8192 else 3, length, 4, stream)
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
                          "note": "per-launch time from trains of back-to-back launches between one HIP event pair, median "
                                  "over trains, rotating buffer sets, bf16"}))
        return
    if args.split_sweep:
        K1, H, P, N2 = 1024, 8192, 8, 3584
        comm = overlapping_stream(tw, torch, [stream])
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
            k_policy = tw.policy_split_row(T, K1, H, P, N2, cus)     # the smart row, or T: both were timed
            rows.append({"T": T, "policy_row": k_policy, "policy_us": timed[k_policy] if k_policy < T else unsplit_us,
                         "equal_split_row": half, "equal_us": timed[half],
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
        def over_best(pick):
            ratio = [pick(r) / min(r["unsplit_us"], r["measured_best_us"]) for r in rows]
            return {"mean": round(float(np.mean(ratio)), 4), "worst": round(float(np.max(ratio)), 4)}
        t_built_in = tw.split_threshold(K1, H, P, N2, cus)
        policy_quality = {
            "built_in_rule_over_best": over_best(lambda r: r["policy_us"]),
            "threshold_alone_over_best": over_best(lambda r: r["smart_us"] if r["T"] >= t_built_in else r["unsplit_us"]),
            "always_split_over_best": over_best(lambda r: r["smart_us"]),
            "never_split_over_best": over_best(lambda r: r["unsplit_us"]),
            "rule_picks_the_faster_of_its_two": sum(
                (r["policy_row"] < r["T"]) == (r["smart_us"] <= r["unsplit_us"]) for r in rows),
            "token_counts": len(rows)}
        print(json.dumps({"split_sweep": rows, "policy_quality": policy_quality, "threshold_sweep": thr, "threshold_sweep_mlp_side": thr_mlp,
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
        comm = overlapping_stream(tw, torch, [stream])
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
    if args.counters_run == "train":
        # three unsplit and three woven trains of eight boundaries (attention side, MLP side alternating)
        # at T = 8192, each followed by a device synchronisation
        T, H, P, L = 8192, 8192, 8, 8
        gen = torch.Generator(device=dev)
        gen.manual_seed(0)

        def rnd(shape, std):
            return torch.empty(shape, dtype=torch.bfloat16, device=dev).normal_(0.0, std, generator=gen)
        shapes = [(1024, 3584), (3584, 1280)]
        weight = gpu(W.uniform_bf16((H,), 0.5, 1.5, 0, W.STREAM_WEIGHT))
        bufs = [dict(X1=rnd((T, K1), 0.02), W1=rnd((H, K1), 0.02), partials=[rnd((T, H), 0.25) for _ in range(P)],
                     residual=rnd((T, H), 1.0), weight=weight, eps=1e-5, W2=rnd((N2, H), 0.02),
                     out=torch.empty((T, H), dtype=torch.bfloat16, device=dev),
                     residual_out=torch.empty((T, H), dtype=torch.bfloat16, device=dev),
                     Y=torch.empty((T, N2), dtype=torch.bfloat16, device=dev)) for (K1, N2) in shapes]
        train = [bufs[i % 2] for i in range(L)]
        comm = overlapping_stream(tw, torch, [stream])
        torch.cuda.synchronize()
        for cut in (0, 0, 0, T // 2, T // 2, T // 2):
            with torch.cuda.stream(stream):
                tw.weave_train(train, cut, stream, comm, parent=stream, use_parent=True, join=True)
            torch.cuda.synchronize()
        print(json.dumps({"counters_run": "train", "T": T, "boundaries": L, "split_row": T // 2,
                          "order": ["unsplit"] * 3 + ["woven"] * 3}))
        return
    if args.counters_run == "gemm":
        # the three tile shapes the library builds: the overlap demo's product takes 256 x 128 tiles, the
        # MLP-side down projection of the same layer ([2048 x 8192] x [8192 x 1280], 80 wide tiles) 256 x 64,
        # a large square product 256 x 256
        gc = W.CONFIGS["c5_overlap_tp8"]["gemm"]
        shapes = [(gc["M"], gc["K"], gc["N"]), (gc["M"], gc["K"], 1280), (8192, 8192, 8192)]   # the last: 256 x 256
        for (M, K, N) in shapes:
            gen = torch.Generator(device=dev)
            gen.manual_seed(M + N)
            A = torch.empty((M, K), dtype=torch.bfloat16, device=dev).normal_(0.0, gc["std"], generator=gen)
            B = torch.empty((N, K), dtype=torch.bfloat16, device=dev).normal_(0.0, gc["std"], generator=gen)
            C = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
            torch.cuda.synchronize()
            for i in range(12):
                tw.gemm_bf16(A, B, C=C, cu_budget=0, stream=stream)
            torch.cuda.synchronize()
        print(json.dumps({"counters_run": "gemm", "launches_per_shape": 12,
                          "flops_per_launch": [2.0 * M * K * N for (M, K, N) in shapes]}))
        return
    if args.counters_run == "probe":
        # plain streaming kernels with the fused kernel's budgeted launch shape, for the L1 request counters
        pb = 192 << 20
        src = torch.empty(pb, dtype=torch.uint8, device=dev).random_()
        dst = torch.empty(pb, dtype=torch.uint8, device=dev)
        sb = pb // 12
        sb -= sb % 16384
        torch.cuda.synchronize()
        for i in range(8):
            tw.hbm_probe(src, dst, pb, tw.PROBE_READ, cu_budget=args.budget, stream=stream)
            tw.hbm_probe_mixed(src, dst, sb, 9, 2, cu_budget=args.budget, stream=stream)
        torch.cuda.synchronize()
        print(json.dumps({"counters_run": "probe", "read_bytes": pb, "mixed_bytes_read": 9 * sb,
                          "mixed_bytes_written": 2 * sb, "cu_budget": args.budget}))
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
    # The timed region holds the K steps and nothing else: one HIP event before the first and one after
    # the last, on the launch stream. (Event pairs around every single launch, as an earlier version had,
    # put two extra queue packets between consecutive kernels and read ~2 us more per launch than the
    # profiler's kernel trace.)
    ev_begin, ev_end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev_begin.record(stream)
    for i in range(args.steps):
        launches[i % 4]()
    ev_end.record(stream)
    stream.synchronize()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    avg_us = float(ev_begin.elapsed_time(ev_end)) * 1e3 / args.steps
    # spread of single launches, outside the timed region: an event pair around each of 100 launches
    kern_us = event_times(launches, min(100, max(10, args.steps)), 4, stream)
    value = nbytes / (ms_per_step * 1e-3) / 1e9
    achieved = nbytes / (avg_us * 1e-6) / 1e9
    thin = args.budget <= 0 or args.budget >= tw.device_cu_count()
    kernel_name = "tw::fused_thin_kernel<8, 4, false, false>" if thin else "tw::fused_kernel<8, 1, false, false>"

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
                     "traffic": None, "traffic_bytes_per_launch": None,
                     "kernel": kernel_name, "avg_launch_us": round(avg_us, 2),
                     "avg_launch_us_is": "HIP events on the launch stream around the K timed steps, / K",
                     "single_launch_event_pair_us": {"p10": round(float(np.percentile(kern_us, 10)), 2),
                                                     "p50": round(float(np.percentile(kern_us, 50)), 2),
                                                     "p90": round(float(np.percentile(kern_us, 90)), 2),
                                                     "note": "outside the timed region; a pair of events around "
                                                             "one launch reads ~2 us more than the kernel takes"},
                     "target": "north star: >= 0.70 of HBM peak at H=8192, P=8 within <= 32 CUs -- NOT MET, and "
                               "above what 32 compute units can request from HBM on this part (see "
                               "hbm_ceiling_per_cu below and bench.py --ceiling)"},
    }
    tp = TRAFFIC_FROM_PROFILE.get((WORKLOAD, args.budget))
    rf = result["roofline"]
    if tp is None:
        rf["traffic_source"] = "no counter profile for this budget"
    elif tp["kernel_source_sha256_12"] != kernel_source_hash():
        rf["traffic_source"] = ("stale: %s was taken for kernel source %s, this build is %s"
                                % (tp["profile"], tp["kernel_source_sha256_12"], kernel_source_hash()))
    else:
        tbytes = (tp["fetched_KiB"] + tp["written_KiB"]) * 1024
        rf["traffic"] = round(tbytes / (avg_us * 1e-6) / 1e9, 1)
        rf["traffic_bytes_per_launch"] = tbytes
        rf["traffic_source"] = "counters in %s (kernel %s, source %s), not measured in this run" % (
            tp["profile"], tp["kernel"], tp["kernel_source_sha256_12"])
        assert tp["kernel"] == rf["kernel"]

    if not args.no_extras:
        extras(result, tw, W, torch, np, stream, sets, fused_sets, algo_bytes, event_times, train_times,
               interleaved_medians, gpu)
    del sets, launches
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(W, np)
    print(json.dumps(result))


def extras(result, tw, W, torch, np, stream, sets, fused_sets, algo_bytes, event_times, train_times,
               interleaved_medians, gpu):
    """Per-budget table, probe ceilings, split sweep, overlap demo. All outside the timed region."""
    nbytes = algo_bytes(sets[0])

    def fused_fns(ss, budget, st=stream):
        return [tw.prepare_reduce_add_rmsnorm(s["partials"], s["residual"], s["weight"], s["eps"], cu_budget=budget,
                                              out=s["out"], residual_out=s["res_out"], stream=st)[0] for s in ss]

    def device_drawn_sets(cfgname, nsets, N, P=None, H=None):
        """Buffer sets of a configuration's shape and value distributions drawn with torch's generator on
        the GPU (seeded): for batches too large for the host-side counter-based generator to be quick."""
        cfg = W.CONFIGS[cfgname]
        P_, H_ = P or cfg["P"], H or cfg["H"]
        out_ = []
        for k in range(nsets):
            gen = torch.Generator(device="cuda:0")
            gen.manual_seed(7919 * k + N)

            def rnd(shape, std):
                return torch.empty(shape, dtype=torch.bfloat16, device="cuda:0").normal_(0.0, std, generator=gen)
            parts = [rnd((N, H_), cfg["partial_std"]) for _ in range(P_)]
            resid = rnd((N, H_), cfg["residual_std"])
            out_.append(dict(partials=parts, residual=resid, eps=cfg["eps"], N=N, H=H_, P=P_,
                             weight=gpu(W.uniform_bf16((H_,), 0.5, 1.5, 0, W.STREAM_WEIGHT)),
                             out=torch.empty_like(resid), res_out=torch.empty_like(resid)))
        torch.cuda.synchronize()      # drawn on torch's stream, launched on ours
        return out_

    # what a budget can stream: read-only and copy probes over 192 MiB buffers, rotated
    pb = 192 << 20
    srcs = [torch.empty(pb, dtype=torch.uint8, device="cuda:0").random_() for _ in range(4)]
    dsts = [torch.empty(pb, dtype=torch.uint8, device="cuda:0") for _ in range(4)]
    budgets = {}

    def per_launch_us(fns, est_us):
        """Median per-launch time from trains of 10 back-to-back launches (one event pair per train)."""
        trains = int(max(4, min(12, 3000.0 / max(est_us, 1.0))))
        return float(np.median(train_times(fns, trains, 10, 6, stream)))
    for b in (8, 16, 32, 64, 128, 256):
        est = nbytes / (min(b, 110) * 50e3)
        t = per_launch_us(fused_fns(sets, b), est)
        t_pair = float(np.median(event_times(fused_fns(sets, b), 30, 4, stream)))
        row = {"us": round(t, 1), "GBps": round(nbytes / t / 1e3, 1),
               "frac_hbm_peak": round(nbytes / t / 1e3 / HBM_PEAK_GBS, 4),
               "single_launch_event_pair_us": round(t_pair, 1)}
        fns = [(lambda i=i: tw.hbm_probe(srcs[i], dsts[i], pb, tw.PROBE_READ, cu_budget=b, stream=stream))
               for i in range(4)]
        tp = per_launch_us(fns, est)
        row["probe_read_GBps"] = round(pb / tp / 1e3, 1)
        # the fused kernel's own mix: P+1 streams read, 2 written, 16 MiB each, no arithmetic
        sb = pb // 12
        sb -= sb % 16384
        fns = [(lambda i=i: tw.hbm_probe_mixed(srcs[i], dsts[i], sb, 9, 2, cu_budget=b, stream=stream))
               for i in range(4)]
        tp = per_launch_us(fns, est)
        row["probe_mix_9r2w_GBps"] = round(11 * sb / tp / 1e3, 1)
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
        t = per_launch_us(fused_fns(sets[:1], b), nbytes / (min(b, 110) * 50e3))
        budgets[str(b)]["inputs_in_infinity_cache_GBps"] = round(nbytes / t / 1e3, 1)
    t = per_launch_us(fused_fns(sets, tw.CU_SHARED), 35.0)
    t_pair = float(np.median(event_times(fused_fns(sets, tw.CU_SHARED), 30, 4, stream)))
    budgets["shared"] = {"us": round(t, 1), "GBps": round(nbytes / t / 1e3, 1),
                         "frac_hbm_peak": round(nbytes / t / 1e3 / HBM_PEAK_GBS, 4),
                         "single_launch_event_pair_us": round(t_pair, 1),
                         "note": "cu_budget=TW_CU_SHARED run alone: 256-thread workgroups on every CU"}
    result["budgets"] = {"workload": WORKLOAD, "per_budget": budgets,
                         "timing": "us = median per-launch time over trains of 10 back-to-back launches on rotating "
                                   "buffer sets, one HIP event pair per train (agrees with the profiler's kernel "
                                   "trace); single_launch_event_pair_us = an event pair around every launch, which "
                                   "reads ~2 us more",
                         "note": "probe_read = one stream read; probe_mix_9r2w = 9 streams read + 2 written with "
                                 "the fused kernel's launch shape and access pattern but no arithmetic: the "
                                 "ceiling that this many compute units allow. A budget of 256 (every compute "
                                 "unit) is a whole-device launch: at this size it takes the small workgroups of "
                                 "the shared mode"}
    del srcs, dsts
    torch.cuda.empty_cache()

    # 8B-class shape (config 2) per budget
    s2 = fused_sets("c2_8b_tp2", 6)
    nb2 = algo_bytes(s2[0])
    c2 = {}
    for b in (8, 16, 32, 256):
        t = per_launch_us(fused_fns(s2, b), nb2 / (min(b, 110) * 50e3))
        c2[str(b)] = {"us": round(t, 1), "GBps": round(nb2 / t / 1e3, 1),
                      "frac_hbm_peak": round(nb2 / t / 1e3 / HBM_PEAK_GBS, 4)}
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
        t_u = per_launch_us(unf, 50.0)
        t_f = per_launch_us(fused_fns(ss, 0), 35.0)
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

    # token split (config 4): one launch vs two halves on two streams, makespan on the parent, at all
    # four token counts. "Per CU budget" is read strictly: the split run gets the same total budget
    # (b/2 per half); the run where each half gets b (2b compute units in all) is reported beside it.
    sa = overlapping_stream(tw, torch, [stream])
    sb = overlapping_stream(tw, torch, [stream, sa])
    split = {}
    cfg4 = W.CONFIGS["c4_split_sweep_tp4"]
    for N in cfg4["N"]:
        if N <= 1024:
            s4 = fused_sets("c4_split_sweep_tp4", 12 if N <= 256 else 4, N=N)
        else:
            s4 = device_drawn_sets("c4_split_sweep_tp4", 2, N)   # the host generator is slow at this size
        nb4 = algo_bytes(s4[0])
        k = tw.split_point(N, cfg4["split_multiple"])
        iters, warm = (40, 6) if N <= 4096 else (10, 3)
        for b in cfg4["cu_budgets"]:
            t1 = event_times(fused_fns(s4, b), iters, warm, stream)

            def split_fn(s, b_half, k=k):
                def f():
                    with torch.cuda.stream(stream):
                        tw.split_launch(s["partials"], s["residual"], s["weight"], s["eps"], k, sa, sb,
                                        cu_budget=b_half, out=s["out"], residual_out=s["res_out"], parent=stream,
                                        use_parent=True, join=True)
                return f
            t_eq = event_times([split_fn(s, b // 2) for s in s4], iters, warm, stream)
            t_2b = event_times([split_fn(s, b) for s in s4], iters, warm, stream)
            row = {"unsplit_us": round(float(np.median(t1)), 1),
                   "split_same_total_budget_us": round(float(np.median(t_eq)), 1),
                   "split_each_half_full_budget_us": round(float(np.median(t_2b)), 1)}
            if N > 256:     # N = 256 is a latency case: 29 MB, launch- and ramp-bound
                row.update({"unsplit_GBps": round(nb4 / np.median(t1) / 1e3, 1),
                            "split_same_total_budget_GBps": round(nb4 / np.median(t_eq) / 1e3, 1),
                            "split_each_half_full_budget_GBps": round(nb4 / np.median(t_2b) / 1e3, 1)})
            split["N%d_b%d" % (N, b)] = row
        del s4
        torch.cuda.empty_cache()
    result["split"] = {"workload": "c4_split_sweep_tp4 (H=8192, P=4, k=N/2)", "per_case": split,
                       "note": "b = CU budget of the unsplit launch. split_same_total_budget: each half is confined to "
                               "b/2 compute units, so both runs occupy b; split_each_half_full_budget: each half "
                               "gets b (2b occupied). Makespan on the parent stream, fork and join included. N >= "
                               "4096: inputs drawn on the GPU with the config's distributions; N = 256 reported "
                               "as latency only"}

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
    # every pair of streams whose kernels are meant to overlap is checked to sit on different hardware queues
    comm = overlapping_stream(tw, torch, [stream])
    comp = overlapping_stream(tw, torch, [stream, comm])
    cus_total = tw.device_cu_count()
    tf = event_times(fused_fns(s5, 32), 30, 5, stream)
    tg = event_times([lambda: tw.gemm_bf16(A, B, C=C, cu_budget=0, stream=stream)], 30, 5, stream)

    def serial_fn(s):
        def f():
            tw.reduce_add_rmsnorm(s["partials"], s["residual"], s["weight"], s["eps"], cu_budget=32,
                                  out=s["out"], residual_out=s["res_out"], stream=stream)
            tw.gemm_bf16(A, B, C=C, cu_budget=0, stream=stream)
        return f

    def overlap_fn(s, fused_budget, gemm_budget, s_comm=None, s_compute=None):
        # the caller's stream is the compute stream (as in the paper: a compute stream and a
        # communication stream), so only the comm stream is forked from and joined into it
        def f():
            with torch.cuda.stream(stream):
                tw.overlap_launch(dict(partials=s["partials"], residual=s["residual"], weight=s["weight"],
                                       eps=s["eps"], cu_budget=fused_budget, out=s["out"],
                                       residual_out=s["res_out"]),
                                  dict(A=A, B=B, C=C, cu_budget=gemm_budget), s_comm or comm, s_compute or stream,
                                  parent=stream, use_parent=True, join=True)
        return f
    # the same partition enforced by the dispatcher: two streams with disjoint compute-unit masks
    # (an aid from tw_measure.h: if the runtime refuses such a stream the figure is left out)
    try:
        few, rest = tw.CuMaskedStream(0, 32), tw.CuMaskedStream(32, cus_total - 32)
    except tw.TwError:
        few = rest = None
    # the best schedule without overlap on one GPU: no partition, each kernel gets every CU in turn
    def serial_whole_fn(s):
        def f():
            tw.reduce_add_rmsnorm(s["partials"], s["residual"], s["weight"], s["eps"], cu_budget=0,
                                  out=s["out"], residual_out=s["res_out"], stream=stream)
            tw.gemm_bf16(A, B, C=C, cu_budget=0, stream=stream)
        return f
    # the schedules take turns, in rotating order
    schedules = {
        "serial32": [serial_fn(s) for s in s5], "serial_whole": [serial_whole_fn(s) for s in s5],
        "budget32": [overlap_fn(s, 32, cus_total - 32) for s in s5],
        "shared": [overlap_fn(s, tw.CU_SHARED, 0) for s in s5]}
    if few is not None:
        schedules["masked32"] = [overlap_fn(s, 32, cus_total - 32, few.stream, rest.stream) for s in s5]
    ov = interleaved_medians(schedules, rounds=8, iters=10, warm=2)
    torch.cuda.synchronize()
    if few is not None:
        few.close()
        rest.close()

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
    best_serial = min(ov["serial32"], ov["serial_whole"])
    best_overlap = min(ov["budget32"], ov["shared"])
    result["overlap"] = {
        "workload": "c5_overlap_tp8: fused N=2048,H=8192,P=8 @32 CUs || GEMM [2048x8192]x[8192x3584] bf16",
        "gain_best_overlapped_vs_best_serial": round(best_serial / best_overlap, 3),
        "best_serial_schedule": "serial_whole_device" if ov["serial_whole"] <= ov["serial32"] else "serial_budget32",
        "best_overlapped_schedule": "overlapped_shared" if ov["shared"] <= ov["budget32"] else "overlapped_budget32",
        "budgeted_overlap_beats_best_serial": bool(ov["budget32"] < best_serial),
        "fused_alone_us": round(float(np.median(tf)), 1), "gemm_alone_us": round(float(np.median(tg)), 1),
        "gemm_alone_TFLOPs": round(flops / np.median(tg) / 1e6, 1),
        "gemm_frac_mfma_peak": round(flops / np.median(tg) / 1e6 / MFMA_BF16_PEAK_TFLOPS, 4),
        "serial_budget32_us": ov["serial32"],
        "serial_whole_device_us": ov["serial_whole"],
        "overlapped_budget32_us": ov["budget32"],
        "overlapped_shared_us": ov["shared"],
        "overlapped_cu_masked32_us": ov.get("masked32"),
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
                "cu_budget=TW_CU_SHARED: small fused workgroups co-resident with the GEMM's on every CU; overlapped_cu_masked32 = the budgeted "
                "launches on two streams whose compute-unit masks (tw_stream_create_cu_masked) are 32 and 224 disjoint "
                "compute units, both forked from and joined into the caller's stream. The "
                "caller's stream is the compute stream; the schedules take turns in bursts, in rotating order; makespans include fork and join",
    }
    del s5
    torch.cuda.empty_cache()

    # the GEMM stand-in on its own: the demo's product, the attention-side projection of a 4096-token batch
    # (short K) and a large square product, against the dense bf16 MFMA peak
    gem = {}
    for (M_, N_, K_) in ((gc["M"], gc["N"], gc["K"]), (4096, 8192, 1024), (8192, 8192, 8192)):
        gen = torch.Generator(device="cuda:0")
        gen.manual_seed(M_ + K_)
        A_ = torch.empty((M_, K_), dtype=torch.bfloat16, device="cuda:0").normal_(0.0, gc["std"], generator=gen)
        B_ = torch.empty((N_, K_), dtype=torch.bfloat16, device="cuda:0").normal_(0.0, gc["std"], generator=gen)
        C_ = torch.empty((M_, N_), dtype=torch.bfloat16, device="cuda:0")
        torch.cuda.synchronize()
        fl = 2.0 * M_ * N_ * K_
        def vendor():
            with torch.cuda.stream(stream):
                torch.matmul(A_, B_.t(), out=C_)
        # the library's kernel and the vendor library's (through torch.matmul) take turns, twice
        ts, tv = [], []
        for _ in range(2):
            ts.append(train_times([lambda: tw.gemm_bf16(A_, B_, C=C_, cu_budget=0, stream=stream)], 4, 4, 3, stream))
            tv.append(train_times([vendor], 4, 4, 3, stream))
        t, v = float(np.median(np.concatenate(ts))), float(np.median(np.concatenate(tv)))
        gem["%dx%dx%d" % (M_, N_, K_)] = {"us": round(t, 1), "TFLOPs": round(fl / t / 1e6, 1),
                                          "frac_mfma_peak": round(fl / t / 1e6 / MFMA_BF16_PEAK_TFLOPS, 4),
                                          "vendor_library_us": round(v, 1),
                                          "speed_over_vendor_library": round(v / t, 3)}
        del A_, B_, C_
    result["gemm"] = {"per_shape_MxNxK": gem,
                      "note": "tw_gemm_bf16 alone on the whole device, A and B ~ N(0, 0.02^2) drawn on the GPU, trains of "
                              "4 launches; peak = 2500 TFLOP/s dense bf16. The part runs these at its power limit "
                              "(1.2-1.9 GHz against 2.4 GHz idle): a loop of nothing but MFMAs on such operands "
                              "sustains 1990 TFLOP/s. vendor_library_us: torch.matmul (hipBLASLt) on the same tensors, for "
                              "context"}
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
    # the paper's ablation at the level of a layer boundary (Section 5, "fuse only" against the baseline):
    # the same unsplit chain with the pipeline the fused kernel replaces in its place (all-reduce to bf16,
    # then residual add + RMSNorm re-reading it)
    sum_scratch = torch.empty_like(resid)

    def unfused_chain():
        with torch.cuda.stream(stream):
            tw.gemm_bf16(X1, W1, C=parts[0], stream=stream)
            tw.reduce_add_rmsnorm_unfused(parts, resid, weight, d["eps"], out=out, residual_out=res_out,
                                          sum_scratch=sum_scratch, stream=stream)
            tw.gemm_bf16(out, W2, C=Y, stream=stream)
    # the schedules take turns in bursts of 8 calls, in rotating order
    cands = {"unsplit": layer_fn(0, 0, 0), "unsplit_unfused": unfused_chain}
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
    weave = {"unsplit_whole_device_us": med["unsplit"],
             "unsplit_with_the_unfused_pipeline_us": med["unsplit_unfused"],
             "fusion_gain_on_the_layer": round(med["unsplit_unfused"] / med["unsplit"], 3)}
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
                "each kernel on all CUs in turn, one stream, no events; unsplit_with_the_unfused_pipeline = that chain "
                "with tw_reduce_add_rmsnorm_unfused in the fused step's place (what fusing alone saves on the layer); "
                "the schedules take turns in bursts",
    }
    del X1, W1, W2, parts, resid, out, res_out, Y, sum_scratch
    torch.cuda.empty_cache()
    budget_grid(result, tw, W, torch, np, stream, train_times, device_drawn_sets)
    policy_table(result, tw, W, torch, np, stream, comm, interleaved_medians, gpu)
    weave_trains(result, tw, W, torch, np, stream, comm, interleaved_medians)
    decode_trains(result, tw, W, torch, np, stream, gpu)
    result["streams"] = {"second_streams_checked_with": "tw_streams_overlap", "torch_streams_tried": _streams_tried[0],
                         "note": "two streams on one hardware queue never overlap; every second stream used for a "
                                 "split or overlapped schedule here was checked to run side by side with the first"}


def budget_grid(result, tw, W, torch, np, stream, train_times, device_drawn_sets):
    """The analogue of the paper's Fig. 9 / Fig. 22 (latency against the number of SMs, per sequence
    length): the fused kernel's rate per CU budget, per token count, with the smallest budget that reaches
    the plateau and the smallest that reaches 70 % of the HBM peak."""
    H, P = 8192, 8
    grid = {}
    budgets = (8, 16, 32, 64, 128, 256)
    for N in (256, 1024, 4096, 16384):
        per_set = (P + 3) * 2 * H * N
        nsets = max(2, min(12, (600 << 20) // per_set + 1))
        ss = device_drawn_sets("c3_70b_shard_tp8", nsets, N)
        row = {}
        for b in budgets + (tw.CU_SHARED,):
            est_us = per_set / (min(b if b > 0 else 256, 110) * 50e3)      # ~50 GB/s per CU, ~5.5 TB/s at most
            length = int(max(2, min(10, 4000.0 / est_us)))
            trains = int(max(3, min(10, 20e3 / (est_us * length))))
            fns = [tw.prepare_reduce_add_rmsnorm(x["partials"], x["residual"], x["weight"], x["eps"], cu_budget=b,
                                                 out=x["out"], residual_out=x["res_out"], stream=stream)[0]
                   for x in ss]
            t = float(np.median(train_times(fns, trains, length, 3, stream)))
            row["shared" if b == tw.CU_SHARED else str(b)] = {"us": round(t, 1), "GBps": round(per_set / t / 1e3, 1)}
        best = max(v["GBps"] for k_, v in row.items() if k_ != "shared")
        plateau = next(b for b in budgets if row[str(b)]["GBps"] >= 0.95 * best)
        seventy = next((b for b in budgets if row[str(b)]["GBps"] >= 0.70 * HBM_PEAK_GBS), None)
        grid["N%d" % N] = {"per_budget": row, "best_GBps": best, "min_budget_for_plateau": plateau,
                           "min_budget_for_70pct": seventy,
                           "shared_reaches_70pct": bool(row["shared"]["GBps"] >= 0.70 * HBM_PEAK_GBS)}
        del ss
        torch.cuda.empty_cache()
    result["budget_grid"] = {
        "workload": "H=8192, P=8, value distributions of c3 without the outliers, drawn on the GPU; rotating "
                    "buffer sets of > 600 MB in all; per-launch time from trains of back-to-back launches",
        "per_token_count": grid,
        "note": "plateau = smallest budget within 5 % of the best budget's rate; min_budget_for_70pct = smallest "
                "budget at or above 5600 GB/s (null: none reaches it). In the paper 8 SMs are close to optimal at "
                "every length because its kernel is bound by the interconnect; here the kernel is bound by what "
                "a compute unit can request from HBM, so the plateau needs (nearly) every compute unit"}


def policy_table(result, tw, W, torch, np, stream, comm, interleaved_medians, gpu):
    """Fig. 3 / Appendix A 'Selective Enabling': per token count, the layer boundary run never split,
    always split, and under the library's policy (tw_weave_layer_auto with its built-in threshold)."""
    H, P = 8192, 8
    cus = tw.device_cu_count()
    weight = gpu(W.uniform_bf16((H,), 0.5, 1.5, 0, W.STREAM_WEIGHT))
    out_ = {}
    for name, K1, N2 in (("attention_side", 1024, 3584), ("mlp_side", 3584, 1280)):
        gen = torch.Generator(device="cuda:0")
        gen.manual_seed(K1 + N2)

        def rnd(shape, std):
            return torch.empty(shape, dtype=torch.bfloat16, device="cuda:0").normal_(0.0, std, generator=gen)
        W1, W2 = rnd((H, K1), 0.02), rnd((N2, H), 0.02)
        thr = tw.split_threshold(K1, H, P, N2, cus)
        rows = []
        for T in (256, 1024, 2048, 4096, 5120, 6144, 7168, 8192, 12288, 16384, 32768):
            X1, resid = rnd((T, K1), 0.02), rnd((T, H), 1.0)
            parts = [rnd((T, H), 0.25) for _ in range(P)]
            o, r = torch.empty_like(resid), torch.empty_like(resid)
            Y = torch.empty((T, N2), dtype=torch.bfloat16, device="cuda:0")
            torch.cuda.synchronize()
            kw = dict(fused_cu_budget=tw.CU_SHARED, gemm_cu_budget=0, out=o, residual_out=r, Y=Y, parent=stream,
                      use_parent=True, join=True)
            k_smart = tw.smart_split_point(T, 64, [H, N2], cus, gemm_k=[K1, H])[0]
            # the offline search of Algorithm 1, timed: unsplit, the smart row, and two offsets past the middle
            k_tuned, tune_us = tw.weave_tune(X1, W1, parts, resid, weight, 1e-5, W2, stream, comm, offsets=(0, 256),
                                             reps=5, out=o, residual_out=r, Y=Y)
            taken = []

            def never():
                with torch.cuda.stream(stream):
                    tw.weave_layer(X1, W1, parts, resid, weight, 1e-5, W2, 0, stream, comm, **kw)
            sum_scratch = torch.empty_like(resid)

            def never_unfused():      # the baseline of the paper's ablation: no split, no fused kernel
                with torch.cuda.stream(stream):
                    tw.gemm_bf16(X1, W1, C=parts[0], stream=stream)
                    tw.reduce_add_rmsnorm_unfused(parts, resid, weight, 1e-5, out=o, residual_out=r,
                                                  sum_scratch=sum_scratch, stream=stream)
                    tw.gemm_bf16(o, W2, C=Y, stream=stream)

            def always():
                with torch.cuda.stream(stream):
                    tw.weave_layer(X1, W1, parts, resid, weight, 1e-5, W2, k_smart, stream, comm, **kw)

            def policy():
                with torch.cuda.stream(stream):
                    taken.append(tw.weave_layer_auto(X1, W1, parts, resid, weight, 1e-5, W2, stream, comm, **kw)[3])

            def tuned():
                with torch.cuda.stream(stream):
                    tw.weave_layer(X1, W1, parts, resid, weight, 1e-5, W2, 0 if k_tuned == T else k_tuned, stream, comm,
                                   **kw)
            iters = 8 if T <= 8192 else 5
            med = interleaved_medians({"never": never, "always": always, "policy": policy, "tuned": tuned,
                                       "never_unfused": never_unfused}, rounds=4, iters=iters, warm=2)
            best = min(med["never"], med["always"])
            rows.append({"T": T, "never_split_us": med["never"], "always_split_us": med["always"],
                         "policy_us": med["policy"], "tuned_us": med["tuned"],
                         "never_split_unfused_pipeline_us": med["never_unfused"],
                         "policy_over_unfused_baseline": round(med["never_unfused"] / med["policy"], 3),
                         "policy_split_row": taken[-1],
                         "tuned_split_row": k_tuned, "always_split_row": k_smart,
                         "policy_over_best": round(med["policy"] / best, 3),
                         "tuned_over_best": round(med["tuned"] / best, 3)})
            del X1, resid, parts, o, r, Y, sum_scratch
            torch.cuda.empty_cache()
        out_[name] = {"boundary": "[Tx%d]x[%dx8192] -> fused H=8192 P=8 (shared mode) -> [Tx8192]x[8192x%d]"
                                  % (K1, K1, N2),
                      "built_in_threshold_tokens": thr if thr < 2 ** 62 else "never",
                      "rows": rows,
                      "worst_policy_over_best": max(r_["policy_over_best"] for r_ in rows),
                      "worst_tuned_over_best": max(r_["tuned_over_best"] for r_ in rows)}
    result["policy"] = {
        "per_boundary": out_,
        "note": "never = the chain G1, F, G2 unsplit on one stream; always = tw_weave_layer at the row "
                "tw_smart_split_point picks, whatever T; policy = tw_weave_layer_auto with the built-in rule "
                "(tw_policy_split_row: split from tw_split_threshold's tokens up, and above half of that when the cut "
                "costs no GEMM waves); tuned = tw_weave_layer at the row tw_weave_tune reported for "
                "this batch size beforehand (its timed search over: unsplit, the smart row, the middle, the middle "
                "+ 256). A split row equal to T means no split. never_split_unfused_pipeline = the unsplit chain with "
                "tw_reduce_add_rmsnorm_unfused in the fused step's place: the baseline of the paper's ablation (no "
                "fused kernel, no overlap); policy_over_unfused_baseline = what fusion and the policy gain together. "
                "Candidates take turns in bursts, in rotating order; medians of HIP-event timed calls"}


def weave_trains(result, tw, W, torch, np, stream, comm, interleaved_medians):
    """Consecutive layer boundaries as an engine would run them (Fig. 7b continues from layer to layer):
    eight boundaries of a 70B-class TP=8 model (attention side, MLP side, alternating) back to back, unsplit
    on one stream, woven with a fork and a join around every boundary, and woven with the two splits'
    chains running on through the boundaries (tw_weave_train: one fork before the first, one join after the
    last)."""
    H, P, L = 8192, 8, 8
    cus = tw.device_cu_count()
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(11)

    def rnd(shape, std):
        return torch.empty(shape, dtype=torch.bfloat16, device="cuda:0").normal_(0.0, std, generator=gen)
    shapes = [(1024, 3584), (3584, 1280)]
    Ws = [(rnd((H, K1), 0.02), rnd((N2, H), 0.02)) for (K1, N2) in shapes]
    weight = torch.ones(H, dtype=torch.bfloat16, device="cuda:0")
    rows_out = []
    for T in (2048, 3072, 4096, 5120, 7168, 8192, 12288, 16384, 32768):
        bufs = [dict(X1=rnd((T, K1), 0.02), resid=rnd((T, H), 1.0), parts=[rnd((T, H), 0.25) for _ in range(P)],
                     o=torch.empty((T, H), dtype=torch.bfloat16, device="cuda:0"),
                     r=torch.empty((T, H), dtype=torch.bfloat16, device="cuda:0"),
                     Y=torch.empty((T, N2), dtype=torch.bfloat16, device="cuda:0")) for (K1, N2) in shapes]
        torch.cuda.synchronize()
        cut = [tw.smart_split_point(T, 64, [H, N2], cus, gemm_k=[K1, H])[0] for (K1, N2) in shapes]

        def call(i, k, use_parent, join):
            b, (W1, W2) = bufs[i % 2], Ws[i % 2]
            tw.weave_layer(b["X1"], W1, b["parts"], b["resid"], weight, 1e-5, W2, k, stream, comm,
                           fused_cu_budget=tw.CU_SHARED, gemm_cu_budget=0, out=b["o"], residual_out=b["r"], Y=b["Y"],
                           parent=stream, use_parent=use_parent, join=join)

        def unsplit():
            with torch.cuda.stream(stream):
                for i in range(L):
                    call(i, 0, False, False)

        def woven_each():
            with torch.cuda.stream(stream):
                for i in range(L):
                    call(i, cut[i % 2], True, True)
        scratch = torch.empty((T, H), dtype=torch.bfloat16, device="cuda:0")

        def unsplit_unfused():      # neither of the paper's two techniques: the baseline of its ablation
            with torch.cuda.stream(stream):
                for i in range(L):
                    b, (W1, W2) = bufs[i % 2], Ws[i % 2]
                    tw.gemm_bf16(b["X1"], W1, C=b["parts"][0], stream=stream)
                    tw.reduce_add_rmsnorm_unfused(b["parts"], b["resid"], weight, 1e-5, out=b["o"], residual_out=b["r"],
                                                  sum_scratch=scratch, stream=stream)
                    tw.gemm_bf16(b["o"], W2, C=b["Y"], stream=stream)

        train = [dict(X1=bufs[i % 2]["X1"], W1=Ws[i % 2][0], partials=bufs[i % 2]["parts"], residual=bufs[i % 2]["resid"],
                      weight=weight, eps=1e-5, W2=Ws[i % 2][1], out=bufs[i % 2]["o"], residual_out=bufs[i % 2]["r"],
                      Y=bufs[i % 2]["Y"]) for i in range(L)]

        def woven_through():
            with torch.cuda.stream(stream):
                tw.weave_train(train, cut[0], stream, comm, parent=stream, use_parent=True, join=True)
        med = interleaved_medians({"unsplit": unsplit, "woven_each": woven_each, "woven_through": woven_through,
                                   "unsplit_unfused": unsplit_unfused}, rounds=4, iters=4 if T <= 16384 else 2, warm=1)
        rows_out.append({"T": T, "unsplit_unfused_pipeline_us_per_boundary": round(med["unsplit_unfused"] / L, 1),
                         "woven_through_gain_over_unfused_unsplit": round(med["unsplit_unfused"] / med["woven_through"], 3),
                         "unsplit_us_per_boundary": round(med["unsplit"] / L, 1),
                         "woven_fork_join_each_us_per_boundary": round(med["woven_each"] / L, 1),
                         "woven_through_us_per_boundary": round(med["woven_through"] / L, 1),
                         "through_over_unsplit": round(med["woven_through"] / med["unsplit"], 3)})
        del bufs, scratch, train
        torch.cuda.empty_cache()
    result["weave_trains"] = {
        "workload": "8 consecutive layer boundaries (attention side K1=1024, N2=3584 and MLP side K1=3584, N2=1280 "
                    "alternating; H=8192, P=8, shared mode), per boundary",
        "rows": rows_out,
        "note": "unsplit: every boundary on one stream; woven_fork_join_each: tw_weave_layer with a parent stream and "
                "join around every boundary (what the per-boundary tables time); woven_through: tw_weave_train, one fork "
                "before the first boundary and one join after the last, each split's chain running on through the "
                "boundaries on its own stream; unsplit_unfused_pipeline: the unsplit train with "
                "tw_reduce_add_rmsnorm_unfused in the fused step's place (no fused kernel, no overlap), and "
                "woven_through_gain_over_unfused_unsplit what the two techniques gain together"}


def decode_trains(result, tw, W, torch, np, stream, gpu):
    """Appendix B's decode case: an iteration is a train of many small fused steps (two per layer, 80
    layers). 160 back-to-back calls, eager against one HIP graph captured once and replayed."""
    H, P, calls = 8192, 8, 160
    rows = {}
    for N in (1, 16, 32, 64, 256):
        d = W.make_fused_inputs("c3_70b_shard_tp8", N=N)
        parts = [gpu(p) for p in d["partials"]]
        resid, weight = gpu(d["residual"]), gpu(d["weight"])
        o, r = torch.empty_like(resid), torch.empty_like(resid)
        # a decode step has nothing to run beside: a whole-device launch (which takes the small
        # workgroups at these sizes, and up to a few dozen rows their all-at-once form)
        launch = tw.prepare_reduce_add_rmsnorm(parts, resid, weight, d["eps"], cu_budget=0, out=o,
                                               residual_out=r, stream=stream)[0]

        def train():
            for _ in range(calls):
                launch()
        train()
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            train()

        def replay():
            with torch.cuda.stream(stream):
                graph.replay()
        res = {}
        for label, fn in (("eager", train), ("graph", replay)):
            wall, host, dev_us = [], [], []
            for rep in range(12):
                stream.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                t0 = time.perf_counter()
                e0.record(stream)
                fn()
                e1.record(stream)
                t1 = time.perf_counter()
                stream.synchronize()
                t2 = time.perf_counter()
                if rep >= 2:
                    host.append((t1 - t0) * 1e6 / calls)
                    wall.append((t2 - t0) * 1e6 / calls)
                    dev_us.append(e0.elapsed_time(e1) * 1e3 / calls)
            res[label] = {"wall_us_per_launch": round(float(np.median(wall)), 2),
                          "device_us_per_launch": round(float(np.median(dev_us)), 2),
                          "host_us_per_call": round(float(np.median(host)), 2)}
        res["graph_speedup_wall"] = round(res["eager"]["wall_us_per_launch"] / res["graph"]["wall_us_per_launch"], 3)
        rows["N%d" % N] = res
        del graph
    result["decode_trains"] = {
        "workload": "160 back-to-back tw_reduce_add_rmsnorm calls (H=8192, P=8, whole-device launches, same buffers: inputs "
                    "stay in cache as in a decode step), per call",
        "per_token_count": rows,
        "note": "eager: 160 calls through the C ABI (arguments marshalled once), then one synchronisation; graph: "
                "the same 160 launches captured once with hipStreamBeginCapture and replayed. wall = submit + "
                "drain per launch; host = time for the calls (or the replay call) to return, per launch; device = "
                "HIP events around the train"}


def gemm_phases(tw, torch, np, stream, train_times):
    """Per-wave shader clocks of the phases of the 256x256 tile's pipeline (tw_gemm_bf16_traced), next to
    the plain kernel's time for the same product, for a long-K, a square and a short-K product."""
    rows = []
    names = tw.GEMM_PHASE_NAMES
    for (M, N, K) in ((8192, 8192, 8192), (4096, 4096, 4096), (16384, 8192, 1024)):
        gen = torch.Generator(device="cuda:0")
        gen.manual_seed(M + K)
        A = torch.empty((M, K), dtype=torch.bfloat16, device="cuda:0").normal_(0.0, 0.02, generator=gen)
        B = torch.empty((N, K), dtype=torch.bfloat16, device="cuda:0").normal_(0.0, 0.02, generator=gen)
        C = torch.empty((M, N), dtype=torch.bfloat16, device="cuda:0")
        torch.cuda.synchronize()
        plain_us = train_times([lambda: tw.gemm_bf16(A, B, C=C, b_layout=tw.B_NK, stream=stream)], trains=6, length=4,
                               warm=3, on_stream=stream)
        for _ in range(3):
            _, cyc = tw.gemm_bf16_traced(A, B, C=C, stream=stream)
        stream.synchronize()
        traced_us = train_times([lambda: tw.gemm_bf16_traced(A, B, C=C, stream=stream)], trains=4, length=2, warm=1,
                                on_stream=stream)
        c = cyc.cpu().numpy().astype(np.float64)
        ran = c[:, names.index("tiles")] > 0
        c = c[ran]
        tiles = c[:, names.index("tiles")]
        steps = tiles * (K // 64)
        per_step = {n: round(float((c[:, names.index(n)] / steps).mean()), 1)
                    for n in ("sub_step_0", "wait_landed", "barrier", "sub_step_1")}
        per_tile = {n: round(float((c[:, names.index(n)] / tiles).mean()), 0) for n in ("tile_fill", "tile_stores")}
        k_step = sum(per_step.values())
        rows.append({"MxNxK": "%dx%dx%d" % (M, N, K), "plain_us": round(float(np.median(plain_us)), 1),
                     "traced_us": round(float(np.median(traced_us)), 1), "waves": int(ran.sum()),
                     "tiles_per_wave": float(tiles.mean()), "K_steps_per_tile": K // 64,
                     "clocks_per_K_step": per_step, "clocks_per_K_step_total": round(k_step, 1),
                     "matrix_work_clocks_per_K_step": 2048, "clocks_per_tile": per_tile,
                     "kernel_clocks_per_wave": round(float(c[:, names.index("kernel")].mean()), 0),
                     "share_of_kernel": {
                         "matrix_work": round(float((2048 * steps / c[:, names.index("kernel")]).mean()), 3),
                         "K_loop": round(float((k_step * steps / c[:, names.index("kernel")]).mean()), 3),
                         "tile_fill": round(float((c[:, names.index("tile_fill")] / c[:, names.index("kernel")]).mean()), 3),
                         "tile_stores": round(float((c[:, names.index("tile_stores")] / c[:, names.index("kernel")]).mean()), 3)}})
        del A, B, C
        torch.cuda.empty_cache()
    print(json.dumps({"gemm_phases": rows,
                      "note": "tw_gemm_bf16_traced: shader clocks per wave, means over the waves that ran; a K step of "
                              "64 is 128 MFMAs 16x16x32 per wave = 2048 clocks of matrix work on its SIMD; the traced "
                              "kernel reads the clock around its waits and is a few percent slower than the plain one"}))


def ceiling_sweep(tw, torch, np, stream, train_times):
    """What one compute unit can pull from / push to HBM, and what it does not depend on: budgets x
    workgroup sizes x accesses in flight for a read-only and a copy stream, budgets x workgroup sizes for
    the fused kernel's own mix (9 streams read, 2 written). One workgroup per compute unit throughout."""
    pb = 192 << 20
    srcs = [torch.empty(pb, dtype=torch.uint8, device="cuda:0").random_() for _ in range(4)]
    dsts = [torch.empty(pb, dtype=torch.uint8, device="cuda:0") for _ in range(4)]
    torch.cuda.synchronize()
    budgets = (1, 2, 4, 8, 16, 32)
    table = []
    for mode, mname in ((tw.PROBE_READ, "read"), (tw.PROBE_COPY, "copy")):
        for threads in (256, 512, 1024):
            for depth in (1, 2, 4, 8, 16):
                row = {"stream": mname, "threads_per_workgroup": threads, "accesses_in_flight_per_thread": depth,
                       "KiB_in_flight_per_cu": threads * depth * 16 // 1024}
                for b in budgets:
                    # small budgets move less so that a cell stays in the tens of milliseconds
                    nbytes = min(pb, (b * 24) << 20)
                    fns = [(lambda i=i: tw.hbm_probe_shaped(srcs[i], dsts[i], nbytes, mode, cu_budget=b,
                                                            threads=threads, in_flight=depth, stream=stream))
                           for i in range(4)]
                    t = float(np.median(train_times(fns, 3, 4, 2, stream)))
                    moved = nbytes * (2 if mode == tw.PROBE_COPY else 1)
                    row["GBps_per_cu_b%d" % b] = round(moved / t / 1e3 / b, 1)
                table.append(row)
    sb = pb // 12
    sb -= sb % 16384
    for threads in (256, 512, 1024):
        row = {"stream": "9 read + 2 written", "threads_per_workgroup": threads,
               "accesses_in_flight_per_thread": 9, "KiB_in_flight_per_cu": threads * 9 * 16 // 1024}
        for b in budgets:
            per = min(sb, ((b * 2) << 20) // 16384 * 16384)
            fns = [(lambda i=i: tw.hbm_probe_mixed_shaped(srcs[i], dsts[i], per, 9, 2, cu_budget=b, threads=threads,
                                                          stream=stream)) for i in range(4)]
            t = float(np.median(train_times(fns, 3, 4, 2, stream)))
            row["GBps_per_cu_b%d" % b] = round(11 * per / t / 1e3 / b, 1)
        table.append(row)
    best = {}
    for b in budgets:
        for sname in ("read", "copy", "9 read + 2 written"):
            best["%s_b%d" % (sname.split()[0] if sname != "9 read + 2 written" else "mix", b)] = max(
                r["GBps_per_cu_b%d" % b] for r in table if r["stream"] == sname)
    print(json.dumps({"ceiling": table, "best_GBps_per_cu": best,
                      "needed_for_70pct_of_hbm_peak_in_32_cus_GBps_per_cu": round(0.7 * HBM_PEAK_GBS / 32, 1),
                      "note": "GB/s per compute unit (copy and mix: bytes read + bytes written); one workgroup per "
                              "compute unit (each requests 96 KiB of LDS); buffers of 192 MiB rotated four ways, so "
                              "nothing is served from the 256 MB Infinity Cache; per-launch time from trains of 4 "
                              "back-to-back launches, median of 3"}))


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
