#!/usr/bin/env python3
"""Benchmark of the densify hot path on one MI355X.

A step is one whole ts_densify call (sort, row reduce with the dense add fused,
combine of cut rows) on the transformer-big worker share: V=32768, d=1024, fp32,
encoder + decoder contributions of 8192 rows each laid end to end (n=16384), ids
Zipf(1.1).  Inputs are resident in HBM before the timed region; the calls rotate
over several independent buffer sets so that no call finds its lines in the
memory-side cache.

Prints ONE JSON line: whole-call throughput in algorithmic GB/s (`value`), the
roofline of the dominant kernel measured with HIP events inside the same timed
region, and the CPU checker timed on the host as a baseline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0

# HBM bytes per reduce_kernel launch with default tuning, per workload, from the two
# rocprofv3 --pmc runs summarised in profiles/ (FETCH_SIZE x 1.985 + WRITE_SIZE x 0.995, the
# factors a plain copy of known size gives: profiles/counter_calibration.md).  Only valid for
# the kernel source it was taken with: when the source's hash differs, `traffic` is reported
# as null.
COUNTED_TRAFFIC = {
    "source_sha256": "d8a97e2228c41f6397e8d07345f6ef92847fa4099b2c55f05a629d0f02c6d588",
    "reduce_kernel_bytes_per_launch": {
        "transformer_big": 294.79e6,
        "transformer_base": 113.20e6,
        "large_batch_bf16": 568.29e6,
        "multi_shard_stress": 1387.21e6,
    },
}


def algorithmic_bytes(n, d, V, elem, out_elem=4):
    """Read dense_in, write dense_out, read every id and value row once."""
    return (4 + out_elem) * V * d + n * (4 + elem * d)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", default="transformer_big",
                    choices=["transformer_base", "transformer_big", "large_batch_bf16", "multi_shard_stress"])
    ap.add_argument("--tokens", type=int, default=0,
                    help="instead of a named workload: one worker's share at a per-worker batch of this many "
                         "tokens (the paper's scaling runs use 2,048 to 25,600, Section 5): V=32768, d=1024, "
                         "fp32, an encoder and a decoder contribution of that many pairs each, Zipf 1.1")
    ap.add_argument("--sets", type=int, default=0,
                    help="independent buffer sets to rotate over (0 = at least 3, and as many as it takes to "
                         "pass 1 GB in all, so that no call finds its data in the 256 MB memory-side cache)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--overlap-mib", type=float, default=-1.0,
                    help="dense bytes copied beside each sort launch (tuning; -1 = library default)")
    ap.add_argument("--piece-tokens", type=int, default=0, help="tuning; 0 = library default")
    ap.add_argument("--sort-part", type=int, default=0, help="tuning; 0 = library default")
    ap.add_argument("--short-rows", type=int, default=-1, help="tuning; -1 = library default, 0 = in the pieces, 1 = row by row")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run the same launches with n = 0: a plain [V, d] copy of known size, used to "
                         "scale hardware byte counters")
    ap.add_argument("--compare-rules", action="store_true",
                    help="time ts_accumulate under Algorithm 1 (gather) and Algorithm 2 (convert and reduce) "
                         "on the workload's three gradients and print both buffers' sizes (Fig. 5 of the "
                         "paper, for one worker)")
    ap.add_argument("--out", default="fp32", choices=["fp32", "bf16"],
                    help="with --scale: time ts_densify_scaled (write-back epilogue) instead; bf16 halves "
                         "the bytes written")
    ap.add_argument("--scale", type=float, default=None, help="epilogue factor, e.g. 0.0625 for an average of 16")
    ap.add_argument("--no-events", action="store_true",
                    help="do not record per-kernel HIP events inside the timed region")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_1905_04035_amd import binding as ts
    from paper_1905_04035_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    ts.lib()      # fail loudly if the HIP library has not been built
    if args.overlap_mib >= 0:
        ts.ts_set_overlap_bytes(int(args.overlap_mib * (1 << 20)))
    if args.piece_tokens:
        ts.ts_set_piece_tokens(args.piece_tokens)
    if args.sort_part:
        ts.ts_set_sort_part(args.sort_part)
    if args.short_rows >= 0:
        ts.ts_set_short_rows(args.short_rows)

    if args.tokens > 0:
        args.workload = f"per_worker_batch_{args.tokens}_tokens"
        w = wl.make_custom(V=32768, d=1024, n_list=[args.tokens, args.tokens], zipf_s=1.1,
                           seed=190504035 + args.tokens, sigma_rows=0.01, sigma_dense=1.0)
    else:
        w = wl.make(args.workload)
    V, d, n = w.V, w.d, w.n_total
    elem = 2 if w.row_dtype == wl.ROW_BF16 else 4
    multi = args.workload == "multi_shard_stress"
    epilogue = args.scale is not None or args.out == "bf16"
    scale = 1.0 if args.scale is None else args.scale
    out_elem = 2 if args.out == "bf16" else 4
    ids_h, rows_h = w.concatenated()

    def dev_rows(a):
        return torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).to(dev)

    if args.sets <= 0:
        per_set = 4 * V * d + out_elem * V * d + n * (4 + elem * d)
        args.sets = max(3, -(-10 ** 9 // per_set))
    sets = []
    for _ in range(args.sets):
        s = dict(dense_in=torch.from_numpy(w.dense_in).to(dev),
                 dense_out=torch.empty((V, d), dtype=torch.int16 if out_elem == 2 else torch.float32, device=dev))
        if multi or epilogue:
            ik, rk = w.grouped(2)
            s["ids"] = [torch.from_numpy(i).to(dev) for i in ik]
            s["rows"] = [dev_rows(r) for r in rk]
        else:
            s["ids"] = torch.from_numpy(ids_h).to(dev)
            s["rows"] = dev_rows(rows_h)
        sets.append(s)
    ws = ts.Workspace(n, d, V, dev)
    stream = torch.cuda.current_stream()

    if args.calibrate_copy:
        empty_ids = torch.empty(0, dtype=torch.int32, device=dev)
        empty_rows = torch.empty((0, d), dtype=torch.float32, device=dev)
        for i in range(args.warmup + args.steps):
            s = sets[i % len(sets)]
            ts.ts_densify(empty_ids, empty_rows, d, V, s["dense_in"], s["dense_out"], stream)
        torch.cuda.synchronize()
        info = ts.ts_last_launch_info()
        x = info["sort_copy_rows_end"]
        print(json.dumps({"calibration": "ts_densify with n = 0 copies dense_in to dense_out",
                          "launches_per_step": {"sort_kernel": {"read_bytes": 4 * d * x, "write_bytes": 4 * d * x},
                                                "reduce_kernel": {"read_bytes": 4 * d * (V - x),
                                                                  "write_bytes": 4 * d * (V - x)}},
                          "steps": args.warmup + args.steps}))
        ws.close()
        return

    if args.compare_rules:
        assert not multi and elem == 4, "--compare-rules takes a two-contribution fp32 workload"
        n0 = len(w.ids[0])
        res = {}
        for rule, name in ((ts.TS_RULE_TF, "algorithm_1_gather"), (ts.TS_RULE_PROPOSED, "algorithm_2_convert_and_reduce")):
            outs = [dict(ids=torch.empty(V + n, dtype=torch.int32, device=dev),
                         rows=torch.empty((V + n, d), dtype=torch.float32, device=dev)) for _ in sets] \
                if rule == ts.TS_RULE_TF else [None] * len(sets)

            def acc_step(i):
                s = sets[i % len(sets)]
                grads = [("slices", s["ids"][:n0], s["rows"][:n0]), ("slices", s["ids"][n0:], s["rows"][n0:]),
                         ("dense", s["dense_in"])]
                o = outs[i % len(sets)]
                return ts.ts_accumulate(grads, rule, d, V, s["dense_out"], o and o["ids"], o and o["rows"], stream)

            for i in range(args.warmup):
                st, total = acc_step(i)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(args.steps):
                acc_step(i)
            torch.cuda.synchronize()
            us = (time.perf_counter() - t0) * 1e6 / args.steps
            out_bytes = total * (4 + 4 * d) if total is not None else 4 * V * d
            res[name] = {"strategy": st, "accumulate_buffer_bytes": out_bytes, "us_per_call": round(us, 2)}
        a, b = res["algorithm_1_gather"], res["algorithm_2_convert_and_reduce"]
        print(json.dumps({"comparison": "tensor accumulate, sparse gather vs dense reduce, one worker",
                          "workload": args.workload, "V": V, "d": d, "n_pairs": n, **res,
                          "buffer_ratio": round(a["accumulate_buffer_bytes"] / b["accumulate_buffer_bytes"], 3),
                          "note": "the gathered buffer grows with the number of workers (x k after an "
                                  "all-gather), the dense one does not"}))
        ws.close()
        return

    def step(i):
        s = sets[i % len(sets)]
        if epilogue:
            ts.ts_densify_scaled(s["ids"], s["rows"], w.row_dtype, d, V, s["dense_in"], s["dense_out"], scale, stream)
        elif multi:
            ts.ts_densify_multi(s["ids"], s["rows"], w.row_dtype, d, V, s["dense_in"], s["dense_out"], stream)
        elif w.row_dtype == wl.ROW_BF16:
            ts.ts_densify_bf16(s["ids"], s["rows"], d, V, s["dense_in"], s["dense_out"], stream)
        else:
            ts.ts_densify(s["ids"], s["rows"], d, V, s["dense_in"], s["dense_out"], stream)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # timed region: exactly `steps` calls, nothing else on the stream
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    info = ts.ts_last_launch_info()

    # the same `steps` calls again, now with a HIP event pair that the library has stamped with
    # the begin and end of every launch of the row-reduce kernel, on the stream it runs on.  Kept out of the region
    # above because the extra event packets lengthen a whole call by several microseconds.
    use_events = not args.no_events and args.steps <= 4096
    kernel_ms = []
    ms_per_step_with_events = None
    if use_events:
        ts.ts_profile_begin(args.steps)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for i in range(args.steps):
            step(i)
        torch.cuda.synchronize()
        ms_per_step_with_events = (time.perf_counter() - t2) * 1e3 / args.steps
        kernel_ms = ts.ts_profile_end(args.steps)

    # a third pass: every call bracketed by its own pair of events on the stream (median and
    # minimum of single calls; the event packets add a few microseconds to each)
    per_call = None
    if use_events:
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
        evs[0].record(stream)
        for i in range(args.steps):
            step(i)
            evs[i + 1].record(stream)
        torch.cuda.synchronize()
        us = np.array([evs[i].elapsed_time(evs[i + 1]) * 1e3 for i in range(args.steps)])
        per_call = {"median_us": round(float(np.median(us)), 2), "min_us": round(float(us.min()), 2),
                    "calls": int(args.steps), "measured": "one event pair per call, same stream"}

    alg = algorithmic_bytes(n, d, V, elem, out_elem)
    gbps = alg / (ms_per_step * 1e-3) / 1e9
    rows_per_s = n / (ms_per_step * 1e-3)

    # per-row pair counts of the last call, from the library's own views
    count = ts.ts_read_views(V, n)[0].numpy()

    # Algorithmic bytes of one launch of the row-reduce kernel: every value row once; dense_in
    # read and dense_out written for every output row that received pairs (all of them are
    # finished in this launch) and for each untouched row of the range it copies.  The other
    # untouched rows are copied beside the sort launches; ids are read by the sort.
    x0, x1 = info["sort_copy_rows_end"], info["reduce_copy_rows_end"]
    touched = int((count > 0).sum())
    untouched_mid = int((count[x0:x1] == 0).sum())
    alg_reduce = n * elem * d + (4 + out_elem) * d * (touched + untouched_mid)
    roofline = None
    traffic = None
    default_tuning = (args.overlap_mib < 0 and not args.piece_tokens and not args.sort_part and args.short_rows < 0 and not epilogue)
    if default_tuning and args.workload in COUNTED_TRAFFIC["reduce_kernel_bytes_per_launch"]:
        import hashlib
        src = os.path.join(ROOT, "paper_1905_04035_amd", "csrc", "ts_densify.hip")
        if os.path.exists(src) and hashlib.sha256(open(src, "rb").read()).hexdigest() == COUNTED_TRAFFIC["source_sha256"]:
            traffic = COUNTED_TRAFFIC["reduce_kernel_bytes_per_launch"][args.workload]
    if kernel_ms:
        k_ms = float(np.mean(kernel_ms))
        ach = alg_reduce / (k_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": "reduce_kernel", "achieved": round(ach, 1),
                    "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBPS, 4),
                    "traffic": traffic, "avg_kernel_us": round(k_ms * 1e3, 2),
                    "median_kernel_us": round(float(np.median(kernel_ms)) * 1e3, 2),
                    "algorithmic_bytes_per_launch": alg_reduce,
                    "share_of_call_bytes": round(alg_reduce / alg, 4),
                    "measured": "HIP events stamped with the begin and end of every reduce_kernel launch, in a second pass of the same steps",
                    "ms_per_step_with_events": round(ms_per_step_with_events, 5)}

    # The CPU baseline leg: the checker (test infrastructure) timed on this host, and, since it
    # has run anyway, the last timed GPU output compared with its result.
    cpu = None
    parity_ok = None
    if not args.no_cpu_baseline:
        import oracle
        r = oracle.densify(w.ids, w.rows, d, V, w.dense_in, w.row_dtype, scale=scale if epilogue else None)
        out = sets[(args.steps - 1) % len(sets)]["dense_out"].cpu().numpy()
        tol = 1e-5 * r.abs_sum
        if out_elem == 2:
            # bf16 output: rounding is monotonic, so the result must lie between the roundings of
            # the ends of the fp32 tolerance interval
            def val(bits):
                return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
            from oracle import reference as oref
            v = val(out.view(np.uint16))
            parity_ok = bool(np.all((v >= val(oref.bf16_round(r.exact - tol))) & (v <= val(oref.bf16_round(r.exact + tol)))))
        else:
            parity_ok = bool(np.all(np.abs(out.astype(np.float64) - r.exact) <= tol))
        parity_ok = parity_ok and bool(np.array_equal(count, r.count))
        t_one = oracle.densify_timed(ids_h, rows_h, d, V, w.dense_in, w.row_dtype, repeats=1)[0]
        reps = int(min(40, max(3, round(15.0 / max(t_one, 1e-3)))))
        times = oracle.densify_timed(ids_h, rows_h, d, V, w.dense_in, w.row_dtype, repeats=reps)
        t_med = float(np.median(times))
        cpu = {"value": round(alg / t_med / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": f"the whole {args.workload} call (n={n} pairs), median of {reps} runs after one warm-up",
               "ms_per_call": round(t_med * 1e3, 2), "rows_per_s": round(n / t_med, 1),
               "host_cores_available": os.cpu_count()}

    gathered, dense_b = ts.ts_buffer_bytes(16 if multi else 1, n // (16 if multi else 1), d, V, w.row_dtype)
    line = {
        "metric": "densify throughput (algorithmic HBM GB/s of the whole ts_densify call)",
        "value": round(gbps, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": args.workload, "V": V, "d": d, "n_pairs": n,
                   "value_rows": "fp32" if elem == 4 else "bf16 (widened exactly, summed in fp32)",
                   "ids": f"zipf(s={w.spec.zipf_s}) over V, random rank->id permutation",
                   "buffer_sets": len(sets), "entry_point": "ts_densify_scaled" if epilogue else
                   ("ts_densify_multi" if multi else ("ts_densify_bf16" if elem == 2 else "ts_densify")),
                   **({"epilogue": {"scale": scale, "out": args.out}} if epilogue else {})},
        "pct_of_hbm_peak": round(100.0 * gbps / HBM_PEAK_GBPS, 2),
        "rows_per_s": round(rows_per_s, 1),
        "algorithmic_bytes_per_step": alg,
        "unique_ids": int((count > 0).sum()),
        "max_count": int(count.max()) if count.size else 0,
        "gathered_vs_dense_bytes": [gathered, dense_b],
        "parity_ok": parity_ok,
        "launch_split": info,
        "per_call_events": per_call,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    ws.close()
    print(json.dumps(line))
    if parity_ok is False:
        sys.exit(1)


if __name__ == "__main__":
    main()
