#!/usr/bin/env python3
"""Benchmark of the GAF filter-and-average hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

One "step" is one pass of the whole hot path over one batch of synthetic
micro-gradients already resident in HBM: a full gaf_aggregate (batch
workloads), N gaf_step calls (streaming), or gaf_aggregate_with_matrix
(diagnostic: distance matrix plus filter). Prints ONE JSON line.

Vectors of 2^21 .. 2^26 elements: the batch call guesses each call's accept set from the previous
call's. Timing one batch over and over would make every guess right, which no training run
does; so for those sizes the steps cycle through several independently drawn batches
(--batches, default 4), and the run with one repeated batch is reported separately under
other_schedules as the all-guesses-right bound.

value = effective HBM GB/s = (bytes the method itself must move) / time:
    per visited gradient  s*P (read g_i) + 4*P (read the aggregate) + 4*P if accepted (write it),
    once per batch        s*P + 4*P for the seed,
    pairwise              N*s*P (every gradient read once).
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBPS = 8000.0        # MI355X HBM3E, published
PEAK_MFMA_F32_TFLOPS = 157.3  # MI355X dense fp32 matrix, published
PEAK_MFMA_BF16_TFLOPS = 2500.0  # MI355X dense bf16 matrix, published
PEAK_VALU_F64_TFLOPS = 78.6   # MI355X fp64 vector, published


def source_digest():
    """Hash of the kernel sources' code: line comments and blank lines do not count, so that the
    profiler figures stay attached to the kernels until their code changes."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2412_18052_amd", "csrc")
    for fn in sorted(os.listdir(csrc)):
        h.update(fn.encode() + b"\0")
        with open(os.path.join(csrc, fn), "r") as fh:
            for line in fh:
                code = line.split("//", 1)[0].strip()
                if code:
                    h.update(code.encode() + b"\n")
    return h.hexdigest()[:16]


def bmin_bytes(w, mask):
    s, P = w.elem_bytes, w.P
    total = s * P + 4 * P
    for i in range(1, w.N):
        total += s * P + 4 * P + (4 * P if mask[i] else 0)
    if w.mode == "pairwise":
        total += w.N * s * P
    return total


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="large",
                    choices=["tiny", "resnet18", "streaming", "large", "diagnostic"])
    ap.add_argument("--schedule", default="auto", choices=["auto", "sequential", "gram"],
                    help="schedule of the batch call (auto = Gram-first for N <= 64)")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step in a HIP graph and time its replays (launch-bound sizes)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--P", type=int, default=None, help="override the vector length")
    ap.add_argument("--N", type=int, default=None, help="override the number of micro-gradients")
    ap.add_argument("--batches", type=int, default=0,
                    help="independently drawn batches (seeds seed, seed+1, ...) the steps cycle through; "
                         "0 = 4 where the library carries guesses from call to call, else 1")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="ELEMS",
                    help="before anything else run one plain copy of ELEMS binary32 elements through "
                         "the library (a single-gradient batch: reads 4*ELEMS bytes, writes 4*ELEMS): "
                         "the known-size dispatch that profiler byte counters are scaled by")
    ap.add_argument("--only-profile-loop", action="store_true",
                    help="for runs under a profiler: skip the timed loop, the other schedules, the ceilings "
                         "and the CPU baseline, so that the last --steps launches of every kernel are exactly "
                         "the ones the per-kernel figures (roofline) are computed from")
    ap.add_argument("--cpu-seconds", type=float, default=15.0,
                    help="target CPU time of the oracle baseline sample (0 disables it)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: the library runs on one GPU only (no collectives, no sharding); "
                 "use --gpus 1")
    return args



def hbm_roof(alg_bytes, avg_ms):
    ach = alg_bytes / (avg_ms * 1e-3) / 1e9
    return {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
            "frac": ach / PEAK_HBM_GBPS}


def kernel_rooflines(w, steps, B, per_kernel, records, masks, counts):
    """Roofline of each streaming kernel from its launch durations in the per-kernel loop:
    {kernel: (roofline dict, mean launch ms, algorithmic bytes per launch, total ms)}.
    records: the library's record of guesses after each step of that loop ([] where nothing is
    guessed); masks, counts: accept mask and count of each of the B batches."""
    P, N, s = w.P, w.N, w.elem_bytes
    roofs = {}
    if "gram" in per_kernel:
        # one launch reads every gradient once
        dur = per_kernel["gram"]
        avg_ms = sum(dur) / len(dur)
        alg_bytes = float(N * s * P)
        if records:                 # launches that also wrote the mean of their guess
            assert len(dur) == len(records)
            alg_bytes += 4.0 * P * sum(r["write"] for r in records) / len(records)
        r = hbm_roof(alg_bytes, avg_ms)
        if N <= 8:
            # vector-ALU kernel: one binary64 FMA per pair (i <= j) per element
            flops = 2.0 * (N * (N + 1) // 2) * P
            frac2 = flops / (avg_ms * 1e-3) / 1e12 / PEAK_VALU_F64_TFLOPS
            if frac2 > r["frac"]:
                r = {"bound": "alu", "achieved": flops / (avg_ms * 1e-3) / 1e12,
                     "peak": PEAK_VALU_F64_TFLOPS, "unit": "TFLOP/s", "frac": frac2, "hbm_frac": r["frac"]}
            else:
                r["alu_frac"] = frac2
        else:
            # matrix-core kernel: 16-row groups, one 16x16 tile per pair of groups. binary32 rows in
            # three or four groups are multiplied through a three-way bfloat16 split (six bf16 MFMAs
            # per product), everything else in its own type.
            ng = (N + 15) // 16
            flops = 2.0 * (ng * (ng + 1) // 2) * 256 * P
            peak_tf = PEAK_MFMA_F32_TFLOPS if w.dtype == "f32" else PEAK_MFMA_BF16_TFLOPS
            if w.dtype == "f32" and ng >= 3:
                flops *= 6
                peak_tf = PEAK_MFMA_BF16_TFLOPS
            mfma_frac = flops / (avg_ms * 1e-3) / 1e12 / peak_tf
            if mfma_frac > r["frac"]:
                r = {"bound": "mfma", "achieved": flops / (avg_ms * 1e-3) / 1e12, "peak": peak_tf,
                     "unit": "TFLOP/s", "frac": mfma_frac, "hbm_frac": r["frac"]}
            else:
                r["mfma_frac"] = mfma_frac
        roofs["gram"] = (r, avg_ms, alg_bytes, sum(dur))
    if "mean" in per_kernel:
        # accepted gradients read once, result written once; a launch that finds the result in
        # place (right guess) returns at once and is left out
        dur = per_kernel["mean"]
        assert len(dur) == steps
        live = [k for k in range(steps) if not (records and records[k]["valid"])]
        if live:
            avg_ms = sum(dur[k] for k in live) / len(live)
            alg_bytes = sum(float(counts[k % B] * s * P + 4 * P) for k in live) / len(live)
            roofs["mean"] = (hbm_roof(alg_bytes, avg_ms), avg_ms, alg_bytes, sum(dur[k] for k in live))
    if "reduce" in per_kernel:
        # launch k of a batch's reducing passes visits gradient i = k + 2 and stores the update of
        # gradient i - 1 if that one was accepted; a streaming reduce never stores.
        if w.mode == "step":
            # the launch for the seed returns at once (nothing to compare with): not counted
            per_launch = ([None] + [(4 + s) * P] * (N - 1)) * steps
        else:
            per_launch = [(4 + s) * P + (4 * P if masks[k % B][i - 1] else 0)
                          for k in range(steps) for i in range(2, N)]
        dur = per_kernel["reduce"]
        assert len(dur) == len(per_launch), (len(dur), len(per_launch))
        dur = [d for k, d in enumerate(dur) if per_launch[k] is not None]
        alg = sum(b for b in per_launch if b is not None)
        avg_ms = sum(dur) / max(1, len(dur))
        alg_bytes = alg / max(1, len(dur))
        roofs["reduce"] = (hbm_roof(alg_bytes, avg_ms), avg_ms, alg_bytes, sum(dur))
    return roofs


def measure_ceilings(gaf, torch):
    """What this GPU's memory system delivers to the simplest kernels of the library, measured now:
    a read-only pass (inner products of two binary32 vectors of 2^28 elements: 2 GiB read) and a
    plain copy (a single-gradient batch: 1 GiB read, 1 GiB written)."""
    try:
        E = 1 << 28
        a_c = torch.ones(E, dtype=torch.float32, device="cuda")
        b_c = torch.full((E,), 0.5, dtype=torch.float32, device="cuda")
        cal = gaf.gaf_create(max_P=E, max_N=2)
        o_c = gaf.gaf_aggregate(cal, [a_c], 1.0)
        d_c = gaf.gaf_pairwise(cal, [a_c, b_c])
        torch.cuda.synchronize()
        gaf.gaf_profile_begin(cal, 256)
        for _ in range(5):
            gaf.gaf_aggregate(cal, [a_c], 1.0, *o_c)
            gaf.gaf_pairwise(cal, [a_c, b_c], d_c)
        kt = {}
        for name, ms in gaf.gaf_profile_end(cal, 256):
            kt.setdefault(name, []).append(ms)
        gaf.gaf_destroy(cal)
        return {"read_only": 2 * 4 * E / (min(kt["gram"]) * 1e-3) / 1e9,
                "copy": 2 * 4 * E / (min(kt["update"]) * 1e-3) / 1e9, "unit": "GB/s",
                "how": "best of 5 launches each: inner products of two 2^28-element binary32 vectors "
                       "(read-only), single-gradient batch of one such vector (copy)"}
    except (torch.OutOfMemoryError, KeyError) as e:      # the workload left no room, or a kernel was renamed
        return {"error": repr(e)}


def cpu_baseline(w, grads, seed, cpu_seconds, wl, np):
    """The oracle, as it stands, on a bounded sample of the same workload: all N micro-gradients,
    the first Ps coordinates of each, Ps sized for about cpu_seconds of work."""
    from oracle import gaf_oracle
    P, N = w.P, w.N
    cores = gaf_oracle.num_threads()
    rate_guess = 1.2e8 * cores          # element visits per second, refined by a probe
    probe = min(P, 1 << 20)
    host = [wl.to_host_array(g[:probe]) for g in grads]
    tp = time.perf_counter()
    gaf_oracle.aggregate(host, np.float32(w.tau))
    tp = time.perf_counter() - tp
    rate_guess = max(rate_guess, N * probe / max(tp, 1e-4))
    Ps = int(min(P, max(probe, cpu_seconds * rate_guess / N)))
    if w.mode == "pairwise":
        Ps = int(min(P, max(1 << 16, Ps // 24)))   # the pair loop costs ~N/2 more passes
    host = [wl.to_host_array(g[:Ps]) for g in grads]
    tc = time.perf_counter()
    if w.mode == "pairwise":
        gaf_oracle.pairwise(host)
    if w.mode == "step":
        acc64 = np.empty(Ps, dtype=np.float64)
        cnt, o_mask = 0, []
        for h in host:
            _, a_i, cnt = gaf_oracle.step(acc64, cnt, h, np.float32(w.tau))
            o_mask.append(a_i)
    else:
        _, o_mask, _, _ = gaf_oracle.aggregate(host, np.float32(w.tau))
    tc = time.perf_counter() - tc
    ws = wl.spec(w.name, seed, P=Ps, N=N)
    cpu_bytes = bmin_bytes(ws, list(o_mask))
    return {"value": cpu_bytes / tc / 1e9, "unit": "GB/s", "cores": cores, "kind": "oracle",
            "seconds": tc, "micro_gradients_per_s": N / tc * (Ps / P),
            "sample": "all %d micro-gradients, first %d of %d coordinates each "
                      "(%.3g of the workload); micro_gradients_per_s is scaled to full length"
                      % (N, Ps, P, Ps / P)}


def main():
    args = parse_args()

    import numpy as np
    import torch
    from paper_2412_18052_amd import gaf
    from paper_2412_18052_amd import workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    torch.cuda.set_device(0)
    gaf.load()

    if args.calibrate_copy > 0:
        cal_ctx = gaf.gaf_create(max_P=args.calibrate_copy, max_N=1)
        src = torch.ones(args.calibrate_copy, dtype=torch.float32, device="cuda")
        gaf.gaf_aggregate(cal_ctx, [src], 1.0)
        torch.cuda.synchronize()
        gaf.gaf_destroy(cal_ctx)
        del src

    t0 = time.time()
    w, grads = wl.generate(args.workload, args.seed, P=args.P, N=args.N, device="cuda")
    torch.cuda.synchronize()
    gen_s = time.time() - t0
    P, N, s = w.P, w.N, w.elem_bytes
    ctx = gaf.gaf_create(max_P=P, max_N=max(N, 64))
    gaf.gaf_set_schedule(ctx, args.schedule)
    if w.mode == "step":
        schedule_used = "streaming"
    elif args.schedule == "sequential" or not (2 <= N <= 64):
        schedule_used = "sequential"
    else:
        schedule_used = "gram_first"
    # long vectors on the matrix-core path: the Gram pass also writes the mean of a guessed accept set
    fused = schedule_used == "gram_first" and args.schedule == "auto" and P >= (1 << 26)
    if fused:
        schedule_used = "gram_first_fused_mean"
    # shorter vectors: the guess is the previous call's accept set
    carried = schedule_used == "gram_first" and args.schedule == "auto" and (1 << 21) <= P < (1 << 26)
    B = args.batches if args.batches > 0 else (4 if carried and not args.graph else 1)
    batches = [grads] + [wl.generate(args.workload, args.seed + j, P=args.P, N=args.N, device="cuda")[1]
                         for j in range(1, B)]
    torch.cuda.synchronize()

    out = torch.empty(P, dtype=torch.float32, device="cuda")
    mask = torch.empty(N, dtype=torch.uint8, device="cuda")
    dist = torch.empty(N, dtype=torch.float32, device="cuda")
    count = torch.zeros(1, dtype=torch.int32, device="cuda")
    D = torch.empty((N, N), dtype=torch.float32, device="cuda") if w.mode == "pairwise" else None
    G = torch.empty((N, N), dtype=torch.float64, device="cuda") if w.mode == "pairwise" else None

    state = {"schedule": args.schedule}

    def step(k=0):
        grads = batches[k % B]
        if w.mode == "step":
            count.zero_()
            for i, g in enumerate(grads):
                gaf.gaf_step(ctx, out, count, g, w.tau, dist[i:i + 1], mask[i:i + 1])
        else:
            if w.mode == "pairwise" and state["schedule"] != "sequential":
                # the distance matrix and the filter share one Gram pass
                gaf.gaf_aggregate_with_matrix(ctx, grads, w.tau, out, mask, dist, count, D, G)
                return
            if w.mode == "pairwise":
                gaf.gaf_pairwise(ctx, grads, D=D)
            gaf.gaf_aggregate(ctx, grads, w.tau, out, mask, dist, count)

    # every batch once: its accept mask (for the bytes the method must move) and a warm-up
    masks, dists, counts = [], [], []
    for b in range(B):
        step(b)
        torch.cuda.synchronize()
        masks.append(mask.cpu().numpy().tolist())
        dists.append(dist.cpu().numpy().tolist())
        counts.append(int(count.item()))
    for k in range(args.warmup):
        step(k)
    torch.cuda.synchronize()
    run_step = step
    if args.graph:
        # the library neither allocates nor synchronises in its calls, so a step can be captured
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        run_step = lambda k=0: graph.replay()
        run_step()
        torch.cuda.synchronize()
    mask_h, dist_h, c_h = masks[0], dists[0], counts[0]
    step_bytes = sum(bmin_bytes(w, masks[k % B]) for k in range(args.steps)) / args.steps
    ms_per_step = ms_per_step_events = value = None
    if not args.only_profile_loop:
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        ev0.record()
        for k in range(args.steps):
            run_step(k)
        ev1.record()
        torch.cuda.synchronize()
        wall_s = time.perf_counter() - t0
        ms_per_step = 1e3 * wall_s / args.steps
        ms_per_step_events = ev0.elapsed_time(ev1) / args.steps
        value = step_bytes / (ms_per_step * 1e-3) / 1e9

    # ---- per-kernel durations over the same steps, HIP events on the launch stream; where the
    # Gram pass may write the mean of a guess, the library's record says after each step whether
    # it did and whether the guess was right (reading it waits for the device: not in the timed loop)
    gaf.gaf_profile_begin(ctx, 65536)
    records = []
    for k in range(args.steps):
        step(k)
        if fused or carried:
            records.append(gaf.gaf_fused_mean_record(ctx))
    times = gaf.gaf_profile_end(ctx, 65536)
    per_kernel = {}
    for name, ms in times:
        per_kernel.setdefault(name, []).append(ms)
    launches_per_step = len(times) // args.steps

    roofs = kernel_rooflines(w, args.steps, B, per_kernel, records, masks, counts)
    dom = max(roofs, key=lambda k: roofs[k][3])      # the kernel the step spends most time in
    roof, avg_ms, alg_bytes, _ = roofs[dom]
    roof["kernel"] = dom
    roof["avg_launch_ms"] = avg_ms
    roof["algorithmic_bytes_per_launch"] = alg_bytes
    roof["traffic"] = None
    roof["other_kernels"] = {k: {"frac": v[0]["frac"], "bound": v[0]["bound"], "avg_launch_ms": v[1],
                                 "algorithmic_bytes_per_launch": v[2]}
                             for k, v in roofs.items() if k != dom}
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        with open(tpath) as fh:
            tj = json.load(fh)
        # measured HBM bytes per launch of this kernel in the profiler run, as a ratio to the
        # algorithmic bytes per launch of that same run; scaled to this run's launches
        ent = tj.get("%s/%s/%s" % (w.name, schedule_used, dom))
        if ent and ent.get("source_digest") == source_digest() and ent.get("P") == P:
            roof["traffic"] = ent["hbm_bytes_over_algorithmic"] * alg_bytes
            roof["traffic_over_algorithmic"] = ent["hbm_bytes_over_algorithmic"]

    # ---- the other schedules of the batch call, for comparison (fewer steps) ----
    other = None
    if w.mode != "step" and args.schedule == "auto" and 2 <= N <= 64 and not args.only_profile_loop:
        other = []
        # (label, schedule); all on the first batch, repeated
        runs = [("gram_two_pass", "gram")] if fused or carried else []
        if carried and not args.graph:
            runs.append(("gram_first_one_batch_repeated_every_guess_right", "auto"))
        runs.append(("sequential", "sequential"))
        for label, sched in runs:
            gaf.gaf_set_schedule(ctx, sched)
            state["schedule"] = sched
            # short steps: as many as the main loop, or the host's launch overhead shows
            k = args.steps if ms_per_step < 1.0 else max(3, args.steps // 4)
            step()
            step()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(k):
                step()
            torch.cuda.synchronize()
            ms_o = 1e3 * (time.perf_counter() - t0) / k
            gaf.gaf_profile_begin(ctx, 65536)      # per-kernel times in a loop of their own: the event
            for _ in range(k):                     # brackets cost time between launches
                step()
            kt = {}
            for name, ms in gaf.gaf_profile_end(ctx, 65536):
                kt.setdefault(name, []).append(ms)
            entry = {"schedule": label, "steps": k,
                     "ms_per_step": ms_o, "value": bmin_bytes(w, masks[0]) / (ms_o * 1e-3) / 1e9,
                     "kernel_ms": {n: sum(v) / len(v) for n, v in kt.items()}}
            if sched == "gram" and "gram" in kt:
                g_ms = sum(kt["gram"]) / len(kt["gram"])
                entry["gram_kernel_hbm_frac"] = N * s * P / (g_ms * 1e-3) / 1e9 / PEAK_HBM_GBPS
            other.append(entry)
        gaf.gaf_set_schedule(ctx, args.schedule)
        state["schedule"] = args.schedule

    # ---- the memory system's own ceilings; the dominant kernel's rate is also reported as a fraction
    # of whichever of the two matches its read/write mix
    ceilings = None
    if not args.only_profile_loop:
        ceilings = measure_ceilings(gaf, torch)
        if "error" not in ceilings:
            writes = ((dom == "gram" and any(r["write"] for r in records)) or dom == "mean" or
                      (dom == "reduce" and w.mode != "step"))
            roof["frac_of_measured_ceiling"] = (roof["achieved"] / ceilings["copy" if writes else "read_only"]
                                                if roof["bound"] == "hbm" else None)

    # ---- CPU baseline ----
    cpu = None
    if args.cpu_seconds > 0 and not args.only_profile_loop:
        cpu = cpu_baseline(w, grads, args.seed, args.cpu_seconds, wl, np)

    line = {
        "metric": "gaf_filter_average_effective_hbm_gbps",
        "value": value,
        "unit": "GB/s",
        "pct_of_hbm_peak": None if value is None else 100.0 * value / PEAK_HBM_GBPS,
        "micro_gradients_per_s": None if ms_per_step is None else N / (ms_per_step * 1e-3),
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "ms_per_step_hip_events": ms_per_step_events,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "dtype_detail": "%s gradients, binary32 running mean and output, binary64 inner products"
                        % w.dtype,
        "data": "synthetic",
        "config": {"workload": w.name, "N": N, "P": P, "input_dtype": w.dtype, "tau": w.tau,
                   "mode": w.mode, "schedule": schedule_used, "hip_graph": bool(args.graph), "seed": args.seed, "accepted": c_h,
                   "batches": B, "accepted_per_batch": counts,
                   "guesses": ({"source": "sample of this call's gradients" if fused else "previous call's accept set",
                                "mean_written_by_gram_pass": sum(r["write"] for r in records),
                                "right": sum(r["valid"] for r in records), "steps": len(records)}
                               if records else None),
                   "generator": "g_i = a_i (s_i sqrt(rho_i) c + sqrt(1 - rho_i) z_i); rho, s, a from numpy Philox keyed by "
                                "the seed, c and z_i from a torch.Generator on the device (" + w.noise + "); see workloads.py",
                   "algorithmic_bytes_per_step": step_bytes,
                   "launches_per_step": launches_per_step, "generate_seconds": gen_s},
        "roofline": roof,
        "measured_ceilings": ceilings,
        "cpu_baseline": cpu,
        "other_schedules": other,
        "kernel_ms": {k: sum(v) / len(v) for k, v in per_kernel.items()},
        "accept_mask": mask_h,
        "cos_dist": [round(x, 6) for x in dist_h],
        "paper_reference": "no throughput reported; experiments ran on 2x NVIDIA A40 with k = 2",
    }
    print(json.dumps(line))
    gaf.gaf_destroy(ctx)


if __name__ == "__main__":
    main()
