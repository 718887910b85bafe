#!/usr/bin/env python3
"""Throughput of the HBM-PS mini-batch pull+push on one MI355X.

One "step" = hps_pull + hps_push of one synthetic mini-batch (all five stages of the
path: dedup, lookup-or-insert, gather + pool, reduce by key, Adagrad update), inputs
already resident in HBM.  Prints ONE JSON line:

  value      unique keys per second over the timed steps (whole job, one GPU) of the headline
             workload: `large`, the 10^9-key table, the largest that fits one GPU
  roofline   the stage that takes the most time, its algorithmic HBM bytes per launch
             over its HIP-event duration, against the 8 TB/s peak
  cpu_baseline  the CPU oracle timed on a bounded sample of the same workload
  others     the other workloads (tiny, mid, insert_heavy, skewed, skewed_shifted) in the same launch
             configuration, each with its own fresh table: ms per step, unique keys/s,
             fraction of peak, stage times; insert_heavy runs its 50 consecutive steps and
             reports the first, the last and the mean

Schedule of the timed steps (default): hps_pull(i); hps_push(i) on one stream, so that the
stages' HIP-event times add up to the step.  --pipelined times pull_prepared(i); prepare(i+1)
on a second stream; push(i) -- every mini-batch still goes through all five stages, the dedup
of the next one overlaps the push of the current one; the default run reports that schedule
as `pipelined_ms_per_step` as well.

python bench.py [--gpus 1] [--steps K] [--warmup W] [--config large] [--others none]
"""
import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
OTHER_WORKLOADS = "tiny,mid,insert_heavy,skewed,skewed_shifted"


def measured_traffic(workload, stage):
    """HBM bytes per launch of a stage from the committed rocprofv3 counter summary
    (profiles/<workload>_hbm_counters.md, lines 'traffic <stage> <bytes>'), or None."""
    path = os.path.join(ROOT, "profiles", "%s_hbm_counters.md" % workload)
    try:
        with open(path) as f:
            for line in f:
                parts = line.split()
                if len(parts) == 3 and parts[0] == "traffic" and parts[1] == stage:
                    return int(float(parts[2]))
    except OSError:
        pass
    return None


def stage_bytes(n, u, bags, d, wb=4, acc=1):
    """Algorithmic HBM bytes of one step, per stage: what the method itself has to move
    once, with 4-byte indices and each distinct row crossing HBM once per direction.
    wb = bytes per stored weight (4, or 2 for bfloat16 rows); acc = accumulators per row
    (1, or d for the elementwise Adagrad)."""
    return {
        "dedup": 8 * n + 4 * n + 8 * u,                     # read keys, write inverse, write uniq
        "lookup": 8 * u + 4 * u,                            # one slot key per unique, row id
        "pool": wb * d * u + 4 * n + 4 * bags + 4 * d * bags,  # rows, inverse, offsets, pooled
        "push": 4 * d * bags + 4 * n + 2 * (wb * d + 4 * acc) * u,  # grads, grouping, row+acc r/w
    }


def host_description():
    """The box the CPU figure was taken on: core count, CPU model, memory."""
    model, mem_gib = "unknown", None
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
        with open("/proc/meminfo") as f:
            for line in f:
                if line.startswith("MemTotal"):
                    mem_gib = round(int(line.split()[1]) / 2**20, 1)
                    break
    except OSError:
        pass
    return {"cpus": os.cpu_count(), "cpu_model": model, "mem_gib": mem_gib}


STAGE_BITS = {"dedup": 0b00011, "lookup": 0b00100, "pool": 0b01000, "push": 0b10000}
STAGE_KERNELS = {
    "dedup": "bucket_count, scan_tiles, scatter_pass (once or twice, with digit_count and "
             "scan_tiles between), region_borders, region_sort, region_emit (a table's first "
             "two dedups, and very large ones: sort_prepare, n_pass x onesweep_pass, "
             "unique_emit, fix_mixed_runs, unique_emit)",
    "lookup": "lookup_keys<0>, insert_missing",
    "pool": "pool_bags",
    "push": "push_main (short | medium | chunk roles), push_long",
}


def merge_stage_times(times):
    out = {}
    out["dedup"] = (times["sort"][0] + times["unique"][0], times["sort"][1])
    for k in ("lookup", "pool", "push"):
        out[k] = times[k]
    return out


def random_row_ceiling(hps, torch, dim, rows_log2=26):
    """Random rows of dim float32 values per second from a large array, read by a kernel that
    does nothing else (hps_probe_random_rows), and by a plain library gather."""
    n_rows = (1 << rows_log2) * 16 // dim
    big = torch.zeros((n_rows, dim), dtype=torch.float32, device="cuda")
    sink = torch.empty(262144, dtype=torch.float32, device="cuda")
    n_acc = 1 << 25 if dim == 16 else 1 << 23
    hps.probe_random_rows(big, n_acc, sink)
    torch.cuda.synchronize()
    g0 = time.perf_counter()
    for _ in range(3):
        hps.probe_random_rows(big, n_acc, sink)
    torch.cuda.synchronize()
    ceiling = 3 * n_acc / (time.perf_counter() - g0)
    idx = torch.randint(0, n_rows, (1 << 22,), device="cuda")
    torch.index_select(big, 0, idx)
    torch.cuda.synchronize()
    g0 = time.perf_counter()
    for _ in range(3):
        torch.index_select(big, 0, idx)
    torch.cuda.synchronize()
    lib_rate = 3 * idx.numel() / (time.perf_counter() - g0)
    del big, idx, sink
    return ceiling, lib_rate


def run_workload(name, args, headline):
    """Builds the workload's table, runs its steps and returns the measurements."""
    import numpy as np
    import torch

    import paper_2003_05622_amd as hps
    import synth

    cfg = synth.CONFIGS[name]
    elementwise = args.adagrad == "elementwise"
    whole_run = name == "insert_heavy"      # the workload IS its 50 consecutive steps
    steps = cfg.steps if whole_run else (args.steps if headline else min(args.steps, 20))
    warmup = 0 if whole_run else (args.warmup if headline else min(args.warmup, 3))
    # all-stage timing run after the timed region (insert_heavy is its 50 consecutive steps and
    # nothing else: its stages are timed inside them)
    extra_steps = 0 if whole_run else 5
    serial = not args.pipelined
    # the other schedule afterwards, for comparison
    other_steps = 8 if headline and not args.one_schedule else 0
    n_batches = args.batches or min(steps + warmup + extra_steps + other_steps, 64)
    if whole_run:
        n_batches = steps                   # never reused: every step inserts fresh keys

    def dev_keys(a):
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint64).view(np.int64)).cuda()

    # ---- inputs: generated on the host, resident in HBM before the timed region -------
    t0 = time.time()
    stream = synth.BatchStream(cfg)
    host_batches, dev_batches = [], []
    for _ in range(n_batches):
        b = stream.next()
        host_batches.append(b)
        dev_batches.append((dev_keys(b.keys), torch.from_numpy(b.offsets).cuda(),
                            torch.from_numpy(b.grads).cuda()))
    n_max = max(b.n_keys for b in host_batches)
    uniques = [int(np.unique(b.keys).shape[0]) for b in host_batches]
    table = hps.HpsTable(cfg.capacity, cfg.dim, n_max, cfg.n_bags, lr=cfg.lr, eps=cfg.eps,
                         init_acc=cfg.init_acc, init_range=cfg.init_range,
                         init_seed=cfg.init_seed,
                         opt=hps.ADAGRAD_ELEMENTWISE if elementwise else hps.ADAGRAD_ROWWISE,
                         row_format={"bf16": hps.ROWS_BF16, "f32wide": hps.ROWS_F32_WIDE}.get(args.rows, hps.ROWS_F32))
    chunk = 1 << 23
    for lo in range(0, cfg.n_prefill, chunk):
        table.insert(dev_keys(synth.prefill_keys(lo, min(lo + chunk, cfg.n_prefill))))
    torch.cuda.synchronize()
    table.check("prefill")
    size_before = int(table.stats().size)
    pooled = torch.empty((cfg.n_bags, cfg.dim), dtype=torch.float32, device="cuda")
    setup_s = time.time() - t0

    side = torch.cuda.Stream()          # default priority

    def prepare(i):
        k, o, _ = dev_batches[i % n_batches]
        with torch.cuda.stream(side):
            table.prepare(k, o, cfg.n_examples, cfg.n_slots)

    def step(i, more=True):
        """One step = dedup + lookup/insert + pool + reduce + update of mini-batch i.  In the
        pipelined form the dedup of mini-batch i was enqueued during step i-1 and that of
        mini-batch i+1 is enqueued here, between this step's pull and push."""
        k, o, g = dev_batches[i % n_batches]
        if serial:
            table.pull(k, o, cfg.n_examples, cfg.n_slots, pooled)
        else:
            table.pull_prepared(pooled)
            if more:
                prepare(i + 1)
        table.push(g)

    if headline and args.calibrate_copy:
        src = torch.ones(64 << 20, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                  # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    # ---- warm-up, and a look at which stage dominates ---------------------------------
    table.set_stage_timing(0b11111)
    if not serial:
        prepare(0)
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    calib = merge_stage_times(table.stage_times())
    if warmup == 0 or calib["dedup"][1] == 0:
        dominant = "dedup"
    else:
        dominant = max(calib, key=lambda s: calib[s][0])
    # inside the timed region only the dominant stage is timed (fewer events on the stream),
    # and for the workloads beside the headline one nothing; all stages are timed in a few
    # further steps afterwards
    table.set_stage_timing(0b11111 if whole_run else STAGE_BITS[dominant] if headline else 0)

    # ---- timed region --------------------------------------------------------------------
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)] if whole_run else None
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(warmup, warmup + steps):
        if marks:
            marks[i - warmup].record()
        step(i, more=i + 1 < warmup + steps)
    if marks:
        marks[steps].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    timed = merge_stage_times(table.stage_times())
    table.check("timed steps")

    idx = [i % n_batches for i in range(warmup, warmup + steps)]
    sum_u = sum(uniques[i] for i in idx)
    sum_n = sum(host_batches[i].n_keys for i in idx)
    mean_n, mean_u = sum_n / steps, sum_u / steps
    per_stage = stage_bytes(mean_n, mean_u, cfg.n_bags, cfg.dim, 2 if args.rows == "bf16" else 4,
                            cfg.dim if elementwise else 1)
    dom_ms = timed[dominant][0] / max(timed[dominant][1], 1)
    achieved = per_stage[dominant] / (dom_ms * 1e-3) / 1e9 if dom_ms > 0 else 0.0
    step_bytes = sum(per_stage.values())

    # ---- all stages once more, outside the timed region, for the record -------------------
    allst = timed
    if extra_steps:
        table.set_stage_timing(0b11111)
        last = warmup + steps + extra_steps - 1
        if not serial:
            prepare(warmup + steps)
        for i in range(warmup + steps, last + 1):
            step(i, more=i < last)
        torch.cuda.synchronize()
        allst = merge_stage_times(table.stage_times())
    stages = {s: {"ms": round(allst[s][0] / max(allst[s][1], 1), 4),
                  "alg_bytes": int(per_stage[s]),
                  "gbps": round(per_stage[s] / max(allst[s][0] / max(allst[s][1], 1), 1e-9) / 1e6, 1)}
              for s in allst}
    other_ms = None
    if other_steps:
        # the schedule that was not timed, for comparison (no stage events)
        table.set_stage_timing(0)
        first = warmup + steps + extra_steps
        if not serial:                      # the pipelined run left no mini-batch prepared
            k, o, g = dev_batches[first % n_batches]
            table.pull(k, o, cfg.n_examples, cfg.n_slots, pooled)      # one untimed step
            table.push(g)
            torch.cuda.synchronize()
            c0 = time.perf_counter()
            for i in range(first + 1, first + other_steps):
                k, o, g = dev_batches[i % n_batches]
                table.pull(k, o, cfg.n_examples, cfg.n_slots, pooled)
                table.push(g)
        else:
            prepare(first)
            table.pull_prepared(pooled)                                # one untimed step
            prepare(first + 1)
            table.push(dev_batches[first % n_batches][2])
            torch.cuda.synchronize()
            c0 = time.perf_counter()
            for i in range(first + 1, first + other_steps):
                table.pull_prepared(pooled)
                if i + 1 < first + other_steps:
                    prepare(i + 1)
                table.push(dev_batches[i % n_batches][2])
        torch.cuda.synchronize()
        other_ms = (time.perf_counter() - c0) / (other_steps - 1) * 1e3
    st = table.stats()
    assert st.error == 0

    res = {
        "value": round(sum_u / elapsed, 1),
        "ms_per_step": round(elapsed / steps * 1e3, 4),
        "steps": steps,
        "warmup": warmup,
        "occurrences_per_s": round(sum_n / elapsed, 1),
        "step_alg_bytes": int(step_bytes),
        "step_gbps": round(step_bytes / (elapsed / steps) / 1e9, 1),
        "step_frac_of_peak": round(step_bytes / (elapsed / steps) / 1e9 / HBM_PEAK_GBS, 4),
        "stages": stages,
        ("pipelined_ms_per_step" if serial else "serial_ms_per_step"):
            None if other_ms is None else round(other_ms, 4),
        "config": {"workload": cfg.name,
                   "schedule": "serial: pull then push on one stream" if serial
                               else "dedup of batch i+1 overlaps push of batch i",
                   "table_keys": int(st.size), "capacity": cfg.capacity, "rows": args.rows,
                   "adagrad": args.adagrad,
                   "dim": cfg.dim, "n_examples": cfg.n_examples, "n_slots": cfg.n_slots,
                   "keys_per_step": round(mean_n, 1), "unique_per_step": round(mean_u, 1),
                   "zipf_s": cfg.zipf_s, "fresh_frac": cfg.fresh_frac,
                   "distinct_batches": n_batches},
        "roofline": {"bound": "hbm", "kernel": dominant + ": " + STAGE_KERNELS[dominant],
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": measured_traffic(cfg.name, dominant),
                     "launch_ms": round(dom_ms, 4), "launches_timed": int(timed[dominant][1]),
                     "alg_bytes_per_launch": int(per_stage[dominant])},
        "setup_s": round(setup_s, 1),
    }
    if marks:
        per_step = [marks[i].elapsed_time(marks[i + 1]) for i in range(steps)]
        n_slots_table = int(st.n_slots)
        res["consecutive_steps"] = {
            "first_ms": round(per_step[0], 4), "second_ms": round(per_step[1], 4),
            "last_ms": round(per_step[-1], 4),
            "mean_ms": round(sum(per_step) / steps, 4),
            "mean_after_the_first_two_ms": round(sum(per_step[2:]) / max(steps - 2, 1), 4),
            "load_factor_first": round(size_before / n_slots_table, 4),
            "load_factor_last": round(int(st.size) / n_slots_table, 4),
            "what": "HIP-event time of each of the %d consecutive steps; a table's first two "
                    "dedups take the plain form" % steps}

    # ---- the rate at which this GPU returns random rows of this width ---------------------
    # Pooling and push are gathers of rows: at least 3U row accesses (pool reads, push reads
    # and writes each unique row) and N gradient-row gathers per step.  Their bound is the
    # random-access rate of the memory system, not its streaming bandwidth.  That rate is
    # measured here with a kernel that does nothing but read random rows of a 4 GiB array in
    # the pooling kernel's access shape (hps_probe_random_rows), and, for comparison, with a
    # plain library gather (torch.index_select) over the same array.
    if headline and args.gather_rows and cfg.dim in (16, 64) and args.rows != "bf16":
        ceiling, lib_rate = random_row_ceiling(hps, torch, cfg.dim)
        pp_ms = stages["pool"]["ms"] + stages["push"]["ms"]
        path_rate = (3 * mean_u + mean_n) / (pp_ms * 1e-3)
        # What the two kernels issue: pooling reads a row per OCCURRENCE (a frequent key's row
        # is fetched again unless L2 still holds it), the push reads a gradient row per
        # occurrence and reads and writes the weights and the accumulator(s) of every unique
        # key (two places unless they lie side by side: the elementwise Adagrad's layout).
        per_unique = 2 if (elementwise and args.rows == "f32") or args.rows == "f32wide" else 4
        issued_rate = (2 * mean_n + per_unique * mean_u) / (pp_ms * 1e-3)
        res["random_row_access"] = {
            "what": "random %d-byte row accesses per second; pooling + push need at least 3U + N "
                    "of them per step (path_per_s) and issue 2N + %dU (issued_per_s: a row per "
                    "occurrence in pooling, reads and writes of weights and accumulators in the "
                    "push); ceiling = a kernel that only reads random rows of a 4 GiB "
                    "array (hps_probe_random_rows); library = torch.index_select over the same "
                    "array" % (4 * cfg.dim, per_unique),
            "row_bytes": 4 * cfg.dim,
            "path_per_s": round(path_rate, 1), "ceiling_per_s": round(ceiling, 1),
            "frac": round(path_rate / ceiling, 3),
            "issued_per_s": round(issued_rate, 1), "issued_frac": round(issued_rate / ceiling, 3),
            "library_per_s": round(lib_rate, 1)}

    # ---- CPU oracle on a bounded sample of the same workload ------------------------------
    if headline and args.cpu_seconds > 0:
        import oracle
        ot = oracle.OracleTable(cfg.capacity, cfg.dim, lr=cfg.lr, eps=cfg.eps,
                                init_acc=cfg.init_acc, init_range=cfg.init_range,
                                init_seed=cfg.init_seed,
                                opt=oracle.ADAGRAD_ELEMENTWISE if elementwise else oracle.ADAGRAD_ROWWISE,
                                row_format=oracle.ROWS_BF16 if args.rows == "bf16" else oracle.ROWS_F32)
        ot.declare_resident(cfg.n_prefill)
        spent, done_u, done = 0.0, 0, 0
        for b in host_batches:
            resident, _ = synth.resident_split(cfg, b)
            ot.materialize(resident)            # stands in for the prefill: not timed
            c0 = time.perf_counter()
            ot.pull(b.keys, b.offsets)
            ot.push(b.grads)
            spent += time.perf_counter() - c0
            done_u += ot.n_unique
            done += 1
            if spent > args.cpu_seconds:
                break
        res["cpu_baseline"] = {
            "value": round(done_u / spent, 1), "unit": "unique keys/s", "cores": 1,
            "kind": "oracle",
            "sample": "%d mini-batch(es) of the '%s' workload, pull+push, single thread, "
                      "%.1f s" % (done, cfg.name, spent),
            "host": host_description()}
        del ot
    del table, pooled, dev_batches, host_batches
    gc.collect()
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="large",
                    help="the headline workload (default: large, the 10^9-key table)")
    ap.add_argument("--others", default=OTHER_WORKLOADS,
                    help="comma-separated workloads measured as well, each on a fresh table of its "
                         "own ('none': only the headline workload)")
    ap.add_argument("--batches", type=int, default=0,
                    help="distinct pre-generated batches (0: one per step run, at most 64)")
    ap.add_argument("--pipelined", action="store_true",
                    help="time hps_prepare of the next mini-batch on a second stream while the "
                         "current one is pushed (default: plain hps_pull + hps_push per step)")
    ap.add_argument("--one-schedule", action="store_true",
                    help="skip the few steps of the other schedule that the headline workload runs "
                         "after its timed region for comparison (for profiles: every dispatch of a "
                         "kernel then belongs to the same schedule)")
    ap.add_argument("--serial", action="store_true", help="the default schedule (kept for old command lines)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy, so that a counter run of this "
                         "command can scale FETCH_SIZE / WRITE_SIZE by a kernel of known traffic")
    ap.add_argument("--rows", choices=("f32", "bf16", "f32wide"), default="f32",
                    help="how the table stores weights (the arithmetic is float32 either way)")
    ap.add_argument("--adagrad", choices=("rowwise", "elementwise"), default="rowwise",
                    help="one accumulator per row (the default) or one per element")
    ap.add_argument("--gather-rows", type=int, default=1,
                    help="0: skip the random-row ceiling and the library gather")
    ap.add_argument("--cpu-seconds", type=float, default=15.0,
                    help="time budget of the CPU oracle leg (0 disables it)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one GPU's shard of the table, no "
              "collectives); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2

    import torch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)

    head = run_workload(args.config, args, headline=True)
    others = {}
    if args.others != "none":
        for name in args.others.split(","):
            if name and name != args.config:
                r = run_workload(name, args, headline=False)
                keep = ("value", "ms_per_step", "steps", "warmup", "step_alg_bytes", "step_gbps",
                        "step_frac_of_peak", "stages", "consecutive_steps")
                others[name] = {k: r[k] for k in keep if k in r}
                others[name]["keys_per_step"] = r["config"]["keys_per_step"]
                others[name]["unique_per_step"] = r["config"]["unique_per_step"]

    out = {
        "metric": "unique keys/sec pull+push (1 MI355X) and achieved HBM GB/s vs peak",
        "value": head["value"],
        "unit": "unique keys/s",
        "n_gpus": 1,
        "steps": head["steps"],
        "warmup": head["warmup"],
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": head["config"],
        "occurrences_per_s": head["occurrences_per_s"],
        "step_alg_bytes": head["step_alg_bytes"],
        "step_gbps": head["step_gbps"],
        "step_frac_of_peak": head["step_frac_of_peak"],
        "roofline": head["roofline"],
        "stages": head["stages"],
        "random_row_access": head.get("random_row_access"),
        "pipelined_ms_per_step": head.get("pipelined_ms_per_step"),
        "serial_ms_per_step": head.get("serial_ms_per_step"),
        "cpu_baseline": head.get("cpu_baseline"),
        "others": others,
        "setup_s": head["setup_s"],
    }
    if "consecutive_steps" in head:
        out["consecutive_steps"] = head["consecutive_steps"]
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
