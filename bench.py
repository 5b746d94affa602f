#!/usr/bin/env python3
"""Benchmark of the feature-extraction hot path on one MI355X.

A step is one fbx_extract call: the whole path (every kernel the call enqueues
plus its one synchronisation) over one batch of synthetic records that is
already resident in HBM.  Two batches of the workload are held in HBM (records
[0, R) and [R, 2R) of the same generator) and the timed calls alternate between
them, so that every timed call sizes its ragged arrays from a call on *other*
records, as a pipeline's calls do.  Prints ONE JSON line: records/s, signs/s,
the roofline of the dominant kernel (HIP-event time on the call's stream,
measured live), what the first-call launch sequence costs, how many timed calls
fell back to it, and the CPU oracle timed on a bounded sample of the same
workload (all host cores, and one thread).
"""
from __future__ import annotations

import argparse
import glob
import hashlib
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
# vector instructions the chip can issue per second: one per wavefront, SIMD and 4 cycles
# (256 compute units x 4 SIMDs x 2.4 GHz / 4); 64 lanes each, i.e. the 157.3 TFLOP/s fp32 vector
# peak counted in (packed, fused) instructions instead of flops
VALU_PEAK_PER_S = 256 * 4 * 2.4e9 / 4


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def source_digest() -> str:
    """Digest of the kernel and host sources of the library: counter readings in profiles/ name the
    digest they were taken at and are quoted only while it still matches."""
    h = hashlib.sha256()
    files = sorted(f for f in glob.glob(os.path.join(ROOT, "paper_2210_07768_amd", "csrc", "*"))
                   if os.path.basename(f) != "fbx_clean.hip")     # (the cleaning stage is no part of the extraction path)
    for f in files + [os.path.join(ROOT, "include", "fbx.h")]:
        if os.path.isfile(f):
            h.update(os.path.basename(f).encode() + b"\0" + open(f, "rb").read() + b"\0")
    return h.hexdigest()[:16]


def measured_counters(workload, records, launch, compile_for_plan):
    """Counter readings of the dominant kernel for this configuration from the summaries in
    profiles/ (lines that start with 'bench-key:'), or {} when none was taken at these sources."""
    want = {"workload": workload, "records": str(records), "launch": launch, "compile": str(compile_for_plan),
            "sources": source_digest()}
    found = {}
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.md"))):
        for line in open(path):
            if not line.startswith("bench-key:"):
                continue
            kv = dict(item.split("=", 1) for item in line[len("bench-key:"):].split())
            if all(kv.get(k) == v for k, v in want.items()):
                found.update({k: int(v) for k, v in kv.items() if k not in want})
    return found


def build_inputs(w, first_record=0, chunk_records=500_000, tag=""):
    """Generate records [first_record, first_record + n) chunk by chunk on the host and assemble them in HBM."""
    import numpy as np
    import torch

    n = w.n_records
    probe, _ = w.generate(first_record, min(n, 2048))
    est = int(probe.size / min(n, 2048) * n * 1.03) + (1 << 20)
    d_raw = torch.empty(est, dtype=torch.uint8, device="cuda")
    d_off = torch.empty(n + 1, dtype=torch.int64, device="cuda")
    pos, r = 0, 0
    t0 = time.time()
    while r < n:
        m = min(chunk_records, n - r)
        raw, off = w.generate(first_record + r, m)
        if pos + raw.size > d_raw.numel():
            grown = torch.empty(int((pos + raw.size) * 1.1), dtype=torch.uint8, device="cuda")
            grown[:pos].copy_(d_raw[:pos])
            d_raw = grown
        d_raw[pos:pos + raw.size].copy_(torch.from_numpy(raw))
        d_off[r:r + m].copy_(torch.from_numpy((off[:-1] + np.uint64(pos)).astype(np.int64)))
        pos += raw.size
        r += m
        if r == n or (r // chunk_records) % 8 == 0:
            log(f"[bench] batch {tag}: generated {r}/{n} records, {pos / 1e9:.2f} GB, {time.time() - t0:.0f}s")
    d_off[n:].fill_(pos)
    torch.cuda.synchronize()
    return d_raw[:pos], d_off


def cpu_baseline(w, budget_s=10.0):
    """The oracle as it stands on the first records of the workload: over disjoint record ranges on
    all host cores (the figure reported as `value`), and in one thread."""
    from concurrent.futures import ThreadPoolExecutor

    from oracle import fbx_oracle as O
    from oracle import ranges

    n = min(256, w.n_records)
    raw, off = w.generate(0, n)
    t = time.time()
    O.extract(w.spec, raw, off)
    dt = max(time.time() - t, 1e-4)
    m1 = int(min(w.n_records, max(n, n * budget_s / dt)))
    raw, off = w.generate(0, m1)
    t = time.time()
    res = O.extract(w.spec, raw, off)
    dt1 = time.time() - t
    cores = ranges.host_workers()
    mc = int(min(w.n_records, m1 * cores))
    if mc > m1:
        raw, off = w.generate(0, mc)
    t = time.time()
    with ThreadPoolExecutor(cores) as pool:
        parts = ranges.extract_ranges(w.spec, raw, off, pool, cores * 4)
    dtc = time.time() - t
    signs_c = sum(p.n_values_total for _, _, p in parts)
    return {"value": mc / dtc, "unit": "records/s", "cores": cores, "kind": "oracle",
            "signs_per_s": signs_c / dtc,
            "sample": f"first {mc} records of {w.name} ({raw.size / 1e6:.1f} MB), {dtc:.1f} s on {cores} threads "
                      f"(the single-threaded oracle over disjoint record ranges)",
            "single_thread": {"value": m1 / dt1, "unit": "records/s", "cores": 1, "signs_per_s": res.n_values_total / dt1,
                              "sample": f"first {m1} records, {dt1:.1f} s"}}


def side_stage(args, w, B, torch):
    """Timings of the two stages beside the benchmark line: one ragged operator with in-kernel
    allocation (unordered output) against the same operator through the ordered path, and the toy
    cleaning stage.  HIP events around each call, median of --steps calls; one JSON line."""
    R = w.n_records
    d_raw, d_off = build_inputs(w, 0, tag="A")

    def timed(call):
        for _ in range(max(args.warmup, 1)):
            call()
        ms = []
        for _ in range(args.steps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(); call(); b.record()
            torch.cuda.synchronize()
            ms.append(a.elapsed_time(b))
        return statistics.median(ms)

    if args.stage == "unordered":
        line = next(ln for ln in w.spec.split("\n") if " multi=1" in ln and " emit=1" in ln)
        slot = int(line.split("slot=")[1].split()[0])
        spec = "\n".join(w.spec.split("\n")[:2] + [line]) + "\n"
        plan = B.Plan(spec)
        res, ws = B.extract_with_retry(plan, d_raw, d_off, slack=1.1)
        n_signs = res.n_values_total
        pool = torch.empty(int(8 * n_signs * 1.05) + (R // 256 + 1) * 128 + 4096, dtype=torch.uint8, device="cuda")
        state = torch.zeros(4, dtype=torch.int64, device="cuda")
        toff = torch.empty(R, dtype=torch.int64, device="cuda")
        lens = torch.empty(R, dtype=torch.int32, device="cuda")
        t_un = timed(lambda: plan.extract_unordered(slot, d_raw, d_off, pool, state, toff, lens))
        plan.set_option("one_launch", 0)
        t_cw = timed(lambda: plan.extract(d_raw, d_off))
        plan.set_option("one_launch", 1)
        plan.extract(d_raw, d_off)
        t_one = timed(lambda: plan.extract(d_raw, d_off))
        plan.set_option("placement", 1)
        t_arr = timed(lambda: plan.extract(d_raw, d_off))
        alg = d_raw.numel() + 8 * (R + 1) + 8 * n_signs + 8 * (R + 1)
        print(json.dumps({"stage": "unordered", "workload": w.name, "records": R, "operator": line, "signs": int(n_signs),
                          "ms": {"in_kernel_allocation_unordered": t_un, "ordered_count_scan_write": t_cw, "ordered_one_launch_look_back": t_one,
                                 "tile_kernel_arrival_order": t_arr},
                          "algorithmic_GBps": {"in_kernel_allocation_unordered": alg / t_un / 1e6, "ordered_count_scan_write": alg / t_cw / 1e6,
                                               "ordered_one_launch_look_back": alg / t_one / 1e6, "tile_kernel_arrival_order": alg / t_arr / 1e6},
                          "note": "the operator's field is one of many: every variant reads the whole text once (twice with a counting launch)"}))
        plan.close()
        return
    k = next(i for i, f in enumerate(w.fields) if f.kind == 0)   # a single-valued categorical field
    spec = ("fbxclean 1\n" + f"fields {w.n_fields}\n" + f"fill field={k} value={b'none'.hex()}\n"
            + f"keep field={k} prefix=\n" + f"fill field={w.n_fields - 1} value=30\n")
    clean = B.Clean(spec)
    scratch = torch.empty(clean.scratch_hint(R), dtype=torch.uint8, device="cuda")
    d_out = torch.empty(d_raw.numel() + 8 * R, dtype=torch.uint8, device="cuda")
    d_out_off = torch.empty(R + 1, dtype=torch.int64, device="cuda")
    res = clean.run(d_raw, d_off, d_out, d_out_off, scratch)
    t = timed(lambda: clean.run(d_raw, d_off, d_out, d_out_off, scratch))
    alg = d_raw.numel() + 8 * (R + 1) + res.out_len + 8 * (res.n_kept + 1)
    print(json.dumps({"stage": "clean", "workload": w.name, "records": R, "kept": int(res.n_kept), "spec": spec, "ms": t,
                      "algorithmic_GBps": alg / t / 1e6, "frac_of_hbm_peak": alg / t / 1e6 / HBM_PEAK_GBPS,
                      "note": "two launches over tiles of records staged in LDS (measure, write) and a scan between them"}))
    clean.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=5, help="workload 1..5 (default: the largest)")
    ap.add_argument("--records", type=int, default=None, help="override the record count (debugging)")
    ap.add_argument("--fused", type=int, default=1)
    ap.add_argument("--lds-pad", type=int, default=0)
    ap.add_argument("--compile", type=int, default=1,
                    help="1: the tile kernel is compiled for the plan at run time, during the warm-up calls "
                         "(plan option compile, default); 0: the generic kernel")
    ap.add_argument("--opt", action="append", default=[], metavar="KEY=VALUE",
                    help="extra plan option (tuning), e.g. --opt tile_log2=4")
    ap.add_argument("--one-batch", action="store_true",
                    help="time every call on the batch the sizes were learned on (what profiles of one kernel use)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-arrival", action="store_true", help="skip the calls with ragged slots placed in arrival order")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="only run a device-to-device copy of this many MiB (3 times) and exit: the known "
                         "traffic against which FETCH_SIZE / WRITE_SIZE readings of rocprofv3 are scaled")
    ap.add_argument("--launch-overhead", action="store_true",
                    help="only measure what Table 1 of the paper measures, on this device, and exit: 1 / 10 / 100 / "
                         "1,000 / 10,000 back-to-back launches of an empty kernel with five pointer arguments")
    ap.add_argument("--stage", choices=["extract", "unordered", "clean"], default="extract",
                    help="what to time: the extraction path (default, the benchmark line); 'unordered': one ragged "
                         "operator of layer 1 with in-kernel allocation (fbx_extract_unordered) beside the ordered path "
                         "on a plan that holds only that operator; 'clean': the toy cleaning stage (fbx_clean_run)")
    ap.add_argument("--print-source-digest", action="store_true",
                    help="print the digest of the library's sources that counter summaries in profiles/ are keyed on")
    args = ap.parse_args()
    if args.print_source_digest:
        print(source_digest())
        return
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (records are independent: a batch shards by record range); use --gpus 1")

    import numpy as np
    import torch

    from paper_2210_07768_amd import binding as B
    from paper_2210_07768_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.copy_calibration:
        src = torch.empty(args.copy_calibration << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": src.numel(), "copy_bytes_written": src.numel(), "copies": 3}))
        return
    B.lib()  # fails loudly when libfbx.so is missing
    if args.launch_overhead:
        st = torch.cuda.current_stream().cuda_stream
        B.launch_overhead(100, st)   # (the first launch of a kernel loads its code)
        table = {}
        for n in (1, 10, 100, 1000, 10000):
            runs = sorted(B.launch_overhead(n, st) for _ in range(7))
            table[str(n)] = {"median_us": round(runs[3], 2), "min_us": round(runs[0], 2), "per_launch_us": round(runs[3] / n, 3)}
        print(json.dumps({"empty_kernel_launches": table, "arguments": "five pointers", "timed": "host clock, first launch call to end of stream wait",
                          "paper_table_1_us_on_V100": {"1": 4, "10": 35, "100": 360, "1000": 3619, "10000": 34515}}))
        return
    w = W.get(args.config, args.records)
    R = w.n_records
    log(f"[bench] workload {w.name}: {R} records x {w.n_fields} fields, {w.n_ops} ops, {w.n_layers} layers")
    if args.stage != "extract":
        side_stage(args, w, B, torch)
        return
    batches = [build_inputs(w, 0, tag="A")]
    if not args.one_batch:
        batches.append(build_inputs(w, R, tag="B"))

    plan = B.Plan(w.spec)
    plan.set_option("profile", 1)
    plan.set_option("fused", args.fused)
    plan.set_option("compile", args.compile)
    if args.lds_pad:
        plan.set_option("lds_pad", args.lds_pad)
    for kv in args.opt:
        k, v = kv.split("=")
        plan.set_option(k, int(v))
    # the first call sizes the workspace (a few percent of headroom, as a serving loop would keep; both batches must fit)
    res, ws = B.extract_with_retry(plan, *batches[0], slack=1.05)
    log(f"[bench] workspace {ws.numel() / 1e9:.2f} GB, {res.n_values_total} signs, "
        f"{len(res.slot_ids)} slots, malformed {res.n_malformed_numeric}")

    notes = [res.note] if res.note else []
    for i in range(max(args.warmup, 1 if len(batches) > 1 else 0)):
        r = plan.extract(*batches[(i + 1) % len(batches)])
        if r.note:
            notes.append(r.note)
    torch.cuda.synchronize()
    n_compiled, compile_ms = plan.compiled()
    if args.compile:
        log(f"[bench] {n_compiled} tile kernels compiled for the plan in {compile_ms / 1e3:.1f} s (before the timed calls)")

    # what a call costs that cannot use the sizes of the call before it (a plan's first call, or a
    # batch that outgrows its arrays): counting launch, scan, writing launch, with compiled kernels
    cold = None
    if res.tile_launches and args.fused:
        plan.set_option("one_launch", 0)
        t0 = time.perf_counter()
        rc = plan.extract(*batches[0])
        torch.cuda.synchronize()
        cold = {"ms": (time.perf_counter() - t0) * 1e3, "tile_launches": rc.tile_launches, "kernel_ms": {}}
        for which, name in ((1, "count"), (2, "scan"), (3, "alloc"), (101, "tile")):
            try:
                cold["kernel_ms"][name] = round(plan.kernel_ms(which), 4)
            except B.FbxError:
                pass
        plan.set_option("one_launch", 1)
        for kv in args.opt:  # (an explicit one_launch=0 on the command line stays)
            k, v = kv.split("=")
            if k == "one_launch":
                plan.set_option(k, int(v))

    kernel_ms, step_ms, step_bytes, fell_back = {}, [], [], 0
    events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    first_timed = len(batches) - 1   # (the cold call above ran on batch A: the first timed call takes the other one)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    # (inside the timed loop: the call, two event records and the library's own kernel timers, which the
    # next call overwrites; what the results hold is looked at afterwards)
    timer_ids = [0, 1, 2, 3] + [101 + k for k in range(1 if args.fused else w.n_layers)]
    results = []
    for i in range(args.steps):
        d_raw, d_off = batches[(first_timed + i) % len(batches)]
        events[i][0].record()
        res = plan.extract(d_raw, d_off)
        events[i][1].record()
        results.append((res, plan.kernel_ms_all(timer_ids)))
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    step_ms = [a.elapsed_time(b) for a, b in events]
    for i, (res, timers) in enumerate(results):
        for which, ms in timers.items():
            kernel_ms.setdefault(which, []).append(ms)
        n_ragged_emitted = sum(1 for s in res.slot_ids if res.slots[s].offsets is not None)
        step_bytes.append(batches[(first_timed + i) % len(batches)][0].numel() + 8 * (R + 1) + 8 * res.n_values_total
                          + 8 * (R + 1) * n_ragged_emitted)
        fell_back += 1 if (res.tile_launches == 2 and "fell back" in res.note) else 0

    ms_per_step = elapsed / args.steps * 1e3
    n_signs = res.n_values_total
    alg_bytes = float(np.mean(step_bytes))
    raw_len = batches[(first_timed + args.steps - 1) % len(batches)][0].numel()

    # algorithmic bytes per tile-kernel launch: each input read once, each output written once,
    # intermediates and re-reads count zero
    _, _, layers, _ = plan.info()
    emitted_ops = [i for i, ln in enumerate(w.spec.strip().split("\n")[2:]) if " emit=1" in ln]
    per_layer = {}
    for slot_pos, op in enumerate(emitted_ops):
        s = res.slots[res.slot_ids[slot_pos]]
        b = 8 * s.n_values + (8 * (R + 1) if s.offsets is not None else 0)
        per_layer[layers[op]] = per_layer.get(layers[op], 0) + b
    launches = {}
    if args.fused:
        launches[101] = alg_bytes
    else:
        for l in range(1, w.n_layers + 1):
            launches[100 + l] = per_layer.get(l, 0) + (raw_len + 8 * (R + 1) if l == 1 else 0)
    avg = {k: float(np.mean(v)) for k, v in kernel_ms.items() if v}
    dom = max(launches, key=lambda k: avg.get(k, 0.0))
    dom_ms = avg[dom]
    achieved = launches[dom] / (dom_ms * 1e-3) / 1e9
    names = {0: "validate", 1: "count", 2: "scan", 3: "alloc"}
    kernels = {names.get(k, f"tile_layer{k - 100}" if not args.fused else "tile"): round(v, 4)
               for k, v in sorted(avg.items())}
    if not args.fused:
        launch, kname = "per_layer", f"fbx::k_walk, layer {dom - 100}"
    elif res.tile_launches == 0:
        launch, kname = "walk_fused", "fbx::k_walk"
    elif res.tile_launches == 1:
        # no ragged slot at all: the writing launch alone; else counting and writing in one launch
        has_ragged = any(" multi=1" in ln or " ngram " in ln or " filter " in ln for ln in w.spec.split("\n"))
        launch, kname = ("one_launch", "fbx::k_tile<2>") if has_ragged else ("write", "fbx::k_tile<1>")
    else:
        launch, kname = "count+write", "fbx::k_tile<1>"
    compiled_now = plan.compiled()[0]
    if compiled_now and res.tile_launches and "generic kernel" not in " ".join(notes + [res.note]):
        kname = f"fbx_tile_fixed_{kname[-2]} ({kname} compiled for the plan)"

    counters = measured_counters(w.name, R, launch, args.compile)
    traffic = counters["fetch_bytes"] + counters["write_bytes"] if "fetch_bytes" in counters and "write_bytes" in counters else None
    out = {
        "metric": "records/s", "value": R / (ms_per_step * 1e-3), "unit": "records/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u64", "data": "synthetic",
        "config": {"workload": w.name, "records": R, "fields": w.n_fields, "ops": w.n_ops, "layers": w.n_layers,
                   "raw_bytes": raw_len, "signs": int(n_signs), "launch": launch, "compile": args.compile,
                   "batches": ("one batch, every call on the records its sizes were learned on" if len(batches) == 1 else
                               f"two batches of {R} records alternate: every timed call sizes its ragged arrays from a call on other records")},
        "ms_per_step_median_hip_events": statistics.median(step_ms),
        "signs_per_s": n_signs / (ms_per_step * 1e-3),
        "path_algorithmic_GBps": alg_bytes / (ms_per_step * 1e-3) / 1e9,
        "path_frac_of_hbm_peak": alg_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "kernel_ms": kernels,
        "timed_calls_that_fell_back": fell_back,
        "first_call_sequence": cold,
        "roofline": {"bound": "hbm", "kernel": kname,
                     "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": traffic,
                     "algorithmic_bytes_per_launch": int(launches[dom]), "avg_launch_ms": dom_ms},
    }
    if "valu" in counters:
        # what actually bounds the kernel: vector instruction issue.  The count per launch is the
        # profiled one (same sources, same configuration), the duration this run's.
        rate = counters["valu"] / (dom_ms * 1e-3)
        out["roofline_alu"] = {"bound": "alu", "kernel": kname, "achieved": rate, "peak": VALU_PEAK_PER_S,
                               "unit": "wavefront vector instructions/s", "frac": rate / VALU_PEAK_PER_S,
                               "valu_instructions_per_launch": counters["valu"], "per_record": counters["valu"] / R}
    if args.compile:
        # host time spent compiling, all of it before the timed calls unless compiled_in_timed_calls says otherwise
        out["compile"] = {"kernels": compiled_now, "ms": round(plan.compiled()[1], 1),
                          "compiled_in_timed_calls": compiled_now - n_compiled}
    if res.note:
        notes.append(res.note)
    if notes:
        out["note"] = "; ".join(dict.fromkeys(notes))
    # Beside the line: the same calls with the tiles of a ragged slot placed in the order in which they
    # arrive (plan option placement=1: one atomic add per slot and tile instead of the look-back; each
    # record's lists are the same, the arrays are no longer in record order).  Not the benchmark's
    # value: the path's result is the record-ordered CSR.
    has_ragged = any(s_.offsets is not None for s_ in res.slots.values())
    if args.fused and res.tile_launches and has_ragged and not args.no_arrival and not any(kv.startswith("placement=") for kv in args.opt):
        plan.set_option("placement", 1)
        for i in range(2):  # (compiles the kernel of that mode)
            plan.extract(*batches[(first_timed + i) % len(batches)])
        a_ms, a_kernel, a_res, a_fell = [], [], None, 0
        for i in range(args.steps):
            d_raw, d_off = batches[(first_timed + i) % len(batches)]
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            a_res = plan.extract(d_raw, d_off)
            e1.record()
            torch.cuda.synchronize()
            a_ms.append(e0.elapsed_time(e1))
            a_kernel.append(plan.kernel_ms(101))
            a_fell += 1 if "fell back" in a_res.note else 0
        k_ms = float(np.mean(a_kernel))
        out["arrival_order"] = {"ms_per_step_median_hip_events": statistics.median(a_ms), "tile_kernel_ms": round(k_ms, 4),
                                "records_per_s": R / (statistics.median(a_ms) * 1e-3),
                                "tile_kernel_frac_of_hbm_peak": alg_bytes / (k_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                                "tile_launches": a_res.tile_launches, "arrival_tile_records": a_res.arrival_tile_records,
                                "timed_calls_that_fell_back": a_fell,
                                "note": "plan option placement=1; ragged arrays hold the tiles' shares in arrival order"}
        plan.set_option("placement", 0)
    if not args.no_cpu:
        log("[bench] timing the CPU oracle on a bounded sample ...")
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out), flush=True)
    plan.close()


if __name__ == "__main__":
    main()
