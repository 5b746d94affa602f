#!/usr/bin/env python3
"""Benchmark of the feature-extraction hot path on one MI355X.

A step is one fbx_extract call: the whole path (every kernel the call enqueues
plus its one synchronisation) over one batch of synthetic records that is
already resident in HBM.  Prints ONE JSON line: records/s, signs/s, the roofline
of the dominant kernel (HIP-event time on the call's stream, measured live), and
the CPU oracle timed on a bounded sample of the same workload.
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

HBM_PEAK_GBPS = 8000.0
# vector instructions the chip can issue per second: one per wavefront, SIMD and 4 cycles
# (256 compute units x 4 SIMDs x 2.4 GHz / 4); 64 lanes each, i.e. the 157.3 TFLOP/s fp32 vector
# peak counted in (packed, fused) instructions instead of flops
VALU_PEAK_PER_S = 256 * 4 * 2.4e9 / 4

# HBM traffic of one launch of the dominant kernel as rocprofv3 counted it (FETCH_SIZE and
# WRITE_SIZE, each scaled by what the same counter reads for a device-to-device copy of known
# size), for the workloads that were profiled: see profiles/.  Other runs report null.
MEASURED_TRAFFIC = {
    # (workload, records, launch sequence, compiled for the plan): bytes per launch; profiles/k_tile_config5_hbm_traffic.md
    ("config5", 16000000, "one_launch", 1): 42406717805,
    ("config5", 16000000, "one_launch", 0): 42386037351,
}
# Vector instructions (SQ_INSTS_VALU) of one launch of the dominant kernel, same keys;
# profiles/k_tile_config5_instruction_mix.md
MEASURED_VALU = {
    ("config5", 16000000, "one_launch", 1): 7693398336,
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_inputs(w, chunk_records=500_000):
    """Generate the workload chunk by chunk on the host and assemble it in HBM."""
    import numpy as np
    import torch

    n = w.n_records
    probe, _ = w.generate(0, min(n, 2048))
    est = int(probe.size / min(n, 2048) * n * 1.03) + (1 << 20)
    d_raw = torch.empty(est, dtype=torch.uint8, device="cuda")
    d_off = torch.empty(n + 1, dtype=torch.int64, device="cuda")
    pos, r = 0, 0
    t0 = time.time()
    while r < n:
        m = min(chunk_records, n - r)
        raw, off = w.generate(r, m)
        if pos + raw.size > d_raw.numel():
            grown = torch.empty(int((pos + raw.size) * 1.1), dtype=torch.uint8, device="cuda")
            grown[:pos].copy_(d_raw[:pos])
            d_raw = grown
        d_raw[pos:pos + raw.size].copy_(torch.from_numpy(raw))
        d_off[r:r + m].copy_(torch.from_numpy((off[:-1] + np.uint64(pos)).astype(np.int64)))
        pos += raw.size
        r += m
        log(f"[bench] generated {r}/{n} records, {pos / 1e9:.2f} GB, {time.time() - t0:.0f}s")
    d_off[n:].fill_(pos)
    torch.cuda.synchronize()
    return d_raw[:pos], d_off


def cpu_baseline(w, budget_s=12.0):
    """The oracle as it stands, single-threaded, on the first records of the workload."""
    from oracle import fbx_oracle as O

    n = min(256, w.n_records)
    raw, off = w.generate(0, n)
    t = time.time()
    O.extract(w.spec, raw, off)
    dt = max(time.time() - t, 1e-4)
    m = int(min(w.n_records, max(n, n * budget_s / dt)))
    raw, off = w.generate(0, m)
    t = time.time()
    res = O.extract(w.spec, raw, off)
    dt = time.time() - t
    return {"value": m / dt, "unit": "records/s", "cores": 1, "kind": "oracle",
            "signs_per_s": res.n_values_total / dt,
            "sample": f"first {m} records of {w.name} ({raw.size / 1e6:.1f} MB), {dt:.1f} s, single thread"}


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
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="only run a device-to-device copy of this many MiB (3 times) and exit: the known "
                         "traffic against which FETCH_SIZE / WRITE_SIZE readings of rocprofv3 are scaled")
    args = ap.parse_args()
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
    w = W.get(args.config, args.records)
    log(f"[bench] workload {w.name}: {w.n_records} records x {w.n_fields} fields, {w.n_ops} ops, {w.n_layers} layers")
    d_raw, d_off = build_inputs(w)
    raw_len, R = d_raw.numel(), w.n_records

    plan = B.Plan(w.spec)
    plan.set_option("profile", 1)
    plan.set_option("fused", args.fused)
    plan.set_option("compile", args.compile)
    if args.lds_pad:
        plan.set_option("lds_pad", args.lds_pad)
    for kv in args.opt:
        k, v = kv.split("=")
        plan.set_option(k, int(v))
    res, ws = B.extract_with_retry(plan, d_raw, d_off, slack=1.03)  # a few percent of headroom, as a serving loop would keep
    log(f"[bench] workspace {ws.numel() / 1e9:.2f} GB, {res.n_values_total} signs, "
        f"{len(res.slot_ids)} slots, malformed {res.n_malformed_numeric}")

    notes = [res.note] if res.note else []
    for _ in range(args.warmup):
        r = plan.extract(d_raw, d_off)
        if r.note:
            notes.append(r.note)
    torch.cuda.synchronize()
    n_compiled, compile_ms = plan.compiled()
    if args.compile:
        log(f"[bench] {n_compiled} tile kernels compiled for the plan in {compile_ms / 1e3:.1f} s (before the timed calls)")
    kernel_ms = {}
    t0 = time.perf_counter()
    for _ in range(args.steps):
        res = plan.extract(d_raw, d_off)
        for which in [0, 1, 2, 3] + [101 + k for k in range(1 if args.fused else w.n_layers)]:
            try:
                kernel_ms.setdefault(which, []).append(plan.kernel_ms(which))
            except B.FbxError:
                pass
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    # reading the event times sits inside the timed loop: a few microseconds per step

    ms_per_step = elapsed / args.steps * 1e3
    n_signs = res.n_values_total
    n_ragged_emitted = sum(1 for s in res.slot_ids if res.slots[s].offsets is not None)
    alg_bytes = raw_len + 8 * (R + 1) + 8 * n_signs + 8 * (R + 1) * n_ragged_emitted

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

    out = {
        "metric": "records/s", "value": R / (ms_per_step * 1e-3), "unit": "records/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u64", "data": "synthetic",
        "config": {"workload": w.name, "records": R, "fields": w.n_fields, "ops": w.n_ops, "layers": w.n_layers,
                   "raw_bytes": raw_len, "signs": int(n_signs), "launch": launch, "compile": args.compile},
        "signs_per_s": n_signs / (ms_per_step * 1e-3),
        "path_algorithmic_GBps": alg_bytes / (ms_per_step * 1e-3) / 1e9,
        "path_frac_of_hbm_peak": alg_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "kernel_ms": kernels,
        "roofline": {"bound": "hbm", "kernel": kname,
                     "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": MEASURED_TRAFFIC.get((w.name, R, launch, args.compile)),
                     "algorithmic_bytes_per_launch": int(launches[dom]), "avg_launch_ms": dom_ms},
    }
    valu = MEASURED_VALU.get((w.name, R, launch, args.compile))
    if valu:
        # what actually bounds the kernel: vector instruction issue.  The count per launch is the
        # profiled one, the duration this run's.
        rate = valu / (dom_ms * 1e-3)
        out["roofline_alu"] = {"bound": "alu", "kernel": kname, "achieved": rate, "peak": VALU_PEAK_PER_S,
                               "unit": "wavefront vector instructions/s", "frac": rate / VALU_PEAK_PER_S,
                               "valu_instructions_per_launch": valu, "per_record": valu / R}
    if args.compile:
        # host time spent compiling, all of it before the timed calls unless compiled_in_timed_calls says otherwise
        out["compile"] = {"kernels": compiled_now, "ms": round(plan.compiled()[1], 1),
                          "compiled_in_timed_calls": compiled_now - n_compiled}
    if res.note:
        notes.append(res.note)
    if notes:
        out["note"] = "; ".join(dict.fromkeys(notes))
    if not args.no_cpu:
        log("[bench] timing the CPU oracle on a bounded sample ...")
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out), flush=True)
    plan.close()


if __name__ == "__main__":
    main()
