"""The CPU oracle over disjoint record ranges on several host cores.

Test infrastructure, like the rest of this directory: only tests, the smoke check and the
benchmark's CPU-baseline leg may import it.  Records are independent (every operator computes on
one row; Section 3, "Extract features"), so the single-threaded oracle can be called on disjoint
ranges of records from several threads (it keeps no state between calls, and ctypes releases the
interpreter lock during a call); its per-range results laid end to end are its result on the whole
batch.  The oracle itself (fbx_oracle.c) is untouched by this and stays single-threaded.
"""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from oracle import fbx_oracle as O


def host_workers(limit=16):
    return max(1, min(limit, os.cpu_count() or 1))


def extract_ranges(spec, raw, off, pool, pieces):
    """[(first record, count, OracleResult)] for `pieces` disjoint ranges that cover the records."""
    n = len(off) - 1
    cuts = np.unique(np.linspace(0, n, pieces + 1).astype(np.int64))
    jobs = []
    for a, b in zip(cuts[:-1], cuts[1:]):
        a, b = int(a), int(b)
        lo, hi = int(off[a]), int(off[b])
        jobs.append((a, b - a, pool.submit(O.extract, spec, raw[lo:hi], off[a:b + 1] - off[a])))
    return [(a, c, f.result()) for a, c, f in jobs]


def extract_parallel(spec, raw, off, workers=None):
    """{slot: (values, offsets, arity)}, n_values_total, n_malformed of the whole batch, computed range by range."""
    workers = workers or host_workers()
    raw = np.ascontiguousarray(raw, dtype=np.uint8)
    off = np.ascontiguousarray(off, dtype=np.uint64)
    with ThreadPoolExecutor(workers) as pool:
        parts = extract_ranges(spec, raw, off, pool, workers * 2)
    slots, total, malformed = {}, 0, 0
    for s in parts[0][2].slot_ids:
        vals = np.concatenate([p.slots[s][0] for _, _, p in parts])
        offs, base = [np.zeros(1, np.uint64)], np.uint64(0)
        for _, _, p in parts:
            offs.append(p.slots[s][1][1:] + base)
            base = base + p.slots[s][1][-1]
        slots[s] = (vals, np.concatenate(offs), parts[0][2].slots[s][2])
    for _, _, p in parts:
        total += p.n_values_total
        malformed += p.n_malformed_numeric
    return slots, parts[0][2].slot_ids, total, malformed
