"""The CPU oracle over disjoint record ranges on all host cores, and a complete comparison of a
large GPU result with it, chunk by chunk.

Test infrastructure: records are independent (every operator computes on one row; Section 3,
"Extract features"), so the single-threaded oracle can be called on disjoint ranges of records
from several threads (it keeps no state between calls and ctypes releases the interpreter lock
during a call) and its per-range results laid end to end are its result on the whole batch.
The oracle itself is untouched; nothing in the product package imports this module.
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


def check_every_sign(spec, res, d_raw, d_off, chunk_records=250_000, workers=None, label="", progress=None):
    """Every slot's values and offsets of a GPU result (binding.ExtractResult over device buffers
    d_raw / d_off) against the oracle, byte for byte: records are taken in chunks, each chunk's text
    is copied to the host, the oracle runs on sub-ranges of it on all cores, and every slot's
    slice of the result is copied back and compared.  Returns (signs compared, malformed numerics
    the oracle counted)."""
    workers = workers or host_workers()
    R = d_off.numel() - 1
    assert res.n_records == R, label
    slot_ids = list(res.slot_ids)
    running = {s: 0 for s in slot_ids}      # signs of the records before the chunk, per slot
    compared = malformed = 0
    with ThreadPoolExecutor(workers) as pool:
        for first in range(0, R, chunk_records):
            count = min(chunk_records, R - first)
            off = d_off[first:first + count + 1].cpu().numpy().astype(np.uint64)
            raw = d_raw[int(off[0]):int(off[-1])].cpu().numpy()
            parts = extract_ranges(spec, raw, off - off[0], pool, workers * 2)
            assert sorted(parts[0][2].slot_ids) == sorted(slot_ids), label
            malformed += sum(p.n_malformed_numeric for _, _, p in parts)

            def one_slot(s):
                slot = res.slots[s]
                arity = parts[0][2].slots[s][2]
                assert slot.fixed_arity == arity, f"{label} slot {s}: arity"
                want_v = np.concatenate([p.slots[s][0] for _, _, p in parts])
                n = want_v.size
                lo = running[s]
                if slot.offsets is None:
                    assert lo == first * arity and n == count * arity, f"{label} slot {s}: sign count"
                else:
                    want_o, base = [np.full(1, lo, np.uint64)], np.uint64(lo)
                    for _, _, p in parts:
                        want_o.append(p.slots[s][1][1:] + base)
                        base = base + p.slots[s][1][-1]
                    got_o = slot.offsets[first:first + count + 1].cpu().numpy().view(np.uint64)
                    assert np.array_equal(got_o, np.concatenate(want_o)), \
                        f"{label} slot {s}: offsets of records {first}..{first + count} differ"
                got_v = slot.values[lo:lo + n].cpu().numpy().view(np.uint64)
                if not np.array_equal(got_v, want_v):
                    bad = np.nonzero(got_v != want_v)[0] if got_v.size == want_v.size else [-1]
                    raise AssertionError(f"{label} slot {s}: signs of records {first}..{first + count} differ "
                                         f"({len(bad)} of {n}, first at {lo + int(bad[0])})")
                return n

            for s, n in zip(slot_ids, pool.map(one_slot, slot_ids)):
                running[s] += n
                compared += n
            if progress:
                progress(first + count, R)
    for s in slot_ids:
        assert running[s] == res.slots[s].n_values, f"{label} slot {s}: {running[s]} signs compared, {res.slots[s].n_values} reported"
    assert compared == res.n_values_total, label
    assert malformed == res.n_malformed_numeric, label
    return compared, malformed
