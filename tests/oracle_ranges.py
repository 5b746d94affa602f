"""A complete comparison of a large GPU result with the CPU oracle, chunk by chunk, the oracle
running over disjoint record ranges on all host cores (oracle/ranges.py).  Nothing in the product
package imports this module."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from oracle.ranges import extract_parallel, extract_ranges, host_workers  # noqa: F401  (re-exported for the tests)


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
