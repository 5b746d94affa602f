"""Helpers for the GPU parity tests: run libfbx through its C ABI binding and
compare every emitted slot with the CPU oracle, bit for bit."""
import numpy as np

from oracle import fbx_oracle as O
from paper_2210_07768_amd import binding as B


def to_device(raw: np.ndarray, off: np.ndarray, misalign: int = 0):
    import torch

    buf = torch.empty(raw.size + misalign + 64, dtype=torch.uint8, device="cuda")
    d_raw = buf[misalign:misalign + raw.size]
    if raw.size:
        d_raw.copy_(torch.from_numpy(np.array(raw, dtype=np.uint8)))
    d_off = torch.from_numpy(np.ascontiguousarray(off).astype(np.int64)).cuda()
    return d_raw, d_off


def expand(slot, n_records):
    """(values, explicit offsets) as numpy uint64 from a binding Slot."""
    vals = slot.values.cpu().numpy().view(np.uint64)
    if slot.offsets is None:
        offs = (np.arange(n_records + 1, dtype=np.uint64) * np.uint64(slot.fixed_arity))
    else:
        offs = slot.offsets.cpu().numpy().view(np.uint64)
    return vals, offs


def run_gpu(spec, raw, off, options=None, misalign=0, workspace_bytes=None):
    plan = B.Plan(spec)
    for k, v in (options or {}).items():
        plan.set_option(k, v)
    d_raw, d_off = to_device(np.asarray(raw, dtype=np.uint8), np.asarray(off, dtype=np.uint64), misalign)
    if workspace_bytes is None:
        res, ws = B.extract_with_retry(plan, d_raw, d_off)
    else:
        import torch
        ws = torch.empty(workspace_bytes, dtype=torch.uint8, device="cuda")
        plan.set_workspace(ws)
        res = plan.extract(d_raw, d_off)
    n = len(off) - 1
    out = {s: expand(res.slots[s], n) for s in res.slot_ids}
    return out, res, plan


def assert_same(gpu_out, gpu_res, oracle_res, label=""):
    assert sorted(gpu_out) == sorted(oracle_res.slots), label
    for s in oracle_res.slot_ids:
        ov, oo, arity = oracle_res.slots[s]
        gv, go = gpu_out[s]
        assert gpu_res.slots[s].fixed_arity == arity, f"{label} slot {s} arity"
        assert np.array_equal(go, oo), f"{label} slot {s}: offsets differ"
        if not np.array_equal(gv, ov):
            bad = np.nonzero(gv != ov)[0]
            raise AssertionError(f"{label} slot {s}: {bad.size} of {ov.size} signs differ, first at {bad[0]}")
    assert gpu_res.n_values_total == oracle_res.n_values_total, label
    assert gpu_res.n_malformed_numeric == oracle_res.n_malformed_numeric, label


def check(spec, raw, off, options=None, misalign=0, label=""):
    raw = np.frombuffer(raw, dtype=np.uint8) if isinstance(raw, (bytes, bytearray)) else np.asarray(raw, np.uint8)
    off = np.asarray(off, dtype=np.uint64)
    want = O.extract(spec, raw, off)
    out, res, plan = run_gpu(spec, raw, off, options, misalign)
    assert_same(out, res, want, label)
    plan.close()
    return res, want


def device_workload(w, chunk_records=500_000):
    """A whole synthetic workload assembled in device memory chunk by chunk: (raw bytes, record offsets)."""
    import torch

    n = w.n_records
    probe, _ = w.generate(0, min(n, 2048))
    est = int(probe.size / min(n, 2048) * n * 1.03) + (1 << 20)
    d_raw = torch.empty(est, dtype=torch.uint8, device="cuda")
    d_off = torch.empty(n + 1, dtype=torch.int64, device="cuda")
    pos = r = 0
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
    d_off[n:].fill_(pos)
    torch.cuda.synchronize()
    return d_raw[:pos], d_off


def check_window(spec, res, d_raw, d_off, first, count, label=""):
    """Records [first, first + count) of a large result against the oracle run on just those records."""
    off = d_off[first:first + count + 1].cpu().numpy().astype(np.uint64)
    raw = d_raw[int(off[0]):int(off[-1])].cpu().numpy()
    want = O.extract(spec, raw, off - off[0])
    assert sorted(res.slot_ids) == sorted(want.slots), label
    for s in want.slot_ids:
        ov, oo, arity = want.slots[s]
        slot = res.slots[s]
        assert slot.fixed_arity == arity, f"{label} slot {s} arity"
        if slot.offsets is None:
            lo, hi = first * arity, (first + count) * arity
        else:
            go = slot.offsets[first:first + count + 1].cpu().numpy().view(np.uint64)
            assert np.array_equal(go - go[0], oo), f"{label} slot {s}: offsets of records {first}.. differ"
            lo, hi = int(go[0]), int(go[-1])
        gv = slot.values[lo:hi].cpu().numpy().view(np.uint64)
        assert np.array_equal(gv, ov), f"{label} slot {s}: signs of records {first}..{first + count} differ"
