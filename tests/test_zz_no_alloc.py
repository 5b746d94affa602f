"""The entry point that allocates nothing (fbx_extract_static) against fbx_extract, through the C ABI."""
import numpy as np
import pytest

from paper_2210_07768_amd import binding as B
from paper_2210_07768_amd import workloads as W
from gpu_harness import expand, to_device

pytestmark = pytest.mark.gpu


def _same(a, b, n, label):
    assert list(a.slot_ids) == list(b.slot_ids), label
    assert a.n_values_total == b.n_values_total and a.n_malformed_numeric == b.n_malformed_numeric, label
    for s in a.slot_ids:
        av, ao = expand(a.slots[s], n)
        bv, bo = expand(b.slots[s], n)
        assert a.slots[s].fixed_arity == b.slots[s].fixed_arity, f"{label} slot {s}"
        assert np.array_equal(ao, bo), f"{label} slot {s}: offsets differ"
        assert np.array_equal(av, bv), f"{label} slot {s}: signs differ"


def test_static_entry_point_matches_extract_on_two_calls_in_a_row():
    """Two calls in a row on the library's own table array, the second with a smaller input (and
    another plan, so that the tables there change hands), each against fbx_extract with a workspace;
    then the first plan again, whose second call knows its ragged sizes and places in one launch."""
    import torch

    assert B.lib().fbx_static_scratch_bytes() == 64 << 20
    cases = [(W.get(4, 3000), 0), (W.get(5, 700), 0), (W.get(4, 3000), 0)]
    plans = {}
    out = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
    for w, begin in cases:
        raw, off = w.generate(begin, w.n_records)
        n = w.n_records
        d_raw, d_off = to_device(raw, off)
        ref_plan = B.Plan(w.spec)
        ref, ws = B.extract_with_retry(ref_plan, d_raw, d_off)
        plan = plans.get(w.name) or B.Plan(w.spec)
        plans[w.name] = plan
        out.fill_(0x77)
        got = plan.extract(d_raw, d_off, out_buffer=out)
        _same(got, ref, n, f"{w.name} static")
        out.fill_(0x99)
        again = plan.extract(d_raw, d_off, out_buffer=out)   # (sizes known now: one launch where the plan allows it)
        _same(again, ref, n, f"{w.name} static, second call")
        ref_plan.close()
    # an output buffer that is too small says how much would do, and that much does
    w = W.get(2, 500)
    raw, off = w.generate()
    d_raw, d_off = to_device(raw, off)
    plan = B.Plan(w.spec)
    with pytest.raises(B.FbxError) as e:
        plan.extract(d_raw, d_off, out_buffer=out[:4096])
    assert e.value.status == B.E_NOMEM and e.value.required_bytes > 4096
    need = e.value.required_bytes
    got = plan.extract(d_raw, d_off, out_buffer=out[:need])
    ref_plan = B.Plan(w.spec)
    ref, ws = B.extract_with_retry(ref_plan, d_raw, d_off)
    _same(got, ref, 500, "config2 static, exact buffer")
    # a batch whose tables outgrow the array is refused with a clear message, before anything runs
    spec = "fbx 1\nfields 1\n" + "".join(f"op m{k} hash slot={k} seed={k} emit=1 field=0 multi=1\n" for k in range(40))
    recs = [b"a,b\n"] * 200_000
    big = B.Plan(spec)
    big.set_option("tile_log2", 0)          # one record a tile: 200,000 tiles x 40 ragged operators x 12 bytes
    raw = np.frombuffer(b"".join(recs), np.uint8)
    off = np.arange(len(recs) + 1, dtype=np.uint64) * 4
    d_raw, d_off = to_device(raw, off)
    with pytest.raises(B.FbxError) as e:
        big.extract(d_raw, d_off, out_buffer=out)
    assert e.value.status == B.E_ARG and "allocates nothing" in str(e.value)
    for p in list(plans.values()) + [plan, ref_plan, big]:
        p.close()
