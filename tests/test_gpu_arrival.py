"""Plan option placement=1: in a call that skips the counting launch every tile takes its share of a
ragged slot with one atomic add (Section 5, Algorithm 1 with a tile's share as the block), so tiles
land in the order in which they arrive.  What is unique is compared with the oracle (every record's
list of every slot, fixed-arity slots bit for bit in record order), the rest is checked to be valid
(the tiles' shares are disjoint and cover the slot's array)."""
import random

import numpy as np
import pytest

from oracle import fbx_oracle as O
from paper_2210_07768_amd import binding as B
from paper_2210_07768_amd import workloads as W
from helpers import FOLLOW_SPEC, random_dag
from gpu_harness import assert_same, expand, to_device
from oracle_ranges import extract_parallel

pytestmark = pytest.mark.gpu


def assert_same_in_arrival_order(res, want, n, label=""):
    k = res.arrival_tile_records
    assert k > 0 and (k & (k - 1)) == 0, label
    n_tiles = -(-n // k)
    last_of_tile = np.minimum((np.arange(n_tiles) + 1) * k, n) - 1
    assert sorted(res.slot_ids) == sorted(want.slots), label
    total = 0
    for s in want.slot_ids:
        ov, oo, arity = want.slots[s]
        slot = res.slots[s]
        assert slot.fixed_arity == arity, f"{label} slot {s}: arity"
        gv = slot.values.cpu().numpy().view(np.uint64)
        total += gv.size
        if arity:
            assert slot.tile_ends is None and np.array_equal(gv, ov), f"{label} slot {s}: a fixed-arity slot stays in record order"
            continue
        assert gv.size == ov.size, f"{label} slot {s}: sign count"
        start = slot.offsets.cpu().numpy().view(np.uint64)
        ends_of_tiles = slot.tile_ends.cpu().numpy().view(np.uint64)
        assert ends_of_tiles.size == n_tiles and start.size == n + 1
        end = start[1:].copy()
        end[last_of_tile] = ends_of_tiles
        assert start[n] == ends_of_tiles[-1], f"{label} slot {s}: the last record's end"
        begin = start[:n]
        want_len = oo[1:] - oo[:-1]
        assert np.array_equal(end - begin, want_len), f"{label} slot {s}: list lengths differ"
        # every record's list: gather the oracle's signs to where the library put the record
        if ov.size:
            dest = np.repeat(begin - oo[:-1], want_len.astype(np.int64)) + np.arange(ov.size, dtype=np.uint64)
            assert int(dest.max()) < gv.size, f"{label} slot {s}: a list outside the array"
            moved = np.empty_like(ov)
            moved[dest.astype(np.int64)] = ov
            assert np.array_equal(gv, moved), f"{label} slot {s}: signs differ"
        # the tiles' shares: disjoint, end to end, covering the array
        first_of_tile = np.arange(n_tiles) * k
        share_begin = begin[first_of_tile]
        order = np.argsort(share_begin, kind="stable")
        nonempty = order[(ends_of_tiles - share_begin)[order] > 0]
        if nonempty.size:
            assert share_begin[nonempty[0]] == 0 and ends_of_tiles[nonempty[-1]] == gv.size, f"{label} slot {s}: shares do not cover the array"
            assert np.array_equal(share_begin[nonempty[1:]], ends_of_tiles[nonempty[:-1]]), f"{label} slot {s}: shares overlap or leave gaps"
    assert res.n_values_total == want.n_values_total == total, label
    assert res.n_malformed_numeric == want.n_malformed_numeric, label


class _Want:
    """The oracle's result over disjoint record ranges on all host cores, in the shape O.extract gives."""

    def __init__(self, spec, raw, off):
        self.slots, self.slot_ids, self.n_values_total, self.n_malformed_numeric = extract_parallel(spec, raw, off)


def _arrival_calls(spec, raw, off, options, label, want_one_launch=True, may_fall_back=False):
    n = len(off) - 1
    want = O.extract(spec, raw, off) if n < 50_000 else _Want(spec, raw, off)
    plan = B.Plan(spec)
    plan.set_option("placement", 1)
    for key, v in options.items():
        plan.set_option(key, v)
    d_raw, d_off = to_device(raw, off)
    res, ws = B.extract_with_retry(plan, d_raw, d_off, slack=1.05)
    # the first call has no sizes to go by: counting launch, record order
    assert res.arrival_tile_records == 0
    assert_same({s: expand(res.slots[s], n) for s in res.slot_ids}, res, want, label + " first call")
    for call in (1, 2):
        ws.fill_(0x3C)
        plan.set_workspace(ws)
        res = plan.extract(d_raw, d_off)
        if want_one_launch is None or (want_one_launch and res.arrival_tile_records == 0 and res.tile_launches == 1):
            # (no ragged operator in the plan: one launch, nothing to place, record order)
            assert res.tile_launches == 1 and res.arrival_tile_records == 0, res.note
            assert_same({s: expand(res.slots[s], n) for s in res.slot_ids}, res, want, f"{label} call {call}")
        elif may_fall_back and res.tile_launches == 2 and ("fell back" in res.note or "not tried" in res.note):
            # (records of very different lengths: a tile's text did not fit the LDS section, the counting sequence answered)
            assert res.arrival_tile_records == 0
            assert_same({s: expand(res.slots[s], n) for s in res.slot_ids}, res, want, f"{label} call {call}")
        elif want_one_launch:
            assert res.tile_launches == 1, res.note
            assert_same_in_arrival_order(res, want, n, f"{label} call {call}")
        else:
            assert res.arrival_tile_records == 0
            assert_same({s: expand(res.slots[s], n) for s in res.slot_ids}, res, want, f"{label} call {call}")
    plan.close()


@pytest.mark.parametrize("cfg,n,options", [
    (5, 6000, {}), (5, 6000, {"compile": 1}), (5, 40_000, {"compile": 1, "grid_limit": 8}),
    (2, 900, {}),            # many ragged operators on tiles of four records: one launch in this order only
    (2, 900, {"compile": 1}),
    (4, 1500, {}), (3, 5000, {"compile": 1}),
    (5, 6000, {"compile": 1, "tile_log2": 6, "lds_budget": 160 * 1024, "lane_ops": 2}),   # generated straight-line operators
    (4, 1500, {"compile": 1}),
    (5, 1_000_000, {"compile": 1}),   # far more tiles than workgroups that run at the same time
    (2, 120_000, {"compile": 1}),
], ids=["config5", "config5_compiled", "config5_compiled_8_workgroups", "config2", "config2_compiled", "config4", "config3_compiled",
        "config5_generated_operators", "config4_compiled",
        "config5_a_million_records", "config2_30000_tiles"])
def test_workloads_in_arrival_order(cfg, n, options):
    w = W.get(cfg, n)
    raw, off = w.generate()
    _arrival_calls(w.spec, raw, off, options, w.name)


@pytest.mark.parametrize("tile_log2", [0, 3, 6])
def test_operators_over_lists_in_arrival_order(tile_log2):
    rng = random.Random(31 + tile_log2)
    word = lambda: "".join(rng.choice("abcdefg") for _ in range(rng.randint(0, 9)))
    recs = [("\t".join([word(), word(), ",".join(word() for _ in range(rng.randint(1, 6))),
                        ",".join(word() for _ in range(rng.randint(1, 3)))]) + ("\n" if i % 3 else "")).encode() for i in range(3000)]
    raw = np.frombuffer(b"".join(recs), np.uint8)
    off = np.cumsum([0] + [len(r) for r in recs]).astype(np.uint64)
    _arrival_calls(FOLLOW_SPEC, raw, off, {"tile_log2": tile_log2}, f"T={1 << tile_log2}")


@pytest.mark.parametrize("seed", range(8))
def test_random_dags_in_arrival_order(seed):
    """Operator DAGs drawn at random (every kind of root on any field, crosses and concats of anything earlier, emitted or
    not) on records whose fields are lists, numbers, text or missing; generic and compiled kernels, several tile sizes."""
    rng = random.Random(7000 + seed)

    def field():
        kind = rng.randrange(5)
        if kind == 0:
            return ",".join("".join(rng.choice("abcxyz") for _ in range(rng.randint(0, 6))) for _ in range(rng.randint(1, 7)))
        if kind == 1:
            return f"{rng.randint(-200, 200)}.{rng.randint(0, 999)}"
        if kind == 2:
            return "".join(rng.choice("abcdefgh ,") for _ in range(rng.randint(0, 30)))
        return "".join(rng.choice("abc") for _ in range(rng.randint(0, 5)))

    while True:
        spec, ids, deps = random_dag(rng, rng.randrange(2, 9), rng.randrange(1, 9))
        n = rng.choice([300, 1000, 2500])
        recs = [("\t".join(field() for _ in range(rng.randint(1, 5))) + ("\n" if i % 3 else "")).encode() for i in range(n)]
        raw = np.frombuffer(b"".join(recs), np.uint8)
        off = np.cumsum([0] + [len(r) for r in recs]).astype(np.uint64)
        try:
            want = O.extract(spec, raw, off)
        except O.OracleError:
            continue                       # (a cross of crosses that outgrows the sign limit: draw again)
        if want.n_values_total <= 3_000_000:
            break
    has_ragged = any(arity == 0 for _, _, arity in want.slots.values()) or " multi=1" in spec or " ngram " in spec or " filter " in spec
    for options in ({}, {"compile": 1}, {"tile_log2": rng.choice([0, 2, 4])}):
        _arrival_calls(spec, raw, off, options, f"seed {seed} {options}", want_one_launch=None if not has_ragged else True, may_fall_back=True)


def test_arrival_order_falls_back_to_record_order():
    """Sizes learned on a batch with short lists, then a batch with long ones: the arrays are too small, no tile writes
    beyond them, and the counting sequence answers the call in record order."""
    spec = ("fbx 1\nfields 2\n"
            "op a hash slot=0 seed=1 emit=1 field=0 multi=1\n"
            "op b hash slot=1 seed=2 emit=1 field=1 multi=0\n"
            "op c cross slot=2 seed=3 emit=1 a=b b=a\n")
    short = [b"x,y\tq\n"] * 4000
    long_ = [b"x,y,z,w,v,u,t,s\tq\n"] * 4000
    cat = lambda recs: (np.frombuffer(b"".join(recs), np.uint8), np.cumsum([0] + [len(r) for r in recs]).astype(np.uint64))
    plan = B.Plan(spec)
    plan.set_option("placement", 1)
    d_raw, d_off = to_device(*cat(long_))
    res, ws = B.extract_with_retry(plan, d_raw, d_off, slack=1.2)   # (a workspace that holds the long batch)
    d_raw1, d_off1 = to_device(*cat(short))
    res = plan.extract(d_raw1, d_off1)
    res = plan.extract(d_raw1, d_off1)
    assert res.tile_launches == 1 and res.arrival_tile_records > 0
    res = plan.extract(d_raw, d_off)
    assert res.tile_launches == 2 and res.arrival_tile_records == 0 and "fell back" in res.note
    assert_same({s: expand(res.slots[s], 4000) for s in res.slot_ids}, res, O.extract(spec, *cat(long_)), "after the fall-back")
    res = plan.extract(d_raw, d_off)
    assert res.tile_launches == 1
    assert_same_in_arrival_order(res, O.extract(spec, *cat(long_)), 4000, "with the new sizes")
    plan.close()
