"""Pins of the CPU oracle against things other than itself: published hash
vectors, Python library routines, hand-built records, invariants, and a
pure-Python brute force.  No GPU is needed."""
import bisect
import random
from decimal import Decimal

import numpy as np
import pytest

from oracle import brute
from oracle import fbx_oracle as O
from paper_2210_07768_amd import workloads as W
from helpers import BAD_SPECS, FRAMING_SPEC, FRAMING_RECORDS

M64 = (1 << 64) - 1


# ---------------------------------------------------------------- hash pins
def test_fnv_published_vectors_pin_brute_and_oracle(golden):
    for msg_hex, want in golden("fnv1a64_vectors.txt"):
        msg = b"" if msg_hex == "-" else bytes.fromhex(msg_hex)
        assert brute.fnv1a64(msg) == int(want, 16)
        if len(msg) >= 8:
            # the oracle hashes le64(seed) || token: split a published message there
            seed = int.from_bytes(msg[:8], "little")
            assert O.hash_bytes(seed, msg[8:]) == int(want, 16)


def test_seeded_hash_is_fnv_of_prefixed_message():
    rng = random.Random(1)
    for _ in range(2000):
        seed = rng.getrandbits(64)
        m = bytes(rng.getrandbits(8) for _ in range(rng.randrange(0, 70)))
        assert O.hash_bytes(seed, m) == brute.fnv1a64(seed.to_bytes(8, "little") + m)


def test_fnv_step_structure():
    # appending one byte c to a message multiplies (h ^ c) by the prime: checks the
    # xor-then-multiply order (FNV-1a, not FNV-1) without re-typing the loop
    rng = random.Random(2)
    for _ in range(200):
        seed = rng.getrandbits(64)
        m = bytes(rng.getrandbits(8) for _ in range(rng.randrange(0, 20)))
        c = rng.getrandbits(8)
        h0 = O.hash_bytes(seed, m)
        assert O.hash_bytes(seed, m + bytes([c])) == ((h0 ^ c) * 0x100000001B3) & M64


def test_splitmix_published_outputs(golden):
    gamma = 0x9E3779B97F4A7C15
    for k, want in golden("splitmix64_vectors.txt"):
        x = (int(k) * gamma) & M64
        assert O.mix64(x) == int(want, 16)
        assert brute.mix64(x) == int(want, 16)


def test_mix64_is_a_bijection_on_samples():
    xs = np.random.default_rng(3).integers(0, 1 << 63, size=200000, dtype=np.uint64)
    xs = np.unique(xs)
    ys = {O.mix64(int(x)) for x in xs[:50000]}
    assert len(ys) == 50000
    assert O.mix64(0) == 0


def test_contract_worked_values(golden):
    g = {k: int(v, 16) for k, v in golden("contract_values.txt")}
    assert O.hash_bytes(0, b"") == g["hash_seed0_empty"]
    assert O.hash_bytes(1, b"abc") == g["hash_seed1_abc"]
    assert O.hash_bytes(0xDEADBEEF, b"hello") == g["hash_seeddeadbeef_hello"]
    assert O.hash_bytes(2, b"xy") == g["hash_seed2_xy"]
    assert O.mix64(0) == g["mix64_0"] and O.mix64(1) == g["mix64_1"]
    K = O.mix64(7)
    assert K == g["mix64_7"]
    a, b = O.hash_bytes(1, b"abc"), O.hash_bytes(2, b"xy")
    assert O.cross(K, a, b) == g["cross_K7_abc_xy"]
    assert O.cross(K, b, a) == g["cross_K7_xy_abc"]
    assert O.mix64((K + 3) & M64) == g["bucket_sign_K7_idx3"]
    # the hand-built record of the contract: F = 3, field 1 multi-valued with an empty item
    spec = ("fbx 1\nfields 3\n"
            "op t hash slot=5 seed=11 emit=1 field=1 multi=1\n"
            "op n bucket slot=6 seed=7 emit=1 field=2 multi=0 bounds=-5,0,0,10,1000000\n")
    raw = b"ab\tx,y,,z\t1.5\n"
    r = O.extract(spec, raw, [0, len(raw)])
    vals, offs, _ = r.slots[5]
    assert [int(v) for v in vals] == [g[f"field1_seed11_tok{i}"] for i in range(4)]
    assert offs.tolist() == [0, 4]
    # 1.5 -> 1500000 micro-units -> all five boundaries are <= it
    assert int(r.slots[6][0][0]) == O.mix64((K + 5) & M64)


def test_cross_is_not_commutative_and_matches_brute():
    rng = random.Random(4)
    for _ in range(500):
        K, a, b = (rng.getrandbits(64) for _ in range(3))
        assert O.cross(K, a, b) == brute.cross(K, a, b)
    K = O.mix64(7)
    assert O.cross(K, 1, 2) != O.cross(K, 2, 1)


# ------------------------------------------------------------- numeric pins
def test_parse_micro_hand_table():
    table = {b"0": 0, b"1": 1000000, b"1.5": 1500000, b"0.000001": 1, b"0.0000019": 1,
             b"-2.25": -2250000, b".5": 500000, b"12x": 12000000, b"": 0, b"-": 0, b".": 0,
             b"-.5": -500000, b"1.": 1000000, b"1.2.3": 1200000, b"-0": 0, b"007": 7000000,
             b"+1": 0, b" 1": 0, b"1e3": 1000000, b"123456.654321": 123456654321,
             b"0.9999999": 999999, b"-0.9999999": -999999}
    malformed = {b"12x", b"", b"-", b".", b"1.2.3", b"+1", b" 1", b"1e3"}
    for tok, want in table.items():
        v, bad = O.parse_micro(tok)
        assert v == want, tok
        assert bad == (tok in malformed), tok
        assert brute.micro_any(tok) == (want, tok in malformed), tok


def test_parse_micro_matches_decimal_on_wellformed_text():
    rng = random.Random(5)
    for _ in range(5000):
        ip = rng.randrange(0, 10 ** rng.randrange(1, 12))
        k = rng.randrange(0, 10)
        txt = ("-" if rng.random() < 0.3 else "") + str(ip)
        if k:
            txt += "." + "".join(rng.choice("0123456789") for _ in range(k))
        want = int(Decimal(txt) * 10 ** 6)
        v, bad = O.parse_micro(txt.encode())
        assert (v, bad) == (want, False), txt


def test_parse_micro_overflow_wraps():
    v, bad = O.parse_micro(b"99999999999999999999999")
    want = (99999999999999999999999 * 10 ** 6) & M64
    want = want - (1 << 64) if want >> 63 else want
    assert v == want and not bad


def test_bucket_index_is_bisect_right():
    bounds = [-5, 0, 0, 10, 1000000]
    got = [O.bucket_index(bounds, v) for v in (-6, -5, 0, 9, 10, 999999, 1000000, 5000000)]
    assert got == [0, 1, 3, 3, 4, 4, 5, 5]
    rng = np.random.default_rng(6)
    b = np.sort(rng.integers(-10 ** 9, 10 ** 9, size=64))
    for v in rng.integers(-2 * 10 ** 9, 2 * 10 ** 9, size=2000).tolist() + b.tolist():
        assert O.bucket_index(b, v) == bisect.bisect_right(b.tolist(), v)
        assert O.bucket_index(b, v) == int(np.searchsorted(b, v, side="right"))
    assert O.bucket_index([], 5) == 0


# --------------------------------------------------------- framing pins
def _run_both(spec, records):
    raw = b"".join(records)
    offs = np.cumsum([0] + [len(r) for r in records]).astype(np.uint64)
    got = O.extract(spec, raw, offs)
    want, want_bad = brute.extract(spec, records)
    assert sorted(got.slots) == sorted(want)
    for s, (vals, offsets) in want.items():
        gv, go, _ = got.slots[s]
        assert go.tolist() == offsets, f"slot {s} offsets"
        assert [int(x) for x in gv] == vals, f"slot {s} values"
    assert got.n_malformed_numeric == want_bad
    return got


def test_hand_built_records_against_python_split():
    records = FRAMING_RECORDS
    got = _run_both(FRAMING_SPEC, records)
    # sign count equals token count (#commas + 1) for the multi-valued hash slot
    _, offs, _ = got.slots[1]
    counts = np.diff(offs.astype(np.int64)).tolist()
    toks = []
    for r in records:
        r = r[:-1] if r.endswith(b"\n") else r
        f = r.split(b"\t")
        toks.append((f[1] if len(f) > 1 else b"").count(b",") + 1)
    assert counts == toks


def test_invariants_on_random_small_records():
    rng = random.Random(7)
    alphabet = b"ab,x\t1.-9 \n"
    for trial in range(60):
        records = []
        for _ in range(rng.randrange(1, 8)):
            n = rng.randrange(0, 40)
            body = bytes(rng.choice(alphabet) for _ in range(n)).replace(b"\n", b"z")
            records.append(body + (b"\n" if rng.random() < 0.7 else b""))
        got = _run_both(FRAMING_SPEC, records)
        R = len(records)
        total = 0
        for s, (vals, offs, arity) in got.slots.items():
            assert offs[0] == 0 and offs[-1] == vals.size and offs.size == R + 1
            assert np.all(np.diff(offs.astype(np.int64)) >= 0)
            if arity:
                assert np.all(np.diff(offs.astype(np.int64)) == arity)
            total += vals.size
        assert total == got.n_values_total
        # cross count is the product of the input list lengths
        cb = np.diff(got.slots[1][1].astype(np.int64))
        cc = np.diff(got.slots[2][1].astype(np.int64))
        assert np.array_equal(np.diff(got.slots[6][1].astype(np.int64)), cb * cc)
        # concat count is the sum
        ca = np.diff(got.slots[0][1].astype(np.int64))
        assert np.array_equal(np.diff(got.slots[7][1].astype(np.int64)), cb * cc + ca)


def test_ngram_widths_and_counts():
    for n in range(1, 9):
        spec = f"fbx 1\nfields 1\nop g ngram slot=0 seed=1 emit=1 field=0 n={n}\n"
        recs = [b"abcdefghij\n", b"ab\n", b"\n", b"abcdefgh"]
        got = _run_both(spec, recs)
        counts = np.diff(got.slots[0][1].astype(np.int64)).tolist()
        assert counts == [max(len(r.rstrip(b"\n")) - n + 1, 0) for r in recs]


def test_config1_matches_brute_force():
    w = W.get(1, 300)
    raw, off = w.generate()
    got = O.extract(w.spec, raw, off)
    b = raw.tobytes()
    records = [b[int(off[i]):int(off[i + 1])] for i in range(300)]
    want, _ = brute.extract(w.spec, records)
    assert len(want) == 24
    for s, (vals, offsets) in want.items():
        gv, go, arity = got.slots[s]
        assert arity == 1
        assert go.tolist() == offsets
        assert [int(x) for x in gv] == vals


@pytest.mark.parametrize("cfg,n", [(2, 40), (3, 60), (4, 40), (5, 40)])
def test_other_configs_match_brute_force(cfg, n):
    w = W.get(cfg, n)
    raw, off = w.generate()
    got = O.extract(w.spec, raw, off)
    b = raw.tobytes()
    records = [b[int(off[i]):int(off[i + 1])] for i in range(n)]
    want, bad = brute.extract(w.spec, records)
    assert got.n_malformed_numeric == bad == 0
    for s, (vals, offsets) in want.items():
        gv, go, _ = got.slots[s]
        assert go.tolist() == offsets
        assert [int(x) for x in gv] == vals


def test_config1_oracle_is_fast_enough():
    import time
    w = W.get(1)
    raw, off = w.generate()
    t = time.time()
    got = O.extract(w.spec, raw, off)
    assert time.time() - t < 2.0
    assert got.n_values_total == 4096 * 24


# ------------------------------------------------------------- spec / layers
def test_layer_rule_on_paper_example(golden):
    rows = golden("dag_example.txt")
    lines = ["fbx 1", "fields 1"]
    for i, (op, inp, _) in enumerate(rows):
        if inp == "-":
            lines.append(f"op {op} hash slot={i} seed={i} emit=1 field=0 multi=0")
        else:
            lines.append(f"op {op} concat slot={i} emit=1 a={inp} b={inp}")
    layers, _ = O.spec_layers("\n".join(lines) + "\n")
    assert layers == [int(r[2]) for r in rows]


@pytest.mark.parametrize("name", sorted(BAD_SPECS))
def test_oracle_rejects_bad_specs(name):
    with pytest.raises(O.OracleError) as e:
        O.extract(BAD_SPECS[name], b"x\n", [0, 2])
    assert e.value.status == O.E_SPEC


def test_duplicate_slot_is_fine_when_not_emitted():
    spec = ("fbx 1\nfields 1\nop a hash slot=0 seed=0 emit=0 field=0 multi=0\n"
            "op b hash slot=0 seed=1 emit=1 field=0 multi=0\n")
    r = O.extract(spec, b"x\n", [0, 2])
    assert r.slot_ids == [0]


def test_oracle_rejects_bad_offsets():
    spec = "fbx 1\nfields 1\nop a hash slot=0 seed=0 emit=1 field=0 multi=0\n"
    for offs in ([0, 5], [2, 1], [0, 1, 0]):
        with pytest.raises(O.OracleError) as e:
            O.extract(spec, b"ab\n", offs)
        assert e.value.status == O.E_INPUT


def test_results_do_not_depend_on_op_order():
    # the same DAG written in two topologically valid orders gives the same slots
    a = ("fbx 1\nfields 2\n"
         "op p hash slot=0 seed=1 emit=1 field=0 multi=1\n"
         "op q hash slot=1 seed=2 emit=1 field=1 multi=0\n"
         "op x cross slot=2 seed=3 emit=1 a=p b=q\n"
         "op y concat slot=3 emit=1 a=x b=p\n")
    b = ("fbx 1\nfields 2\n"
         "op q hash slot=1 seed=2 emit=1 field=1 multi=0\n"
         "op p hash slot=0 seed=1 emit=1 field=0 multi=1\n"
         "op x cross slot=2 seed=3 emit=1 a=p b=q\n"
         "op y concat slot=3 emit=1 a=x b=p\n")
    raw = b"u,v,w\tz\nk\tm\n"
    ra, rb = O.extract(a, raw, [0, 8, 12]), O.extract(b, raw, [0, 8, 12])
    for s in range(4):
        assert np.array_equal(ra.slots[s][0], rb.slots[s][0])
        assert np.array_equal(ra.slots[s][1], rb.slots[s][1])
