"""The toy "clean views" stage of the library (fbx_clean_*) against its oracle, byte for byte, and
cleaned text handed on to fbx_extract without leaving the device."""
import random

import numpy as np
import pytest

from oracle import fbx_clean_oracle as C
from oracle import fbx_oracle as O
from paper_2210_07768_amd import binding as B
from gpu_harness import assert_same, expand, to_device
from test_clean_oracle_pins import SPEC

pytestmark = pytest.mark.gpu


def _cat(records):
    return np.frombuffer(b"".join(records), np.uint8), np.cumsum([0] + [len(r) for r in records]).astype(np.uint64)


def _gpu_clean(spec, raw, off, out_cap=None, misalign=0):
    import torch
    n = len(off) - 1
    clean = B.Clean(spec)
    d_raw, d_off = to_device(raw, off, misalign)
    scratch = torch.empty(clean.scratch_hint(n), dtype=torch.uint8, device="cuda").fill_(0x6B)
    d_out = torch.empty(raw.size + 64 * n + 64 if out_cap is None else out_cap, dtype=torch.uint8, device="cuda").fill_(0x21)
    d_out_off = torch.full((n + 1,), -1, dtype=torch.int64, device="cuda")
    res = clean.run(d_raw, d_off, d_out, d_out_off, scratch)
    clean.close()
    return res, d_out, d_out_off


def _random_case(rng, n):
    F = rng.randint(1, 6)
    lines = ["fbxclean 1", f"fields {F}"]
    for _ in range(rng.randint(0, 7)):
        kind = rng.choice(["fill", "key", "keep"])
        arg = "".join(rng.choice("abck") for _ in range(rng.randint(0 if kind != "fill" else 1, 2))).encode().hex()
        lines.append(f"{kind} field={rng.randrange(F)} {dict(fill='value', key='name', keep='prefix')[kind]}={arg}")
    field = lambda: "".join(rng.choice("abc:;k") for _ in range(rng.randint(0, 12)))
    recs = [("\t".join(field() for _ in range(rng.randint(0, F + 1))) + ("\n" if rng.random() < 0.7 else "")).encode()
            for _ in range(n)]
    return "\n".join(lines) + "\n", recs


@pytest.mark.parametrize("seed", range(8))
def test_clean_matches_the_oracle(seed):
    rng = random.Random(100 + seed)
    spec, recs = _random_case(rng, rng.choice([1, 255, 256, 257, 5000]))
    raw, off = _cat(recs)
    want_raw, want_off = C.clean(spec, raw, off)
    res, d_out, d_out_off = _gpu_clean(spec, raw, off, misalign=seed % 3)
    assert res.n_kept == len(want_off) - 1 and res.out_len == want_raw.size
    assert np.array_equal(d_out_off[:res.n_kept + 1].cpu().numpy().view(np.uint64), want_off)
    assert np.array_equal(d_out[:res.out_len].cpu().numpy(), want_raw)
    assert bool((d_out[res.out_len:] == 0x21).all()), "written beyond the cleaned text"


def _wide_case(rng, F, n, long_every=0, n_ops=12, width=10, keep_all=False):
    """n records of about F fields (some fewer, some more) of 0..width bytes, operators on random fields;
    every long_every-th record holds one field of 30 to 70 KB."""
    lines = ["fbxclean 1", f"fields {F}"]
    for o in range(n_ops):
        kind = "keep" if o == n_ops // 2 else rng.choice(["fill", "fill", "key"])  # (one filter: more would drop nearly every record)
        arg = "".join(rng.choice("abk") for _ in range(rng.randint(0 if kind != "fill" else 1, {"fill": 9, "key": 2, "keep": 0 if keep_all else 1}[kind]))).encode().hex()
        lines.append(f"{kind} field={rng.randrange(F)} {dict(fill='value', key='name', keep='prefix')[kind]}={arg}")
    field = lambda: "".join(rng.choice("abc:;k") for _ in range(rng.randint(0, width)))
    recs = []
    for i in range(n):
        fields = [field() for _ in range(F + rng.choice([0, 0, 0, 0, -1, 1, -F // 2]))]
        if long_every and i % long_every == long_every - 1 and fields:
            fields[rng.randrange(len(fields))] = "".join(rng.choice("ab;:k") for _ in range(64)) * rng.randint(470, 1100)
        recs.append(("\t".join(fields) + ("\n" if rng.random() < 0.8 else "")).encode())
    return "\n".join(lines) + "\n", recs


@pytest.mark.parametrize("F,n,long_every,n_ops,width", [
    (130, 3000, 0, 40, 10),      # tiles of 16 records, two turns of a wavefront per record
    (130, 3001, 0, 40, 10),      # the same with a filter that keeps every record
    (100, 2500, 97, 30, 8),      # now and then a tile whose text does not fit the section: read in place
    (1, 9000, 0, 2, 6),          # tiles of 64 short records
    (7, 700, 5, 6, 300),         # long fields: few records per tile, many tiles read in place
    (5000, 24, 0, 50, 3),        # more fields than the tables in LDS hold: one record per thread
])
def test_clean_tiles_of_every_shape(F, n, long_every, n_ops, width):
    rng = random.Random(F * 1000 + n)
    spec, recs = _wide_case(rng, F, n, long_every, n_ops, width, keep_all=n % 2 == 1)
    raw, off = _cat(recs)
    want_raw, want_off = C.clean(spec, raw, off)
    assert 0 < len(want_off) - 1, "the case keeps no record"
    res, d_out, d_out_off = _gpu_clean(spec, raw, off, out_cap=want_raw.size + 1000, misalign=n % 5)
    assert res.n_kept == len(want_off) - 1 and res.out_len == want_raw.size
    assert np.array_equal(d_out_off[:res.n_kept + 1].cpu().numpy().view(np.uint64), want_off)
    assert np.array_equal(d_out[:res.out_len].cpu().numpy(), want_raw)
    assert bool((d_out[res.out_len:] == 0x21).all()), "written beyond the cleaned text"


def test_clean_edge_cases_and_errors():
    import torch
    recs = [b"ann\tage:3;city:rome;x:1\tok1\t5\n", b"\tcity:;age:4\tokay\t\n", b"bob\tage:3\tok\t1", b"cy\tcity:oslo\tnot ok\t2\n",
            b"", b"\t\tok\t\n"] * 100
    raw, off = _cat(recs)
    want_raw, want_off = C.clean(SPEC, raw, off)
    # an empty batch
    res, d_out, d_out_off = _gpu_clean(SPEC, raw[:0], off[:1])
    assert res.n_kept == 0 and res.out_len == 0 and int(d_out_off[0]) == 0
    # an output buffer that is too small: nothing written, the need reported, and that much suffices
    with pytest.raises(B.FbxError) as e:
        _gpu_clean(SPEC, raw, off, out_cap=want_raw.size - 1)
    assert e.value.status == B.E_NOMEM and e.value.required_bytes == want_raw.size
    res, d_out, d_out_off = _gpu_clean(SPEC, raw, off, out_cap=want_raw.size)
    assert np.array_equal(d_out.cpu().numpy(), want_raw)
    # scratch too small, bad offsets, bad spec
    clean = B.Clean(SPEC)
    d_raw, d_off = to_device(raw, off)
    d_out = torch.empty(raw.size * 2, dtype=torch.uint8, device="cuda")
    d_out_off = torch.empty(len(recs) + 1, dtype=torch.int64, device="cuda")
    with pytest.raises(B.FbxError) as e:
        clean.run(d_raw, d_off, d_out, d_out_off, torch.empty(1024, dtype=torch.uint8, device="cuda"))
    assert e.value.status == B.E_NOMEM
    bad = off.copy(); bad[7] = bad[9]
    d_raw2, d_off2 = to_device(raw, bad)
    with pytest.raises(B.FbxError) as e:
        clean.run(d_raw2, d_off2, d_out, d_out_off, torch.empty(clean.scratch_hint(len(recs)), dtype=torch.uint8, device="cuda"))
    assert e.value.status == B.E_INPUT
    clean.close()
    for spec in ("fields 2\n", "fbxclean 1\nfields 2\nfill field=2 value=61\n", "fbxclean 1\nfields 2\nfill field=0 value=09\n",
                 "fbxclean 1\nfields 2\nkeep field=0\n", "fbxclean 1\nfields 2\nfrob field=0 value=61\n"):
        with pytest.raises(B.FbxError) as e:
            B.Clean(spec)
        assert e.value.status == B.E_SPEC


def test_cleaned_text_feeds_extraction_on_the_device():
    """Clean, then extract, both on the device, against the two oracles chained on the host."""
    import torch
    rng = random.Random(77)
    word = lambda: "".join(rng.choice("abcdxyz") for _ in range(rng.randint(1, 8)))
    recs = []
    for i in range(4000):
        attrs = ";".join(f"{k}:{word()}" for k in rng.sample(["city", "age", "tag", "os"], rng.randint(0, 4)))
        terms = ",".join(word() for _ in range(rng.randint(1, 5))) if i % 9 else ""
        price = f"{rng.randint(0, 300)}.{rng.randint(0, 99)}" if i % 7 else ""
        recs.append(f"{word() if i % 5 else ''}\t{attrs}\t{terms}\t{price}\t{rng.choice(['click', 'view', 'skip'])}\n".encode())
    clean_spec = ("fbxclean 1\nfields 5\n"
                  f"fill field=0 value={b'anon'.hex()}\n"
                  f"key field=1 name={b'city'.hex()}\n"
                  f"fill field=1 value={b'nowhere'.hex()}\n"
                  f"fill field=2 value={b'none'.hex()}\n"
                  f"fill field=3 value={b'0'.hex()}\n"
                  f"keep field=4 prefix={b'cli'.hex()}\n")
    extract_spec = ("fbx 1\nfields 5\n"
                    "op u hash slot=0 seed=1 emit=1 field=0 multi=0\n"
                    "op c hash slot=1 seed=2 emit=1 field=1 multi=0\n"
                    "op t hash slot=2 seed=3 emit=1 field=2 multi=1\n"
                    "op p bucket slot=3 seed=4 emit=1 field=3 multi=0 bounds=1000000,10000000,100000000\n"
                    "op uc cross slot=4 seed=5 emit=1 a=u b=c\n"
                    "op ct cross slot=5 seed=6 emit=1 a=c b=t\n")
    raw, off = _cat(recs)
    want_raw, want_off = C.clean(clean_spec, raw, off)
    want = O.extract(extract_spec, want_raw, want_off)
    assert 0 < len(want_off) - 1 < len(recs) and want.n_malformed_numeric == 0
    res, d_out, d_out_off = _gpu_clean(clean_spec, raw, off)
    plan = B.Plan(extract_spec)
    got, ws = B.extract_with_retry(plan, d_out[:res.out_len], d_out_off[:res.n_kept + 1])
    assert_same({s: expand(got.slots[s], res.n_kept) for s in got.slot_ids}, got, want, "clean then extract")
    plan.close()
