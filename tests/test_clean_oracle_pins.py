"""Pins of the oracle of the toy "clean views" stage: Python's own bytes.split / partition /
startswith on hand-built and random records, hand-written expected outputs, and invariants."""
import random

import numpy as np
import pytest

from oracle import brute
from oracle import fbx_clean_oracle as C

SPEC = ("fbxclean 1\nfields 4\n"
        "fill field=0 value=" + b"unknown".hex() + "\n"
        "key field=1 name=" + b"city".hex() + "\n"
        "fill field=1 value=" + b"nowhere".hex() + "\n"
        "keep field=2 prefix=" + b"ok".hex() + "\n"
        "fill field=3 value=30\n")


def _cat(records):
    return np.frombuffer(b"".join(records), np.uint8), np.cumsum([0] + [len(r) for r in records]).astype(np.uint64)


def _records_of(data, offs):
    b = data.tobytes()
    return [b[int(offs[i]):int(offs[i + 1])] for i in range(len(offs) - 1)]


def test_hand_written_expected_output():
    recs = [b"ann\tage:3;city:rome;x:1\tok1\t5\n",          # everything there
            b"\tcity:;age:4\tokay\t\n",                       # nulls filled; the key is there with an empty value -> filled too
            b"bob\tage:3\tok\t1",                             # no such key -> filled; no trailing newline
            b"cy\tcity:oslo\tnot ok\t2\n",                    # dropped by the filter
            b"dee\tcity\tok\t3\textra\tfields\n",             # a pair without ':' never matches; extra fields dropped
            b"eve\tcityx:1;city:a:b;city:second\tok\n",       # exact key match; value keeps later ':'; first match wins; missing field 3
            b"",                                              # all fields missing: field 2 is empty -> dropped
            b"\t\tok\t\n"]
    want = [b"ann\trome\tok1\t5\n", b"unknown\tnowhere\tokay\t0\n", b"bob\tnowhere\tok\t1\n",
            b"dee\tnowhere\tok\t3\n", b"eve\ta:b\tok\t0\n", b"unknown\tnowhere\tok\t0\n"]
    data, offs = C.clean(SPEC, *_cat(recs))
    assert _records_of(data, offs) == want
    assert brute.clean(SPEC, recs) == want


def test_random_records_against_python():
    rng = random.Random(5)
    alphabet = "abc:;k"
    def field():
        return "".join(rng.choice(alphabet) for _ in range(rng.randint(0, 10)))
    for trial in range(30):
        F = rng.randint(1, 5)
        lines = ["fbxclean 1", f"fields {F}"]
        for _ in range(rng.randint(0, 6)):
            kind = rng.choice(["fill", "key", "keep"])
            arg = "".join(rng.choice("abck") for _ in range(rng.randint(0 if kind != "fill" else 1, 2))).encode().hex()
            lines.append(f"{kind} field={rng.randrange(F)} {dict(fill='value', key='name', keep='prefix')[kind]}={arg}")
        spec = "\n".join(lines) + "\n"
        recs = [("\t".join(field() for _ in range(rng.randint(0, F + 1))) + ("\n" if rng.random() < 0.7 else "")).encode()
                for _ in range(200)]
        data, offs = C.clean(spec, *_cat(recs))
        assert _records_of(data, offs) == brute.clean(spec, recs), spec


def test_invariants():
    rng = random.Random(9)
    recs = [("\t".join("".join(rng.choice("ab:;") for _ in range(rng.randint(0, 6))) for _ in range(rng.randint(0, 4))) + "\n").encode()
            for _ in range(500)]
    spec = "fbxclean 1\nfields 3\nfill field=0 value=7a\nfill field=1 value=7a\nfill field=2 value=7a\n"
    data, offs = C.clean(spec, *_cat(recs))
    out = _records_of(data, offs)
    assert len(out) == len(recs)                                    # no filter: nothing is dropped
    for r in out:
        fields = r[:-1].split(b"\t")
        assert len(fields) == 3 and all(fields) and r.endswith(b"\n")   # exactly F fields, none empty after filling
    kept = []
    for p in (b"", b"a", b"ab", b"aba"):                               # a longer prefix never keeps more
        d, o = C.clean(spec + f"keep field=0 prefix={p.hex()}\n", *_cat(recs))
        kept.append(len(o) - 1)
    assert kept[0] == len(recs) and kept == sorted(kept, reverse=True) and kept[-1] < kept[0]


@pytest.mark.parametrize("spec", ["fields 2\n", "fbxclean 1\n", "fbxclean 1\nfields 0\n", "fbxclean 1\nfields 2\nfill field=2 value=61\n",
                                  "fbxclean 1\nfields 2\nfill field=0 value=\n", "fbxclean 1\nfields 2\nfill field=0 value=09\n",
                                  "fbxclean 1\nfields 2\nkey field=0 name=6\n", "fbxclean 1\nfields 2\nkeep field=0\n",
                                  "fbxclean 1\nfields 2\nfrob field=0 value=61\n", "fbxclean 1\nfields 2\nkeep field=0 prefix=61 prefix=62\n"])
def test_bad_specs(spec):
    with pytest.raises(C.CleanOracleError) as e:
        C.clean(spec, *_cat([b"a\tb\n"]))
    assert e.value.status == C.E_SPEC
