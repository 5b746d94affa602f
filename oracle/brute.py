"""Pure-Python brute force of the extraction contract, for tiny inputs only.

Test infrastructure only.  Its job is to pin the C oracle to something other
than itself: wherever the contract coincides with a Python library routine the
routine is used (``bytes.split`` for field and item framing,
``bytes.startswith`` for the prefix filter, ``bisect.bisect_right`` for the
bucket index, ``decimal.Decimal`` for well-formed numerics), and the two hash
primitives are three-line loops over Python integers that the tests check
against the published FNV-1a-64 and SplitMix64 values.

The paper (Section 3, "Extract features"; Section 5, first paragraph) only
says that operators are evaluated per row of a table and that strings are split
at a delimiter; all operator semantics below are this repository's readings.
"""
from __future__ import annotations

import bisect
from decimal import Decimal
from typing import Dict, List, Tuple

M64 = (1 << 64) - 1


def fnv1a64(data: bytes) -> int:
    h = 0xCBF29CE484222325
    for b in data:
        h = ((h ^ b) * 0x100000001B3) & M64
    return h


def hash_bytes(seed: int, m: bytes) -> int:
    return fnv1a64(seed.to_bytes(8, "little") + m)


def mix64(x: int) -> int:
    x &= M64
    x ^= x >> 30
    x = (x * 0xBF58476D1CE4E5B9) & M64
    x ^= x >> 27
    x = (x * 0x94D049BB133111EB) & M64
    x ^= x >> 31
    return x


def cross(K: int, a: int, b: int) -> int:
    return mix64(mix64((a + K) & M64) + b)


def micro_wellformed(tok: bytes) -> int:
    """Micro-units of a well-formed decimal token, via exact Decimal arithmetic."""
    return int(Decimal(tok.decode()) * 10 ** 6)  # int() truncates toward zero


def micro_any(tok: bytes) -> Tuple[int, bool]:
    """Micro-units and malformed flag of any token: take the longest prefix of the
    shape -?digits*(.digits*)? and hand it to Decimal."""
    i, n = 0, len(tok)
    if i < n and tok[i:i + 1] == b"-":
        i += 1
    j = i
    while j < n and tok[j:j + 1].isdigit():
        j += 1
    k = j
    if k < n and tok[k:k + 1] == b".":
        k += 1
        while k < n and tok[k:k + 1].isdigit():
            k += 1
    body = tok[:k]
    ndig = sum(1 for c in body if 48 <= c <= 57)
    malformed = k < n or ndig == 0
    if ndig == 0:
        return 0, malformed
    txt = body.decode()
    if txt.endswith("."):
        txt += "0"
    if txt.startswith("-."):
        txt = "-0" + txt[1:]
    elif txt.startswith("."):
        txt = "0" + txt
    v = int(Decimal(txt) * 10 ** 6)
    # the contract wraps modulo 2^64 and reads the result as two's complement
    v &= M64
    return (v - (1 << 64) if v >> 63 else v), malformed


def parse_spec(spec: str):
    lines = [ln.strip() for ln in spec.split("\n")]
    lines = [ln for ln in lines if ln and not ln.startswith("#")]
    assert lines[0].split() == ["fbx", "1"]
    assert lines[1].split()[0] == "fields"
    n_fields = int(lines[1].split()[1])
    ops = []
    for ln in lines[2:]:
        parts = ln.split()
        assert parts[0] == "op"
        op = {"id": parts[1], "kind": parts[2]}
        for kv in parts[3:]:
            k, v = kv.split("=", 1)
            op[k] = v
        ops.append(op)
    return n_fields, ops


def extract(spec: str, records: List[bytes]) -> Tuple[Dict[int, Tuple[List[int], List[int]]], int]:
    """Returns ({slot: (values, offsets)}, n_malformed)."""
    _, ops = parse_spec(spec)
    out: Dict[int, Tuple[List[int], List[int]]] = {}
    for op in ops:
        if op["emit"] == "1":
            out[int(op["slot"])] = ([], [0])
    malformed = 0
    for rec in records:
        if rec.endswith(b"\n"):
            rec = rec[:-1]
        fields = rec.split(b"\t")
        lists: Dict[str, List[int]] = {}
        for op in ops:
            kind = op["kind"]
            res: List[int] = []
            if kind in ("cross", "concat"):
                A, B = lists[op["a"]], lists[op["b"]]
                if kind == "cross":
                    K = mix64(int(op["seed"]))
                    res = [cross(K, a, b) for a in A for b in B]
                else:
                    res = list(A) + list(B)
            else:
                k = int(op["field"])
                fld = fields[k] if k < len(fields) else b""
                seed = int(op["seed"])
                if kind == "ngram":
                    n = int(op["n"])
                    res = [hash_bytes(seed, fld[i:i + n]) for i in range(len(fld) - n + 1)]
                else:
                    toks = fld.split(b",") if op["multi"] == "1" else [fld]
                    if kind == "hash":
                        res = [hash_bytes(seed, t) for t in toks]
                    elif kind == "filter":
                        p = bytes.fromhex(op["prefix"])
                        res = [hash_bytes(seed, t) for t in toks if t.startswith(p)]
                    elif kind == "bucket":
                        bounds = [int(x) for x in op["bounds"].split(",")] if op["bounds"] else []
                        K = mix64(seed)
                        for t in toks:
                            v, bad = micro_any(t)
                            malformed += int(bad)
                            res.append(mix64(K + bisect.bisect_right(bounds, v)))
                    else:
                        raise ValueError(kind)
            lists[op["id"]] = res
            if op["emit"] == "1":
                vals, offs = out[int(op["slot"])]
                vals.extend(res)
                offs.append(len(vals))
    return out, malformed


# ---------------------------------------------------------------- the toy "clean views" stage
def clean(spec: str, records):
    """Kept records (bytes, each ending in a newline) of the cleaning spec, with Python's own
    split / partition / startswith (Section 3, "Clean views": fill nulls, take one key out of a flat
    key:value list, drop instances by a filter)."""
    lines = [ln.split("#")[0].split() for ln in spec.splitlines()]
    lines = [ln for ln in lines if ln]
    assert lines[0] == ["fbxclean", "1"] and lines[1][0] == "fields"
    n_fields = int(lines[1][1])
    ops = []
    for ln in lines[2:]:
        kv = dict(item.split("=", 1) for item in ln[1:])
        arg = bytes.fromhex(kv[{"fill": "value", "key": "name", "keep": "prefix"}[ln[0]]])
        ops.append((ln[0], int(kv["field"]), arg))
    out = []
    for rec in records:
        if rec.endswith(b"\n"):
            rec = rec[:-1]
        fields = (rec.split(b"\t") + [b""] * n_fields)[:n_fields]
        keep = True
        for kind, k, arg in ops:
            if kind == "fill":
                if not fields[k]:
                    fields[k] = arg
            elif kind == "key":
                value = b""
                for pair in fields[k].split(b";"):
                    key, sep, val = pair.partition(b":")
                    if sep and key == arg:
                        value = val
                        break
                fields[k] = value
            elif not fields[k].startswith(arg):
                keep = False
                break
        if keep:
            out.append(b"\t".join(fields) + b"\n")
    return out
