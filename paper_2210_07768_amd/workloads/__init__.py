"""Seeded synthetic workloads: raw record bytes plus the operator-DAG spec text.

The five workloads mirror the benchmark configurations this build is measured
on (record counts, field mixes, token-length and list-length distributions).
They stand in for the paper's proprietary click logs (Section 6, "Models").

This module holds none of the extraction method's arithmetic: it draws random
text (through ``fbxgen.c``) and writes spec lines.  Both the oracle's tests and
the GPU path's tests use it, and neither side imports the other.
"""
from __future__ import annotations

import ctypes
import os
import random
import subprocess
from dataclasses import dataclass, field as dc_field
from typing import List, Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fbxgen.c")
_LIB = os.path.join(_HERE, "libfbxgen.so")

CAT_SINGLE, CAT_MULTI, NUMERIC, TEXT = 0, 1, 2, 3
MASTER_SEED = 20221014


class _Field(ctypes.Structure):
    _fields_ = [
        ("kind", ctypes.c_int32),
        ("len_lo", ctypes.c_int32),
        ("len_hi", ctypes.c_int32),
        ("frac_digits", ctypes.c_int32),
        ("zipf_s", ctypes.c_double),
        ("vocab", ctypes.c_double),
        ("lam", ctypes.c_double),
        ("ln_mu", ctypes.c_double),
        ("ln_sigma", ctypes.c_double),
    ]


def build(force: bool = False) -> str:
    """Compile the generator with gcc (host only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.fbxgen_generate.restype = ctypes.c_uint64
        _lib.fbxgen_generate.argtypes = [
            ctypes.c_uint64, ctypes.POINTER(_Field), ctypes.c_int32,
            ctypes.c_uint64, ctypes.c_uint64,
            ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p,
        ]
    return _lib


@dataclass
class FieldSpec:
    kind: int
    len_lo: int = 4
    len_hi: int = 8
    frac_digits: int = -1
    zipf_s: float = 1.1
    vocab: float = 1e5
    lam: float = 3.0
    ln_mu: float = 0.0
    ln_sigma: float = 2.0


@dataclass
class Workload:
    name: str
    seed: int
    n_records: int
    fields: List[FieldSpec]
    spec: str                       # operator-DAG spec text
    n_ops: int = 0
    n_layers: int = 0
    notes: str = ""
    emitted_slots: List[int] = dc_field(default_factory=list)

    @property
    def n_fields(self) -> int:
        return len(self.fields)

    def generate(self, rec_begin: int = 0, n_records: Optional[int] = None,
                 out: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
        """Raw bytes (uint8) and record offsets (uint64, n+1) of a record range."""
        n = self.n_records - rec_begin if n_records is None else n_records
        return generate_records(self.seed, self.fields, rec_begin, n, out=out)


def generate_records(seed: int, fields: List[FieldSpec], rec_begin: int, n_records: int,
                     out: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    lib = _load()
    arr = (_Field * len(fields))()
    for i, f in enumerate(fields):
        arr[i] = _Field(f.kind, f.len_lo, f.len_hi, f.frac_digits, f.zipf_s,
                        float(f.vocab), f.lam, f.ln_mu, f.ln_sigma)
    rec_off = np.zeros(n_records + 1, dtype=np.uint64)
    if out is None:
        probe_n = min(n_records, 512)
        probe_off = np.zeros(probe_n + 1, dtype=np.uint64)
        probe = lib.fbxgen_generate(seed, arr, len(fields), rec_begin, probe_n, None, 0,
                                    probe_off.ctypes.data)
        cap = int(probe / max(probe_n, 1) * n_records * 1.15) + (1 << 16)
        out = np.empty(cap, dtype=np.uint8)
    while True:
        total = lib.fbxgen_generate(seed, arr, len(fields), rec_begin, n_records,
                                    out.ctypes.data, out.size, rec_off.ctypes.data)
        if total <= out.size:
            return out[:total], rec_off
        out = np.empty(int(total), dtype=np.uint8)


# --------------------------------------------------------------------------
# spec text helpers
# --------------------------------------------------------------------------
def _root_line(op_id, kind, slot, seed, emit, fld, **kw) -> str:
    extra = "".join(f" {k}={v}" for k, v in kw.items())
    return f"op {op_id} {kind} slot={slot} seed={seed} emit={emit} field={fld}{extra}"


def _seed64(rng: random.Random) -> int:
    return rng.getrandbits(64)


def _lognormal_bounds(rng: random.Random, n: int, mu: float, sigma: float) -> List[int]:
    vals = sorted(int(rng.lognormvariate(mu, sigma) * 1e6) for _ in range(n))
    return vals


def _records(scale_records: Optional[int], full: int) -> int:
    return full if scale_records is None else int(scale_records)


def config1(n_records: Optional[int] = None) -> Workload:
    """4,096 records x 16 single-valued fields; 16 hashes + 8 pairwise crosses."""
    seed = MASTER_SEED + 1
    rng = random.Random(seed)
    F = 16
    fields = [FieldSpec(CAT_SINGLE, 4, 32, zipf_s=1.1, vocab=1e5) for _ in range(F)]
    lines = ["fbx 1", f"fields {F}"]
    for k in range(F):
        lines.append(_root_line(f"h{k}", "hash", k, _seed64(rng), 1, k, multi=0))
    pairs = set()
    while len(pairs) < 8:
        a, b = rng.randrange(F), rng.randrange(F)
        if a != b:
            pairs.add((a, b))
    for i, (a, b) in enumerate(sorted(pairs)):
        lines.append(f"op x{i} cross slot={100 + i} seed={_seed64(rng)} emit=1 a=h{a} b=h{b}")
    return Workload("config1", seed, _records(n_records, 4096), fields, "\n".join(lines) + "\n",
                    n_ops=24, n_layers=2)


def config2(n_records: Optional[int] = None) -> Workload:
    """1M records x 64 fields (48 multi-valued); per-token hash + 32 list crosses."""
    seed = MASTER_SEED + 2
    rng = random.Random(seed)
    F = 64
    fields = [FieldSpec(CAT_SINGLE if k < 16 else CAT_MULTI, 4, 48, zipf_s=1.1, vocab=1e7, lam=3.0)
              for k in range(F)]
    lines = ["fbx 1", f"fields {F}"]
    for k in range(F):
        lines.append(_root_line(f"h{k}", "hash", k, _seed64(rng), 1, k, multi=0 if k < 16 else 1))
    pairs = set()
    while len(pairs) < 32:
        a, b = rng.randrange(F), rng.randrange(F)
        if a != b:
            pairs.add((a, b))
    for i, (a, b) in enumerate(sorted(pairs)):
        lines.append(f"op x{i} cross slot={1000 + i} seed={_seed64(rng)} emit=1 a=h{a} b=h{b}")
    return Workload("config2", seed, _records(n_records, 1_000_000), fields, "\n".join(lines) + "\n",
                    n_ops=96, n_layers=2)


def config3(n_records: Optional[int] = None) -> Workload:
    """4M records x 32 numeric fields bucketised + one query field as char 3-grams."""
    seed = MASTER_SEED + 3
    rng = random.Random(seed)
    fields = [FieldSpec(NUMERIC, frac_digits=-1, ln_mu=0.0, ln_sigma=2.0) for _ in range(32)]
    fields.append(FieldSpec(TEXT, 16, 256))
    lines = ["fbx 1", "fields 33"]
    for k in range(32):
        bounds = ",".join(str(b) for b in _lognormal_bounds(rng, 64, 0.0, 2.0))
        lines.append(_root_line(f"b{k}", "bucket", k, _seed64(rng), 1, k, multi=0, bounds=bounds))
    lines.append(_root_line("q", "ngram", 32, _seed64(rng), 1, 32, n=3))
    return Workload("config3", seed, _records(n_records, 4_000_000), fields, "\n".join(lines) + "\n",
                    n_ops=33, n_layers=1)


def config4(n_records: Optional[int] = None) -> Workload:
    """2M records x 96 mixed fields through a 4-layer DAG of 200 operators."""
    seed = MASTER_SEED + 4
    rng = random.Random(seed)
    fields: List[FieldSpec] = []
    for k in range(96):
        if k < 48:
            fields.append(FieldSpec(CAT_SINGLE, 4, 24, zipf_s=1.1, vocab=1e7))
        elif k < 72:
            fields.append(FieldSpec(CAT_MULTI, 4, 24, zipf_s=1.1, vocab=1e7, lam=3.0))
        else:
            fields.append(FieldSpec(NUMERIC, frac_digits=-1, ln_mu=0.0, ln_sigma=2.0))
    lines = ["fbx 1", "fields 96"]
    ops = []  # (id, layer, expected_len)
    slot = 0

    def add(op_id, layer, explen, line):
        ops.append([op_id, layer, explen, line, False])

    for k in range(96):
        if k < 48:
            add(f"r{k}", 1, 1.0, _root_line(f"r{k}", "hash", "{slot}", _seed64(rng), "{emit}", k, multi=0))
        elif k < 72:
            add(f"r{k}", 1, 4.0, _root_line(f"r{k}", "hash", "{slot}", _seed64(rng), "{emit}", k, multi=1))
        else:
            bounds = ",".join(str(b) for b in _lognormal_bounds(rng, 64, 0.0, 2.0))
            add(f"r{k}", 1, 1.0, _root_line(f"r{k}", "bucket", "{slot}", _seed64(rng), "{emit}", k,
                                             multi=0, bounds=bounds))
    alphabet = "0123456789abcdefghijklmnopqrstuvwxyz"
    for i in range(12):
        k = rng.randrange(72)
        plen = 1 + rng.randrange(2)
        prefix = "".join(rng.choice(alphabet[:8]) for _ in range(plen)).encode().hex()
        multi = 0 if k < 48 else 1
        explen = (1.0 if k < 48 else 4.0) * (36.0 ** -plen)
        add(f"f{i}", 1, explen,
            _root_line(f"f{i}", "filter", "{slot}", _seed64(rng), "{emit}", k, multi=multi, prefix=prefix))
    for i in range(12):
        k = rng.randrange(72)
        add(f"g{i}", 1, 1.0 if k < 48 else 4.0,
            _root_line(f"g{i}", "hash", "{slot}", _seed64(rng), "{emit}", k, multi=0 if k < 48 else 1))
    assert len(ops) == 120
    consumed = set()
    for layer, count in ((2, 40), (3, 25), (4, 15)):
        for i in range(count):
            while True:
                prev = [o for o in ops if o[1] == layer - 1]
                earlier = [o for o in ops if o[1] < layer]
                a, b = rng.choice(prev), rng.choice(earlier)
                if rng.random() < 0.5:
                    a, b = b, a
                kind = "cross" if rng.random() < 0.7 else "concat"
                explen = a[2] * b[2] if kind == "cross" else a[2] + b[2]
                if kind == "cross" and explen > 64:
                    continue
                break
            op_id = f"L{layer}_{i}"
            if kind == "cross":
                line = f"op {op_id} cross slot={{slot}} seed={_seed64(rng)} emit={{emit}} a={a[0]} b={b[0]}"
            else:
                line = f"op {op_id} concat slot={{slot}} emit={{emit}} a={a[0]} b={b[0]}"
            consumed.add(a[0]); consumed.add(b[0])
            add(op_id, layer, explen, line)
    assert len(ops) == 200
    for o in ops:
        emit = 1 if (rng.random() < 0.8 or o[0] not in consumed) else 0
        lines.append(o[3].format(slot=slot, emit=emit))
        slot += 1
    return Workload("config4", seed, _records(n_records, 2_000_000), fields, "\n".join(lines) + "\n",
                    n_ops=200, n_layers=4)


def config5(n_records: Optional[int] = None) -> Workload:
    """16M records x 100 mixed fields (~12 GB raw); 100 root ops + 64 crosses."""
    seed = MASTER_SEED + 5
    rng = random.Random(seed)
    fields: List[FieldSpec] = []
    for k in range(100):
        if k < 88:
            fields.append(FieldSpec(CAT_SINGLE, 3, 8, zipf_s=1.05, vocab=1e8))
        elif k < 92:
            fields.append(FieldSpec(CAT_MULTI, 3, 8, zipf_s=1.05, vocab=1e8, lam=5.0))
        else:
            fields.append(FieldSpec(NUMERIC, frac_digits=-1, ln_mu=0.0, ln_sigma=2.0))
    lines = ["fbx 1", "fields 100"]
    for k in range(100):
        if k < 88:
            lines.append(_root_line(f"r{k}", "hash", k, _seed64(rng), 1, k, multi=0))
        elif k < 92:
            lines.append(_root_line(f"r{k}", "hash", k, _seed64(rng), 1, k, multi=1))
        else:
            bounds = ",".join(str(b) for b in _lognormal_bounds(rng, 64, 0.0, 2.0))
            lines.append(_root_line(f"r{k}", "bucket", k, _seed64(rng), 1, k, multi=0, bounds=bounds))
    pairs = set()
    while len(pairs) < 60:
        a, b = rng.randrange(88), rng.randrange(88)
        if a != b:
            pairs.add((a, b))
    pairs = sorted(pairs)
    for m in range(88, 92):
        pairs.append((rng.randrange(88), m))
    for i, (a, b) in enumerate(pairs):
        lines.append(f"op x{i} cross slot={1000 + i} seed={_seed64(rng)} emit=1 a=r{a} b=r{b}")
    return Workload("config5", seed, _records(n_records, 16_000_000), fields, "\n".join(lines) + "\n",
                    n_ops=164, n_layers=2)


CONFIGS = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}


def get(config: int, n_records: Optional[int] = None) -> Workload:
    return CONFIGS[config](n_records)
