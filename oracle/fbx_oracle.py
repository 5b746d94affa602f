"""ctypes loader for the C oracle (``fbx_oracle.c``).

Test infrastructure only.  Nothing in the product package may import this
module; it exists so that tests, the smoke check and the benchmark's CPU
baseline can run the plain CPU definition of the extraction path.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, List, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fbx_oracle.c")
_LIB = os.path.join(_HERE, "libfbx_oracle.so")

OK, E_ARG, E_SPEC, E_NOMEM, E_INPUT = 0, -1, -2, -3, -4


class OracleError(Exception):
    def __init__(self, status: int, msg: str):
        super().__init__(f"oracle status {status}: {msg}")
        self.status = status


class _Slot(ctypes.Structure):
    _fields_ = [("slot_id", ctypes.c_uint32), ("fixed_arity", ctypes.c_uint32),
                ("n_values", ctypes.c_uint64),
                ("values", ctypes.POINTER(ctypes.c_uint64)),
                ("offsets", ctypes.POINTER(ctypes.c_uint64))]


class _Result(ctypes.Structure):
    _fields_ = [("n_records", ctypes.c_uint64), ("n_values_total", ctypes.c_uint64),
                ("n_malformed_numeric", ctypes.c_uint64), ("n_slots", ctypes.c_uint32),
                ("n_layers", ctypes.c_uint32), ("slots", ctypes.POINTER(_Slot))]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc: -O2, no threads, no intrinsics."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-std=c11", "-D_GNU_SOURCE", "-O2", "-Wall", "-shared", "-fPIC",
                               "-o", _LIB, _SRC])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.fbxo_hash_bytes.restype = ctypes.c_uint64
        L.fbxo_hash_bytes.argtypes = [ctypes.c_uint64, ctypes.c_char_p, ctypes.c_size_t]
        L.fbxo_mix64.restype = ctypes.c_uint64
        L.fbxo_mix64.argtypes = [ctypes.c_uint64]
        L.fbxo_cross.restype = ctypes.c_uint64
        L.fbxo_cross.argtypes = [ctypes.c_uint64] * 3
        L.fbxo_parse_micro.restype = ctypes.c_int64
        L.fbxo_parse_micro.argtypes = [ctypes.c_char_p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_int)]
        L.fbxo_bucket_index.restype = ctypes.c_uint32
        L.fbxo_bucket_index.argtypes = [ctypes.c_void_p, ctypes.c_uint32, ctypes.c_int64]
        L.fbxo_extract.restype = ctypes.c_int
        L.fbxo_extract.argtypes = [ctypes.c_char_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_uint64,
                                   ctypes.c_void_p, ctypes.c_uint64, ctypes.POINTER(_Result),
                                   ctypes.c_char_p, ctypes.c_size_t]
        L.fbxo_free.restype = None
        L.fbxo_free.argtypes = [ctypes.POINTER(_Result)]
        L.fbxo_spec_layers.restype = ctypes.c_int
        L.fbxo_spec_layers.argtypes = [ctypes.c_char_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int32,
                                       ctypes.c_void_p, ctypes.c_char_p, ctypes.c_size_t]
        _lib = L
    return _lib


def hash_bytes(seed: int, m: bytes) -> int:
    return lib().fbxo_hash_bytes(seed, m, len(m))


def mix64(x: int) -> int:
    return lib().fbxo_mix64(x)


def cross(K: int, a: int, b: int) -> int:
    return lib().fbxo_cross(K, a, b)


def parse_micro(tok: bytes) -> Tuple[int, bool]:
    bad = ctypes.c_int(0)
    v = lib().fbxo_parse_micro(tok, len(tok), ctypes.byref(bad))
    return v, bool(bad.value)


def bucket_index(bounds, v: int) -> int:
    b = np.ascontiguousarray(np.asarray(bounds, dtype=np.int64))
    return lib().fbxo_bucket_index(b.ctypes.data if b.size else None, b.size, v)


def spec_layers(spec: str) -> Tuple[List[int], List[int]]:
    """(layer, fixed arity) of every operator in spec order."""
    s = spec.encode()
    err = ctypes.create_string_buffer(256)
    n = lib().fbxo_spec_layers(s, len(s), None, 0, None, err, 256)
    if n < 0:
        raise OracleError(n, err.value.decode())
    layers = np.zeros(max(n, 1), dtype=np.int32)
    arity = np.zeros(max(n, 1), dtype=np.uint32)
    lib().fbxo_spec_layers(s, len(s), layers.ctypes.data, n, arity.ctypes.data, err, 256)
    return layers[:n].tolist(), arity[:n].tolist()


class OracleResult:
    """Per-slot ``values`` (uint64) and explicit ``offsets`` (uint64, n_records+1)."""

    def __init__(self):
        self.n_records = 0
        self.n_values_total = 0
        self.n_malformed_numeric = 0
        self.n_layers = 0
        self.slot_ids: List[int] = []
        self.slots: Dict[int, Tuple[np.ndarray, np.ndarray, int]] = {}


def extract(spec: str, raw, rec_off) -> OracleResult:
    raw = np.ascontiguousarray(np.frombuffer(raw, dtype=np.uint8) if isinstance(raw, (bytes, bytearray)) else raw,
                               dtype=np.uint8)
    rec_off = np.ascontiguousarray(rec_off, dtype=np.uint64)
    n_records = max(rec_off.size - 1, 0)
    s = spec.encode() if isinstance(spec, str) else spec
    res = _Result()
    err = ctypes.create_string_buffer(256)
    rc = lib().fbxo_extract(s, len(s), raw.ctypes.data if raw.size else None, raw.size,
                            rec_off.ctypes.data if rec_off.size else None, n_records,
                            ctypes.byref(res), err, 256)
    if rc != OK:
        raise OracleError(rc, err.value.decode())
    out = OracleResult()
    out.n_records = res.n_records
    out.n_values_total = res.n_values_total
    out.n_malformed_numeric = res.n_malformed_numeric
    out.n_layers = res.n_layers
    for i in range(res.n_slots):
        sl = res.slots[i]
        vals = np.ctypeslib.as_array(sl.values, shape=(sl.n_values,)).copy() if sl.n_values else np.zeros(0, np.uint64)
        offs = np.ctypeslib.as_array(sl.offsets, shape=(n_records + 1,)).copy()
        out.slot_ids.append(sl.slot_id)
        out.slots[sl.slot_id] = (vals, offs, sl.fixed_arity)
    lib().fbxo_free(ctypes.byref(res))
    return out
