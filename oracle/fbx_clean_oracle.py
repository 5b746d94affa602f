"""ctypes loader for the C oracle of the toy "clean views" stage (``fbx_clean_oracle.c``).

Test infrastructure only: nothing in the product package may import this module.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fbx_clean_oracle.c")
_LIB = os.path.join(_HERE, "libfbx_clean_oracle.so")

OK, E_ARG, E_SPEC, E_NOMEM, E_INPUT = 0, -1, -2, -3, -4


class CleanOracleError(Exception):
    def __init__(self, status: int, msg: str):
        super().__init__(f"clean oracle status {status}: {msg}")
        self.status = status


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-std=c11", "-D_GNU_SOURCE", "-O2", "-Wall", "-shared", "-fPIC", "-o", _LIB, _SRC])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.fbxo_clean.restype = ctypes.c_int
        L.fbxo_clean.argtypes = [ctypes.c_char_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p,
                                 ctypes.c_uint64, ctypes.POINTER(ctypes.c_void_p), ctypes.POINTER(ctypes.c_uint64),
                                 ctypes.POINTER(ctypes.c_void_p), ctypes.POINTER(ctypes.c_uint64), ctypes.c_char_p, ctypes.c_size_t]
        L.fbxo_clean_free.restype = None
        L.fbxo_clean_free.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        _lib = L
    return _lib


def clean(spec: str, raw, rec_off) -> Tuple[np.ndarray, np.ndarray]:
    """(cleaned bytes, offsets of the kept records: n_kept + 1 entries)."""
    raw = np.ascontiguousarray(np.frombuffer(raw, dtype=np.uint8) if isinstance(raw, (bytes, bytearray)) else raw, dtype=np.uint8)
    rec_off = np.ascontiguousarray(rec_off, dtype=np.uint64)
    n = max(rec_off.size - 1, 0)
    s = spec.encode() if isinstance(spec, str) else spec
    out_raw, out_off = ctypes.c_void_p(), ctypes.c_void_p()
    out_len, n_kept = ctypes.c_uint64(), ctypes.c_uint64()
    err = ctypes.create_string_buffer(256)
    rc = lib().fbxo_clean(s, len(s), raw.ctypes.data if raw.size else None, raw.size, rec_off.ctypes.data, n,
                          ctypes.byref(out_raw), ctypes.byref(out_len), ctypes.byref(out_off), ctypes.byref(n_kept), err, 256)
    if rc != OK:
        raise CleanOracleError(rc, err.value.decode())
    data = np.ctypeslib.as_array(ctypes.cast(out_raw, ctypes.POINTER(ctypes.c_uint8)), shape=(max(out_len.value, 1),))[:out_len.value].copy()
    offs = np.ctypeslib.as_array(ctypes.cast(out_off, ctypes.POINTER(ctypes.c_uint64)), shape=(n_kept.value + 1,)).copy()
    lib().fbxo_clean_free(out_raw, out_off)
    return data, offs
