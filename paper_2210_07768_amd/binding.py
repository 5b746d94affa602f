"""Thin ctypes binding over the C ABI of ``libfbx.so`` (see ``include/fbx.h``).

Argument marshalling only: every step of the extraction path runs in the
library's HIP kernels.  PyTorch appears solely as the owner of device memory
and streams.  If the library has not been built the import of this module
fails loudly; there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, List, Optional, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfbx.so")

OK, E_ARG, E_SPEC, E_NOMEM, E_INPUT, E_HIP = 0, -1, -2, -3, -4, -5

EXPORTS = [
    "fbx_plan_create", "fbx_plan_destroy", "fbx_plan_workspace_hint", "fbx_plan_set_workspace",
    "fbx_extract", "fbx_last_error", "fbx_status_str", "fbx_plan_info", "fbx_plan_set_option",
    "fbx_plan_kernel_ms", "fbx_plan_compiled", "fbx_arena_alloc", "fbx_arena_reset",
    "fbx_extract_static", "fbx_static_scratch_bytes", "fbx_plan_kernel_source",
    "fbx_launch_overhead", "fbx_extract_unordered",
    "fbx_clean_create", "fbx_clean_destroy", "fbx_clean_last_error", "fbx_clean_scratch_hint", "fbx_clean_run",
]


class FbxError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"fbx status {status}: {msg}")
        self.status = status
        self.required_bytes = 0


class SlotView(ctypes.Structure):
    _fields_ = [("slot_id", ctypes.c_uint32), ("fixed_arity", ctypes.c_uint32),
                ("n_values", ctypes.c_uint64), ("values", ctypes.c_void_p), ("offsets", ctypes.c_void_p),
                ("tile_ends", ctypes.c_void_p)]


class Result(ctypes.Structure):
    _fields_ = [("n_records", ctypes.c_uint64), ("n_values_total", ctypes.c_uint64),
                ("n_malformed_numeric", ctypes.c_uint64), ("arena_high_water", ctypes.c_uint64),
                ("n_slots", ctypes.c_uint32), ("n_layers", ctypes.c_uint32),
                ("slots", ctypes.POINTER(SlotView)),
                ("tile_launches", ctypes.c_uint32), ("arrival_tile_records", ctypes.c_uint32)]


class CleanResult(ctypes.Structure):
    _fields_ = [("n_kept", ctypes.c_uint64), ("out_len", ctypes.c_uint64), ("required_scratch", ctypes.c_uint64)]


class UnorderedResult(ctypes.Structure):
    _fields_ = [("n_values", ctypes.c_uint64), ("n_malformed_numeric", ctypes.c_uint64), ("pool_head", ctypes.c_uint64)]


_lib = None


def lib():
    """Load libfbx.so (built beforehand by ``paper_2210_07768_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2210_07768_amd.build` first")
        # PyTorch ships its own HIP runtime; load it first so that libfbx binds to the
        # same runtime instance that owns the device memory and streams it is handed.
        import torch  # noqa: F401

        L = ctypes.CDLL(LIB_PATH)
        vp, u64, u32 = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32
        L.fbx_plan_create.restype = ctypes.c_int
        L.fbx_plan_create.argtypes = [ctypes.c_char_p, ctypes.c_size_t, ctypes.POINTER(vp)]
        L.fbx_plan_destroy.restype = None
        L.fbx_plan_destroy.argtypes = [vp]
        L.fbx_plan_workspace_hint.restype = ctypes.c_int
        L.fbx_plan_workspace_hint.argtypes = [vp, u64, u64, ctypes.POINTER(u64)]
        L.fbx_plan_set_workspace.restype = ctypes.c_int
        L.fbx_plan_set_workspace.argtypes = [vp, vp, u64]
        L.fbx_extract.restype = ctypes.c_int
        L.fbx_extract.argtypes = [vp, vp, u64, vp, u64, vp, ctypes.POINTER(Result)]
        L.fbx_extract_static.restype = ctypes.c_int
        L.fbx_extract_static.argtypes = [vp, vp, u64, vp, u64, vp, u64, vp, ctypes.POINTER(Result)]
        L.fbx_static_scratch_bytes.restype = u64
        L.fbx_static_scratch_bytes.argtypes = []
        L.fbx_plan_kernel_source.restype = ctypes.c_int
        L.fbx_plan_kernel_source.argtypes = [vp, u64, u64, ctypes.c_int, ctypes.c_char_p, ctypes.c_size_t,
                                             ctypes.POINTER(ctypes.c_size_t)]
        L.fbx_extract_unordered.restype = ctypes.c_int
        L.fbx_extract_unordered.argtypes = [vp, u32, vp, u64, vp, u64, vp, u64, vp, ctypes.c_int, vp, vp, vp,
                                            ctypes.POINTER(UnorderedResult)]
        L.fbx_clean_create.restype = ctypes.c_int
        L.fbx_clean_create.argtypes = [ctypes.c_char_p, ctypes.c_size_t, ctypes.POINTER(vp)]
        L.fbx_clean_destroy.restype = None
        L.fbx_clean_destroy.argtypes = [vp]
        L.fbx_clean_last_error.restype = ctypes.c_char_p
        L.fbx_clean_last_error.argtypes = [vp]
        L.fbx_clean_scratch_hint.restype = ctypes.c_int
        L.fbx_clean_scratch_hint.argtypes = [vp, u64, ctypes.POINTER(u64)]
        L.fbx_clean_run.restype = ctypes.c_int
        L.fbx_clean_run.argtypes = [vp, vp, u64, vp, u64, vp, u64, vp, vp, u64, vp, ctypes.POINTER(CleanResult)]
        L.fbx_launch_overhead.restype = ctypes.c_int
        L.fbx_launch_overhead.argtypes = [u32, vp, ctypes.POINTER(ctypes.c_double)]
        L.fbx_last_error.restype = ctypes.c_char_p
        L.fbx_last_error.argtypes = [vp]
        L.fbx_status_str.restype = ctypes.c_char_p
        L.fbx_status_str.argtypes = [ctypes.c_int]
        L.fbx_plan_compiled.restype = ctypes.c_int
        L.fbx_plan_compiled.argtypes = [vp, ctypes.POINTER(u32), ctypes.POINTER(ctypes.c_double)]
        L.fbx_plan_info.restype = ctypes.c_int
        L.fbx_plan_info.argtypes = [vp, ctypes.POINTER(u32), ctypes.POINTER(u32), vp, vp]
        L.fbx_plan_set_option.restype = ctypes.c_int
        L.fbx_plan_set_option.argtypes = [vp, ctypes.c_char_p, ctypes.c_int64]
        L.fbx_plan_kernel_ms.restype = ctypes.c_int
        L.fbx_plan_kernel_ms.argtypes = [vp, u32, ctypes.POINTER(ctypes.c_float)]
        L.fbx_arena_alloc.restype = ctypes.c_int
        L.fbx_arena_alloc.argtypes = [vp, vp, u64, vp, u32, vp]
        L.fbx_arena_reset.restype = ctypes.c_int
        L.fbx_arena_reset.argtypes = [vp, u64, vp]
        _lib = L
    return _lib


class Slot:
    """One emitted slot of a result; ``values`` / ``offsets`` are torch views of the workspace
    (made when first asked for: a result with hundreds of slots costs nothing to hand over)."""

    def __init__(self, slot_id, fixed_arity, n_values, ws64, values_at, offsets_at, n_offsets, tile_ends_at=None, n_tiles=0):
        self.slot_id, self.fixed_arity, self.n_values = slot_id, fixed_arity, n_values
        self._ws64, self._values_at, self._offsets_at, self._n_offsets = ws64, values_at, offsets_at, n_offsets
        self._tile_ends_at, self._n_tiles = tile_ends_at, n_tiles
        self._values = self._offsets = None

    @property
    def tile_ends(self):
        """Arrival order only (ExtractResult.arrival_tile_records != 0, ragged slot): where each tile's share ends."""
        if self._tile_ends_at is None:
            return None
        return self._ws64[self._tile_ends_at:self._tile_ends_at + self._n_tiles]

    @property
    def values(self):
        if self._values is None:
            self._values = self._ws64[self._values_at:self._values_at + self.n_values]
        return self._values

    @property
    def offsets(self):
        """None for a slot of fixed arity (offsets are implicit)."""
        if self._offsets_at is None:
            return None
        if self._offsets is None:
            self._offsets = self._ws64[self._offsets_at:self._offsets_at + self._n_offsets]
        return self._offsets


class ExtractResult:
    """What fbx_extract reported.  ``slots`` (slot id -> Slot) and ``slot_ids`` (in emission order)
    are built from the library's slot table when first asked for."""

    def __init__(self):
        self.n_records = 0
        self.n_values_total = 0
        self.n_malformed_numeric = 0
        self.arena_high_water = 0
        self.n_layers = 0
        self.tile_launches = 0
        self.arrival_tile_records = 0   # 0: ragged slots in record order; k: tiles of k records in arrival order (fbx.h)
        self.note = ""
        self._table = None   # (bytes of the library's slot table, workspace as int64, its base address, offsets per slot)
        self._slots = None
        self._slot_ids = None

    def _build(self):
        table, ws64, base, n_offsets = self._table
        k = self.arrival_tile_records
        n_tiles = -(-(n_offsets - 1) // k) if k else 0
        n = len(table) // ctypes.sizeof(SlotView)
        self._slots, self._slot_ids = {}, []
        for sv in ((SlotView * n).from_buffer_copy(table) if n else ()):
            v0 = ((sv.values or base) - base) // 8
            o0 = (sv.offsets - base) // 8 if sv.offsets else None
            # (the table of tile ends lies in the workspace; with the entry point that allocates nothing it does not, and no view is made)
            inside = sv.tile_ends and base <= sv.tile_ends < base + ws64.numel() * 8
            t0 = (sv.tile_ends - base) // 8 if inside else None
            self._slots[sv.slot_id] = Slot(sv.slot_id, sv.fixed_arity, sv.n_values, ws64, v0, o0, n_offsets, t0, n_tiles)
            self._slot_ids.append(sv.slot_id)

    @property
    def slots(self) -> Dict[int, Slot]:
        if self._slots is None:
            self._build()
        return self._slots

    @property
    def slot_ids(self) -> List[int]:
        if self._slot_ids is None:
            self._build()
        return self._slot_ids


class Plan:
    """fbx_plan_create / fbx_plan_set_workspace / fbx_extract / fbx_plan_destroy."""

    def __init__(self, spec: str):
        self._h = ctypes.c_void_p()
        s = spec.encode() if isinstance(spec, str) else spec
        st = lib().fbx_plan_create(s, len(s), ctypes.byref(self._h))
        if st != OK:
            self._h = ctypes.c_void_p()
            raise FbxError(st, lib().fbx_last_error(None).decode())
        self._ws = None

    def close(self):
        if getattr(self, "_h", None) and self._h.value:
            lib().fbx_plan_destroy(self._h)
            self._h = ctypes.c_void_p()
        self._ws = None

    __del__ = close

    def _check(self, st: int):
        if st != OK:
            raise FbxError(st, lib().fbx_last_error(self._h).decode())

    def info(self) -> Tuple[int, int, List[int], List[int]]:
        n_ops, n_layers = ctypes.c_uint32(), ctypes.c_uint32()
        self._check(lib().fbx_plan_info(self._h, ctypes.byref(n_ops), ctypes.byref(n_layers), None, None))
        layers = (ctypes.c_uint32 * max(n_ops.value, 1))()
        arity = (ctypes.c_uint32 * max(n_ops.value, 1))()
        self._check(lib().fbx_plan_info(self._h, None, None, layers, arity))
        return n_ops.value, n_layers.value, list(layers)[:n_ops.value], list(arity)[:n_ops.value]

    def compiled(self) -> Tuple[int, float]:
        """(tile kernels compiled for this plan so far, milliseconds spent compiling them)."""
        n, ms = ctypes.c_uint32(), ctypes.c_double()
        self._check(lib().fbx_plan_compiled(self._h, ctypes.byref(n), ctypes.byref(ms)))
        return n.value, ms.value

    def kernel_source(self, raw_len: int, n_records: int, mode: int) -> str:
        """The text that compile=1 hands to the run-time compiler for a batch of this shape."""
        need = ctypes.c_size_t()
        self._check(lib().fbx_plan_kernel_source(self._h, raw_len, n_records, mode, None, 0, ctypes.byref(need)))
        buf = ctypes.create_string_buffer(need.value)
        self._check(lib().fbx_plan_kernel_source(self._h, raw_len, n_records, mode, buf, need.value, None))
        return buf.value.decode()

    def set_option(self, key: str, value: int):
        self._check(lib().fbx_plan_set_option(self._h, key.encode(), int(value)))

    def workspace_hint(self, raw_len: int, n_records: int) -> int:
        out = ctypes.c_uint64()
        self._check(lib().fbx_plan_workspace_hint(self._h, raw_len, n_records, ctypes.byref(out)))
        return out.value

    def set_workspace(self, ws):
        """ws: a torch uint8 CUDA tensor; the caller keeps ownership (a reference is held here)."""
        self._check(lib().fbx_plan_set_workspace(self._h, ws.data_ptr(), ws.numel()))
        self._ws = ws

    def kernel_ms(self, which: int) -> float:
        ms = ctypes.c_float()
        self._check(lib().fbx_plan_kernel_ms(self._h, which, ctypes.byref(ms)))
        return ms.value

    def kernel_ms_all(self, which_ids) -> Dict[int, float]:
        """fbx_plan_kernel_ms for every timer of the list that the last call used (no exception for the others)."""
        out, ms, fn = {}, ctypes.c_float(), lib().fbx_plan_kernel_ms
        for which in which_ids:
            if fn(self._h, which, ctypes.byref(ms)) == 0:
                out[which] = ms.value
        return out

    def extract_unordered(self, slot_id: int, d_raw, d_rec_off, pool, state, thread_offsets, lengths, reset: bool = True,
                          stream: Optional[int] = None) -> UnorderedResult:
        """fbx_extract_unordered: pool (uint8), state (4 x int64), thread_offsets (int64, one per record) and
        lengths (int32, one per record) are CUDA tensors owned by the caller."""
        import torch

        if stream is None:
            stream = torch.cuda.current_stream().cuda_stream
        res = UnorderedResult()
        st = lib().fbx_extract_unordered(self._h, slot_id, d_raw.data_ptr() if d_raw.numel() else 0, d_raw.numel(),
                                         d_rec_off.data_ptr(), d_rec_off.numel() - 1, pool.data_ptr(), pool.numel(),
                                         state.data_ptr(), 1 if reset else 0, thread_offsets.data_ptr(), lengths.data_ptr(),
                                         stream, ctypes.byref(res))
        if st != OK:
            err = FbxError(st, lib().fbx_last_error(self._h).decode())
            err.required_bytes = res.pool_head if st == E_NOMEM else 0
            raise err
        return res

    def extract_raw(self, raw_ptr: int, raw_len: int, off_ptr: int, n_records: int, stream: int = 0) -> Result:
        res = Result()
        st = lib().fbx_extract(self._h, raw_ptr, raw_len, off_ptr, n_records, stream, ctypes.byref(res))
        if st != OK:
            err = FbxError(st, lib().fbx_last_error(self._h).decode())
            err.required_bytes = res.arena_high_water if st == E_NOMEM else 0
            raise err
        return res

    def extract(self, d_raw, d_rec_off, stream: Optional[int] = None, out_buffer=None) -> ExtractResult:
        """d_raw: uint8 CUDA tensor; d_rec_off: int64/uint64 CUDA tensor of n_records + 1 entries.
        With out_buffer (a uint8 CUDA tensor, 256-byte aligned) the call goes to fbx_extract_static:
        no workspace, results in out_buffer."""
        import torch

        if stream is None:
            stream = torch.cuda.current_stream().cuda_stream
        n_records = d_rec_off.numel() - 1
        raw_ptr = d_raw.data_ptr() if d_raw.numel() else 0
        if out_buffer is None:
            res = self.extract_raw(raw_ptr, d_raw.numel(), d_rec_off.data_ptr(), n_records, stream)
            home = self._ws
        else:
            res = Result()
            st = lib().fbx_extract_static(self._h, raw_ptr, d_raw.numel(), d_rec_off.data_ptr(), n_records,
                                          out_buffer.data_ptr(), out_buffer.numel(), stream, ctypes.byref(res))
            if st != OK:
                err = FbxError(st, lib().fbx_last_error(self._h).decode())
                err.required_bytes = res.arena_high_water if st == E_NOMEM else 0
                raise err
            home = out_buffer
        out = ExtractResult()
        out.n_records, out.n_values_total = res.n_records, res.n_values_total
        out.n_malformed_numeric, out.arena_high_water = res.n_malformed_numeric, res.arena_high_water
        out.n_layers = res.n_layers
        out.tile_launches = res.tile_launches
        out.arrival_tile_records = res.arrival_tile_records
        out.note = lib().fbx_last_error(self._h).decode()
        # the library's slot table is overwritten by the next call: copy the plain numbers out now
        ws64 = home[: home.numel() // 8 * 8].view(torch.int64)
        table = ctypes.string_at(res.slots, res.n_slots * ctypes.sizeof(SlotView)) if res.n_slots else b""
        out._table = (table, ws64, home.data_ptr(), n_records + 1)
        return out


def extract_with_retry(plan: Plan, d_raw, d_rec_off, device="cuda", slack: float = 1.0):
    """Allocate a workspace from the hint, run, and grow once if the library asks for more."""
    import torch

    n_records = d_rec_off.numel() - 1
    need = plan.workspace_hint(d_raw.numel(), n_records)
    for _ in range(3):
        ws = torch.empty(int(need * slack) + 256, dtype=torch.uint8, device=device)
        plan.set_workspace(ws)
        try:
            return plan.extract(d_raw, d_rec_off), ws
        except FbxError as e:
            if e.status != E_NOMEM or not e.required_bytes:
                raise
            need = e.required_bytes
    raise RuntimeError("workspace kept growing")


def arena_alloc(d_head, d_sizes, d_offsets, block_threads: int = 256, stream: int = 0):
    st = lib().fbx_arena_alloc(d_head.data_ptr(), d_sizes.data_ptr(), d_sizes.numel(), d_offsets.data_ptr(),
                               block_threads, stream)
    if st != OK:
        raise FbxError(st, lib().fbx_status_str(st).decode())


def arena_reset(d_head, value: int, stream: int = 0):
    st = lib().fbx_arena_reset(d_head.data_ptr(), value, stream)
    if st != OK:
        raise FbxError(st, lib().fbx_status_str(st).decode())


def launch_overhead(n_launches: int, stream: int = 0) -> float:
    """Microseconds for n_launches back-to-back launches of an empty kernel with five pointer arguments."""
    us = ctypes.c_double()
    st = lib().fbx_launch_overhead(n_launches, stream, ctypes.byref(us))
    if st != OK:
        raise FbxError(st, lib().fbx_status_str(st).decode())
    return us.value


class Clean:
    """fbx_clean_create / fbx_clean_run / fbx_clean_destroy: the toy "clean views" stage."""

    def __init__(self, spec: str):
        self._h = ctypes.c_void_p()
        s = spec.encode() if isinstance(spec, str) else spec
        st = lib().fbx_clean_create(s, len(s), ctypes.byref(self._h))
        if st != OK:
            self._h = ctypes.c_void_p()
            raise FbxError(st, lib().fbx_clean_last_error(None).decode())

    def close(self):
        if getattr(self, "_h", None) and self._h.value:
            lib().fbx_clean_destroy(self._h)
            self._h = ctypes.c_void_p()

    __del__ = close

    def scratch_hint(self, n_records: int) -> int:
        out = ctypes.c_uint64()
        st = lib().fbx_clean_scratch_hint(self._h, n_records, ctypes.byref(out))
        if st != OK:
            raise FbxError(st, "bad argument")
        return out.value

    def run(self, d_raw, d_rec_off, d_out, d_out_off, scratch, stream: Optional[int] = None) -> CleanResult:
        """All arguments are CUDA tensors owned by the caller (uint8, int64, uint8, int64, uint8)."""
        import torch

        if stream is None:
            stream = torch.cuda.current_stream().cuda_stream
        res = CleanResult()
        st = lib().fbx_clean_run(self._h, d_raw.data_ptr() if d_raw.numel() else 0, d_raw.numel(), d_rec_off.data_ptr(),
                                 d_rec_off.numel() - 1, d_out.data_ptr() if d_out.numel() else 0, d_out.numel(),
                                 d_out_off.data_ptr(), scratch.data_ptr(), scratch.numel(), stream, ctypes.byref(res))
        if st != OK:
            err = FbxError(st, lib().fbx_clean_last_error(self._h).decode())
            err.required_bytes = res.out_len if st == E_NOMEM else 0
            raise err
        return res
