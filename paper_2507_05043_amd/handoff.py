"""ctypes binding of the chunked payload hand-off (argument marshalling only)."""
from __future__ import annotations

import ctypes
from typing import List, Sequence

import torch

from .stage import load_library

DECODE, PREFILL = 0, 1


class HandoffError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"handoff error {code}: {message}")
        self.code = code


class HandoffRecord(ctypes.Structure):
    _fields_ = [("ticket", ctypes.c_int64), ("kind", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("offset", ctypes.c_int64), ("bytes", ctypes.c_int64), ("pick", ctypes.c_int64),
                ("begin_ms", ctypes.c_double), ("end_ms", ctypes.c_double)]

    def as_tuple(self):
        return (self.ticket, self.kind, self.offset, self.bytes)


_ready = False


def _lib():
    global _ready
    lib = load_library()
    if not _ready:
        i32p, i64p = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64)
        recp = ctypes.POINTER(HandoffRecord)
        lib.handoff_plan.argtypes = [ctypes.c_int32, i32p, ctypes.c_int64, ctypes.c_int64, recp, ctypes.c_int32, i32p]
        lib.handoff_sender_create.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.POINTER(ctypes.c_void_p)]
        lib.handoff_sender_submit.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                              ctypes.c_int32, i32p, ctypes.c_int64, i64p]
        lib.handoff_sender_wait.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32]
        lib.handoff_sender_visible_pick.argtypes = [ctypes.c_void_p, ctypes.c_int64, i64p]
        lib.handoff_sender_picks.argtypes = [ctypes.c_void_p, i64p]
        lib.handoff_sender_log.argtypes = [ctypes.c_void_p, recp, ctypes.c_int32, i32p]
        lib.handoff_sender_destroy.argtypes = [ctypes.c_void_p]
        lib.handoff_sender_destroy.restype = None
        lib.handoff_last_error.restype = ctypes.c_char_p
        for n in ("handoff_plan", "handoff_sender_create", "handoff_sender_submit", "handoff_sender_wait",
                  "handoff_sender_visible_pick", "handoff_sender_picks", "handoff_sender_log"):
            getattr(lib, n).restype = ctypes.c_int
        _ready = True
    return lib


def _check(rc: int) -> None:
    if rc != 0:
        raise HandoffError(rc, _lib().handoff_last_error().decode())


def _q_array(q_lens: Sequence[int]):
    arr = (ctypes.c_int32 * len(q_lens))(*[int(q) for q in q_lens])
    return arr, len(q_lens)


def plan(q_lens: Sequence[int], row_bytes: int, chunk_bytes: int) -> List[tuple]:
    """[(kind, offset, bytes)] of one payload: decode runs, then prefill chunks."""
    lib = _lib()
    arr, n = _q_array(q_lens)
    count = ctypes.c_int32()
    rc = lib.handoff_plan(n, arr, row_bytes, chunk_bytes, None, 0, ctypes.byref(count))
    if rc not in (0, -3):
        _check(rc)
    recs = (HandoffRecord * max(count.value, 1))()
    _check(lib.handoff_plan(n, arr, row_bytes, chunk_bytes, recs, count.value, ctypes.byref(count)))
    return [(recs[i].kind, recs[i].offset, recs[i].bytes) for i in range(count.value)]


class Sender:
    def __init__(self, chunk_bytes: int, device: str = "cuda:0"):
        self.device = torch.device(device)
        h = ctypes.c_void_p()
        _check(_lib().handoff_sender_create(self.device.index or 0, chunk_bytes, ctypes.byref(h)))
        self._h = h

    def submit(self, payload: torch.Tensor, host: torch.Tensor, q_lens: Sequence[int]) -> int:
        """payload: contiguous device [T, row] tensor; host: pinned host tensor of the same bytes."""
        if not payload.is_contiguous() or not host.is_contiguous() or not host.is_pinned():
            raise ValueError("payload must be contiguous and host a contiguous pinned tensor")
        if host.numel() * host.element_size() != payload.numel() * payload.element_size():
            raise ValueError("host buffer and payload differ in size")
        arr, n = _q_array(q_lens)
        row_bytes = payload.shape[1] * payload.element_size()
        ticket = ctypes.c_int64()
        stream = torch.cuda.current_stream(self.device).cuda_stream
        _check(_lib().handoff_sender_submit(self._h, ctypes.c_void_p(stream), payload.data_ptr(), host.data_ptr(), n, arr,
                                            row_bytes, ctypes.byref(ticket)))
        return ticket.value

    def wait(self, ticket: int, kind: int = PREFILL) -> None:
        _check(_lib().handoff_sender_wait(self._h, ticket, kind))

    def visible_pick(self, ticket: int) -> int:
        out = ctypes.c_int64()
        _check(_lib().handoff_sender_visible_pick(self._h, ticket, ctypes.byref(out)))
        return out.value

    def picks(self) -> int:
        out = ctypes.c_int64()
        _check(_lib().handoff_sender_picks(self._h, ctypes.byref(out)))
        return out.value

    def log(self) -> List[HandoffRecord]:
        lib = _lib()
        count = ctypes.c_int32()
        rc = lib.handoff_sender_log(self._h, None, 0, ctypes.byref(count))
        if rc not in (0, -3):
            _check(rc)
        recs = (HandoffRecord * max(count.value, 1))()
        _check(lib.handoff_sender_log(self._h, recs, max(count.value, 1), ctypes.byref(count)))
        return [recs[i] for i in range(count.value)]

    def close(self) -> None:
        if getattr(self, "_h", None):
            _lib().handoff_sender_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()
