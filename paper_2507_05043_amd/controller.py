"""ctypes binding of the micro-batch controller (argument marshalling only)."""
from __future__ import annotations

import ctypes
from typing import Dict, List, Optional, Sequence, Tuple

from .stage import load_library


class ControllerError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"controller error {code}: {message}")
        self.code = code


class _Point(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("ms", ctypes.c_double)]


class _Profile(ctypes.Structure):
    _fields_ = [("points", ctypes.POINTER(_Point)), ("num_points", ctypes.c_int32)]


class _Link(ctypes.Structure):
    _fields_ = [("latency_ms", ctypes.c_double), ("bytes_per_ms", ctypes.c_double)]


class Choice(ctypes.Structure):
    _fields_ = [("num_microbatches", ctypes.c_int32), ("batch_per_microbatch", ctypes.c_int32),
                ("period_ms", ctypes.c_double), ("round_trip_ms", ctypes.c_double), ("busiest_ms", ctypes.c_double)]


_ready = False


def _lib():
    global _ready
    lib = load_library()
    if not _ready:
        common = [ctypes.c_int32, ctypes.POINTER(_Profile), ctypes.POINTER(_Link), ctypes.c_int32, ctypes.c_double,
                  ctypes.c_double]
        lib.mbc_evaluate.argtypes = common + [ctypes.c_int32, ctypes.POINTER(Choice)]
        lib.mbc_choose.argtypes = common + [ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(Choice)]
        lib.mbc_evaluate.restype = lib.mbc_choose.restype = ctypes.c_int
        lib.mbc_last_error.restype = ctypes.c_char_p
        _ready = True
    return lib


def _marshal(profiles: Sequence[Sequence[Tuple[int, float]]], links: Sequence[Tuple[float, float]]):
    keep = []
    prof = (_Profile * len(profiles))()
    for i, pts in enumerate(profiles):
        arr = (_Point * len(pts))(*[_Point(int(b), float(ms)) for b, ms in pts])
        keep.append(arr)
        prof[i].points = arr
        prof[i].num_points = len(pts)
    lk = (_Link * len(links))(*[_Link(float(lat), float(bw)) for lat, bw in links])
    return prof, lk, keep


def _check(rc: int) -> None:
    if rc != 0:
        raise ControllerError(rc, _lib().mbc_last_error().decode())


def evaluate(profiles, links, num_seqs: int, activation_bytes_per_seq: float, token_bytes_per_seq: float,
             num_microbatches: int) -> Choice:
    """profiles: per stage [(batch, ms), ...]; links: per stage (latency_ms, bytes_per_ms)."""
    prof, lk, keep = _marshal(profiles, links)
    out = Choice()
    _check(_lib().mbc_evaluate(len(profiles), prof, lk, num_seqs, activation_bytes_per_seq, token_bytes_per_seq,
                               num_microbatches, ctypes.byref(out)))
    return out


def choose(profiles, links, num_seqs: int, activation_bytes_per_seq: float, token_bytes_per_seq: float,
           max_batch_per_microbatch: int = 0, max_microbatches: int = 1 << 30) -> Choice:
    prof, lk, keep = _marshal(profiles, links)
    out = Choice()
    _check(_lib().mbc_choose(len(profiles), prof, lk, num_seqs, activation_bytes_per_seq, token_bytes_per_seq,
                             max_batch_per_microbatch, max_microbatches, ctypes.byref(out)))
    return out
