"""ctypes binding of the host-side batching queue (include/symb_batcher.h): marshalling only."""
from __future__ import annotations

import ctypes as C
from typing import List, Tuple

from . import binding as sb


class symb_request(C.Structure):
    _fields_ = [("id", C.c_int64), ("client", C.c_int32), ("n_tokens", C.c_int32),
                ("latency_sensitive", C.c_int32), ("reserved", C.c_int32), ("arrival_us", C.c_double)]


class symb_batch_policy(C.Structure):
    _fields_ = [("base_wait_us", C.c_double), ("per_token_wait_us", C.c_double), ("max_wait_us", C.c_double),
                ("max_tokens", C.c_int32), ("reserved", C.c_int32)]


EXPORTS = ("symb_batcher_create", "symb_batcher_destroy", "symb_batcher_submit", "symb_batcher_pending",
           "symb_batcher_next_due", "symb_batcher_take")

_ready = False


def _lib():
    global _ready
    l = sb.lib()
    if not _ready:
        vp = C.c_void_p
        l.symb_batcher_create.argtypes = [C.POINTER(vp), C.POINTER(symb_batch_policy), C.c_int32]
        l.symb_batcher_destroy.argtypes = [vp]
        l.symb_batcher_submit.argtypes = [vp, C.c_int32, C.POINTER(symb_request)]
        l.symb_batcher_pending.argtypes = [vp, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int64)]
        l.symb_batcher_next_due.argtypes = [vp, C.c_int32, C.POINTER(C.c_double)]
        l.symb_batcher_take.argtypes = [vp, C.c_int32, C.c_double, C.c_int32, C.POINTER(C.c_int64),
                                        C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        for n in EXPORTS:
            getattr(l, n).restype = C.c_int
        _ready = True
    return l


def _check(st: int) -> None:
    if st != sb.SYMB_OK:
        raise sb.SymbError(st, sb.lib().symb_status_string(st).decode())


class Batcher:
    def __init__(self, base_wait_us: float, per_token_wait_us: float, max_wait_us: float, max_tokens: int,
                 num_layers: int = 1):
        self._h = C.c_void_p()
        pol = symb_batch_policy(base_wait_us, per_token_wait_us, max_wait_us, int(max_tokens), 0)
        _check(_lib().symb_batcher_create(C.byref(self._h), C.byref(pol), int(num_layers)))

    def close(self) -> None:
        if self._h:
            _check(_lib().symb_batcher_destroy(self._h))
            self._h = C.c_void_p()

    def submit(self, layer: int, rid: int, client: int, n_tokens: int, latency_sensitive: bool, arrival_us: float) -> None:
        r = symb_request(int(rid), int(client), int(n_tokens), 1 if latency_sensitive else 0, 0, float(arrival_us))
        _check(_lib().symb_batcher_submit(self._h, int(layer), C.byref(r)))

    def pending(self, layer: int) -> Tuple[int, int]:
        n, t = C.c_int32(0), C.c_int64(0)
        _check(_lib().symb_batcher_pending(self._h, int(layer), C.byref(n), C.byref(t)))
        return n.value, t.value

    def next_due(self, layer: int) -> float:
        d = C.c_double(0)
        _check(_lib().symb_batcher_next_due(self._h, int(layer), C.byref(d)))
        return d.value

    def take(self, layer: int, now_us: float, capacity: int = 4096) -> Tuple[List[int], List[int]]:
        ids = (C.c_int64 * capacity)()
        off = (C.c_int32 * (capacity + 1))()
        n = C.c_int32(0)
        _check(_lib().symb_batcher_take(self._h, int(layer), float(now_us), int(capacity), ids, off, C.byref(n)))
        return list(ids[:n.value]), list(off[:n.value + 1])
