"""ctypes binding of libsymb.so: argument marshalling only.

Every function here has the name of the C entry point it calls (include/symb.h) and
does nothing but turn torch tensors into device pointers and host lists into C arrays.
All arithmetic runs in the HIP kernels; there is no CPU or PyTorch fallback: if the
library is missing, `lib()` raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsymb.so")

SYMB_OK, SYMB_ERR_INVALID_ARG, SYMB_ERR_BAD_SEGMENTS, SYMB_ERR_UNSUPPORTED, \
    SYMB_ERR_WORKSPACE_TOO_SMALL, SYMB_ERR_DEVICE = range(6)
SYMB_ADAPTER_NONE, SYMB_ADAPTER_LORA, SYMB_ADAPTER_IA3, SYMB_ADAPTER_IA3_IN = range(4)
SYMB_OP_FWD, SYMB_OP_BWD_INPUT, SYMB_OP_ADAPTER_GRAD, SYMB_OP_FWD_INPLACE, SYMB_OP_BWD_INPUT_INPLACE = range(5)
SYMB_OPT_DESCRIPTOR_REUSE, SYMB_OPT_K_SPLIT, SYMB_OPT_SMALL_BATCH_KERNELS, SYMB_OPT_SKINNY_DEEP = range(4)
SYMB_STATIC_SCRATCH_BYTES = 32 << 20
SYMB_BWD_FULL, SYMB_BWD_BASE_ONLY, SYMB_BWD_REUSE_DH = 0, 1, 2
SYMB_GRAD_OVERWRITE, SYMB_GRAD_ACCUMULATE, SYMB_GRAD_REUSE_DH, SYMB_GRAD_REUSE_HS = 0, 1, 2, 4
SYMB_MAX_RANK = 128
SYMB_WEIGHT_LINEAR, SYMB_WEIGHT_CONV1D = 0, 1

EXPORTS = ("symb_create", "symb_destroy", "symb_validate_batch", "symb_debug_row_segment_map",
           "symb_plan_row_tiles", "symb_workspace_bytes", "symb_base_linear_fwd",
           "symb_base_linear_bwd_input", "symb_base_linear_bwd_input_ex", "symb_adapter_grad", "symb_adapter_grad_ex",
           "symb_noise_add", "symb_base_linear_fwd_denoise", "symb_base_linear_fwd_seg", "symb_base_linear_bwd_input_seg",
           "symb_adapter_grad_seg",
           "symb_status_string", "symb_last_error",
           "symb_batcher_create", "symb_batcher_destroy", "symb_batcher_submit", "symb_batcher_pending",
           "symb_batcher_next_due", "symb_batcher_take",
           "symb_debug_gemm_timing_enable", "symb_debug_gemm_timing_read", "symb_debug_descriptor_stats",
           "symb_debug_set_option", "symb_debug_xcd_rule", "symb_base_linear_fwd_static")


class symb_adapter(C.Structure):
    _fields_ = [("kind", C.c_int32), ("rank", C.c_int32), ("scale", C.c_float),
                ("A", C.c_void_p), ("B", C.c_void_p), ("dA", C.c_void_p), ("dB", C.c_void_p)]


class symb_noise(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("rows", C.c_int32), ("reserved", C.c_int32)]


class symb_batch(C.Structure):
    _fields_ = [("d_in", C.c_int32), ("d_out", C.c_int32), ("num_segments", C.c_int32),
                ("seg_offsets", C.POINTER(C.c_int32)), ("adapters", C.POINTER(symb_adapter)),
                ("weight_layout", C.c_int32)]


class SymbError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{text} (status {status})")
        self.status = status


_lib = None


def lib() -> C.CDLL:
    """Loads libsymb.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2507_03220_amd.build` "
                               "(or __graft_entry__.build()) first; there is no fallback path")
        l = C.CDLL(LIB_PATH)
        vp, i32, u32, sz = C.c_void_p, C.c_int32, C.c_uint32, C.c_size_t
        bp = C.POINTER(symb_batch)
        l.symb_create.argtypes = [C.POINTER(vp), C.c_int]
        l.symb_destroy.argtypes = [vp]
        l.symb_validate_batch.argtypes = [bp]
        l.symb_debug_row_segment_map.argtypes = [bp, C.POINTER(i32)]
        l.symb_plan_row_tiles.argtypes = [bp, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]
        l.symb_workspace_bytes.argtypes = [bp, i32, C.POINTER(sz)]
        l.symb_base_linear_fwd.argtypes = [vp, bp, vp, vp, vp, vp, vp, vp, sz, vp]
        l.symb_base_linear_bwd_input.argtypes = [vp, bp, vp, vp, vp, u32, vp, sz, vp]
        l.symb_adapter_grad.argtypes = [vp, bp, vp, vp, vp, u32, vp, sz, vp]
        l.symb_base_linear_bwd_input_ex.argtypes = [vp, bp, vp, vp, vp, vp, u32, vp, sz, vp]
        l.symb_adapter_grad_ex.argtypes = [vp, bp, vp, vp, vp, vp, u32, vp, sz, vp]
        l.symb_base_linear_fwd_seg.argtypes = [vp, bp, C.POINTER(vp), vp, vp, C.POINTER(vp), vp, sz, vp]
        l.symb_base_linear_bwd_input_seg.argtypes = [vp, bp, C.POINTER(vp), vp, C.POINTER(vp), u32, vp, sz, vp]
        l.symb_adapter_grad_seg.argtypes = [vp, bp, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), u32, vp, sz, vp]
        l.symb_noise_add.argtypes = [vp, bp, vp, C.POINTER(symb_noise), vp, vp]
        l.symb_base_linear_fwd_denoise.argtypes = [vp, bp, vp, vp, vp, C.POINTER(symb_noise), vp, vp, sz, vp]
        l.symb_debug_gemm_timing_enable.argtypes = [vp, i32]
        l.symb_debug_gemm_timing_read.argtypes = [vp, i32, C.POINTER(C.c_double), C.POINTER(C.c_int64),
                                                  C.POINTER(C.c_double)]
        l.symb_debug_descriptor_stats.argtypes = [vp, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
        l.symb_debug_set_option.argtypes = [vp, i32, i32]
        l.symb_debug_xcd_rule.argtypes = [vp, C.POINTER(i32), C.POINTER(i32)]
        l.symb_base_linear_fwd_static.argtypes = [vp, bp, vp, vp, vp, vp, vp, vp]
        l.symb_status_string.argtypes = [C.c_int]
        l.symb_status_string.restype = C.c_char_p
        l.symb_last_error.argtypes = [vp]
        l.symb_last_error.restype = C.c_char_p
        for name in EXPORTS:
            if name not in ("symb_status_string", "symb_last_error"):
                getattr(l, name).restype = C.c_int
        _lib = l
    return _lib


def _ptr(t) -> Optional[int]:
    """Device (or host) address of a tensor, None for None; ints pass through."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _check(status: int, handle=None) -> None:
    if status != SYMB_OK:
        l = lib()
        msg = l.symb_last_error(handle).decode() or l.symb_status_string(status).decode()
        raise SymbError(status, f"{l.symb_status_string(status).decode()}: {msg}")


@dataclass
class Adapter:
    """One segment's adapter; tensors are torch device tensors (or raw addresses)."""
    kind: int = SYMB_ADAPTER_NONE
    rank: int = 0
    scale: float = 0.0
    A: object = None
    B: object = None
    dA: object = None
    dB: object = None


class Batch:
    """Owns the C arrays of one symb_batch (host offsets + per-segment descriptors)."""

    def __init__(self, d_in: int, d_out: int, seg_offsets: Sequence[int], adapters: Sequence[Adapter],
                 weight_layout: int = 0):
        S = len(adapters)
        if len(seg_offsets) != S + 1:
            raise ValueError("seg_offsets must have num_segments + 1 entries")
        self._off = (C.c_int32 * (S + 1))(*[int(x) for x in seg_offsets])
        self._ad = (symb_adapter * max(S, 1))()
        self._keep = list(adapters)
        for i, a in enumerate(adapters):
            d = self._ad[i]
            d.kind, d.rank, d.scale = int(a.kind), int(a.rank), float(a.scale)
            d.A, d.B, d.dA, d.dB = _ptr(a.A), _ptr(a.B), _ptr(a.dA), _ptr(a.dB)
        self.c = symb_batch(int(d_in), int(d_out), S, self._off, self._ad, int(weight_layout))
        self.d_in, self.d_out, self.S = int(d_in), int(d_out), S
        self.T = int(seg_offsets[-1]) if S >= 0 and len(seg_offsets) else 0

    def ref(self):
        return C.byref(self.c)


# ---- entry points, same names as the C ABI ----------------------------------------------------
def symb_create(device: int = 0) -> int:
    h = C.c_void_p()
    _check(lib().symb_create(C.byref(h), int(device)))
    return h.value


def symb_destroy(handle) -> None:
    _check(lib().symb_destroy(handle))


def symb_validate_batch(batch: Batch) -> int:
    return int(lib().symb_validate_batch(batch.ref()))


def symb_debug_row_segment_map(batch: Batch):
    import numpy as np
    out = np.empty(max(batch.T, 0), dtype=np.int32)
    _check(lib().symb_debug_row_segment_map(batch.ref(), out.ctypes.data_as(C.POINTER(C.c_int32))))
    return out


def symb_plan_row_tiles(batch: Batch, tile_m: int):
    import numpy as np
    n = max((batch.T + tile_m - 1) // tile_m, 0) if tile_m > 0 else 0
    lo = np.empty(max(n, 1), dtype=np.int32)
    hi = np.empty(max(n, 1), dtype=np.int32)
    cnt = C.c_int32(0)
    _check(lib().symb_plan_row_tiles(batch.ref(), int(tile_m), lo.ctypes.data_as(C.POINTER(C.c_int32)),
                                     hi.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(cnt)))
    return lo[:cnt.value], hi[:cnt.value]


def symb_workspace_bytes(batch: Batch, op: int) -> int:
    out = C.c_size_t(0)
    _check(lib().symb_workspace_bytes(batch.ref(), int(op), C.byref(out)))
    return int(out.value)


def _ws_args(ws):
    if ws is None:
        return None, 0
    return ws.data_ptr(), ws.numel() * ws.element_size()


def symb_base_linear_fwd(handle, batch: Batch, X, W, bias, Y, Ybase=None, ws=None, stream: int = 0) -> None:
    wp, wb = _ws_args(ws)
    _check(lib().symb_base_linear_fwd(handle, batch.ref(), _ptr(X), _ptr(W), _ptr(bias), _ptr(Y), _ptr(Ybase),
                                      wp, wb, stream or None), handle)


def symb_base_linear_fwd_static(handle, batch: Batch, X, W, bias, Y, Ybase=None, stream: int = 0) -> None:
    _check(lib().symb_base_linear_fwd_static(handle, batch.ref(), _ptr(X), _ptr(W), _ptr(bias), _ptr(Y), _ptr(Ybase),
                                             stream or None), handle)


def _noise_array(batch: Batch, noise: Sequence):
    """noise: per segment None or a tensor [rows][width] (rows 1 = broadcast) or a (ptr, rows) pair."""
    if len(noise) != batch.S:
        raise ValueError("one noise entry per segment")
    arr = (symb_noise * max(batch.S, 1))()
    for i, n in enumerate(noise):
        if n is None:
            continue
        if isinstance(n, tuple):
            arr[i].ptr, arr[i].rows = _ptr(n[0]), int(n[1])
        else:
            arr[i].ptr, arr[i].rows = _ptr(n), int(n.shape[0]) if n.dim() > 1 else 1
    return arr


def _ptr_array(batch: Batch, tensors: Sequence):
    if len(tensors) != batch.S:
        raise ValueError("one buffer per segment")
    return (C.c_void_p * max(batch.S, 1))(*[_ptr(t) for t in tensors])


def symb_base_linear_fwd_seg(handle, batch: Batch, X_seg: Sequence, W, bias, Y_seg: Sequence, ws=None, stream: int = 0) -> None:
    wp, wb = _ws_args(ws)
    _check(lib().symb_base_linear_fwd_seg(handle, batch.ref(), _ptr_array(batch, X_seg), _ptr(W), _ptr(bias),
                                          _ptr_array(batch, Y_seg), wp, wb, stream or None), handle)


def symb_base_linear_bwd_input_seg(handle, batch: Batch, dY_seg: Sequence, W, dX_seg: Sequence, flags: int = SYMB_BWD_FULL,
                                   ws=None, stream: int = 0) -> None:
    wp, wb = _ws_args(ws)
    _check(lib().symb_base_linear_bwd_input_seg(handle, batch.ref(), _ptr_array(batch, dY_seg), _ptr(W),
                                                _ptr_array(batch, dX_seg), int(flags), wp, wb, stream or None), handle)


def symb_adapter_grad_seg(handle, batch: Batch, X_seg: Sequence, dY_seg: Sequence, Ybase_seg=None,
                          flags: int = SYMB_GRAD_OVERWRITE, ws=None, stream: int = 0) -> None:
    wp, wb = _ws_args(ws)
    _check(lib().symb_adapter_grad_seg(handle, batch.ref(), _ptr_array(batch, X_seg), _ptr_array(batch, dY_seg),
                                       None if Ybase_seg is None else _ptr_array(batch, Ybase_seg), int(flags),
                                       wp, wb, stream or None), handle)


def symb_noise_add(handle, batch: Batch, X, noise: Sequence, Xn, stream: int = 0) -> None:
    arr = _noise_array(batch, noise)
    _check(lib().symb_noise_add(handle, batch.ref(), _ptr(X), arr, _ptr(Xn), stream or None), handle)


def symb_base_linear_fwd_denoise(handle, batch: Batch, Xn, W, bias, noise_effect: Sequence, Y, ws=None,
                                 stream: int = 0) -> None:
    wp, wb = _ws_args(ws)
    arr = _noise_array(batch, noise_effect)
    _check(lib().symb_base_linear_fwd_denoise(handle, batch.ref(), _ptr(Xn), _ptr(W), _ptr(bias), arr, _ptr(Y),
                                              wp, wb, stream or None), handle)


def symb_base_linear_bwd_input(handle, batch: Batch, dY, W, dX, flags: int = SYMB_BWD_FULL, ws=None,
                               stream: int = 0) -> None:
    wp, wb = _ws_args(ws)
    _check(lib().symb_base_linear_bwd_input(handle, batch.ref(), _ptr(dY), _ptr(W), _ptr(dX), int(flags),
                                            wp, wb, stream or None), handle)


def symb_base_linear_bwd_input_ex(handle, batch: Batch, dY, W, dX, dXbase=None, flags: int = SYMB_BWD_FULL, ws=None,
                                  stream: int = 0) -> None:
    wp, wb = _ws_args(ws)
    _check(lib().symb_base_linear_bwd_input_ex(handle, batch.ref(), _ptr(dY), _ptr(W), _ptr(dX), _ptr(dXbase),
                                               int(flags), wp, wb, stream or None), handle)


def symb_adapter_grad_ex(handle, batch: Batch, X, dY, Ybase=None, dXbase=None, flags: int = SYMB_GRAD_OVERWRITE,
                         ws=None, stream: int = 0) -> None:
    wp, wb = _ws_args(ws)
    _check(lib().symb_adapter_grad_ex(handle, batch.ref(), _ptr(X), _ptr(dY), _ptr(Ybase), _ptr(dXbase), int(flags),
                                      wp, wb, stream or None), handle)


def symb_adapter_grad(handle, batch: Batch, X, dY, Ybase=None, flags: int = SYMB_GRAD_OVERWRITE, ws=None,
                      stream: int = 0) -> None:
    wp, wb = _ws_args(ws)
    _check(lib().symb_adapter_grad(handle, batch.ref(), _ptr(X), _ptr(dY), _ptr(Ybase), int(flags),
                                   wp, wb, stream or None), handle)


def symb_debug_gemm_timing_enable(handle, on: bool) -> None:
    _check(lib().symb_debug_gemm_timing_enable(handle, 1 if on else 0), handle)


def symb_debug_descriptor_stats(handle):
    """Returns (sent, in_place): calls that sent their descriptors / found them on the device."""
    a, b = C.c_int64(0), C.c_int64(0)
    _check(lib().symb_debug_descriptor_stats(handle, C.byref(a), C.byref(b)), handle)
    return a.value, b.value


def symb_debug_gemm_timing_read(handle, variant: int):
    """Returns (ms_total, launches, flops_total) of the GEMM launches of `variant` since enable."""
    ms, n, fl = C.c_double(0), C.c_int64(0), C.c_double(0)
    _check(lib().symb_debug_gemm_timing_read(handle, int(variant), C.byref(ms), C.byref(n), C.byref(fl)), handle)
    return ms.value, n.value, fl.value


def symb_debug_set_option(handle, option: int, value: int) -> None:
    _check(lib().symb_debug_set_option(handle, int(option), int(value)), handle)


def symb_debug_xcd_rule(handle):
    """Returns (holds, [XCD id seen for workgroup ids 0..7])."""
    ok = C.c_int32(0)
    ids = (C.c_int32 * 8)()
    _check(lib().symb_debug_xcd_rule(handle, C.byref(ok), ids), handle)
    return bool(ok.value), list(ids)
