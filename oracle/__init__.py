"""ctypes front end of the fp64 CPU oracle (oracle/symb_oracle.c).

TEST INFRASTRUCTURE ONLY.  Importable from tests/, the smoke check and the bench's
cpu_baseline leg; the GPU library and its Python binding never import this package,
and this package never imports them.  It adds no arithmetic of its own: it builds
the C file with gcc, marshals numpy arrays of bf16 bit patterns, and returns fp64.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "symb_oracle.c")
_LIB = os.path.join(_HERE, "libsymb_oracle.so")

NONE, LORA, IA3, IA3_IN = 0, 1, 2, 3


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP over independent rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


class _Adapter(C.Structure):
    _fields_ = [("kind", C.c_int32), ("rank", C.c_int32), ("scale", C.c_double),
                ("A", C.c_void_p), ("B", C.c_void_p)]


@dataclass
class Adapter:
    """Host adapter of one segment: bit patterns (uint16 bf16) in storage layout."""
    kind: int = NONE
    rank: int = 0
    scale: float = 0.0
    A: Optional[np.ndarray] = None  # LoRA [rank, d_in]; IA3 l [d_out]; IA3_IN l [d_in]
    B: Optional[np.ndarray] = None  # LoRA [d_out, rank]


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_num_threads.restype = C.c_int
    return _lib


def num_threads() -> int:
    return int(lib().orc_num_threads())


def _u16(a: Optional[np.ndarray]):
    if a is None:
        return None
    assert a.dtype == np.uint16 and a.flags["C_CONTIGUOUS"], "bf16 bit patterns, contiguous"
    return a.ctypes.data_as(C.c_void_p)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _pack(adapters: Sequence[Adapter], d_in: int, d_out: int):
    arr = (_Adapter * max(1, len(adapters)))()
    for i, a in enumerate(adapters):
        arr[i].kind, arr[i].rank, arr[i].scale = int(a.kind), int(a.rank), float(a.scale)
        if a.kind == LORA:
            assert a.A.shape == (a.rank, d_in) and a.B.shape == (d_out, a.rank)
        elif a.kind == IA3:
            assert a.A.shape == (d_out,)
        elif a.kind == IA3_IN:
            assert a.A.shape == (d_in,)
        arr[i].A = _u16(a.A).value if a.A is not None else None
        arr[i].B = _u16(a.B).value if a.B is not None else None
    return arr


def row_segment_map(off) -> np.ndarray:
    off = _i32(off)
    S = len(off) - 1
    out = np.empty(max(int(off[-1]), 0), dtype=np.int32)
    rc = lib().orc_row_segment_map(C.c_int32(S), off.ctypes.data_as(C.c_void_p),
                                   out.ctypes.data_as(C.c_void_p))
    if rc:
        raise ValueError("invalid segment offsets")
    return out


def forward(off, adapters: Sequence[Adapter], X: np.ndarray, W: np.ndarray,
            bias: Optional[np.ndarray] = None, rows=None, client_bf16: bool = False):
    """Returns (Y0, Y) as fp64 [nrows, d_out] for the listed rows (default: all).  client_bf16: the
    product x * l_i of IA3_IN segments is the bf16 tensor the paper's client would send (client_scale);
    Y0 stays the base output of the unscaled input."""
    if client_bf16 and any(a.kind == IA3_IN for a in adapters):
        Y0, _ = forward(off, adapters, X, W, bias, rows=rows)
        _, Y = forward(off, _without(adapters, IA3_IN), client_scale(off, adapters, X, IA3_IN), W, bias, rows=rows)
        return Y0, Y
    off = _i32(off)
    S = len(off) - 1
    d_out, d_in = W.shape
    assert X.shape[1] == d_in and X.shape[0] >= off[-1]
    rows_a = None if rows is None else _i32(rows)
    n = int(off[-1]) if rows is None else len(rows_a)
    Y0 = np.empty((n, d_out), dtype=np.float64)
    Y = np.empty((n, d_out), dtype=np.float64)
    ad = _pack(adapters, d_in, d_out)
    rc = lib().orc_forward_rows(C.c_int32(d_in), C.c_int32(d_out), C.c_int32(S),
                                off.ctypes.data_as(C.c_void_p), ad, _u16(X), _u16(W), _u16(bias),
                                C.c_int32(n), None if rows_a is None else rows_a.ctypes.data_as(C.c_void_p),
                                Y0.ctypes.data_as(C.c_void_p), Y.ctypes.data_as(C.c_void_p))
    if rc:
        raise ValueError("oracle forward: bad offsets or row index")
    return Y0, Y


def _noise_args(off, noise: Sequence[Optional[np.ndarray]], width: int):
    """noise[i]: None or bf16 bits [rows][width] (rows 1 = broadcast over the segment)."""
    S = len(off) - 1
    assert len(noise) == S
    keep = [None if n is None else np.ascontiguousarray(np.asarray(n, dtype=np.uint16).reshape(-1, width)) for n in noise]
    ptrs = (C.c_void_p * max(S, 1))(*[None if n is None else n.ctypes.data for n in keep])
    rows = np.array([0 if n is None else n.shape[0] for n in keep] or [0], dtype=np.int32)
    return keep, ptrs, rows


def noise_add(off, X: np.ndarray, noise: Sequence[Optional[np.ndarray]]) -> np.ndarray:
    """Client prepass of the privacy flow (Sec. 3.8): bf16 bits of x + n per segment."""
    off = _i32(off)
    S = len(off) - 1
    width = X.shape[1]
    keep, ptrs, rows = _noise_args(off, noise, width)
    Xc = np.ascontiguousarray(X, dtype=np.uint16)
    out = np.empty_like(Xc)
    rc = lib().orc_noise_add(C.c_int32(width), C.c_int32(S), off.ctypes.data_as(C.c_void_p), _u16(Xc), ptrs,
                             rows.ctypes.data_as(C.c_void_p), out.ctypes.data_as(C.c_void_p))
    if rc:
        raise ValueError("oracle noise_add: bad offsets or noise rows")
    return out


def forward_private(off, adapters: Sequence[Adapter], Xn: np.ndarray, W: np.ndarray, bias: Optional[np.ndarray],
                    noise: Sequence[Optional[np.ndarray]], rows=None) -> np.ndarray:
    """y = (layer(xn) + b) - layer_without_bias(n), eqs. (1)-(3) of Sec. 3.8, fp64 [nrows, d_out]."""
    off = _i32(off)
    S = len(off) - 1
    d_out, d_in = W.shape
    assert Xn.shape[1] == d_in and Xn.shape[0] >= off[-1]
    rows_a = None if rows is None else _i32(rows)
    n = int(off[-1]) if rows is None else len(rows_a)
    keep, ptrs, nrows = _noise_args(off, noise, d_in)
    Y = np.empty((n, d_out), dtype=np.float64)
    ad = _pack(adapters, d_in, d_out)
    rc = lib().orc_forward_private_rows(C.c_int32(d_in), C.c_int32(d_out), C.c_int32(S),
                                        off.ctypes.data_as(C.c_void_p), ad, _u16(Xn), _u16(W), _u16(bias), ptrs,
                                        nrows.ctypes.data_as(C.c_void_p), C.c_int32(n),
                                        None if rows_a is None else rows_a.ctypes.data_as(C.c_void_p),
                                        Y.ctypes.data_as(C.c_void_p))
    if rc:
        raise ValueError("oracle forward_private: bad offsets, noise rows or row index")
    return Y


def forward_denoise(off, adapters: Sequence[Adapter], Xn: np.ndarray, W: np.ndarray, bias: Optional[np.ndarray],
                    neff: Sequence[Optional[np.ndarray]], rows=None, client_bf16: bool = False) -> np.ndarray:
    """y = (layer(xn) + b) - neff with the noise effect given as the bf16 tensor the client kept
    (steps (2) and (3) of Sec. 3.8); neff[i]: None or bf16 bits [rows][d_out]; fp64 [nrows, d_out].
    client_bf16: as in forward()."""
    if client_bf16 and any(a.kind == IA3_IN for a in adapters):
        return forward_denoise(off, _without(adapters, IA3_IN), client_scale(off, adapters, Xn, IA3_IN), W, bias, neff, rows=rows)
    off = _i32(off)
    S = len(off) - 1
    d_out, d_in = W.shape
    assert Xn.shape[1] == d_in and Xn.shape[0] >= off[-1]
    rows_a = None if rows is None else _i32(rows)
    n = int(off[-1]) if rows is None else len(rows_a)
    keep, ptrs, nrows = _noise_args(off, neff, d_out)
    Y = np.empty((n, d_out), dtype=np.float64)
    ad = _pack(adapters, d_in, d_out)
    rc = lib().orc_forward_denoise_rows(C.c_int32(d_in), C.c_int32(d_out), C.c_int32(S),
                                        off.ctypes.data_as(C.c_void_p), ad, _u16(Xn), _u16(W), _u16(bias), ptrs,
                                        nrows.ctypes.data_as(C.c_void_p), C.c_int32(n),
                                        None if rows_a is None else rows_a.ctypes.data_as(C.c_void_p),
                                        Y.ctypes.data_as(C.c_void_p))
    if rc:
        raise ValueError("oracle forward_denoise: bad offsets, noise-effect rows or row index")
    return Y


def client_scale(off, adapters: Sequence[Adapter], V: np.ndarray, kind: int) -> np.ndarray:
    """bf16 bits of V * l_i on the rows of every segment of `kind` (IA3: V = dY; IA3_IN: V = X), other rows
    copied: the product an IA3 client forms in 16 bits before the tensor goes to the executor (Sec. 3.2, 4)."""
    off = _i32(off)
    S = len(off) - 1
    width = V.shape[1]
    Vc = np.ascontiguousarray(V, dtype=np.uint16)
    out = np.empty_like(Vc)
    arr = (_Adapter * max(1, len(adapters)))()
    for i, a in enumerate(adapters):
        arr[i].kind = int(a.kind)
        if a.kind == kind:
            assert a.A.shape == (width,)
            arr[i].A = _u16(a.A).value
    rc = lib().orc_client_scale(C.c_int32(width), C.c_int32(S), off.ctypes.data_as(C.c_void_p), arr, C.c_int32(kind),
                                _u16(Vc), out.ctypes.data_as(C.c_void_p))
    if rc:
        raise ValueError("oracle client_scale: bad offsets or kind")
    return out


def _without(adapters: Sequence[Adapter], kind: int):
    return [Adapter() if a.kind == kind else a for a in adapters]


def backward_input(off, adapters: Sequence[Adapter], dY: np.ndarray, W: np.ndarray,
                   rows=None, base_only: bool = False, client_bf16: bool = False) -> np.ndarray:
    """dX in fp64 [nrows, d_in].  client_bf16: the IA3 product dY * l_i is the bf16 tensor the paper's
    client would send (client_scale), not the exact product."""
    if client_bf16 and not base_only and any(a.kind == IA3 for a in adapters):
        return backward_input(off, _without(adapters, IA3), client_scale(off, adapters, dY, IA3), W, rows=rows)
    off = _i32(off)
    S = len(off) - 1
    d_out, d_in = W.shape
    assert dY.shape[1] == d_out and dY.shape[0] >= off[-1]
    rows_a = None if rows is None else _i32(rows)
    n = int(off[-1]) if rows is None else len(rows_a)
    dX = np.empty((n, d_in), dtype=np.float64)
    ad = _pack(adapters, d_in, d_out)
    rc = lib().orc_backward_input_rows(C.c_int32(d_in), C.c_int32(d_out), C.c_int32(S),
                                       off.ctypes.data_as(C.c_void_p), ad, _u16(dY), _u16(W),
                                       C.c_int32(n),
                                       None if rows_a is None else rows_a.ctypes.data_as(C.c_void_p),
                                       C.c_int32(1 if base_only else 0), dX.ctypes.data_as(C.c_void_p))
    if rc:
        raise ValueError("oracle backward: bad offsets or row index")
    return dX


def lora_grad(off, adapters: Sequence[Adapter], X: np.ndarray, dY: np.ndarray, i: int,
              want_dA: bool = True, want_dB: bool = True):
    """Returns (dA [r, d_in], dB [d_out, r]) in fp64 for LoRA segment i."""
    off = _i32(off)
    S = len(off) - 1
    d_in, d_out = X.shape[1], dY.shape[1]
    r = adapters[i].rank
    dA = np.empty((r, d_in), dtype=np.float64) if want_dA else None
    dB = np.empty((d_out, r), dtype=np.float64) if want_dB else None
    ad = _pack(adapters, d_in, d_out)
    rc = lib().orc_lora_grad_segment(C.c_int32(d_in), C.c_int32(d_out), C.c_int32(S),
                                     off.ctypes.data_as(C.c_void_p), ad, _u16(X), _u16(dY), C.c_int32(i),
                                     None if dA is None else dA.ctypes.data_as(C.c_void_p),
                                     None if dB is None else dB.ctypes.data_as(C.c_void_p))
    if rc:
        raise ValueError("oracle lora_grad: bad arguments")
    return dA, dB


def ia3_grad(off, adapters: Sequence[Adapter], X: np.ndarray, dY: np.ndarray, W: np.ndarray,
             bias: Optional[np.ndarray], i: int, cols=None, Y0_saved: Optional[np.ndarray] = None,
             G_saved: Optional[np.ndarray] = None) -> np.ndarray:
    """Returns dl (fp64) of IA3 / IA3_IN segment i for the listed channels (default: all).
    Y0_saved: optional bf16 bits [T, d_out] of the base output the client kept from forward (IA3).
    G_saved: optional bf16 bits [T, d_in] of the input gradient dY W the executor returned (IA3_IN)."""
    off = _i32(off)
    S = len(off) - 1
    d_out, d_in = W.shape
    full = d_out if adapters[i].kind == IA3 else d_in
    cols_a = None if cols is None else _i32(cols)
    n = full if cols is None else len(cols_a)
    dl = np.empty(n, dtype=np.float64)
    ad = _pack(adapters, d_in, d_out)
    rc = lib().orc_ia3_grad_segment(C.c_int32(d_in), C.c_int32(d_out), C.c_int32(S),
                                    off.ctypes.data_as(C.c_void_p), ad, _u16(X), _u16(dY), _u16(W),
                                    _u16(bias), _u16(Y0_saved), C.c_int32(i), C.c_int32(n),
                                    None if cols_a is None else cols_a.ctypes.data_as(C.c_void_p),
                                    dl.ctypes.data_as(C.c_void_p), _u16(G_saved))
    if rc:
        raise ValueError("oracle ia3_grad: bad arguments")
    return dl
