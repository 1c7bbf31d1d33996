"""Runs one problem through the C ABI on the GPU and returns host arrays.

Only marshalling lives here: numpy bf16 bit patterns -> torch device tensors -> the
binding's entry points -> numpy.  Comparisons against the oracle are in the tests.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

import synth
from paper_2507_03220_amd import binding as sb

_handle = None


def handle():
    global _handle
    if _handle is None:
        _handle = sb.symb_create(0)
    return _handle


def to_dev(bits: Optional[np.ndarray]):
    if bits is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16)
    return t.to("cuda", non_blocking=False)


def bf16_to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().view(torch.int16).cpu().numpy().view(np.uint16)


@dataclass
class HostAdapter:
    kind: int = 0
    rank: int = 0
    scale: float = 0.0
    A: Optional[np.ndarray] = None
    B: Optional[np.ndarray] = None
    want_grad: bool = True


@dataclass
class DevAdapters:
    descs: List[sb.Adapter]
    tensors: list = field(default_factory=list)


def upload_adapters(ads: Sequence[HostAdapter], d_in: int, d_out: int, grads: bool, cache: Optional[dict] = None) -> DevAdapters:
    out, keep = [], []
    for a in ads:
        d = sb.Adapter(a.kind, a.rank, a.scale)
        if a.kind == sb.SYMB_ADAPTER_LORA:
            d.A, d.B = to_dev(a.A), to_dev(a.B)
            if grads and a.want_grad:
                d.dA = torch.full((a.rank, d_in), float("nan"), device="cuda", dtype=torch.float32)
                d.dB = torch.full((d_out, a.rank), float("nan"), device="cuda", dtype=torch.float32)
        elif a.kind in (sb.SYMB_ADAPTER_IA3, sb.SYMB_ADAPTER_IA3_IN):
            d.A = to_dev(a.A)
            if grads and a.want_grad:
                d.dA = torch.full((a.A.shape[0],), float("nan"), device="cuda", dtype=torch.float32)
        out.append(d)
        keep.extend([d.A, d.B, d.dA, d.dB])
    return DevAdapters(out, keep)


def workspace(batch: sb.Batch, op: int) -> Optional[torch.Tensor]:
    n = sb.symb_workspace_bytes(batch, op)
    if n == 0:
        return None
    return torch.empty(n, device="cuda", dtype=torch.uint8)


def stream_ptr() -> int:
    return torch.cuda.current_stream().cuda_stream


def weight_to_dev(W: np.ndarray, conv1d: bool):
    """W is given as [d_out][d_in]; an input-major (Conv1D) layer stores its transpose [d_in][d_out]."""
    return to_dev(np.ascontiguousarray(W.T) if conv1d else W)


def forward(off, ads: Sequence[HostAdapter], X, W, bias=None, want_base=True, conv1d=False):
    """Returns (Y, Ybase) device tensors [T, d_out] bf16 (Ybase None if not wanted)."""
    d_out, d_in = W.shape
    dev = upload_adapters(ads, d_in, d_out, grads=False)
    batch = sb.Batch(d_in, d_out, off, dev.descs, sb.SYMB_WEIGHT_CONV1D if conv1d else sb.SYMB_WEIGHT_LINEAR)
    T = int(off[-1])
    Xd, Wd, bd = to_dev(X), weight_to_dev(W, conv1d), to_dev(bias)
    Y = torch.full((T, d_out), float("nan"), device="cuda", dtype=torch.bfloat16)
    Yb = torch.full((T, d_out), float("nan"), device="cuda", dtype=torch.bfloat16) if want_base else None
    ws = workspace(batch, sb.SYMB_OP_FWD)
    sb.symb_base_linear_fwd(handle(), batch, Xd, Wd, bd, Y, Yb, ws, stream_ptr())
    torch.cuda.synchronize()
    return Y, Yb


def backward_input(off, ads: Sequence[HostAdapter], dY, W, base_only=False, conv1d=False):
    d_out, d_in = W.shape
    dev = upload_adapters(ads, d_in, d_out, grads=False)
    batch = sb.Batch(d_in, d_out, off, dev.descs, sb.SYMB_WEIGHT_CONV1D if conv1d else sb.SYMB_WEIGHT_LINEAR)
    T = int(off[-1])
    gd, Wd = to_dev(dY), weight_to_dev(W, conv1d)
    dX = torch.full((T, d_in), float("nan"), device="cuda", dtype=torch.bfloat16)
    ws = workspace(batch, sb.SYMB_OP_BWD_INPUT)
    sb.symb_base_linear_bwd_input(handle(), batch, gd, Wd, dX,
                                  sb.SYMB_BWD_BASE_ONLY if base_only else sb.SYMB_BWD_FULL, ws, stream_ptr())
    torch.cuda.synchronize()
    return dX


def adapter_grad(off, ads: Sequence[HostAdapter], X, dY, Ybase=None, d_in=None, d_out=None,
                 accumulate_into: Optional[DevAdapters] = None):
    """Returns DevAdapters whose descs carry dA/dB (fp32 device tensors)."""
    d_in = X.shape[1] if d_in is None else d_in
    d_out = dY.shape[1] if d_out is None else d_out
    dev = accumulate_into or upload_adapters(ads, d_in, d_out, grads=True)
    batch = sb.Batch(d_in, d_out, off, dev.descs)
    Xd, gd = to_dev(X), to_dev(dY)
    Yb = Ybase if (Ybase is None or isinstance(Ybase, torch.Tensor)) else to_dev(Ybase)
    ws = workspace(batch, sb.SYMB_OP_ADAPTER_GRAD)
    sb.symb_adapter_grad(handle(), batch, Xd, gd, Yb,
                         sb.SYMB_GRAD_ACCUMULATE if accumulate_into is not None else sb.SYMB_GRAD_OVERWRITE,
                         ws, stream_ptr())
    torch.cuda.synchronize()
    return dev
