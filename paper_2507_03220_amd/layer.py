"""Device-resident state of one frozen projection shared by many clients, plus the three
C-ABI calls that make up its forward and backward.  Marshalling only: buffers are torch
tensors, all arithmetic happens inside libsymb.so.

A "layer" of a model shape is a list of such projections run back to back on
independent inputs (client-side attention, norms and activations are not part of the
base executor and are not modelled).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np
import torch

from . import binding as sb


def bits_to_dev(bits: Optional[np.ndarray]) -> Optional[torch.Tensor]:
    """uint16 bf16 bit patterns (host) -> bf16 device tensor, bit for bit."""
    if bits is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16)
    return t.to("cuda")


@dataclass
class SegmentSpec:
    """One client's segment on this projection (host side description)."""
    n_tokens: int
    kind: int = sb.SYMB_ADAPTER_NONE
    rank: int = 0
    scale: float = 0.0
    A: Optional[np.ndarray] = None       # bf16 bits
    B: Optional[np.ndarray] = None
    finetune: bool = True                 # False: inference segment, forward only


class ProjectionRun:
    """Buffers and batches of one projection: forward over all segments, backward over
    the fine-tuning segments only (a batch of its own, as the executor allows)."""

    def __init__(self, handle, name: str, d_in: int, d_out: int, segs: Sequence[SegmentSpec],
                 W: np.ndarray, X: np.ndarray, dY: np.ndarray, bias: Optional[np.ndarray] = None,
                 want_ybase: Optional[bool] = None):
        self.h, self.name, self.d_in, self.d_out = handle, name, d_in, d_out
        self.segs = list(segs)
        self.W = bits_to_dev(W)
        self.bias = bits_to_dev(bias)
        self.X = bits_to_dev(X)
        self.T = int(sum(s.n_tokens for s in segs))
        assert X.shape == (self.T, d_in) and W.shape == (d_out, d_in)
        # forward batch
        self.fwd_ad = []
        for s in self.segs:
            a = sb.Adapter(s.kind, s.rank, s.scale, bits_to_dev(s.A), bits_to_dev(s.B))
            self.fwd_ad.append(a)
        off = np.zeros(len(segs) + 1, dtype=np.int64)
        off[1:] = np.cumsum([s.n_tokens for s in segs])
        self.fwd_off = off
        self.fwd_batch = sb.Batch(d_in, d_out, off, self.fwd_ad)
        self.Y = torch.empty((self.T, d_out), device="cuda", dtype=torch.bfloat16)
        ia3_ft = any(s.kind == sb.SYMB_ADAPTER_IA3 and s.finetune for s in segs)
        self.want_ybase = ia3_ft if want_ybase is None else want_ybase
        self.Ybase = torch.empty_like(self.Y) if self.want_ybase else None
        # backward batch: fine-tuning segments only, gradients wanted
        ft = [i for i, s in enumerate(segs) if s.finetune]
        self.ft_index = ft
        self.bwd_ad = []
        for i in ft:
            s, f = self.segs[i], self.fwd_ad[i]
            a = sb.Adapter(s.kind, s.rank, s.scale, f.A, f.B)
            if s.kind == sb.SYMB_ADAPTER_LORA:
                a.dA = torch.zeros((s.rank, d_in), device="cuda", dtype=torch.float32)
                a.dB = torch.zeros((d_out, s.rank), device="cuda", dtype=torch.float32)
            elif s.kind == sb.SYMB_ADAPTER_IA3:
                a.dA = torch.zeros((d_out,), device="cuda", dtype=torch.float32)
            self.bwd_ad.append(a)
        boff = np.zeros(len(ft) + 1, dtype=np.int64)
        boff[1:] = np.cumsum([segs[i].n_tokens for i in ft])
        self.bwd_off = boff
        self.Tb = int(boff[-1])
        self.bwd_batch = sb.Batch(d_in, d_out, boff, self.bwd_ad)
        assert dY.shape == (self.Tb, d_out)
        self.dY = bits_to_dev(dY)
        self.dX = torch.empty((self.Tb, d_in), device="cuda", dtype=torch.bfloat16)
        # rows of the forward batch that belong to the backward batch (for X and Ybase)
        if len(ft) == len(segs):
            self.Xb, self.Ybase_b = self.X, self.Ybase
            self._gather = None
        else:
            idx = np.concatenate([np.arange(off[i], off[i + 1]) for i in ft]) if ft else np.zeros(0, np.int64)
            self._gather = torch.from_numpy(idx).to("cuda")
            self.Xb = self.X.index_select(0, self._gather) if self.Tb else self.X[:0]
            self.Ybase_b = torch.empty((self.Tb, d_out), device="cuda", dtype=torch.bfloat16) if self.want_ybase else None
        n = max(sb.symb_workspace_bytes(self.fwd_batch, sb.SYMB_OP_FWD),
                sb.symb_workspace_bytes(self.bwd_batch, sb.SYMB_OP_BWD_INPUT),
                sb.symb_workspace_bytes(self.bwd_batch, sb.SYMB_OP_ADAPTER_GRAD))
        self.ws = torch.empty(max(n, 256), device="cuda", dtype=torch.uint8)

    # -- the three calls -----------------------------------------------------------------------
    def fwd(self, stream: int = 0) -> None:
        sb.symb_base_linear_fwd(self.h, self.fwd_batch, self.X, self.W, self.bias, self.Y, self.Ybase, self.ws, stream)
        self._dh_in_ws = False
        self._dh_from_grad = False
        self._hs_in_ws = self._gather is None      # backward batch == forward batch: Hs stays valid for it

    def sync_saved_output(self) -> None:
        """What a client does between forward and backward: keep its rows of the base output."""
        if self._gather is not None and self.want_ybase and self.Tb:
            torch.index_select(self.Ybase, 0, self._gather, out=self.Ybase_b)

    def bwd_input(self, stream: int = 0, flags: int = sb.SYMB_BWD_FULL, reuse_dh: bool = False) -> None:
        """reuse_dh: the workspace still holds dH from the adapter_grad call just before (same batch, same dY)."""
        if reuse_dh and flags == sb.SYMB_BWD_FULL and getattr(self, "_dh_from_grad", False):
            flags |= sb.SYMB_BWD_REUSE_DH
        sb.symb_base_linear_bwd_input(self.h, self.bwd_batch, self.dY, self.W, self.dX, flags, self.ws, stream)
        self._dh_in_ws = not (flags & sb.SYMB_BWD_BASE_ONLY)
        self._dh_from_grad = False

    def adapter_grad(self, stream: int = 0, flags: int = sb.SYMB_GRAD_OVERWRITE, reuse_dh: bool = False,
                     reuse_hs: bool = False) -> None:
        """reuse_dh: the workspace still holds dH from the bwd_input call just before (same batch, same dY).
        reuse_hs: it still holds Hs from this run's forward call (only when the backward batch is the forward batch)."""
        if reuse_dh and getattr(self, "_dh_in_ws", False):
            flags |= sb.SYMB_GRAD_REUSE_DH
        if reuse_hs and getattr(self, "_hs_in_ws", False):
            flags |= sb.SYMB_GRAD_REUSE_HS
        sb.symb_adapter_grad(self.h, self.bwd_batch, self.Xb, self.dY, self.Ybase_b, flags, self.ws, stream)
        self._dh_in_ws = False
        # a gradient call computes dH of every LoRA segment that wants dA (all of them here) into the workspace
        self._dh_from_grad = any(s.kind == sb.SYMB_ADAPTER_LORA for s in self.segs)

    # -- algorithmic work (flops) ----------------------------------------------------------------
    def flops(self) -> dict:
        """Algorithmic FLOPs: base 2*d_in*d_out per token per direction; LoRA forward
        2 r (d_in+d_out), LoRA backward 4 r (d_in+d_out); IA3 d_out forward, 2 d_out backward."""
        di, do = self.d_in, self.d_out
        f = dict(base_fwd=2.0 * self.T * di * do, base_bwd=2.0 * self.Tb * di * do, ad_fwd=0.0, ad_bwd=0.0,
                 gemm_fwd=2.0 * self.T * di * do, gemm_bwd=2.0 * self.Tb * di * do)
        for s in self.segs:
            if s.kind == sb.SYMB_ADAPTER_LORA:
                f["ad_fwd"] += 2.0 * s.n_tokens * s.rank * (di + do)
                f["gemm_fwd"] += 2.0 * s.n_tokens * s.rank * do          # the expand runs inside the GEMM
                if s.finetune:
                    f["ad_bwd"] += 4.0 * s.n_tokens * s.rank * (di + do)
                    f["gemm_bwd"] += 2.0 * s.n_tokens * s.rank * di
            elif s.kind == sb.SYMB_ADAPTER_IA3:
                f["ad_fwd"] += 1.0 * s.n_tokens * do
                if s.finetune:
                    f["ad_bwd"] += 2.0 * s.n_tokens * do
        f["total"] = f["base_fwd"] + f["base_bwd"] + f["ad_fwd"] + f["ad_bwd"]
        return f
