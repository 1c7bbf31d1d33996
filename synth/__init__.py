"""Seeded synthetic inputs for the segmented base+adapter linear layer.

This module only draws random numbers, rounds them to bf16 bit patterns and
lays out client segments.  It holds none of the layer's arithmetic and is the
only code shared by the CPU oracle's tests and the GPU path's tests/bench:
both sides receive the *same* uint16 bf16 bit patterns.

Recipe (value laws of the tiny plumbing configuration, reused at every size):
  X ~ N(0,1), W ~ N(0,1/d_in), A_i ~ N(0,1/d_in), B_i ~ N(0,1/r_i),
  dY ~ N(0,1), IA3 vector l ~ 1 + N(0, std 0.1); every value rounded to bf16
  (round-to-nearest-even) on the host.  Generator: numpy Philox (counter based),
  keyed by (base seed, tensor tag, chunk index), so a tensor's bits do not
  depend on how many threads generated it.
"""
from __future__ import annotations

import math
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

BASE_SEED = 20250703

KIND_NONE, KIND_LORA, KIND_IA3, KIND_IA3_IN = 0, 1, 2, 3

_CHUNK = 1 << 22  # elements per independently keyed chunk


# ----------------------------------------------------------------------------
# bf16 helpers (storage format only: 1 sign, 8 exponent, 7 mantissa bits)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 values to bf16 (nearest, ties to even); returns uint16."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to float32 exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(b).astype(np.float64)


def _tag_key(seed: int, tag: str, chunk: int) -> List[int]:
    # 64-bit FNV-1a of the tag keeps keys stable across runs and platforms.
    h = 0xCBF29CE484222325
    for c in tag.encode():
        h = ((h ^ c) * 0x100000001B3) & 0xFFFFFFFFFFFFFFFF
    return [(h ^ (seed * 0x9E3779B97F4A7C15)) & 0xFFFFFFFFFFFFFFFF, chunk]


def _threads() -> int:
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:  # pragma: no cover
        n = os.cpu_count() or 1
    return max(1, min(n, int(os.environ.get("OMP_NUM_THREADS", n)), 16))


def normal_bf16(shape: Sequence[int], std: float, tag: str, seed: int = BASE_SEED,
                mean: float = 0.0) -> np.ndarray:
    """i.i.d. mean + std*N(0,1), rounded to bf16; returns uint16 array of `shape`."""
    n = int(np.prod(shape)) if len(shape) else 1
    out = np.empty(n, dtype=np.uint16)
    nchunks = (n + _CHUNK - 1) // _CHUNK

    def fill(c: int) -> None:
        lo, hi = c * _CHUNK, min(n, (c + 1) * _CHUNK)
        g = np.random.Generator(np.random.Philox(key=_tag_key(seed, tag, c)))
        v = g.standard_normal(hi - lo, dtype=np.float32)
        v *= np.float32(std)
        if mean != 0.0:
            v += np.float32(mean)
        out[lo:hi] = f32_to_bf16_bits(v)

    if nchunks <= 1:
        if nchunks == 1:
            fill(0)
    else:
        with ThreadPoolExecutor(_threads()) as ex:
            list(ex.map(fill, range(nchunks)))
    return out.reshape(shape)


def _rng(tag: str, seed: int = BASE_SEED) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=_tag_key(seed, tag, 0)))


# ----------------------------------------------------------------------------
# Workload descriptions
# ----------------------------------------------------------------------------
@dataclass
class Client:
    """One client (= one token segment) of a flattened batch."""
    n_tokens: int
    kind: int = KIND_NONE
    rank: int = 0
    scale: float = 0.0
    finetune: bool = True  # False: inference segment, never runs backward
    uid: int = 0           # stable identity, keys this client's adapter draws


@dataclass
class Projection:
    name: str
    d_in: int
    d_out: int
    adapted: bool = True   # False: every client runs this projection with kind NONE


@dataclass
class Workload:
    name: str
    projections: List[Projection]
    clients: List[Client]
    seed: int = BASE_SEED
    notes: Dict[str, object] = field(default_factory=dict)

    @property
    def offsets(self) -> np.ndarray:
        off = np.zeros(len(self.clients) + 1, dtype=np.int32)
        np.cumsum([c.n_tokens for c in self.clients], out=off[1:])
        return off

    @property
    def T(self) -> int:
        return int(sum(c.n_tokens for c in self.clients))

    def backward_clients(self) -> List[Client]:
        """The backward batch: fine-tuning segments only, in forward order."""
        return [c for c in self.clients if c.finetune]


def offsets_of(clients: Sequence[Client]) -> np.ndarray:
    off = np.zeros(len(clients) + 1, dtype=np.int32)
    if clients:
        np.cumsum([c.n_tokens for c in clients], out=off[1:])
    return off


@dataclass
class AdapterTensors:
    """Host bit patterns of one client's adapter on one projection."""
    kind: int
    rank: int
    scale: float
    A: Optional[np.ndarray] = None  # LoRA: uint16 [rank, d_in]; IA3: l [d_out]; IA3_IN: l [d_in]
    B: Optional[np.ndarray] = None  # LoRA: uint16 [d_out, rank]


def make_adapter(wl: Workload, proj: Projection, c: Client) -> AdapterTensors:
    if not proj.adapted or c.kind == KIND_NONE:
        return AdapterTensors(KIND_NONE, 0, 0.0)
    tag = f"{wl.name}/{proj.name}/client{c.uid}"
    if c.kind == KIND_LORA:
        A = normal_bf16((c.rank, proj.d_in), 1.0 / math.sqrt(proj.d_in), tag + "/A", wl.seed)
        B = normal_bf16((proj.d_out, c.rank), 1.0 / math.sqrt(c.rank), tag + "/B", wl.seed)
        return AdapterTensors(KIND_LORA, c.rank, c.scale, A, B)
    if c.kind == KIND_IA3:
        l = normal_bf16((proj.d_out,), 0.1, tag + "/l", wl.seed, mean=1.0)
        return AdapterTensors(KIND_IA3, 0, 0.0, l)
    if c.kind == KIND_IA3_IN:
        l = normal_bf16((proj.d_in,), 0.1, tag + "/l", wl.seed, mean=1.0)
        return AdapterTensors(KIND_IA3_IN, 0, 0.0, l)
    raise ValueError(c.kind)


def make_X(wl: Workload, proj: Projection, T: Optional[int] = None, which: str = "X") -> np.ndarray:
    T = wl.T if T is None else T
    return normal_bf16((T, proj.d_in), 1.0, f"{wl.name}/{proj.name}/{which}", wl.seed)


def make_dY(wl: Workload, proj: Projection, T: int) -> np.ndarray:
    return normal_bf16((T, proj.d_out), 1.0, f"{wl.name}/{proj.name}/dY", wl.seed)


def make_W(wl: Workload, proj: Projection) -> np.ndarray:
    return normal_bf16((proj.d_out, proj.d_in), 1.0 / math.sqrt(proj.d_in),
                       f"{wl.name}/{proj.name}/W", wl.seed)


def make_bias(wl: Workload, proj: Projection) -> np.ndarray:
    return normal_bf16((proj.d_out,), 0.5, f"{wl.name}/{proj.name}/bias", wl.seed)


# ----------------------------------------------------------------------------
# The five configurations
# ----------------------------------------------------------------------------
def cfg1_tiny() -> Workload:
    clients = [Client(64, KIND_LORA, 8, 16.0 / 8, True, i) for i in range(4)]
    return Workload("cfg1_tiny", [Projection("lin", 768, 768)], clients)


_LLAMA7B = [("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096), ("o", 4096, 4096),
            ("gate", 4096, 11008), ("up", 4096, 11008), ("down", 11008, 4096)]


def cfg2_llama7b(seed: int = BASE_SEED) -> Workload:
    g = _rng("cfg2/clients", seed)
    lens = g.choice([512, 1024, 2048], size=8)
    ranks = g.choice([8, 16, 32, 64], size=8)
    clients = [Client(int(n), KIND_LORA, int(r), 2.0, True, i) for i, (n, r) in enumerate(zip(lens, ranks))]
    adapted = {"q", "v", "gate", "down"}
    projs = [Projection(n, i, o, n in adapted) for n, i, o in _LLAMA7B]
    return Workload("cfg2_llama7b", projs, clients, seed)


def cfg3_granite20b() -> Workload:
    clients = [Client(1024, KIND_LORA, 8, 2.0, True, i) for i in range(16)]
    projs = [Projection("q", 6144, 6144), Projection("kv", 6144, 256), Projection("o", 6144, 6144),
             Projection("fc", 6144, 24576), Projection("proj", 24576, 6144)]
    return Workload("cfg3_granite20b", projs, clients)


def cfg4_gemma27b(seed: int = BASE_SEED) -> Workload:
    g = _rng("cfg4/clients", seed)
    ranks = g.choice([8, 16], size=20)
    clients = [Client(1024, KIND_LORA, int(r), 2.0, True, i) for i, r in enumerate(ranks)]
    projs = [Projection("q", 4608, 4096), Projection("k", 4608, 2048), Projection("v", 4608, 2048),
             Projection("o", 4096, 4608), Projection("gate", 4608, 36864), Projection("up", 4608, 36864),
             Projection("down", 36864, 4608)]
    return Workload("cfg4_gemma27b", projs, clients, seed)


def bounded_zipf(g: np.random.Generator, a: float, lo: int, hi: int, size: int) -> np.ndarray:
    """P(L=k) proportional to k^-a on the integers lo..hi, by inverse CDF."""
    k = np.arange(lo, hi + 1, dtype=np.float64)
    cdf = np.cumsum(k ** (-a))
    cdf /= cdf[-1]
    u = g.random(size)
    return (lo + np.searchsorted(cdf, u, side="left")).astype(np.int64)


def cfg5_mixed(seed: int = BASE_SEED, arbitrary_ranks: bool = False) -> Workload:
    """48 one-token decode segments + 16 fine-tuning segments, shuffled together."""
    g = _rng("cfg5/clients", seed)
    ft_lens = bounded_zipf(g, 1.1, 16, 4096, 16)
    n = [1] * 48 + [int(x) for x in ft_lens]
    ft = [False] * 48 + [True] * 16
    if arbitrary_ranks:
        ranks = np.rint(2.0 ** g.uniform(2.0, 7.0, size=64)).astype(np.int64)
    else:
        ranks = 2 ** g.integers(2, 8, size=64)
    is_ia3 = g.random(64) < 0.5
    clients = []
    for i in range(64):
        if is_ia3[i]:
            clients.append(Client(n[i], KIND_IA3, 0, 0.0, ft[i], i))
        else:
            clients.append(Client(n[i], KIND_LORA, int(ranks[i]), 2.0, ft[i], i))
    order = g.permutation(64)
    clients = [clients[j] for j in order]
    projs = [Projection(nm, i, o, True) for nm, i, o in _LLAMA7B]
    name = "cfg5_mixed_anyrank" if arbitrary_ranks else "cfg5_mixed"
    return Workload(name, projs, clients, seed)


CONFIGS = {
    "cfg1": cfg1_tiny, "cfg2": cfg2_llama7b, "cfg3": cfg3_granite20b,
    "cfg4": cfg4_gemma27b, "cfg5": cfg5_mixed,
}


def sample_rows(off: np.ndarray, per_segment_random: int, tag: str, seed: int = BASE_SEED,
                block: int = 0) -> np.ndarray:
    """Rows to spot-check: per segment its first two, last two and `per_segment_random` seeded
    random rows; with `block` > 0 also one seeded row of every run of `block` consecutive rows of
    the flattened batch (block = 128: both 128-row halves of every 256-row tile are covered)."""
    g = _rng("rows/" + tag, seed)
    rows: List[int] = []
    for i in range(len(off) - 1):
        lo, hi = int(off[i]), int(off[i + 1])
        if hi <= lo:
            continue
        pick = {lo, min(lo + 1, hi - 1), hi - 1, max(hi - 2, lo)}
        if hi - lo > 4 and per_segment_random > 0:
            pick.update(int(x) for x in g.integers(lo, hi, size=per_segment_random))
        rows.extend(pick)
    T = int(off[-1])
    if block > 0:
        for b0 in range(0, T, block):
            rows.append(int(g.integers(b0, min(T, b0 + block))))
    return np.asarray(sorted(set(rows)), dtype=np.int32)
