"""Plain reference of the opportunistic batching rule (Sec. 3.7): TEST INFRASTRUCTURE ONLY.

Written from the rule itself, with Python lists and no shared code with the library's queue:
a request may be held for min(max_wait, base_wait + per_token_wait * n_tokens); a layer's
queue is due at the smallest arrival + allowed wait, or at the arrival that brings the queued
tokens to the cap; a batch takes, of the requests that have arrived, the latency-sensitive
ones in arrival order, then the others, skipping what does not fit under the cap (the first
always fits).
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Tuple


@dataclass
class Request:
    rid: int
    n_tokens: int
    latency_sensitive: bool
    arrival_us: float


class ReferenceBatcher:
    def __init__(self, base_wait_us: float, per_token_wait_us: float, max_wait_us: float, max_tokens: int):
        self.base, self.per_tok, self.max_wait, self.cap = base_wait_us, per_token_wait_us, max_wait_us, max_tokens
        self.queue: List[Request] = []

    def wait_of(self, n_tokens: int) -> float:
        return min(self.max_wait, self.base + self.per_tok * n_tokens)

    def submit(self, r: Request) -> None:
        assert r.n_tokens >= 1 and (not self.queue or r.arrival_us >= self.queue[-1].arrival_us)
        self.queue.append(r)

    def next_due(self) -> float:
        due, tokens = math.inf, 0
        for r in self.queue:
            due = min(due, r.arrival_us + self.wait_of(r.n_tokens))
            tokens += r.n_tokens
            if tokens >= self.cap:
                return min(due, r.arrival_us)
        return due

    def take(self, now_us: float, capacity: int = 1 << 30) -> Tuple[List[int], List[int]]:
        if not self.queue or self.next_due() > now_us:
            return [], [0]
        here = [r for r in self.queue if r.arrival_us <= now_us]
        ordered = [r for r in here if r.latency_sensitive] + [r for r in here if not r.latency_sensitive]
        chosen, tokens = [], 0
        for r in ordered:
            if len(chosen) == capacity:
                break
            if chosen and tokens + r.n_tokens > self.cap:
                continue
            chosen.append(r)
            tokens += r.n_tokens
        ids = [r.rid for r in chosen]
        self.queue = [r for r in self.queue if r.rid not in set(ids)]
        off = [0]
        for r in chosen:
            off.append(off[-1] + r.n_tokens)
        return ids, off
