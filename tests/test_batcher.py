"""Host-side batching queue (include/symb_batcher.h) against the plain reference in oracle/batching.py,
bit-exactly, on seeded arrival sequences; plus what the rule itself fixes (Sec. 3.7): every request
is served exactly once, nobody is held beyond its size-dependent wait while the executor is free,
small requests are not held back by large ones, a batch never exceeds the token cap unless it is
a single oversized request, latency-sensitive requests come first when a batch is cut."""
import math

import numpy as np
import pytest

from oracle.batching import ReferenceBatcher, Request
from paper_2507_03220_amd import batcher as bt
from paper_2507_03220_amd import binding as sb


@pytest.fixture(scope="module", autouse=True)
def _built():
    from paper_2507_03220_amd import build
    build.build(force=False)


def _arrivals(seed, n, rate_per_ms=2.0):
    rng = np.random.default_rng(seed)
    t, out = 0.0, []
    for i in range(n):
        t += float(rng.exponential(1000.0 / rate_per_ms))
        decode = rng.random() < 0.7
        n_tok = int(rng.integers(1, 5)) if decode else int(rng.choice([256, 512, 1024, 2048, 5000]))
        out.append(Request(i, n_tok, bool(decode), t))
    return out


POLICIES = [dict(base_wait_us=50.0, per_token_wait_us=0.5, max_wait_us=800.0, max_tokens=4096),
            dict(base_wait_us=0.0, per_token_wait_us=0.0, max_wait_us=0.0, max_tokens=1 << 20),      # no waiting at all
            dict(base_wait_us=200.0, per_token_wait_us=0.0, max_wait_us=200.0, max_tokens=1024)]


@pytest.mark.parametrize("seed", [1, 2, 3])
@pytest.mark.parametrize("pol", POLICIES)
def test_batches_match_the_reference_on_a_simulated_executor(seed, pol):
    reqs = _arrivals(seed, 300)
    lib_b, ref_b = bt.Batcher(num_layers=2, **pol), ReferenceBatcher(**pol)
    served, batches = set(), []
    now, i, busy_until = 0.0, 0, 0.0
    while i < len(reqs) or ref_b.queue:
        # next event: an arrival, or the queue becoming due once the executor is free
        due = max(ref_b.next_due(), busy_until)
        assert lib_b.next_due(1) == ref_b.next_due()
        if i < len(reqs) and reqs[i].arrival_us <= due:
            r = reqs[i]
            now = r.arrival_us
            lib_b.submit(1, r.rid, 0, r.n_tokens, r.latency_sensitive, r.arrival_us)
            ref_b.submit(r)
            i += 1
            continue
        now = due
        ids, off = lib_b.take(1, now)
        rids, roff = ref_b.take(now)
        assert ids == rids and off == roff
        assert ids, "a due queue must yield a batch"
        tokens = off[-1]
        assert tokens <= pol["max_tokens"] or len(ids) == 1
        by_id = {r.rid: r for r in reqs}
        flags = [by_id[x].latency_sensitive for x in ids]
        assert flags == sorted(flags, reverse=True), "latency-sensitive requests first"
        for cls in (True, False):
            arr = [by_id[x].arrival_us for x in ids if by_id[x].latency_sensitive == cls]
            assert arr == sorted(arr), "arrival order inside a class"
        for x in ids:
            assert x not in served
            served.add(x)
            # held no longer than its own allowance once the executor was free
            assert now <= max(by_id[x].arrival_us + ref_b.wait_of(by_id[x].n_tokens), busy_until) + 1e-9
        batches.append((now, ids))
        busy_until = now + 20.0 + 0.05 * tokens          # a made-up service time
    assert served == set(range(len(reqs)))
    assert lib_b.pending(1) == (0, 0) and lib_b.pending(0) == (0, 0)
    lib_b.close()


class _Library:
    """The library's queue (layer 0) behind the four calls the hand-computed cases use."""
    def __init__(self, *policy):
        self.b = bt.Batcher(*policy)
    def submit(self, rid, n_tokens, latency_sensitive, arrival_us):
        self.b.submit(0, rid, 0, n_tokens, latency_sensitive, arrival_us)
    def next_due(self):
        return self.b.next_due(0)
    def take(self, now_us):
        ids, off = self.b.take(0, now_us)
        return ids, off
    def pending(self):
        return self.b.pending(0)
    def close(self):
        self.b.close()


class _Reference:
    """The plain reference behind the same four calls: the hand-computed cases pin it directly."""
    def __init__(self, *policy):
        self.b = ReferenceBatcher(*policy)
    def submit(self, rid, n_tokens, latency_sensitive, arrival_us):
        self.b.submit(Request(rid, n_tokens, latency_sensitive, arrival_us))
    def next_due(self):
        return self.b.next_due()
    def take(self, now_us):
        ids, off = self.b.take(now_us)
        return ids, off
    def pending(self):
        return len(self.b.queue), sum(r.n_tokens for r in self.b.queue)
    def close(self):
        pass


# Expected values below are worked out by hand from the rule as Sec. 3.7 states it (wait grows with the
# request's size; inference first; a pre-determined cap), not taken from either implementation.
@pytest.mark.parametrize("impl", [_Reference, _Library])
def test_small_requests_wait_less_than_large_ones(impl):
    b = impl(50.0, 0.5, 800.0, 4096)
    b.submit(1, 2048, False, 0.0)                       # may wait min(800, 50 + 1024) = 800
    assert b.next_due() == 800.0
    b.submit(2, 2, True, 100.0)                         # may wait 51: the queue is now due at 151
    assert b.next_due() == 151.0
    assert b.take(150.0) == ([], [0])
    ids, off = b.take(151.0)
    assert ids == [2, 1] and off == [0, 2, 2050]        # both go, the inference request first
    assert math.isinf(b.next_due())
    b.close()


@pytest.mark.parametrize("impl", [_Reference, _Library])
def test_token_cap_makes_the_queue_due_at_once_and_cuts_the_batch(impl):
    b = impl(1000.0, 0.0, 1000.0, 1000)
    b.submit(1, 600, False, 0.0)
    b.submit(2, 600, False, 10.0)                       # 1200 >= cap: due on arrival
    b.submit(3, 300, True, 20.0)
    assert b.next_due() == 10.0
    ids, off = b.take(20.0)
    assert ids == [3, 1] and off == [0, 300, 900]       # inference first, then what fits; request 2 stays
    assert b.pending() == (1, 600)
    b.submit(4, 5000, False, 30.0)                      # oversized: runs alone when its turn comes
    ids, off = b.take(2000.0)
    assert ids == [2] and off == [0, 600]
    ids, off = b.take(2000.0)
    assert ids == [4] and off == [0, 5000]
    b.close()


@pytest.mark.parametrize("impl", [_Reference, _Library])
def test_only_arrived_requests_are_taken_and_the_wait_is_capped(impl):
    b = impl(10.0, 1.0, 100.0, 10000)
    b.submit(1, 50, True, 0.0)                          # may wait 10 + 50 = 60
    b.submit(2, 500, False, 40.0)                       # may wait min(100, 510) = 100: the cap of the allowance
    b.submit(3, 5, True, 70.0)                          # arrives after the queue is due
    assert b.next_due() == 60.0
    ids, off = b.take(60.0)
    assert ids == [1, 2] and off == [0, 50, 550]        # request 3 has not arrived at t = 60
    assert b.pending() == (1, 5)
    assert b.next_due() == 85.0                         # 70 + (10 + 5)
    assert b.take(84.0) == ([], [0])
    assert b.take(85.0) == ([3], [0, 5])
    b.close()


def test_argument_checks():
    with pytest.raises(sb.SymbError):
        bt.Batcher(-1.0, 0.0, 0.0, 10)
    b = bt.Batcher(1.0, 0.0, 1.0, 10)
    with pytest.raises(sb.SymbError):
        b.submit(3, 1, 0, 1, True, 0.0)                 # no such layer
    with pytest.raises(sb.SymbError):
        b.submit(0, 1, 0, 0, True, 0.0)                 # empty request
    b.submit(0, 1, 0, 1, True, 5.0)
    with pytest.raises(sb.SymbError):
        b.submit(0, 2, 0, 1, True, 4.0)                 # time runs backwards
    b.close()
