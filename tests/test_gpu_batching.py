"""Opportunistic batching end to end on the GPU (Sec. 3.7, Sec. 3.6): seeded arrivals of inference and
fine-tuning requests go through the library's batching queue; every batch it forms runs through
symb_base_linear_fwd as one flattened, padding-free call with each request's own adapter; the
fine-tuning requests then queue for the backward pass in another order, are regrouped into
backward batches by the same queue and run through symb_base_linear_bwd_input.  Every request's
rows must be what the oracle computes for that request ALONE (Sec. 4: batching leaves each client's
output what it would have been on its own), to the usual bar."""
import numpy as np
import pytest
import torch

import oracle
import synth
from helpers import check_dx, check_y

pytestmark = pytest.mark.gpu

D_IN, D_OUT = 512, 384
L, I, N = oracle.LORA, oracle.IA3, oracle.NONE


def _clients(rng):
    nb = lambda shape, std, mean=0.0: synth.f32_to_bf16_bits((mean + std * rng.standard_normal(shape)).astype(np.float32))
    import gpu_harness as gh
    out = []
    for c in range(12):
        kind = [L, L, I, N][c % 4]
        if kind == L:
            r = [8, 16, 5, 64, 128, 24][c % 6]
            out.append(gh.HostAdapter(L, r, 16.0 / r, nb((r, D_IN), D_IN ** -0.5), nb((D_OUT, r), r ** -0.5)))
        elif kind == I:
            out.append(gh.HostAdapter(I, 0, 0.0, nb((D_OUT,), 0.1, 1.0)))
        else:
            out.append(gh.HostAdapter())
    return out


def test_queue_formed_batches_give_each_request_its_own_result():
    import gpu_harness as gh
    from paper_2507_03220_amd import batcher as bt
    from paper_2507_03220_amd import binding as sb
    rng = np.random.default_rng(20250703)
    h = gh.handle()
    clients = _clients(rng)
    dev = gh.upload_adapters(clients, D_IN, D_OUT, grads=False)
    oads = [oracle.Adapter(a.kind, a.rank, a.scale, a.A, a.B) for a in clients]
    W = synth.f32_to_bf16_bits((D_IN ** -0.5 * rng.standard_normal((D_OUT, D_IN))).astype(np.float32))
    bias = synth.f32_to_bf16_bits((0.5 * rng.standard_normal(D_OUT)).astype(np.float32))
    Wd, bd = gh.to_dev(W), gh.to_dev(bias)

    # requests: decode steps (1..4 tokens, latency-sensitive) and fine-tuning passes (48..400 tokens)
    reqs, t = [], 0.0
    for rid in range(48):
        t += float(rng.exponential(400.0))
        decode = rng.random() < 0.6
        n = int(rng.integers(1, 5)) if decode else int(rng.integers(48, 401))
        reqs.append(dict(rid=rid, client=int(rng.integers(0, 12)), n=n, decode=bool(decode), t=t,
                         X=synth.f32_to_bf16_bits(rng.standard_normal((n, D_IN)).astype(np.float32)),
                         dY=synth.f32_to_bf16_bits(rng.standard_normal((n, D_OUT)).astype(np.float32))))
    by_id = {r["rid"]: r for r in reqs}

    def drain(q, layer, pending, run_batch):
        """Feeds `pending` (sorted by arrival) to the queue and runs every batch it forms."""
        now, i, busy_until, nb = 0.0, 0, 0.0, 0
        while i < len(pending) or q.pending(layer)[0]:
            due = max(q.next_due(layer), busy_until)
            if i < len(pending) and pending[i][1] <= due:
                r, at = pending[i]
                q.submit(layer, r["rid"], r["client"], r["n"], r["decode"], at)
                i += 1
                continue
            now = due
            ids, off = q.take(layer, now)
            assert ids, "a due queue must yield a batch"
            run_batch(ids, off)
            nb += 1
            busy_until = now + 30.0 + 0.05 * off[-1]
        return nb

    q = bt.Batcher(base_wait_us=50.0, per_token_wait_us=0.5, max_wait_us=600.0, max_tokens=700, num_layers=2)
    sizes = []

    def run_forward(ids, off):
        batch = sb.Batch(D_IN, D_OUT, off, [dev.descs[by_id[x]["client"]] for x in ids])
        X = gh.to_dev(np.concatenate([by_id[x]["X"] for x in ids], axis=0))
        Y = torch.full((off[-1], D_OUT), float("nan"), device="cuda", dtype=torch.bfloat16)
        sb.symb_base_linear_fwd(h, batch, X, Wd, bd, Y, None, gh.workspace(batch, sb.SYMB_OP_FWD), gh.stream_ptr())
        torch.cuda.synchronize()
        Yh = gh.bf16_to_f64(Y)
        for k, x in enumerate(ids):
            by_id[x]["Y"] = Yh[off[k]:off[k + 1]]
        sizes.append((len(ids), off[-1]))

    n_fwd = drain(q, 0, [(r, r["t"]) for r in reqs], run_forward)
    assert n_fwd < len(reqs), "the queue never batched two requests together"
    assert any(n > 1 and 16 < tok for n, tok in sizes) and any(tok <= 16 for _, tok in sizes)
    for r in reqs:
        alone = np.array([0, r["n"]], dtype=np.int32)
        check_y(r["Y"], alone, [oads[r["client"]]], r["X"], W, bias, f"request {r['rid']} (client {r['client']}, {r['n']} tokens) Y")

    # backward: fine-tuning requests only, arriving in another order -> other groups than in the forward
    ft = [r for r in reqs if not r["decode"]]
    order = rng.permutation(len(ft))
    t, pending = 0.0, []
    for j in order:
        t += float(rng.exponential(150.0))
        pending.append((ft[int(j)], t))
    groups = []

    def run_backward(ids, off):
        batch = sb.Batch(D_IN, D_OUT, off, [dev.descs[by_id[x]["client"]] for x in ids])
        dY = gh.to_dev(np.concatenate([by_id[x]["dY"] for x in ids], axis=0))
        dX = torch.full((off[-1], D_IN), float("nan"), device="cuda", dtype=torch.bfloat16)
        sb.symb_base_linear_bwd_input(h, batch, dY, Wd, dX, sb.SYMB_BWD_FULL, gh.workspace(batch, sb.SYMB_OP_BWD_INPUT), gh.stream_ptr())
        torch.cuda.synchronize()
        dXh = gh.bf16_to_f64(dX)
        for k, x in enumerate(ids):
            by_id[x]["dX"] = dXh[off[k]:off[k + 1]]
        groups.append(tuple(ids))

    drain(q, 1, pending, run_backward)
    q.close()
    assert sorted(x for g in groups for x in g) == sorted(r["rid"] for r in ft)
    for r in ft:
        alone = np.array([0, r["n"]], dtype=np.int32)
        check_dx(r["dX"], alone, [oads[r["client"]]], r["dY"], W, f"request {r['rid']} dX")
