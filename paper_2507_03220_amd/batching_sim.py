#!/usr/bin/env python3
"""Opportunistic batching in front of one frozen layer, on synthetic arrivals (Sec. 3.7, Sec. 4).

A discrete-event simulation whose only real component is the executor: every batch the queue
forms is run on the GPU through symb_base_linear_fwd (flattened rows of all its requests, one
LoRA segment per request) and the measured duration advances the simulated clock.  Clients are
closed-loop, as in the paper's trace replay: an inference client sends a prefill, then decode
steps of one token, each a think time (its own client-side layers) after the previous answer;
fine-tuning clients send 1024-token passes.  Policies compared:
  alone          every request runs by itself, first come first served (the paper's "no-lockstep");
  as-it-comes    no waiting, but whatever queued up while the executor was busy goes together;
  opportunistic  size-dependent wait (base + per-token, capped), inference first.
No trace, dataset or weights: lengths are seeded draws (prefill: bounded Zipf(1.1) on 16..4096).

Run:  python -m paper_2507_03220_amd.batching_sim [--requests 4000] [--d-in 4096 --d-out 4096]
"""
from __future__ import annotations

import argparse
import heapq
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def zipf_bounded(rng, lo, hi, a=1.1):
    k = np.arange(lo, hi + 1)
    p = k ** (-a)
    p /= p.sum()
    return lambda: int(rng.choice(k, p=p))


def simulate(policy_name, pol, args, layer):
    import torch
    from paper_2507_03220_amd import batcher as bt
    from paper_2507_03220_amd import binding as sb

    rng = np.random.default_rng(args.seed)
    draw_prefill = zipf_bounded(rng, 16, 4096)
    q = bt.Batcher(pol["base"], pol["per_tok"], pol["max_wait"], pol["cap"])
    h, X, W, Y, ads, ws = layer
    # client state machines: (kind, steps left in the current generation)
    n_inf, n_ft = args.inference_clients, args.finetune_clients
    future = []            # (arrival time, seq, client, n_tokens, latency_sensitive)
    seq = 0
    steps_left = {}
    for c in range(n_inf):
        heapq.heappush(future, (float(rng.uniform(0, 2000)), seq, c, draw_prefill(), True)); seq += 1
        steps_left[c] = int(rng.integers(8, 33))
    for c in range(n_inf, n_inf + n_ft):
        heapq.heappush(future, (float(rng.uniform(0, 2000)), seq, c, 1024, False)); seq += 1
    info, done = {}, []
    now = busy_until = 0.0
    busy_us = flops = 0.0
    served_tokens = decode_tokens = 0
    batches = []
    rid = 0
    stream = torch.cuda.current_stream()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    while len(done) < args.requests:
        due = max(q.next_due(0), busy_until)
        if future and future[0][0] <= due:
            t, _, c, n_tok, ls = heapq.heappop(future)
            now = t
            q.submit(0, rid, c, n_tok, ls, t)
            info[rid] = (c, n_tok, ls, t)
            rid += 1
            continue
        now = due
        ids, off = q.take(0, now)
        assert ids
        T = off[-1]
        batch = sb.Batch(args.d_in, args.d_out, off, [ads[info[i][0] % len(ads)] for i in ids])
        e0.record(stream)
        sb.symb_base_linear_fwd(h, batch, X, W, None, Y, None, ws, stream.cuda_stream)
        e1.record(stream)
        e1.synchronize()
        dur = e0.elapsed_time(e1) * 1e3
        busy_until = now + dur
        busy_us += dur
        flops += 2.0 * T * args.d_in * args.d_out
        batches.append((T, len(ids)))
        for i in ids:
            c, n_tok, ls, t_arr = info.pop(i)
            done.append((ls, n_tok, busy_until - t_arr))
            served_tokens += n_tok
            think = float(rng.uniform(*args.think_us))
            if c < n_inf:
                if n_tok == 1:
                    decode_tokens += 1
                if steps_left[c] > 0:
                    steps_left[c] -= 1
                    heapq.heappush(future, (busy_until + think, seq, c, 1, True)); seq += 1
                else:
                    steps_left[c] = int(rng.integers(8, 33))
                    heapq.heappush(future, (busy_until + 4 * think, seq, c, draw_prefill(), True)); seq += 1
            else:
                heapq.heappush(future, (busy_until + 10 * think, seq, c, 1024, False)); seq += 1
    q.close()
    lat_dec = np.array([l for ls, n, l in done if ls and n == 1])
    lat_big = np.array([l for ls, n, l in done if n > 1])
    Ts = np.array([b[0] for b in batches]); Ss = np.array([b[1] for b in batches])
    return dict(policy=policy_name, sim_ms=busy_until / 1e3, batches=len(batches), mean_T=Ts.mean(), mean_S=Ss.mean(),
                tokens_per_s=served_tokens / (busy_until * 1e-6), decode_tokens_per_s=decode_tokens / (busy_until * 1e-6),
                decode_lat_mean_us=lat_dec.mean() if len(lat_dec) else float("nan"),
                decode_lat_p95_us=np.percentile(lat_dec, 95) if len(lat_dec) else float("nan"),
                big_lat_mean_us=lat_big.mean() if len(lat_big) else float("nan"),
                busy_frac=busy_us / busy_until, tflops_busy=flops / (busy_us * 1e-6) / 1e12)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--requests", type=int, default=4000)
    ap.add_argument("--d-in", type=int, default=4096)
    ap.add_argument("--d-out", type=int, default=4096)
    ap.add_argument("--rank", type=int, default=16)
    ap.add_argument("--inference-clients", type=int, default=32)
    ap.add_argument("--finetune-clients", type=int, default=2)
    ap.add_argument("--think-us", type=float, nargs=2, default=(60.0, 200.0))
    ap.add_argument("--seed", type=int, default=20250703)
    args = ap.parse_args()

    import torch
    from paper_2507_03220_amd import binding as sb
    assert torch.cuda.is_available(), "the simulation runs its batches on the GPU"
    sb.lib()
    h = sb.symb_create(0)
    g = torch.Generator(device="cuda").manual_seed(args.seed)
    max_rows = 65536
    X = torch.randn((max_rows, args.d_in), device="cuda", generator=g).to(torch.bfloat16)
    W = (torch.randn((args.d_out, args.d_in), device="cuda", generator=g) * args.d_in ** -0.5).to(torch.bfloat16)
    Y = torch.empty((max_rows, args.d_out), device="cuda", dtype=torch.bfloat16)
    ads = []
    for _ in range(args.inference_clients + args.finetune_clients):
        A = (torch.randn((args.rank, args.d_in), device="cuda", generator=g) * args.d_in ** -0.5).to(torch.bfloat16)
        B = (torch.randn((args.d_out, args.rank), device="cuda", generator=g) * args.rank ** -0.5).to(torch.bfloat16)
        ads.append(sb.Adapter(sb.SYMB_ADAPTER_LORA, args.rank, 2.0, A, B))
    # Hs of the largest batch, plus room for the fp32 partial tiles of a K-split launch (at most 320 tiles of 64 KiB)
    ws = torch.empty(max_rows * 2 * 16 * ((args.rank + 15) // 16) * 2 + 4096 + (24 << 20), device="cuda", dtype=torch.uint8)
    layer = (h, X, W, Y, ads, ws)
    policies = [("alone", dict(base=0.0, per_tok=0.0, max_wait=0.0, cap=1)),
                ("as-it-comes", dict(base=0.0, per_tok=0.0, max_wait=0.0, cap=max_rows)),
                ("opportunistic", dict(base=40.0, per_tok=0.25, max_wait=600.0, cap=16384))]
    for name, pol in policies:      # one short untimed pass warms up kernels and caches
        simulate(name, pol, argparse.Namespace(**{**vars(args), "requests": 200}), layer)
    print(f"layer {args.d_in}->{args.d_out}, LoRA r={args.rank}; {args.inference_clients} inference + {args.finetune_clients} fine-tuning "
          f"clients, closed loop, think time U{tuple(args.think_us)} us; {args.requests} requests per policy")
    print(f"{'policy':14s} {'batches':>8s} {'mean T':>8s} {'mean S':>7s} {'tok/s':>11s} {'decode tok/s':>13s} {'decode lat us (mean / p95)':>27s} "
          f"{'prefill+FT lat us':>18s} {'busy':>6s} {'TFLOP/s busy':>13s}")
    for name, pol in policies:
        r = simulate(name, pol, args, layer)
        print(f"{r['policy']:14s} {r['batches']:8d} {r['mean_T']:8.1f} {r['mean_S']:7.2f} {r['tokens_per_s']:11.0f} {r['decode_tokens_per_s']:13.0f} "
              f"{r['decode_lat_mean_us']:13.0f} / {r['decode_lat_p95_us']:<11.0f} {r['big_lat_mean_us']:18.0f} {r['busy_frac']:6.2f} {r['tflops_busy']:13.1f}", flush=True)
    sb.symb_destroy(h)
    return 0


if __name__ == "__main__":
    sys.exit(main())
