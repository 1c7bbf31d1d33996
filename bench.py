#!/usr/bin/env python3
"""Benchmark of the segmented base+adapter layer on one MI355X.

A step = one pass of the whole hot path over one synthetic batch: for every projection
of the layer shape, forward (shrink + fused GEMM), adapter gradients (dB and dH in one pass
over dY, then dA; dl) and input gradient (fused GEMM taking that dH), all through the C ABI.  Inputs are resident in HBM before
the timed region.  Default workload: the Gemma2-27B-shaped layer with 20 LoRA clients x
1024 tokens (T = 20480), ranks from {8, 16}.

Prints ONE JSON line: metric, value (whole-step TFLOP/s), timing, the roofline of the dominant GEMM kernel,
per-projection timings and the oracle timed on the host cores.  Run with --gpus 1 only.

What `value` is timed on: K steps back to back on one stream, host wall clock between two device
synchronisations, the library's host work of every call included.  The steps repeat one batch
layout (the same 20 clients with the same lengths, as in a fine-tuning job), so after the warm-up
every call finds its descriptors on the device and sends nothing; `ms_per_step_descriptors_sent`
is the same region timed again with that reuse switched off (every call uploads its descriptors,
as a job whose batch layout changes from call to call does).  `ms_per_step_median` / `_min` are
per-step event times of the same timed region; `fwd_only_ms` / `bwd_only_ms` time the forward calls
and the backward calls (input gradient + adapter gradients) of all projections on their own.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

BF16_MFMA_PEAK_TFLOPS = 2500.0     # MI355X dense bf16 matrix peak (256 CU x 4096 flop/clk x 2.4 GHz)
HBM_PEAK_GBS = 8000.0


def build_layer(cfg: str, handle):
    import numpy as np
    import synth
    from paper_2507_03220_amd import binding as sb
    from paper_2507_03220_amd.layer import ProjectionRun, SegmentSpec

    wl = synth.CONFIGS[cfg]()
    runs = []
    t0 = time.time()
    for pr in wl.projections:
        segs = []
        for c in wl.clients:
            a = synth.make_adapter(wl, pr, c)
            segs.append(SegmentSpec(c.n_tokens, a.kind, a.rank, a.scale, a.A, a.B, c.finetune))
        Tb = sum(c.n_tokens for c in wl.clients if c.finetune)
        run = ProjectionRun(handle, pr.name, pr.d_in, pr.d_out, segs, synth.make_W(wl, pr), synth.make_X(wl, pr),
                            synth.make_dY(wl, pr, Tb))
        runs.append(run)
    return wl, runs, time.time() - t0


def step(runs, stream):
    for r in runs:
        r.fwd(stream)
    for r in runs:
        # same batch, same X, same dY, same workspace: the gradient call takes Hs as the forward left it and
        # forms dB and dH in one pass over dY; the input gradient takes that dH
        r.adapter_grad(stream, reuse_hs=True)
        r.bwd_input(stream, reuse_dh=True)


def cpu_baseline(cfg: str, budget_s: float = 20.0) -> dict:
    """Times the fp64 oracle, as it stands, on a bounded sample of the same workload:
    forward and input-gradient rows of the widest projection plus full LoRA gradients of
    one client on the narrowest one; reports algorithmic TFLOP/s of that sample."""
    import numpy as np
    import oracle
    import synth

    wl = synth.CONFIGS[cfg]()
    pr = max(wl.projections, key=lambda p: p.d_in * p.d_out)
    clients = wl.clients
    off = wl.offsets
    # sample: rows of the first two non-empty segments only, so only those rows are generated
    keep = [i for i, c in enumerate(clients) if c.n_tokens > 0][:2]
    sub_clients = [clients[i] for i in keep]
    sub_off = synth.offsets_of(sub_clients)
    Ts = int(sub_off[-1])
    ads = []
    for c in sub_clients:
        a = synth.make_adapter(wl, pr, c)
        ads.append(oracle.Adapter(a.kind, a.rank, a.scale, a.A, a.B))
    W = synth.make_W(wl, pr)
    X = synth.normal_bf16((Ts, pr.d_in), 1.0, "cpu_baseline/X")
    dY = synth.normal_bf16((Ts, pr.d_out), 1.0, "cpu_baseline/dY")
    per_row = 2.0 * pr.d_in * pr.d_out
    nthreads = oracle.num_threads()
    # calibrate with one row per thread, then size the sample to the budget
    rows = np.arange(min(nthreads, Ts), dtype=np.int32)
    t0 = time.time(); oracle.forward(sub_off, ads, X, W, None, rows=rows); t_cal = time.time() - t0
    n = int(max(nthreads, min(Ts, (budget_s / 2.2) / max(t_cal, 1e-3) * len(rows))))
    n = (n // nthreads) * nthreads or nthreads
    rows = np.linspace(0, Ts - 1, n).astype(np.int32)
    t0 = time.time(); oracle.forward(sub_off, ads, X, W, None, rows=rows); t_f = time.time() - t0
    t0 = time.time(); oracle.backward_input(sub_off, ads, dY, W, rows=rows); t_b = time.time() - t0
    flops = 2 * n * per_row
    t_g, g_flops = 0.0, 0.0
    if ads[0].kind == oracle.LORA:
        # LoRA gradients of one client on a bounded token count
        ng = min(int(sub_off[1]), 256)
        goff = np.array([0, ng], dtype=np.int32)
        t0 = time.time(); oracle.lora_grad(goff, ads[:1], X[:ng], dY[:ng], 0); t_g = time.time() - t0
        g_flops = 4.0 * ng * ads[0].rank * (pr.d_in + pr.d_out) * 1.5   # dA, dB plus recomputed H and dH
    total_t = t_f + t_b + t_g
    return {"value": (flops + g_flops) / total_t / 1e12, "unit": "TFLOP/s", "cores": nthreads, "kind": "oracle",
            "sample": f"{cfg} projection {pr.name} ({pr.d_in}->{pr.d_out}): {n} rows forward ({t_f:.1f}s) + {n} rows "
                      f"input gradient ({t_b:.1f}s)" + (f" + LoRA gradients of one client over {ng} tokens ({t_g:.1f}s)" if t_g else ""),
            "seconds": total_t}


def per_projection(runs, stream_obj, stream, reps: int = 5) -> list:
    """Median event time of each call of each projection, run alone (outside the timed region)."""
    import statistics
    import torch
    out = []

    def timed(fn):
        ts = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream_obj)
            fn()
            e1.record(stream_obj)
            e1.synchronize()
            ts.append(e0.elapsed_time(e1))
        return statistics.median(ts)

    for r in runs:
        fl = r.flops()
        t_f = timed(lambda: r.fwd(stream))
        t_b = timed(lambda: r.bwd_input(stream))
        r.bwd_input(stream)
        t_g = timed(lambda: r.adapter_grad(stream))       # stand-alone: recomputes Hs and dH
        out.append({"name": r.name, "d_in": r.d_in, "d_out": r.d_out,
                    "fwd_ms": round(t_f, 4), "bwd_input_ms": round(t_b, 4), "adapter_grad_ms": round(t_g, 4),
                    "fwd_tflops": round((fl["base_fwd"] + fl["ad_fwd"]) / t_f / 1e9, 1),
                    "bwd_input_tflops": round(fl["base_bwd"] / t_b / 1e9, 1)})
    return out


def measured_traffic(cfg: str, variant: int):
    """HBM/fabric bytes per launch of the dominant GEMM kernel.  Not measured in this run: read from the
    rocprofv3 --pmc summary committed under profiles/ (FETCH_SIZE + WRITE_SIZE, scaled by a plain copy),
    which exists for cfg4's 256x256 instantiations only; None otherwise."""
    if cfg != "cfg4" or variant not in (0, 1):
        return None
    path = os.path.join(ROOT, "profiles", "cfg4_gemm_hbm_traffic.txt")
    key = "traffic_bytes_per_launch_nn:" if variant else "traffic_bytes_per_launch_nt:"
    try:
        for line in open(path):
            if line.startswith(key):
                return float(line.split(":", 1)[1])
    except OSError:
        pass
    return None


def kernel_name(variant: int) -> str:
    return "symb_gemm16_kernel<%d,%s,%s>" % (4 if variant & 2 else 8, "true" if variant & 1 else "false",
                                             "false" if variant & 4 else "true")


def timed_steps(runs, stream_obj, stream, steps: int):
    """K steps back to back; returns (wall ms of the whole region, per-step event times in ms)."""
    import torch
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev[0].record(stream_obj)
    for k in range(steps):
        step(runs, stream)
        ev[k + 1].record(stream_obj)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return wall_ms, [ev[k].elapsed_time(ev[k + 1]) for k in range(steps)]


def phase_only(runs, stream_obj, stream, reps: int = 5):
    """Median event time of all forward calls / all backward calls of the layer, each phase on its own."""
    import statistics
    import torch

    def timed(fn):
        ts = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream_obj)
            fn()
            e1.record(stream_obj)
            e1.synchronize()
            ts.append(e0.elapsed_time(e1))
        return statistics.median(ts)

    def fwd():
        for r in runs:
            r.fwd(stream)

    def bwd():
        for r in runs:
            r.adapter_grad(stream, reuse_hs=True)
            r.bwd_input(stream, reuse_dh=True)
    t_f = timed(fwd)
    fwd()                                                   # Hs of every projection back in its workspace
    return t_f, timed(bwd)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="cfg4", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-detail", action="store_true", help="skip the per-projection timings taken after the timed region")
    ap.add_argument("--cpu-budget", type=float, default=20.0)
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 1 GiB device-to-device copy (counter calibration under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2507_03220_amd import binding as sb

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    sb.lib()
    torch.cuda.set_device(0)
    h = sb.symb_create(0)
    wl, runs, t_gen = build_layer(args.config, h)
    stream_obj = torch.cuda.current_stream()
    stream = stream_obj.cuda_stream
    print(f"[bench] {wl.name}: T={wl.T} S={len(wl.clients)} projections={[r.name for r in runs]} "
          f"inputs generated+uploaded in {t_gen:.1f}s", file=sys.stderr, flush=True)

    if args.copy_probe:     # a plain copy of known size: 1 GiB read + 1 GiB written per launch
        src = torch.empty(1 << 29, device="cuda", dtype=torch.bfloat16).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for r in runs:          # one untimed pass materialises saved outputs where IA3 gradients need them
        r.fwd(stream)
        r.sync_saved_output()
    for _ in range(args.warmup):
        step(runs, stream)
    torch.cuda.synchronize()

    sb.symb_debug_gemm_timing_enable(h, True)
    desc0 = sb.symb_debug_descriptor_stats(h)
    wall_ms, step_ms = timed_steps(runs, stream_obj, stream, args.steps)
    ev_ms = sum(step_ms)
    ms_per_step = wall_ms / args.steps
    desc1 = sb.symb_debug_descriptor_stats(h)

    fl = {k: sum(r.flops()[k] for r in runs) for k in runs[0].flops()}
    tflops = fl["total"] / (ms_per_step * 1e-3) / 1e12
    tokens = wl.T
    timing = {v: sb.symb_debug_gemm_timing_read(h, v) for v in range(8)}
    sb.symb_debug_gemm_timing_enable(h, False)
    dom = max(timing, key=lambda v: timing[v][0])
    ms_tot, n_launch, fl_tot = timing[dom]
    avg_ms = ms_tot / max(n_launch, 1)
    achieved = (fl_tot / max(n_launch, 1)) / (avg_ms * 1e-3) / 1e12 if n_launch else 0.0
    gemm_ms_per_step = sum(t[0] for t in timing.values()) / args.steps
    # the same region with every call sending its descriptors
    sb.symb_debug_set_option(h, sb.SYMB_OPT_DESCRIPTOR_REUSE, 0)
    step(runs, stream)
    wall_sent_ms, _ = timed_steps(runs, stream_obj, stream, args.steps)
    desc2 = sb.symb_debug_descriptor_stats(h)
    sb.symb_debug_set_option(h, sb.SYMB_OPT_DESCRIPTOR_REUSE, 1)
    step(runs, stream)
    fwd_ms, bwd_ms = phase_only(runs, stream_obj, stream)
    import statistics
    out = {
        "metric": "fwd+bwd base+adapter layer TFLOP/s",
        "value": round(tflops, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: {len(wl.clients)} clients, T={wl.T} tokens, "
                               f"projections {','.join(f'{r.name}:{r.d_in}->{r.d_out}' for r in runs)}; "
                               "fwd + dX + adapter grads per projection",
                   "tokens": tokens, "clients": len(wl.clients)},
        "value_timed_on": "descriptors found in place (the steps repeat one batch layout)",
        "ms_per_step_median": round(statistics.median(step_ms), 4),
        "ms_per_step_min": round(min(step_ms), 4),
        "ms_per_step_descriptors_sent": round(wall_sent_ms / args.steps, 4),
        "tflops_descriptors_sent": round(fl["total"] / (wall_sent_ms / args.steps * 1e-3) / 1e12, 2),
        "fwd_only_ms": round(fwd_ms, 4),
        "bwd_only_ms": round(bwd_ms, 4),
        "fwd_only_tflops": round((fl["base_fwd"] + fl["ad_fwd"]) / fwd_ms / 1e9, 1),
        "bwd_only_tflops": round((fl["base_bwd"] + fl["ad_bwd"]) / bwd_ms / 1e9, 1),
        "mfma_util": round(tflops / BF16_MFMA_PEAK_TFLOPS, 4),
        "token_layers_per_s": round(tokens / (ms_per_step * 1e-3), 1),
        "model_equiv_tokens_per_s": round(tokens / (ms_per_step * 1e-3) / 46.0, 1) if args.config == "cfg4" else None,
        "event_ms_per_step": round(ev_ms / args.steps, 4),
        "gemm_ms_per_step": round(gemm_ms_per_step, 4),
        "algorithmic_tflop_per_step": round(fl["total"] / 1e12, 4),
        "roofline": {
            "bound": "mfma",
            "kernel": kernel_name(dom),
            "achieved": round(achieved, 2),
            "peak": BF16_MFMA_PEAK_TFLOPS,
            "unit": "TFLOP/s",
            "frac": round(achieved / BF16_MFMA_PEAK_TFLOPS, 4),
            "avg_launch_ms": round(avg_ms, 4),
            "launches": n_launch,
            "traffic": measured_traffic(args.config, dom),
            "traffic_source": "stored: profiles/cfg4_gemm_hbm_traffic.txt (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE; not measured in this run)"
                              if measured_traffic(args.config, dom) is not None else None,
        },
        "gemm_kernels": {kernel_name(v): {"launches": t[1], "ms_per_step": round(t[0] / args.steps, 4),
                                          "tflops": round(t[2] / (t[0] * 1e-3) / 1e12, 1) if t[0] > 0 else None}
                         for v, t in timing.items() if t[1]},
    }
    # calls of the timed region that sent their descriptors / found them on the device from an earlier step
    out["descriptors"] = {"sent": desc1[0] - desc0[0], "in_place": desc1[1] - desc0[1],
                          "sent_in_second_region": desc2[0] - desc1[0]}
    if not args.no_detail:
        out["per_projection"] = per_projection(runs, stream_obj, stream)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.config, args.cpu_budget)
        out["cpu_baseline"]["value"] = float("%.3g" % out["cpu_baseline"]["value"])
        out["cpu_baseline"]["seconds"] = round(out["cpu_baseline"]["seconds"], 1)
    print(json.dumps(out), flush=True)
    sb.symb_destroy(h)
    return 0


if __name__ == "__main__":
    sys.exit(main())
