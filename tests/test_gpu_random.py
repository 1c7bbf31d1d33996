"""Seeded random batches against the oracle, beyond the hand-picked cases: every run draws the same cases.

(1) Random shapes that reach the 256x256 tile, the split last round, long segments summed in runs, narrow
layers, every adapter kind, ranks 1..128, empty and one-token segments: forward (with and without the
pre-adapter output), input gradient (full and base-only) and all parameter gradients, each tensor in full.
(2) Random client mixes (inference and fine-tuning segments, so the backward batch is a batch of its own)
through the layer runner's call sequence of tests/test_gpu_configs.py: forward as timed, gradients first
with dB + dH in one pass where the layer is wide, the input gradient taking that dH, the other order (dB
bit-identical), a gradient call on its own."""
import numpy as np
import pytest

import oracle
import synth

pytestmark = pytest.mark.gpu

L, I, N = oracle.LORA, oracle.IA3, oracle.NONE


def _random_case(rng, n):
    big_out = rng.random() < 0.5
    small = int(rng.choice([8, 24, 40, 64, 72, 136, 200, 264, 328]))
    S = int(rng.integers(1, 9))
    lens = [int(x) for x in rng.choice([0, 1, 1, 2, 7, 16, 33, 100, 255, 256, 257, 300, 700], size=S)]
    if sum(lens) == 0:
        lens[0] = 130
    T = sum(lens)
    tiles_m = (T + 255) // 256
    wide = max(int(-(-128 // tiles_m) * 256 - 256 + 8 * rng.integers(1, 33)), 8)      # enough column tiles for the 256x256 kernel
    kinds = [int(x) for x in rng.choice([L, L, L, I, N], size=S)]
    ranks = [int(x) for x in rng.choice([1, 4, 5, 8, 16, 17, 32, 40, 64, 100, 128], size=S)]
    fam = rng.random()
    if fam < 0.12:        # the last round of tiles split over K ranges: at least 264 tiles, K of 1024 or more
        lens = [int(x) for x in rng.choice([120, 1, 99, 80, 200, 33], size=int(rng.integers(2, 5)))]
        tiles_m = (sum(lens) + 255) // 256
        wide = int(-(-264 // tiles_m) * 256 + 8 * rng.integers(0, 40) * tiles_m)
        small = int(rng.choice([1032, 1096, 2056]))
        kinds = kinds[:len(lens)]
    elif fam < 0.3:       # long segments (gradients summed in runs), a narrow layer
        lens = [int(x) for x in rng.choice([1537, 1600, 2100, 3000, 40, 1, 1536], size=int(rng.integers(1, 4)))]
        small, wide = int(rng.choice([72, 136, 264])), int(rng.choice([136, 200, 392]))
    d_in, d_out = (small, wide) if big_out else (wide, small)
    return dict(seed=20_000 + n, d_in=d_in, d_out=d_out, lens=lens, kinds=kinds, ranks=ranks, bias=bool(rng.random() < 0.5))


def test_random_batches_in_full():
    import gpu_harness
    import test_gpu_parity as tp
    from paper_2507_03220_amd import binding
    tp.gh, tp.sb = gpu_harness, binding          # (that module's own fixture sets these only for its own tests)
    binding.lib()
    rng = np.random.default_rng(2024)
    n = 0
    while n < 40:
        case = _random_case(rng, n)
        if case["d_in"] * case["d_out"] * max(sum(case["lens"]), 1) > 3.0e9:      # keeps the oracle to seconds
            continue
        print(f"[random {n}] {case}", flush=True)
        c = dict(case)
        p = tp.make_problem(c.pop("seed"), c.pop("d_in"), c.pop("d_out"), c.pop("lens"), c.pop("kinds"), c.pop("ranks"), **c)
        tp.check_all(p, f"random{n}")
        n += 1


def test_random_client_mixes_through_the_runner():
    import test_gpu_configs as tc
    from paper_2507_03220_amd import binding, layer as layer_mod
    tc.sb, tc.layer = binding, layer_mod
    binding.lib()
    tc._h = binding.symb_create(0)
    try:
        rng = np.random.default_rng(2025)
        for n in range(60):
            clients = []
            for i in range(int(rng.integers(1, 10))):
                ntok = int(rng.choice([1, 1, 2, 16, 33, 100, 256, 300, 700, 1600]))
                kind = int(rng.choice([synth.KIND_LORA, synth.KIND_LORA, synth.KIND_IA3, synth.KIND_NONE]))
                rank = int(rng.choice([4, 8, 16, 16, 32, 64, 128, 5, 23])) if kind == synth.KIND_LORA else 0
                clients.append(synth.Client(ntok, kind, rank, 2.0 if kind == synth.KIND_LORA else 0.0, bool(rng.random() < 0.6), i))
            if not any(c.finetune for c in clients):
                clients[0].finetune = True
            if rng.random() < 0.4:          # ranks up to 16 everywhere: dB + dH in one pass where the layer is wide
                for c in clients:
                    if c.kind == synth.KIND_LORA:
                        c.rank = int(rng.choice([4, 8, 16, 12]))
            shape = int(rng.integers(0, 3))
            if shape == 0:
                d_in, d_out = int(8 * rng.integers(8, 200)), int(8 * rng.integers(8, 200))
            elif shape == 1:
                d_in, d_out = int(8 * rng.integers(8, 64)), int(16384 + 8 * rng.integers(0, 300))
            else:
                d_in, d_out = int(8 * rng.integers(700, 1400)), int(8 * rng.integers(8, 64))
            wl = synth.Workload(f"mix{n}", [synth.Projection("p", d_in, d_out, True)], clients, seed=30_000 + n)
            tc.run_projection(wl, wl.projections[0])
    finally:
        import torch
        torch.cuda.synchronize()
        binding.symb_destroy(tc._h)
        tc._h = None
