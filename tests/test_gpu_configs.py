"""GPU parity at the full sizes of the five workload configurations, in the launch
configuration the bench times (same runner, same buffers, same kernels).

The fp64 oracle cannot compute whole tensors at these sizes, so per segment the first
two rows, the last two rows and a few seeded random rows of Y, Ybase and dX are compared
element by element, and the parameter gradients of a seeded subset of the segments are
compared in full.  Same bar as the small cases (see helpers.py).
"""
import numpy as np
import pytest
import torch

import oracle
import synth
from helpers import assert_close

pytestmark = pytest.mark.gpu

sb = None
layer = None
_h = None


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    global sb, layer, _h
    from paper_2507_03220_amd import binding, layer as layer_mod
    sb, layer = binding, layer_mod
    binding.lib()
    _h = binding.symb_create(0)
    yield
    torch.cuda.synchronize()
    binding.symb_destroy(_h)


def _f64(t):
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def run_projection(wl, pr, rows_per_seg, grad_segments, with_ybase=False):
    clients = wl.clients
    host_ads = [synth.make_adapter(wl, pr, c) for c in clients]
    segs = [layer.SegmentSpec(c.n_tokens, a.kind, a.rank, a.scale, a.A, a.B, c.finetune)
            for c, a in zip(clients, host_ads)]
    ft = [i for i, c in enumerate(clients) if c.finetune]
    off = wl.offsets
    boff = synth.offsets_of([clients[i] for i in ft])
    X, W = synth.make_X(wl, pr), synth.make_W(wl, pr)
    dY = synth.make_dY(wl, pr, int(boff[-1]))
    run = layer.ProjectionRun(_h, pr.name, pr.d_in, pr.d_out, segs, W, X, dY, want_ybase=True)
    s = torch.cuda.current_stream().cuda_stream
    tag = f"{wl.name}/{pr.name}"
    print(f"[{tag}] T={run.T} Tb={run.Tb} d_in={pr.d_in} d_out={pr.d_out}", flush=True)

    # ---- forward on every client
    run.fwd(s)
    torch.cuda.synchronize()
    oads = [oracle.Adapter(a.kind, a.rank, a.scale, a.A, a.B) for a in host_ads]
    rows = synth.sample_rows(off, rows_per_seg, tag)
    Y0r, Yr = oracle.forward(off, oads, X, W, None, rows=rows)
    ridx = torch.from_numpy(rows.astype(np.int64)).cuda()
    assert_close(_f64(run.Y.index_select(0, ridx)), Yr, f"{tag} Y", out_bf16=True)
    assert_close(_f64(run.Ybase.index_select(0, ridx)), Y0r, f"{tag} Ybase", out_bf16=True)

    # ---- backward on the fine-tuning clients only (a batch of its own)
    boads = [oads[i] for i in ft]
    Xb = np.ascontiguousarray(X[np.concatenate([np.arange(off[i], off[i + 1]) for i in ft])]) if len(ft) != len(clients) else X
    run.bwd_input(s)
    torch.cuda.synchronize()
    brows = synth.sample_rows(boff, rows_per_seg, tag + "/bwd")
    dXr = oracle.backward_input(boff, boads, dY, W, rows=brows)
    bidx = torch.from_numpy(brows.astype(np.int64)).cuda()
    assert_close(_f64(run.dX.index_select(0, bidx)), dXr, f"{tag} dX", out_bf16=True)

    # ---- adapter gradients; the saved base output fed back is the oracle's, rounded to bf16
    pick = [q for q in grad_segments if q < len(ft)]
    ia3_rows = [np.arange(boff[q], boff[q + 1]) for q in pick if boads[q].kind == oracle.IA3]
    Y0_saved = None
    if ia3_rows:
        need = np.concatenate(ia3_rows).astype(np.int32)
        Y0n, _ = oracle.forward(boff, boads, Xb, W, None, rows=need)
        Y0_saved = np.zeros((int(boff[-1]), pr.d_out), dtype=np.uint16)
        Y0_saved[need] = synth.f32_to_bf16_bits(Y0n.astype(np.float32))
        run.Ybase_b = layer.bits_to_dev(Y0_saved)
    elif any(a.kind == oracle.IA3 for a in boads):
        run.Ybase_b = torch.zeros((run.Tb, pr.d_out), device="cuda", dtype=torch.bfloat16)
    run.adapter_grad(s)
    torch.cuda.synchronize()
    for q in pick:
        a = boads[q]
        d = run.bwd_ad[q]
        if a.kind == oracle.LORA:
            dAr, dBr = oracle.lora_grad(boff, boads, Xb, dY, q)
            assert_close(d.dA.cpu().numpy(), dAr, f"{tag} dA[{q}]")
            assert_close(d.dB.cpu().numpy(), dBr, f"{tag} dB[{q}]")
        elif a.kind == oracle.IA3:
            cols = np.unique(np.concatenate([[0, 1, pr.d_out - 1], np.random.default_rng(q).integers(0, pr.d_out, 61)])).astype(np.int32)
            dlr = oracle.ia3_grad(boff, boads, Xb, dY, W, None, q, cols=cols, Y0_saved=Y0_saved)
            assert_close(d.dA.cpu().numpy()[cols], dlr, f"{tag} dl[{q}]")
    del run
    torch.cuda.empty_cache()


def _grad_pick(wl, n, seed):
    ft = [c for c in wl.clients if c.finetune]
    g = np.random.default_rng(seed)
    idx = {0, len(ft) - 1}
    idx.update(int(x) for x in g.integers(0, len(ft), size=n))
    return sorted(idx)


def test_cfg4_gemma27b_headline():
    wl = synth.cfg4_gemma27b()
    for pr in wl.projections:
        run_projection(wl, pr, rows_per_seg=2, grad_segments=_grad_pick(wl, 1, 4))


def test_cfg2_llama7b():
    wl = synth.cfg2_llama7b()
    for pr in wl.projections:
        run_projection(wl, pr, rows_per_seg=3, grad_segments=_grad_pick(wl, 1, 2))


def test_cfg3_granite20b():
    wl = synth.cfg3_granite20b()
    for pr in wl.projections:
        run_projection(wl, pr, rows_per_seg=2, grad_segments=_grad_pick(wl, 1, 3))


@pytest.mark.parametrize("any_rank", [False, True])
def test_cfg5_mixed_serving_and_tuning(any_rank):
    wl = synth.cfg5_mixed(arbitrary_ranks=any_rank)
    projs = wl.projections if not any_rank else [p for p in wl.projections if p.name in ("q", "gate", "down")]
    for pr in projs:
        run_projection(wl, pr, rows_per_seg=2, grad_segments=_grad_pick(wl, 3, 5))
