"""GPU parity at the full sizes of the five workload configurations, through the runner,
buffers, workspace and call sequence the bench times.

Per projection: (1) a forward that also emits the pre-adapter output (the full-epilogue
instantiation of the GEMM); (2) the forward exactly as the bench launches it -- no bias, no
pre-adapter output, the whole workspace, so the plain-epilogue instantiation with its last
round of tiles split over K ranges where the planner splits it; (3) the adapter
gradients as in a bench step (Hs from the workspace, dB and dH in one pass over dY); (4) the input
gradient taking that dH; (5) the other order (input gradient first, the gradient call taking its
dH), whose dB must have the same bits; (6) a gradient call on its own.

The fp64 oracle cannot compute whole tensors at these sizes, so rows of Y, Ybase and dX are
sampled: per segment its first two and last two rows and 28 seeded random rows, plus one
seeded row of every run of 128 consecutive rows (both wavefront halves of every 256-row
tile); sampled rows are compared element by element.  The parameter gradients of every
fine-tuning segment are compared in full.  Same bar as the small cases (helpers.py).
"""
import time

import numpy as np
import pytest
import torch

import oracle
import synth
from helpers import assert_close, assert_close_client

pytestmark = pytest.mark.gpu

sb = None
layer = None
_h = None

ROWS_PER_SEGMENT = 28      # seeded random rows per segment, besides its boundary rows
ROW_BLOCK = 128            # and one row of every 128 consecutive rows of the batch


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


def run_projection(wl, pr):
    t_start = time.time()
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

    # ---- (1) forward on every client, pre-adapter output wanted
    run.Y.fill_(float("nan"))
    run.fwd(s)
    torch.cuda.synchronize()
    oads = [oracle.Adapter(a.kind, a.rank, a.scale, a.A, a.B) for a in host_ads]
    rows = synth.sample_rows(off, ROWS_PER_SEGMENT, tag, block=ROW_BLOCK)
    Y0r, Yr = oracle.forward(off, oads, X, W, None, rows=rows)
    ridx = torch.from_numpy(rows.astype(np.int64)).cuda()
    assert_close(_f64(run.Y.index_select(0, ridx)), Yr, f"{tag} Y", out_bf16=True)
    assert_close(_f64(run.Ybase.index_select(0, ridx)), Y0r, f"{tag} Ybase", out_bf16=True)

    # ---- (2) the forward as the bench launches it: no pre-adapter output, the whole workspace
    ybase = run.Ybase
    run.Ybase = None
    run.Y.fill_(float("nan"))
    run.fwd(s)
    torch.cuda.synchronize()
    run.Ybase = ybase
    assert_close(_f64(run.Y.index_select(0, ridx)), Yr, f"{tag} Y (as timed)", out_bf16=True)

    # ---- (3) adapter gradients of every fine-tuning segment (a backward batch of its own), as in a bench step:
    # Hs taken from the workspace where the backward batch is the forward batch; dB and dH in one pass
    # over dY where the ranks allow.  The saved base output fed back for the IA3 gradients is the
    # oracle's, rounded to bf16.
    boads = [oads[i] for i in ft]
    Xb = np.ascontiguousarray(X[np.concatenate([np.arange(off[i], off[i + 1]) for i in ft])]) if len(ft) != len(clients) else X
    ia3_rows = [np.arange(boff[q], boff[q + 1]) for q in range(len(ft)) if boads[q].kind == oracle.IA3]
    Y0_saved = None
    if ia3_rows:
        need = np.concatenate(ia3_rows).astype(np.int32)
        Y0n, _ = oracle.forward(boff, boads, Xb, W, None, rows=need)
        Y0_saved = np.zeros((int(boff[-1]), pr.d_out), dtype=np.uint16)
        Y0_saved[need] = synth.f32_to_bf16_bits(Y0n.astype(np.float32))
        run.Ybase_b = layer.bits_to_dev(Y0_saved)
    ref_grads = {}
    for q in range(len(ft)):
        a = boads[q]
        if a.kind == oracle.LORA:
            ref_grads[q] = oracle.lora_grad(boff, boads, Xb, dY, q)
        elif a.kind == oracle.IA3:
            cols = np.unique(np.concatenate([[0, 1, pr.d_out - 1], np.random.default_rng(q).integers(0, pr.d_out, 61)])).astype(np.int32)
            ref_grads[q] = (cols, oracle.ia3_grad(boff, boads, Xb, dY, W, None, q, cols=cols, Y0_saved=Y0_saved))

    def check_grads(route):
        for q, ref in ref_grads.items():
            d = run.bwd_ad[q]
            if boads[q].kind == oracle.LORA:
                assert_close(d.dA.cpu().numpy(), ref[0], f"{tag} dA[{q}] ({route})")
                assert_close(d.dB.cpu().numpy(), ref[1], f"{tag} dB[{q}] ({route})")
            else:
                assert_close(d.dA.cpu().numpy()[ref[0]], ref[1], f"{tag} dl[{q}] ({route})")

    def nan_grads():
        for d in run.bwd_ad:
            for g in (d.dA, d.dB):
                if g is not None:
                    g.fill_(float("nan"))

    nan_grads()
    run.adapter_grad(s, reuse_hs=True)
    torch.cuda.synchronize()
    check_grads("gradients first")
    first_dB = [d.dB.clone() if d.dB is not None else None for d in run.bwd_ad]
    n_grads = len(ref_grads)

    # ---- (4) input gradient taking dH from that gradient call
    brows = synth.sample_rows(boff, ROWS_PER_SEGMENT, tag + "/bwd", block=ROW_BLOCK)
    dXr = oracle.backward_input(boff, boads, dY, W, rows=brows)
    # with IA3 segments in the backward batch: dY * l as the bf16 tensor the paper's client would send (helpers.py)
    dXc = oracle.backward_input(boff, boads, dY, W, rows=brows, client_bf16=True) if any(a.kind == oracle.IA3 for a in boads) else None
    close_dx = lambda got, what: assert_close(got, dXr, what, out_bf16=True) if dXc is None else assert_close_client(got, dXr, dXc, what)
    bidx = torch.from_numpy(brows.astype(np.int64)).cuda()
    run.dX.fill_(float("nan"))
    run.bwd_input(s, reuse_dh=True)
    torch.cuda.synchronize()
    close_dx(_f64(run.dX.index_select(0, bidx)), f"{tag} dX (as timed)")

    # ---- (5) the other order: the input gradient computes dH itself, the gradient call takes it over
    run.dX.fill_(float("nan"))
    run.bwd_input(s)
    torch.cuda.synchronize()
    close_dx(_f64(run.dX.index_select(0, bidx)), f"{tag} dX")
    nan_grads()
    run.adapter_grad(s, reuse_dh=True, reuse_hs=True)
    torch.cuda.synchronize()
    check_grads("input gradient first")
    for b1, d in zip(first_dB, run.bwd_ad):
        if b1 is not None:
            assert torch.equal(b1, d.dB), f"{tag}: dB differs between the one-pass and the two-pass route"
    # ---- (6) a gradient call on its own recomputes Hs and dH
    nan_grads()
    run._hs_in_ws = False
    run.adapter_grad(s)
    torch.cuda.synchronize()
    check_grads("stand-alone")
    print(f"[{tag}] compared {len(rows)} rows of Y/Ybase, {len(brows)} rows of dX, gradients of {n_grads}/{len(ft)} "
          f"fine-tuning segments in {time.time() - t_start:.1f}s", flush=True)
    del run
    torch.cuda.empty_cache()
    return len(rows), len(brows), n_grads


def test_cfg4_gemma27b_headline():
    wl = synth.cfg4_gemma27b()
    for pr in wl.projections:
        nr, nb, ng = run_projection(wl, pr)
        assert nr >= 640 and nb >= 640 and ng == 20


def test_cfg2_llama7b():
    wl = synth.cfg2_llama7b()
    for pr in wl.projections:
        run_projection(wl, pr)


def test_cfg3_granite20b():
    wl = synth.cfg3_granite20b()
    for pr in wl.projections:
        run_projection(wl, pr)


@pytest.mark.parametrize("any_rank", [False, True])
def test_cfg5_mixed_serving_and_tuning(any_rank):
    wl = synth.cfg5_mixed(arbitrary_ranks=any_rank)
    projs = wl.projections if not any_rank else [p for p in wl.projections if p.name in ("q", "gate", "down")]
    for pr in projs:
        run_projection(wl, pr)
