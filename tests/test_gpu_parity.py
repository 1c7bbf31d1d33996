"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle on the
same seeded bf16 bit patterns.  Sizes here let the oracle compute every element in
seconds while still spanning several tiles, ragged tails, segment-straddling tiles,
empty and one-token segments, odd ranks and every adapter kind.

Bar: relative Frobenius error <= 4e-3 and max-abs error <= 2e-2 after scaling the
oracle tensor to unit RMS, per tensor (per segment for parameter gradients); for tensors
delivered in bf16, elements beyond 5 RMS are allowed half a bf16 ulp of their magnitude
where that exceeds 2e-2 RMS (helpers.py); integer work (row->segment map, adapter
selection) bit-exact.
"""
import numpy as np
import pytest
import torch

import oracle
import synth
from helpers import assert_close, assert_close_client, check_dx, check_y, bits_of

pytestmark = pytest.mark.gpu

gh = None
sb = None


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    global gh, sb
    import gpu_harness
    from paper_2507_03220_amd import binding
    gh, sb = gpu_harness, binding
    binding.lib()          # fail loudly if the HIP library is not built
    yield
    torch.cuda.synchronize()


def make_problem(seed, d_in, d_out, lens, kinds, ranks, bias=True, scales=None):
    rng = np.random.default_rng(seed)
    S = len(lens)
    off = np.zeros(S + 1, dtype=np.int32)
    off[1:] = np.cumsum(lens)
    T = int(off[-1])
    nb = lambda shape, std, mean=0.0: synth.f32_to_bf16_bits(
        (mean + std * rng.standard_normal(shape)).astype(np.float32))
    ads = []
    for i in range(S):
        k = kinds[i % len(kinds)]
        if k == oracle.LORA:
            r = ranks[i % len(ranks)]
            s = scales[i % len(scales)] if scales else 16.0 / r
            ads.append(gh.HostAdapter(k, r, s, nb((r, d_in), d_in ** -0.5), nb((d_out, r), r ** -0.5)))
        elif k == oracle.IA3:
            ads.append(gh.HostAdapter(k, 0, 0.0, nb((d_out,), 0.1, 1.0)))
        elif k == oracle.IA3_IN:
            ads.append(gh.HostAdapter(k, 0, 0.0, nb((d_in,), 0.1, 1.0)))
        else:
            ads.append(gh.HostAdapter())
    return dict(off=off, T=T, d_in=d_in, d_out=d_out, ads=ads,
                X=nb((T, d_in), 1.0), W=nb((d_out, d_in), d_in ** -0.5), dY=nb((T, d_out), 1.0),
                bias=nb((d_out,), 0.5) if bias else None)


def oracle_ads(ads):
    return [oracle.Adapter(a.kind, a.rank, a.scale, a.A, a.B) for a in ads]


def check_all(p, tag):
    oads = oracle_ads(p["ads"])
    off = p["off"]
    # forward
    Y, Yb = gh.forward(off, p["ads"], p["X"], p["W"], p["bias"], want_base=True)
    Y0r, Yr = oracle.forward(off, oads, p["X"], p["W"], p["bias"])
    if p["T"]:
        assert_close(gh.bf16_to_f64(Y), Yr, f"{tag} Y", out_bf16=True)
        assert_close(gh.bf16_to_f64(Yb), Y0r, f"{tag} Ybase", out_bf16=True)
        # the call without the pre-adapter output is the one that may split tiles over K ranges
        Y2, _ = gh.forward(off, p["ads"], p["X"], p["W"], p["bias"], want_base=False)
        assert_close(gh.bf16_to_f64(Y2), Yr, f"{tag} Y (no Ybase)", out_bf16=True)
    # backward, both flavours
    for base_only in (False, True):
        dX = gh.backward_input(off, p["ads"], p["dY"], p["W"], base_only=base_only)
        if p["T"]:
            check_dx(gh.bf16_to_f64(dX), off, oads, p["dY"], p["W"], f"{tag} dX base_only={base_only}", base_only=base_only)
    # adapter gradients.  The saved base output a client feeds back is a bf16 tensor: both sides
    # get the same one, the oracle's Y0 rounded to bf16 here (never the GPU's own output).
    Y0_saved = synth.f32_to_bf16_bits(Y0r.astype(np.float32))
    dev = gh.adapter_grad(off, p["ads"], p["X"], p["dY"], Y0_saved, p["d_in"], p["d_out"])
    for i, a in enumerate(p["ads"]):
        d = dev.descs[i]
        empty = off[i + 1] == off[i]
        if a.kind == oracle.LORA:
            dAr, dBr = oracle.lora_grad(off, oads, p["X"], p["dY"], i)
            dA, dB = d.dA.cpu().numpy(), d.dB.cpu().numpy()
            if empty:
                assert not dA.any() and not dB.any(), f"{tag} empty segment {i} must give zero grads"
            else:
                assert_close(dA, dAr, f"{tag} dA[{i}]")
                assert_close(dB, dBr, f"{tag} dB[{i}]")
        elif a.kind == oracle.IA3:
            dlr = oracle.ia3_grad(off, oads, p["X"], p["dY"], p["W"], p["bias"], i, Y0_saved=Y0_saved)
            dl = d.dA.cpu().numpy()
            if empty:
                assert not dl.any()
            else:
                assert_close(dl, dlr, f"{tag} dl[{i}]")
    return Y, Yb


L, I, N = oracle.LORA, oracle.IA3, oracle.NONE


def test_cfg1_tiny_full():
    wl = synth.cfg1_tiny()
    pr = wl.projections[0]
    ads = []
    for c in wl.clients:
        t = synth.make_adapter(wl, pr, c)
        ads.append(gh.HostAdapter(t.kind, t.rank, t.scale, t.A, t.B))
    p = dict(off=wl.offsets, T=wl.T, d_in=pr.d_in, d_out=pr.d_out, ads=ads, X=synth.make_X(wl, pr),
             W=synth.make_W(wl, pr), dY=synth.make_dY(wl, pr, wl.T), bias=None)
    check_all(p, "cfg1")


@pytest.mark.parametrize("case", [
    # several 128-row tiles, ragged tail, tiles that straddle segments, an empty and two 1-token segments
    dict(seed=1, d_in=320, d_out=264, lens=[130, 1, 0, 77, 1, 300, 64], kinds=[L, I, L, N, L, L, I], ranks=[8, 16, 5, 24, 33]),
    # wide enough for the 256x256 variant (>= 128 big tiles): M 1500 (ragged), N 6200/K 136
    dict(seed=2, d_in=136, d_out=6208, lens=[700, 5, 795], kinds=[L, I, L], ranks=[16, 8]),
    dict(seed=3, d_in=6208, d_out=136, lens=[700, 5, 795], kinds=[L, I, L], ranks=[16, 8]),
    # the 256x256 kernel's LoRA steps: ranks that need 1, 2, 3, 4 and 8 steps of 32 extended columns, tiles
    # that hold several LoRA segments (a step fetched while another one multiplies), odd ranks, K tail
    dict(seed=9, d_in=200, d_out=6208, lens=[300, 1, 200, 2, 57, 0, 940], kinds=[L, L, I, L, L, L, L], ranks=[128, 40, 5, 64, 16, 24, 33]),
    dict(seed=10, d_in=6208, d_out=200, lens=[300, 1, 200, 2, 57, 0, 940], kinds=[L, L, N, L, L, L, L], ranks=[128, 40, 5, 64, 16, 24, 33]),
    # the 256x256 kernel on one partial row tile and 129 column tiles, the last of them 8 columns wide
    dict(seed=11, d_in=136, d_out=32776, lens=[100, 1, 49], kinds=[L, I, L], ranks=[16, 8, 40]),
    dict(seed=12, d_in=32776, d_out=136, lens=[100, 1, 49], kinds=[L, N, L], ranks=[16, 8, 40]),      # the same in the input gradient
    # 266 tiles of 256x256: each XCD's run of 34 tiles ends two tiles into a second round; those are split
    # over four K ranges each (fp32 partial tiles in the workspace); ragged last row tile, 8-column last tile
    dict(seed=13, d_in=2056, d_out=33800, lens=[120, 1, 99, 80], kinds=[L, I, L, N], ranks=[16, 8, 40]),
    dict(seed=14, d_in=33800, d_out=2056, lens=[120, 1, 99, 80], kinds=[L, N, L, L], ranks=[16, 8, 40, 24]),   # the same in the input gradient
    # segments of more than 1536 tokens: their LoRA gradients are summed in runs of 1024 tokens (1537: two runs,
    # the second of 513 tokens; 1536 stays whole)
    dict(seed=15, d_in=136, d_out=200, lens=[1700, 3, 2100, 1536, 1537], kinds=[L, L, L, L, L], ranks=[8, 16, 40, 4, 128]),
    # 128x128 tiles split over K ranges (6 tiles, 4 parts each), many short LoRA segments per tile: the parts
    # share the tile's LoRA steps out; ranks of 1 to 8 steps, an IA3 and a plain segment in between, K tail
    dict(seed=16, d_in=2056, d_out=264, lens=[8, 8, 3, 16, 8, 1, 8, 40, 8, 8, 5, 8, 8, 2, 8, 8, 9], kinds=[L, L, I, L, L, L, N, L, L, L, L, L, I, L, L, L, L],
         ranks=[16, 8, 40, 128, 4, 64, 24]),
    dict(seed=17, d_in=264, d_out=2056, lens=[8, 8, 3, 16, 8, 1, 8, 40, 8, 8, 5, 8, 8, 2, 8, 8, 9], kinds=[L, L, N, L, L, L, N, L, L, L, L, L, L, L, L, L, L],
         ranks=[16, 8, 40, 128, 4, 64, 24]),      # the same in the input gradient
    # the plain-epilogue instantiations of the 256x256 kernel (what a batch without bias, IA3 segment or
    # pre-adapter output runs, the measured configurations among them): forward and input gradient,
    # unsplit, and with the last round of 266 tiles split over four K ranges
    dict(seed=22, d_in=136, d_out=6208, lens=[700, 5, 795], kinds=[L, N, L], ranks=[16, 8], bias=False),
    dict(seed=23, d_in=6208, d_out=136, lens=[700, 5, 795], kinds=[L, N, L], ranks=[16, 8], bias=False),
    dict(seed=24, d_in=2056, d_out=33800, lens=[120, 1, 99, 80], kinds=[L, N, L, L], ranks=[16, 8, 40], bias=False),
    dict(seed=25, d_in=33800, d_out=2056, lens=[120, 1, 99, 80], kinds=[L, N, L, L], ranks=[16, 8, 40, 24], bias=False),
    # all kinds NONE: the paper's plain executor
    dict(seed=4, d_in=256, d_out=512, lens=[100, 156], kinds=[N], ranks=[1]),
    # rank 1, rank 128 (max), rank 100, K tail (d_in not a multiple of 64)
    dict(seed=5, d_in=200, d_out=392, lens=[40, 90, 33], kinds=[L], ranks=[1, 128, 100], bias=False),
    # single segment, single token
    dict(seed=6, d_in=64, d_out=64, lens=[1], kinds=[L], ranks=[8]),
    dict(seed=7, d_in=72, d_out=40, lens=[1], kinds=[I], ranks=[1]),
    # the only IA3 (IA3 on the input) segment of the batch is empty: nothing to scale, on either side of the layer
    dict(seed=26, d_in=328, d_out=10976, lens=[33, 256, 16, 257, 0], kinds=[L, L, L, N, I], ranks=[32, 1, 100]),
    dict(seed=27, d_in=328, d_out=392, lens=[0, 33, 256], kinds=[3, L, N], ranks=[8]),
    dict(seed=28, d_in=72, d_out=200, lens=[0, 9], kinds=[I, N], ranks=[1]),
    # many decode rows interleaved with long segments
    dict(seed=8, d_in=512, d_out=384, lens=[1, 1, 200, 1, 1, 1, 90, 1, 257, 1, 1], kinds=[L, I, L, L, I, N, I, L, L, I, L], ranks=[4, 64, 16, 8, 32, 128]),
])
def test_mixed_batches_full(case):
    c = dict(case)
    p = make_problem(c.pop("seed"), c.pop("d_in"), c.pop("d_out"), c.pop("lens"), c.pop("kinds"), c.pop("ranks"), **c)
    check_all(p, f"case{case['seed']}")


def test_empty_batch_and_all_empty_segments():
    p = make_problem(9, 64, 64, [0, 0], [L, I], [8])
    check_all(p, "all-empty")


def test_index_probe_bit_exact():
    """Adapter selection per row, read back through exactly representable values."""
    lens = [3, 0, 1, 130, 1, 1, 0, 260, 2, 129]
    S = len(lens)
    off = np.zeros(S + 1, dtype=np.int32)
    off[1:] = np.cumsum(lens)
    T, d_in, d_out = int(off[-1]), 64, 256
    Xf = np.zeros((T, d_in), np.float32); Xf[:, 0] = 1
    W = bits_of(np.zeros((d_out, d_in)))
    ads, oads = [], []
    for i in range(S):
        Af = np.zeros((2, d_in), np.float32); Af[0, 0] = 1
        Bf = np.zeros((d_out, 2), np.float32); Bf[:, 0] = i + 1
        ads.append(gh.HostAdapter(L, 2, 1.0, bits_of(Af), bits_of(Bf)))
    Y, _ = gh.forward(off, ads, bits_of(Xf), W, None, want_base=False)
    _, Yr = oracle.forward(off, oracle_ads(ads), bits_of(Xf), W)
    got = gh.bf16_to_f64(Y)
    np.testing.assert_array_equal(got, Yr)
    np.testing.assert_array_equal(got[:, 0].astype(np.int32) - 1, oracle.row_segment_map(off))
    batch = sb.Batch(d_in, d_out, off, [sb.Adapter() for _ in range(S)])
    np.testing.assert_array_equal(sb.symb_debug_row_segment_map(batch), oracle.row_segment_map(off))


def test_stateless_and_deterministic():
    p = make_problem(10, 320, 264, [130, 77, 300], [L, I, L], [8, 16])
    a = [gh.bf16_bits(t) for t in gh.forward(p["off"], p["ads"], p["X"], p["W"], p["bias"])]
    gh.backward_input(p["off"], p["ads"], p["dY"], p["W"])          # unrelated call in between
    q = make_problem(11, 64, 72, [5], [L], [4])
    gh.forward(q["off"], q["ads"], q["X"], q["W"], q["bias"])
    b = [gh.bf16_bits(t) for t in gh.forward(p["off"], p["ads"], p["X"], p["W"], p["bias"])]
    np.testing.assert_array_equal(a[0], b[0])
    np.testing.assert_array_equal(a[1], b[1])
    g1 = gh.adapter_grad(p["off"], p["ads"], p["X"], p["dY"], torch.from_numpy(a[1].view(np.int16)).view(torch.bfloat16).cuda())
    g2 = gh.adapter_grad(p["off"], p["ads"], p["X"], p["dY"], torch.from_numpy(a[1].view(np.int16)).view(torch.bfloat16).cuda())
    for d1, d2 in zip(g1.descs, g2.descs):
        if d1.dA is not None:
            assert torch.equal(d1.dA, d2.dA)
        if d1.dB is not None:
            assert torch.equal(d1.dB, d2.dB)


@pytest.mark.parametrize("dims", [(136, 6208), (6208, 136), (2056, 33800), (33800, 2056), (4096, 520)])
def test_large_tile_kernel_is_deterministic(dims):
    """The 256x256 kernel (forward for the first shape, input gradient for the second): two runs of the
    same call, with another call in between, give the same bits.  The last three shapes split tiles
    over K ranges (the last round of 266 tiles; every tile of a small launch): whichever workgroup
    arrives last adds the partial tiles up in the same order."""
    d_in, d_out = dims
    p = make_problem(13, d_in, d_out, [700, 5, 795] if min(dims) < 1000 or max(dims) < 10000 else [120, 1, 99, 80], [L, I, L], [16, 40])
    y1 = gh.bf16_bits(gh.forward(p["off"], p["ads"], p["X"], p["W"], p["bias"], want_base=False)[0])
    x1 = gh.bf16_bits(gh.backward_input(p["off"], p["ads"], p["dY"], p["W"]))
    y2 = gh.bf16_bits(gh.forward(p["off"], p["ads"], p["X"], p["W"], p["bias"], want_base=False)[0])
    x2 = gh.bf16_bits(gh.backward_input(p["off"], p["ads"], p["dY"], p["W"]))
    np.testing.assert_array_equal(y1, y2)
    np.testing.assert_array_equal(x1, x2)


def test_calls_that_find_their_descriptors_in_place():
    """A call whose descriptors are the bytes of an earlier call on the same stream reads the copy already
    on the device.  Three rounds of forward, input gradient and adapter gradients on the same device
    buffers (a launch that splits every tile over K ranges: its arrival counters live with the
    descriptors), the adapter matrices rewritten in place before the last round: every round gives
    the bits a fresh handle gives, and the last one agrees with the oracle."""
    p = make_problem(21, 4096, 520, [700, 5, 795], [L, I, L], [16, 40])
    off, d_in, d_out, T = p["off"], p["d_in"], p["d_out"], p["T"]
    dev = gh.upload_adapters(p["ads"], d_in, d_out, grads=True)
    batch = sb.Batch(d_in, d_out, off, dev.descs)
    Xd, Wd, bd, gd = gh.to_dev(p["X"]), gh.to_dev(p["W"]), gh.to_dev(p["bias"]), gh.to_dev(p["dY"])
    ws = torch.empty(max(sb.symb_workspace_bytes(batch, op) for op in (sb.SYMB_OP_FWD, sb.SYMB_OP_BWD_INPUT, sb.SYMB_OP_ADAPTER_GRAD)),
                     device="cuda", dtype=torch.uint8)
    Y = torch.empty((T, d_out), device="cuda", dtype=torch.bfloat16)
    dX = torch.empty((T, d_in), device="cuda", dtype=torch.bfloat16)
    Yb = gh.forward(off, p["ads"], p["X"], p["W"], p["bias"], want_base=True)[1]

    def run(h):
        Y.fill_(float("nan")); dX.fill_(float("nan"))
        for d in dev.descs:
            for g in (d.dA, d.dB):
                if g is not None:
                    g.fill_(float("nan"))
        sb.symb_base_linear_fwd(h, batch, Xd, Wd, bd, Y, None, ws, gh.stream_ptr())
        sb.symb_base_linear_bwd_input(h, batch, gd, Wd, dX, sb.SYMB_BWD_FULL, ws, gh.stream_ptr())
        sb.symb_adapter_grad(h, batch, Xd, gd, Yb, sb.SYMB_GRAD_OVERWRITE, ws, gh.stream_ptr())
        torch.cuda.synchronize()
        return [gh.bf16_bits(Y), gh.bf16_bits(dX)] + [g.cpu().numpy().copy() for d in dev.descs for g in (d.dA, d.dB) if g is not None]

    fresh = sb.symb_create(0)
    try:
        want = run(fresh)
        assert sb.symb_debug_descriptor_stats(fresh) == (3, 0)
        run(gh.handle())
        before = sb.symb_debug_descriptor_stats(gh.handle())
        for _ in range(2):
            for a, b in zip(run(gh.handle()), want):
                np.testing.assert_array_equal(a, b)
        after = sb.symb_debug_descriptor_stats(gh.handle())
        assert (after[0] - before[0], after[1] - before[1]) == (0, 6)
        q = make_problem(22, d_in, d_out, [700, 5, 795], [L, I, L], [16, 40])
        for d, a in zip(dev.descs, q["ads"]):
            if a.kind == L:
                d.A.copy_(gh.to_dev(a.A)); d.B.copy_(gh.to_dev(a.B))
        got = run(gh.handle())
        assert sb.symb_debug_descriptor_stats(gh.handle()) == (after[0], after[1] + 3)
    finally:
        sb.symb_destroy(fresh)
    assert not np.array_equal(got[0], want[0])
    for i in (0, 2):
        p["ads"][i].A, p["ads"][i].B = q["ads"][i].A, q["ads"][i].B
    _, Yr = oracle.forward(off, oracle_ads(p["ads"]), p["X"], p["W"], p["bias"])
    assert_close(gh.bf16_to_f64(Y), Yr, "descriptors in place: Y", out_bf16=True)


def test_backward_batch_is_independent_of_forward_batch():
    """Backward on a regrouped subset of the forward clients gives the same rows (bitwise)."""
    p = make_problem(12, 264, 320, [130, 1, 77, 300], [L, I, L, N], [8, 16])
    off = p["off"]
    dX = gh.bf16_bits(gh.backward_input(off, p["ads"], p["dY"], p["W"]))
    order = [2, 0]
    idx = np.concatenate([np.arange(off[i], off[i + 1]) for i in order])
    noff = np.zeros(len(order) + 1, dtype=np.int32)
    noff[1:] = np.cumsum([off[i + 1] - off[i] for i in order])
    sub = gh.bf16_bits(gh.backward_input(noff, [p["ads"][i] for i in order], np.ascontiguousarray(p["dY"][idx]), p["W"]))
    np.testing.assert_array_equal(sub, dX[idx])


@pytest.mark.parametrize("lens", [[90, 33], [1700, 33, 2100]])      # the second: segments whose gradients are summed in runs of 1024 tokens
def test_gradient_accumulate_adds(lens):
    p = make_problem(13, 136, 264, lens, [L, I, L][:len(lens)], [8, 1, 24][:len(lens)])
    _, Yb = gh.forward(p["off"], p["ads"], p["X"], p["W"], p["bias"])
    g = gh.adapter_grad(p["off"], p["ads"], p["X"], p["dY"], Yb)
    once = [(d.dA.clone() if d.dA is not None else None, d.dB.clone() if d.dB is not None else None) for d in g.descs]
    gh.adapter_grad(p["off"], p["ads"], p["X"], p["dY"], Yb, accumulate_into=g)
    for (a1, b1), d in zip(once, g.descs):
        if a1 is not None:
            assert torch.equal(d.dA, a1 + a1)
        if b1 is not None:
            assert torch.equal(d.dB, b1 + b1)


def test_inference_segments_get_no_gradient_work():
    p = make_problem(14, 136, 264, [50, 3, 40], [L, L, I], [8])
    p["ads"][1].want_grad = False
    _, Yb = gh.forward(p["off"], p["ads"], p["X"], p["W"], p["bias"])
    g = gh.adapter_grad(p["off"], p["ads"], p["X"], p["dY"], Yb)
    assert g.descs[1].dA is None and g.descs[1].dB is None
    dAr, dBr = oracle.lora_grad(p["off"], oracle_ads(p["ads"]), p["X"], p["dY"], 0)
    assert_close(g.descs[0].dA.cpu().numpy(), dAr, "dA[0]")
    assert_close(g.descs[0].dB.cpu().numpy(), dBr, "dB[0]")


def test_errors_enqueue_nothing_and_leave_handle_usable():
    p = make_problem(15, 64, 72, [5, 6], [L, I], [4])
    dev = gh.upload_adapters(p["ads"], 64, 72, grads=True)
    X, W, dYd = gh.to_dev(p["X"]), gh.to_dev(p["W"]), gh.to_dev(p["dY"])
    Y = torch.full((11, 72), 7.0, device="cuda", dtype=torch.bfloat16)
    h = gh.handle()
    good = sb.Batch(64, 72, p["off"], dev.descs)
    ws = gh.workspace(good, sb.SYMB_OP_FWD)

    def expect(status, fn):
        with pytest.raises(sb.SymbError) as e:
            fn()
        assert e.value.status == status, str(e.value)
        torch.cuda.synchronize()
        assert bool((Y == 7.0).all()), "a failing call must leave the output untouched"

    bad_off = sb.Batch(64, 72, [0, 6, 5], dev.descs)
    expect(sb.SYMB_ERR_BAD_SEGMENTS, lambda: sb.symb_base_linear_fwd(h, bad_off, X, W, None, Y, None, ws))
    expect(sb.SYMB_ERR_INVALID_ARG, lambda: sb.symb_base_linear_fwd(h, good, None, W, None, Y, None, ws))
    expect(sb.SYMB_ERR_WORKSPACE_TOO_SMALL, lambda: sb.symb_base_linear_fwd(h, good, X, W, None, Y, None, None))
    expect(sb.SYMB_ERR_INVALID_ARG, lambda: sb.symb_base_linear_bwd_input(h, good, dYd, W, Y, 5, None))
    expect(sb.SYMB_ERR_INVALID_ARG,            # IA3 segment wants dl but no Ybase given
           lambda: sb.symb_adapter_grad(h, good, X, dYd, None, sb.SYMB_GRAD_OVERWRITE, gh.workspace(good, sb.SYMB_OP_ADAPTER_GRAD)))
    ia3_in = sb.Batch(64, 72, [0, 11], [sb.Adapter(sb.SYMB_ADAPTER_IA3_IN, 0, 0.0, dev.descs[1].A, dA=dev.descs[1].dA)])
    expect(sb.SYMB_ERR_INVALID_ARG,            # IA3_IN segment wants dl but no dXbase given
           lambda: sb.symb_adapter_grad(h, ia3_in, X, dYd, None, sb.SYMB_GRAD_OVERWRITE, None))
    # the handle still works
    sb.symb_base_linear_fwd(h, good, X, W, None, Y, None, ws)
    torch.cuda.synchronize()
    _, Yr = oracle.forward(p["off"], oracle_ads(p["ads"]), p["X"], p["W"])
    assert_close(gh.bf16_to_f64(Y), Yr, "Y after failed calls", out_bf16=True)


def test_adapter_grad_can_reuse_dh_from_the_input_gradient_call():
    """SYMB_GRAD_REUSE_DH / SYMB_GRAD_REUSE_HS: same batch, same X and dY, same workspace -> the same gradients."""
    p = make_problem(16, 264, 392, [150, 1, 70, 33], [L, I, L, L], [8, 24, 5])
    d_in, d_out, off = p["d_in"], p["d_out"], p["off"]
    Xd, dYd, Wd = gh.to_dev(p["X"]), gh.to_dev(p["dY"]), gh.to_dev(p["W"])
    Y0r, _ = oracle.forward(off, oracle_ads(p["ads"]), p["X"], p["W"], p["bias"])
    Yb = gh.to_dev(synth.f32_to_bf16_bits(Y0r.astype(np.float32)))
    h = gh.handle()
    plain = gh.upload_adapters(p["ads"], d_in, d_out, grads=True)
    b1 = sb.Batch(d_in, d_out, off, plain.descs)
    sb.symb_adapter_grad(h, b1, Xd, dYd, Yb, sb.SYMB_GRAD_OVERWRITE, gh.workspace(b1, sb.SYMB_OP_ADAPTER_GRAD))
    reuse = gh.upload_adapters(p["ads"], d_in, d_out, grads=True)
    b2 = sb.Batch(d_in, d_out, off, reuse.descs)
    n = max(sb.symb_workspace_bytes(b2, op) for op in (sb.SYMB_OP_FWD, sb.SYMB_OP_BWD_INPUT, sb.SYMB_OP_ADAPTER_GRAD))
    ws = torch.empty(n, device="cuda", dtype=torch.uint8)
    dX = torch.empty((p["T"], d_in), device="cuda", dtype=torch.bfloat16)
    sb.symb_base_linear_bwd_input(h, b2, dYd, Wd, dX, sb.SYMB_BWD_FULL, ws)
    sb.symb_adapter_grad(h, b2, Xd, dYd, Yb, sb.SYMB_GRAD_OVERWRITE | sb.SYMB_GRAD_REUSE_DH, ws)
    torch.cuda.synchronize()

    def same(x, y):
        # dB does not depend on where dH came from: same bits.  dA does: a stand-alone gradient call of ranks up
        # to 16 forms dH in its one pass over dY (column blocks summed in groups), the input gradient call forms
        # it with the shrink kernel; the two dH agree to rounding, so dA is held to the oracle's bar instead.
        for i, (d1, d2) in enumerate(zip(x.descs, y.descs)):
            if d1.dB is not None:
                assert torch.equal(d1.dB, d2.dB)
            if d1.dA is not None and p["ads"][i].kind == L:
                dAr, _ = oracle.lora_grad(off, oracle_ads(p["ads"]), p["X"], p["dY"], i, want_dB=False)
                assert_close(d1.dA.cpu().numpy(), dAr, f"dA[{i}] stand-alone")
                assert_close(d2.dA.cpu().numpy(), dAr, f"dA[{i}] reusing dH")
            elif d1.dA is not None:
                assert torch.equal(d1.dA, d2.dA)
    same(plain, reuse)
    # forward, input gradient, then gradients taking both Hs and dH from the workspace
    both = gh.upload_adapters(p["ads"], d_in, d_out, grads=True)
    b3 = sb.Batch(d_in, d_out, off, both.descs)
    ws.fill_(0x7f)
    Y = torch.empty((p["T"], d_out), device="cuda", dtype=torch.bfloat16)
    sb.symb_base_linear_fwd(h, b3, Xd, Wd, None, Y, None, ws)
    sb.symb_base_linear_bwd_input(h, b3, dYd, Wd, dX, sb.SYMB_BWD_FULL, ws)
    sb.symb_adapter_grad(h, b3, Xd, dYd, Yb, sb.SYMB_GRAD_OVERWRITE | sb.SYMB_GRAD_REUSE_DH | sb.SYMB_GRAD_REUSE_HS, ws)
    torch.cuda.synchronize()
    same(plain, both)


@pytest.mark.parametrize("shape", [dict(d_in=264, d_out=392, lens=[150, 1, 70, 0, 33]),          # 128x128 tiles
                                   dict(d_in=200, d_out=6208, lens=[700, 5, 795, 2, 40])])       # 256x256 tiles
def test_privacy_flow_noise_add_and_denoised_forward(shape):
    """Sec. 3.8: x + n bit-exact against the oracle's prepass; the noise effect (a bias-free forward of the
    noise rows) and the denoised forward (a stored noise effect taken off in the epilogue) each against the
    oracle on the same inputs, usual bar; and the whole flow gives the plain layer output up to the
    roundings it adds."""
    d_in, d_out, lens = shape["d_in"], shape["d_out"], shape["lens"]
    p = make_problem(31, d_in, d_out, lens, [L, I, N, L, I], [8, 24, 5])
    off, T = p["off"], p["T"]
    rng = np.random.default_rng(77)
    nb = lambda shp: synth.f32_to_bf16_bits(rng.standard_normal(shp).astype(np.float32))
    noise = [nb((lens[0], d_in)), nb((1, d_in)), None, None, nb((1, d_in))]       # per token, broadcast, none
    Xn_ref = oracle.noise_add(off, p["X"], noise)
    h = gh.handle()
    dev = gh.upload_adapters(p["ads"], d_in, d_out, grads=False)
    b = sb.Batch(d_in, d_out, off, dev.descs)
    Xd, Wd, bd = gh.to_dev(p["X"]), gh.to_dev(p["W"]), gh.to_dev(p["bias"])
    nd = [gh.to_dev(n) for n in noise]
    Xn = torch.empty_like(Xd)
    sb.symb_noise_add(h, b, Xd, nd, Xn)
    torch.cuda.synchronize()
    assert np.array_equal(gh.bf16_bits(Xn), Xn_ref), "x + n must match bit for bit"
    # (1) noise effect: the noise rows as a batch of their own, the clients' adapters, no bias
    keep = [i for i, n in enumerate(noise) if n is not None]
    noff = np.zeros(len(keep) + 1, dtype=np.int32)
    noff[1:] = np.cumsum([noise[i].shape[0] for i in keep])
    nbatch = sb.Batch(d_in, d_out, noff, [dev.descs[i] for i in keep])
    Nd = torch.cat([nd[i] for i in keep], dim=0).contiguous()
    Neff = torch.empty((int(noff[-1]), d_out), device="cuda", dtype=torch.bfloat16)
    sb.symb_base_linear_fwd(h, nbatch, Nd, Wd, None, Neff, None, gh.workspace(nbatch, sb.SYMB_OP_FWD))
    torch.cuda.synchronize()
    oads = oracle_ads(p["ads"])
    _, Neff_ref = oracle.forward(noff, [oads[i] for i in keep], np.concatenate([noise[i] for i in keep], axis=0), p["W"], None)
    assert_close(gh.bf16_to_f64(Neff), Neff_ref, "noise effect", out_bf16=True)
    # (2) + (3): the client keeps the noise effect as a 16-bit tensor and hands it in with later calls; both
    # sides get the same one, the oracle's rounded to bf16 here (never the GPU's own output)
    saved_bits = synth.f32_to_bf16_bits(Neff_ref.astype(np.float32))
    saved = [None] * len(noise)
    for q, i in enumerate(keep):
        saved[i] = saved_bits[int(noff[q]):int(noff[q + 1])]
    Y = torch.empty((T, d_out), device="cuda", dtype=torch.bfloat16)
    sb.symb_base_linear_fwd_denoise(h, b, Xn, Wd, bd, [gh.to_dev(n) for n in saved], Y, gh.workspace(b, sb.SYMB_OP_FWD))
    torch.cuda.synchronize()
    Yr = oracle.forward_denoise(off, oads, Xn_ref, p["W"], p["bias"], saved)
    assert_close(gh.bf16_to_f64(Y), Yr, "denoised Y", out_bf16=True)
    # the whole flow on the GPU alone (its own noise effect): the plain layer output up to the roundings the
    # flow adds (x + n and the stored noise effect are 16-bit tensors: not the 4e-3 bar)
    neff = [None] * len(noise)
    for q, i in enumerate(keep):
        neff[i] = Neff[int(noff[q]):int(noff[q + 1])]
    sb.symb_base_linear_fwd_denoise(h, b, Xn, Wd, bd, neff, Y, gh.workspace(b, sb.SYMB_OP_FWD))
    torch.cuda.synchronize()
    _, Yplain = oracle.forward(off, oads, p["X"], p["W"], p["bias"])
    from helpers import rel_fro
    assert rel_fro(gh.bf16_to_f64(Y), Yplain) < 1e-2
    assert rel_fro(gh.bf16_to_f64(Y), oracle.forward_private(off, oads, Xn_ref, p["W"], p["bias"], noise)) < 1e-2
    # a noise tensor with the wrong number of rows is refused before anything is launched
    if lens[0] >= 3:                     # (2 rows are neither one broadcast row nor one per token then)
        bad = list(nd)
        bad[0] = nd[0][:2]
        with pytest.raises(sb.SymbError) as e:
            sb.symb_noise_add(h, b, Xd, bad, Xn)
        assert e.value.status == sb.SYMB_ERR_INVALID_ARG


@pytest.mark.parametrize("case", [
    dict(seed=41, d_in=320, d_out=264, lens=[130, 1, 0, 77, 1, 300, 64], kinds=[L, I, L, N, L, L, I], ranks=[8, 16, 5, 24, 33]),
    dict(seed=42, d_in=136, d_out=6208, lens=[700, 5, 795], kinds=[L, I, L], ranks=[16, 8]),      # 256x256 tiles, forward
    dict(seed=43, d_in=6208, d_out=136, lens=[700, 5, 795], kinds=[L, I, L], ranks=[16, 5]),      # 256x256 tiles, backward
])
def test_input_major_weight_layout(case):
    """Conv1D-style storage W [d_in][d_out] (Sec. 3.7, 3.8: the base layers are nn.Linear or Conv1D):
    the same linear map, so the oracle is unchanged and only the GPU gets the transposed array."""
    c = dict(case)
    p = make_problem(c.pop("seed"), c.pop("d_in"), c.pop("d_out"), c.pop("lens"), c.pop("kinds"), c.pop("ranks"))
    oads, off = oracle_ads(p["ads"]), p["off"]
    Y, Yb = gh.forward(off, p["ads"], p["X"], p["W"], p["bias"], want_base=True, conv1d=True)
    Y0r, Yr = oracle.forward(off, oads, p["X"], p["W"], p["bias"])
    assert_close(gh.bf16_to_f64(Y), Yr, "conv1d Y", out_bf16=True)
    assert_close(gh.bf16_to_f64(Yb), Y0r, "conv1d Ybase", out_bf16=True)
    for base_only in (False, True):
        dX = gh.backward_input(off, p["ads"], p["dY"], p["W"], base_only=base_only, conv1d=True)
        check_dx(gh.bf16_to_f64(dX), off, oads, p["dY"], p["W"], f"conv1d dX base_only={base_only}", base_only=base_only)


@pytest.mark.parametrize("case", [
    dict(seed=51, d_in=320, d_out=264, lens=[130, 1, 0, 77, 1, 300, 64], kinds=[L, 3, L, N, 3, I, 3], ranks=[8, 16, 5]),
    dict(seed=52, d_in=6208, d_out=136, lens=[700, 5, 795], kinds=[3, L, 3], ranks=[16]),        # 256x256 tiles in the input gradient
    dict(seed=53, d_in=136, d_out=6208, lens=[700, 5, 795], kinds=[3, I, L], ranks=[8], conv1d=True),
])
def test_ia3_input_scaling(case):
    """IA3 on the layer's input (kind 3): Y = (X * l) W^T + b; dX = l * (dY W); dl[k] = sum_t X[t][k] (dY W)[t][k],
    the last from the input gradient the executor returned (a bf16 tensor: both sides get the oracle's)."""
    c = dict(case)
    conv1d = c.pop("conv1d", False)
    p = make_problem(c.pop("seed"), c.pop("d_in"), c.pop("d_out"), c.pop("lens"), c.pop("kinds"), c.pop("ranks"))
    oads, off, d_in, d_out, T = oracle_ads(p["ads"]), p["off"], p["d_in"], p["d_out"], p["T"]
    Y, _ = gh.forward(off, p["ads"], p["X"], p["W"], p["bias"], want_base=False, conv1d=conv1d)
    check_y(gh.bf16_to_f64(Y), off, oads, p["X"], p["W"], p["bias"], "IA3_IN Y")
    # input gradient with the pre-scale output
    dev = gh.upload_adapters(p["ads"], d_in, d_out, grads=True)
    b = sb.Batch(d_in, d_out, off, dev.descs, sb.SYMB_WEIGHT_CONV1D if conv1d else sb.SYMB_WEIGHT_LINEAR)
    h = gh.handle()
    gd, Wd, Xd = gh.to_dev(p["dY"]), gh.weight_to_dev(p["W"], conv1d), gh.to_dev(p["X"])
    dX = torch.full((T, d_in), float("nan"), device="cuda", dtype=torch.bfloat16)
    G = torch.full((T, d_in), float("nan"), device="cuda", dtype=torch.bfloat16)
    sb.symb_base_linear_bwd_input_ex(h, b, gd, Wd, dX, G, sb.SYMB_BWD_FULL, gh.workspace(b, sb.SYMB_OP_BWD_INPUT))
    torch.cuda.synchronize()
    check_dx(gh.bf16_to_f64(dX), off, oads, p["dY"], p["W"], "IA3_IN dX")
    Gr = oracle.backward_input(off, oads, p["dY"], p["W"], base_only=True)
    ia3_rows = np.concatenate([np.arange(off[i], off[i + 1]) for i, a in enumerate(p["ads"]) if a.kind == I] or [np.zeros(0, int)]).astype(int)
    keep = np.setdiff1d(np.arange(T), ia3_rows)          # rows of output-scaling segments hold the scaled product there
    assert_close(gh.bf16_to_f64(G)[keep], Gr[keep], "IA3_IN dXbase", out_bf16=True)
    dXb = gh.backward_input(off, p["ads"], p["dY"], p["W"], base_only=True, conv1d=conv1d)
    assert_close(gh.bf16_to_f64(dXb), Gr, "IA3_IN dX base only", out_bf16=True)
    # gradients: both sides take the oracle's G and Y0 rounded to bf16
    Y0r, _ = oracle.forward(off, oads, p["X"], p["W"], p["bias"])
    G_saved, Y0_saved = synth.f32_to_bf16_bits(Gr.astype(np.float32)), synth.f32_to_bf16_bits(Y0r.astype(np.float32))
    sb.symb_adapter_grad_ex(h, b, Xd, gd, gh.to_dev(Y0_saved), gh.to_dev(G_saved), sb.SYMB_GRAD_OVERWRITE,
                            gh.workspace(b, sb.SYMB_OP_ADAPTER_GRAD))
    torch.cuda.synchronize()
    for i, a in enumerate(p["ads"]):
        if a.kind != 3:
            continue
        dl = dev.descs[i].dA.cpu().numpy()
        if off[i + 1] == off[i]:
            assert not dl.any()
        else:
            assert_close(dl, oracle.ia3_grad(off, oads, p["X"], p["dY"], p["W"], p["bias"], i, G_saved=G_saved), f"IA3_IN dl[{i}]")


@pytest.mark.parametrize("case", [
    dict(seed=61, d_in=320, d_out=264, lens=[130, 1, 0, 77, 1, 300, 64], kinds=[L, I, L, N, L, L, I], ranks=[8, 16, 5, 24, 33]),
    dict(seed=62, d_in=136, d_out=6208, lens=[700, 5, 795], kinds=[L, I, L], ranks=[16, 8]),
    dict(seed=63, d_in=6208, d_out=136, lens=[700, 5, 795], kinds=[L, N, L], ranks=[16, 5]),
    # 266 tiles of 256x256 with the last round split over K ranges, rows from and to per-client buffers
    dict(seed=64, d_in=2056, d_out=33800, lens=[120, 1, 99, 80], kinds=[L, I, L, N], ranks=[16, 8, 40]),
    dict(seed=65, d_in=33800, d_out=2056, lens=[120, 1, 99, 80], kinds=[L, N, L, L], ranks=[16, 8, 40, 24]),
    # IA3 on the input (kind 3) among the clients: the forward multiplies a flat scaled copy of the rows
    dict(seed=66, d_in=320, d_out=264, lens=[130, 1, 0, 77, 1, 300, 64], kinds=[L, 3, L, N, 3, I, 3], ranks=[8, 16, 5]),
    dict(seed=67, d_in=136, d_out=6208, lens=[700, 5, 795], kinds=[3, L, 3], ranks=[16]),
    dict(seed=68, d_in=6208, d_out=136, lens=[700, 5, 795], kinds=[L, 3, 3], ranks=[12]),
])
def test_per_segment_buffers(case):
    """Rows read from and written to one buffer per client, carved in shuffled order and with gaps
    from one arena (Sec. 3.5: pre-allocated client buffers), against the flat oracle result."""
    c = dict(case)
    p = make_problem(c.pop("seed"), c.pop("d_in"), c.pop("d_out"), c.pop("lens"), c.pop("kinds"), c.pop("ranks"))
    off, d_in, d_out, T, S = p["off"], p["d_in"], p["d_out"], p["T"], len(p["ads"])
    oads = oracle_ads(p["ads"])
    h = gh.handle()
    dev = gh.upload_adapters(p["ads"], d_in, d_out, grads=False)
    b = sb.Batch(d_in, d_out, off, dev.descs)
    rng = np.random.default_rng(5)

    def carve(width, src_bits=None):
        """One arena; segment i gets its own region (random order, 16-byte aligned gaps of junk between)."""
        order = rng.permutation(S)
        sizes = {int(i): int(off[i + 1] - off[i]) * width for i in order}
        gaps = {int(i): 8 * int(rng.integers(1, 40)) for i in order}
        arena = torch.full((sum(sizes.values()) + sum(gaps.values()) + 8,), float("nan"), device="cuda", dtype=torch.bfloat16)
        views, cur = [None] * S, 0
        for i in order:
            i = int(i)
            cur += gaps[i]
            n = int(off[i + 1] - off[i])
            views[i] = arena[cur:cur + sizes[i]].view(n, width) if n else None
            if n and src_bits is not None:
                views[i].copy_(gh.to_dev(np.ascontiguousarray(src_bits[off[i]:off[i + 1]])))
            cur += sizes[i]
        return arena, views

    def gather(views, width):
        out = np.zeros((T, width))
        for i, v in enumerate(views):
            if v is not None:
                out[off[i]:off[i + 1]] = gh.bf16_to_f64(v)
        return out

    Wd, bd = gh.to_dev(p["W"]), gh.to_dev(p["bias"])
    _, Xv = carve(d_in, p["X"])
    _, Yv = carve(d_out)
    sb.symb_base_linear_fwd_seg(h, b, Xv, Wd, bd, Yv, gh.workspace(b, sb.SYMB_OP_FWD))
    torch.cuda.synchronize()
    check_y(gather(Yv, d_out), off, oads, p["X"], p["W"], p["bias"], "per-segment Y")
    for base_only in (False, True):
        _, Gv = carve(d_out, p["dY"])
        _, DXv = carve(d_in)
        sb.symb_base_linear_bwd_input_seg(h, b, Gv, Wd, DXv, sb.SYMB_BWD_BASE_ONLY if base_only else sb.SYMB_BWD_FULL,
                                          gh.workspace(b, sb.SYMB_OP_BWD_INPUT))
        torch.cuda.synchronize()
        check_dx(gather(DXv, d_in), off, oads, p["dY"], p["W"], f"per-segment dX base_only={base_only}", base_only=base_only)
    # adapter gradients from the same kind of buffers (the IA3 gradient takes the oracle's Y0 rounded to bf16)
    grads = gh.upload_adapters(p["ads"], d_in, d_out, grads=True)
    bg = sb.Batch(d_in, d_out, off, grads.descs)
    Y0r, _ = oracle.forward(off, oads, p["X"], p["W"], p["bias"])
    Y0_saved = synth.f32_to_bf16_bits(Y0r.astype(np.float32))
    _, Gv = carve(d_out, p["dY"])
    _, Y0v = carve(d_out, Y0_saved)
    # a client with IA3 on the input kept its rows of the input gradient before the scale instead (oracle's, in bf16)
    G_saved = synth.f32_to_bf16_bits(oracle.backward_input(off, oads, p["dY"], p["W"], base_only=True).astype(np.float32))
    _, G0v = carve(d_in, G_saved)
    saved = [G0v[i] if a.kind == 3 else Y0v[i] for i, a in enumerate(p["ads"])]
    sb.symb_adapter_grad_seg(h, bg, Xv, Gv, saved, sb.SYMB_GRAD_OVERWRITE, gh.workspace(bg, sb.SYMB_OP_ADAPTER_GRAD))
    torch.cuda.synchronize()
    for i, a in enumerate(p["ads"]):
        if off[i + 1] == off[i]:
            continue
        if a.kind == L:
            dAr, dBr = oracle.lora_grad(off, oads, p["X"], p["dY"], i)
            assert_close(grads.descs[i].dA.cpu().numpy(), dAr, f"per-segment dA[{i}]")
            assert_close(grads.descs[i].dB.cpu().numpy(), dBr, f"per-segment dB[{i}]")
        elif a.kind == I:
            dlr = oracle.ia3_grad(off, oads, p["X"], p["dY"], p["W"], p["bias"], i, Y0_saved=Y0_saved)
            assert_close(grads.descs[i].dA.cpu().numpy(), dlr, f"per-segment dl[{i}]")
        elif a.kind == 3:
            dlr = oracle.ia3_grad(off, oads, p["X"], p["dY"], p["W"], p["bias"], i, G_saved=G_saved)
            assert_close(grads.descs[i].dA.cpu().numpy(), dlr, f"per-segment dl (input scaling) [{i}]")
    if any(a.kind == 3 for a in p["ads"]):
        return                                      # (no window rule for the forward's inputs then)
    # input buffers more than 4 GiB apart are refused before any launch.  Every address handed over is real
    # memory: one segment's rows are copied to the far end of a 4.6 GB allocation, the others to its start.
    nonempty = [i for i in range(S) if Xv[i] is not None]
    if len(nonempty) >= 2:
        span = torch.empty(((1 << 32) + (64 << 20) + 2 * T * d_in) // 2, device="cuda", dtype=torch.bfloat16)
        far, cur = list(Xv), 0
        for i in nonempty[1:]:
            far[i] = span[cur:cur + Xv[i].numel()].view_as(Xv[i])
            far[i].copy_(Xv[i])
            cur += Xv[i].numel() + 8
        first = nonempty[0]
        far[first] = span[span.numel() - Xv[first].numel():].view_as(Xv[first])
        far[first].copy_(Xv[first])
        assert far[first].data_ptr() - far[nonempty[1]].data_ptr() > (1 << 32)
        with pytest.raises(sb.SymbError) as e:
            sb.symb_base_linear_fwd_seg(h, b, far, Wd, bd, Yv, gh.workspace(b, sb.SYMB_OP_FWD))
        assert e.value.status == sb.SYMB_ERR_UNSUPPORTED
        del span, far


@pytest.mark.parametrize("d_in", [40, 64, 72, 128, 192, 200, 320])
def test_large_tile_kernel_with_one_to_five_k_stages(d_in):
    """The 256x256 kernel's main loop has a prologue, a steady loop and two closing stages: shapes with
    0 (remainder only), 1, 2, 3 and 5 full 64-k stages, with and without a K remainder, wide enough to select
    that kernel."""
    p = make_problem(70 + d_in, d_in, 6208, [700, 5, 795], [L, N, I], [16])
    oads, off = oracle_ads(p["ads"]), p["off"]
    Y, Yb = gh.forward(off, p["ads"], p["X"], p["W"], p["bias"], want_base=True)
    Y0r, Yr = oracle.forward(off, oads, p["X"], p["W"], p["bias"])
    assert_close(gh.bf16_to_f64(Y), Yr, f"Y d_in={d_in}", out_bf16=True)
    assert_close(gh.bf16_to_f64(Yb), Y0r, f"Ybase d_in={d_in}", out_bf16=True)
    # the same K extents in the input gradient: d_out takes the role of K there
    q = make_problem(170 + d_in, 6208, d_in, [700, 5, 795], [L, N, I], [16])
    dX = gh.backward_input(q["off"], q["ads"], q["dY"], q["W"])
    check_dx(gh.bf16_to_f64(dX), q["off"], oracle_ads(q["ads"]), q["dY"], q["W"], f"dX d_out={d_in}")


@pytest.mark.parametrize("lens", [[1], [16], [9, 0, 8], [1, 1, 20, 1, 1, 24], [30, 1, 40, 29], [1] * 48, [50, 78]])
def test_forward_of_a_handful_of_rows(lens):
    """Batches of at most 16 rows (decode steps) take a kernel of their own that streams W once, larger
    ones the 128x128 tiles with every tile split over K ranges: 1, 16, 17, 48, 100 and 128 rows; K with
    a remainder, d_out not a multiple of 32; every adapter kind, ranks 1..128, bias."""
    kinds = [L, I, N, L, L, I]
    p = make_problem(90 + len(lens), 200, 392, lens, kinds, [1, 128, 24, 8, 100])
    assert p["T"] <= 128
    Y, _ = gh.forward(p["off"], p["ads"], p["X"], p["W"], p["bias"], want_base=False)
    _, Yr = oracle.forward(p["off"], oracle_ads(p["ads"]), p["X"], p["W"], p["bias"])
    assert_close(gh.bf16_to_f64(Y), Yr, f"small-batch Y lens={lens}", out_bf16=True)
    q = make_problem(190 + len(lens), 4096, 4096, lens, [L], [16], bias=False)          # a decode batch on a real layer width
    Y, _ = gh.forward(q["off"], q["ads"], q["X"], q["W"], None, want_base=False)
    _, Yr = oracle.forward(q["off"], oracle_ads(q["ads"]), q["X"], q["W"], None)
    assert_close(gh.bf16_to_f64(Y), Yr, f"decode batch Y lens={lens}", out_bf16=True)


def test_k_split_rests_on_a_measured_xcd_rule():
    """The K-split leaves out a device-scope fence because all workgroups of one output tile run on one
    XCD (ids that agree mod 8).  The library measures that rule when a handle is created and uses the
    split only if it holds: here the measurement is read back, and launches with and without the split
    (a last round of 256x256 tiles; every 128x128 tile of a small launch) both meet the oracle."""
    h = gh.handle()
    holds, ids = sb.symb_debug_xcd_rule(h)
    print(f"XCD rule holds={holds}, XCD of workgroup ids 0..7: {ids}", flush=True)
    assert holds, f"workgroup id mod 8 does not name the XCD on this device: {ids}"
    assert len(set(ids)) in (1, 8)
    for case in (dict(seed=13, d_in=2056, d_out=33800, lens=[120, 1, 99, 80], kinds=[L, I, L, N], ranks=[16, 8, 40]),
                 dict(seed=21, d_in=4096, d_out=520, lens=[700, 5, 795], kinds=[L, I, L], ranks=[16, 40])):
        c = dict(case)
        p = make_problem(c.pop("seed"), c.pop("d_in"), c.pop("d_out"), c.pop("lens"), c.pop("kinds"), c.pop("ranks"))
        oads = oracle_ads(p["ads"])
        _, Yr = oracle.forward(p["off"], oads, p["X"], p["W"], p["bias"])
        dXr = oracle.backward_input(p["off"], oads, p["dY"], p["W"])
        dXc = oracle.backward_input(p["off"], oads, p["dY"], p["W"], client_bf16=True)   # (an IA3 segment is in the batch)
        got = {}
        try:
            for split in (1, 0):
                sb.symb_debug_set_option(h, sb.SYMB_OPT_K_SPLIT, split)
                Y, _ = gh.forward(p["off"], p["ads"], p["X"], p["W"], p["bias"], want_base=False)
                dX = gh.backward_input(p["off"], p["ads"], p["dY"], p["W"])
                assert_close(gh.bf16_to_f64(Y), Yr, f"Y split={split}", out_bf16=True)
                assert_close_client(gh.bf16_to_f64(dX), dXr, dXc, f"dX split={split}")
                got[split] = (gh.bf16_bits(Y), gh.bf16_bits(dX))
        finally:
            sb.symb_debug_set_option(h, sb.SYMB_OPT_K_SPLIT, 1)
        # the two routes sum K in different orders: equal up to the last rounding, and not the same launch
        assert not (np.array_equal(got[0][0], got[1][0]) and np.array_equal(got[0][1], got[1][1]))


@pytest.mark.parametrize("case", [
    dict(seed=81, d_in=320, d_out=264, lens=[130, 1, 0, 77, 1, 300, 64], kinds=[L, I, L, N, L, L, I], ranks=[8, 16, 5, 24, 33]),
    dict(seed=82, d_in=136, d_out=6208, lens=[700, 5, 795], kinds=[L, I, L], ranks=[16, 8]),       # 256x256 tiles, d_out > d_in
    dict(seed=83, d_in=6208, d_out=136, lens=[700, 5, 795], kinds=[L, N, L], ranks=[16, 5]),       # d_in > d_out
])
def test_one_buffer_per_client_for_input_and_output(case):
    """Sec. 3.5: each client owns ONE pre-allocated buffer of n_i x max(d_in, d_out) elements; a layer's input
    arrives in it and the output goes back into it, forward (X -> Y) and backward (dY -> dX), rows dense
    at their own widths.  Result against the flat oracle; a workspace sized for the plain call is refused."""
    c = dict(case)
    p = make_problem(c.pop("seed"), c.pop("d_in"), c.pop("d_out"), c.pop("lens"), c.pop("kinds"), c.pop("ranks"))
    off, d_in, d_out, T, S = p["off"], p["d_in"], p["d_out"], p["T"], len(p["ads"])
    oads = oracle_ads(p["ads"])
    h = gh.handle()
    dev = gh.upload_adapters(p["ads"], d_in, d_out, grads=False)
    b = sb.Batch(d_in, d_out, off, dev.descs)
    Wd, bd = gh.to_dev(p["W"]), gh.to_dev(p["bias"])
    wmax = max(d_in, d_out)
    rng = np.random.default_rng(7)
    order = rng.permutation(S)
    gaps = {int(i): 8 * int(rng.integers(1, 40)) for i in order}
    arena = torch.full((T * wmax + sum(gaps.values()) + 8,), float("nan"), device="cuda", dtype=torch.bfloat16)
    bufs, cur = [None] * S, 0
    for i in order:
        i = int(i)
        cur += gaps[i]
        n = int(off[i + 1] - off[i])
        bufs[i] = arena[cur:cur + n * wmax] if n else None
        cur += n * wmax

    def view(i, width):
        n = int(off[i + 1] - off[i])
        return bufs[i][:n * width].view(n, width) if n else None

    def load(src_bits, width):
        for i in range(S):
            if bufs[i] is not None:
                bufs[i].fill_(float("nan"))
                view(i, width).copy_(gh.to_dev(np.ascontiguousarray(src_bits[off[i]:off[i + 1]])))

    def gather(width):
        out = np.zeros((T, width))
        for i in range(S):
            if bufs[i] is not None:
                out[off[i]:off[i + 1]] = gh.bf16_to_f64(view(i, width))
        return out

    # forward in place
    load(p["X"], d_in)
    xin = [view(i, d_in) for i in range(S)]
    yout = [view(i, d_out) for i in range(S)]
    # a workspace sized for the plain call has no room for the flat copy (unless its optional region of
    # K-split partial tiles, which the call then gives up, happens to be larger than that copy)
    n_plain, n_inplace = sb.symb_workspace_bytes(b, sb.SYMB_OP_FWD), sb.symb_workspace_bytes(b, sb.SYMB_OP_FWD_INPLACE)
    assert n_inplace >= n_plain + T * d_out * 2
    if n_plain < T * d_out * 2:
        with pytest.raises(sb.SymbError) as e:
            sb.symb_base_linear_fwd_seg(h, b, xin, Wd, bd, yout, gh.workspace(b, sb.SYMB_OP_FWD))
        assert e.value.status == sb.SYMB_ERR_WORKSPACE_TOO_SMALL
        torch.cuda.synchronize()
        k = next(i for i in range(S) if off[i + 1] > off[i])
        assert np.array_equal(gh.bf16_bits(view(k, d_in)), p["X"][off[k]:off[k + 1]]), "a refused call must leave the buffers alone"
    sb.symb_base_linear_fwd_seg(h, b, xin, Wd, bd, yout, gh.workspace(b, sb.SYMB_OP_FWD_INPLACE))
    torch.cuda.synchronize()
    _, Yr = oracle.forward(off, oads, p["X"], p["W"], p["bias"])
    assert_close(gather(d_out), Yr, "in-place Y", out_bf16=True)
    # input gradient in place
    load(p["dY"], d_out)
    gin = [view(i, d_out) for i in range(S)]
    xout = [view(i, d_in) for i in range(S)]
    sb.symb_base_linear_bwd_input_seg(h, b, gin, Wd, xout, sb.SYMB_BWD_FULL, gh.workspace(b, sb.SYMB_OP_BWD_INPUT_INPLACE))
    torch.cuda.synchronize()
    check_dx(gather(d_in), off, oads, p["dY"], p["W"], "in-place dX")


@pytest.mark.parametrize("lens", [[1], [16], [9, 0, 7], [1, 1, 5, 1, 1, 4], [3, 1, 2, 1, 1, 2, 1, 1]])
@pytest.mark.parametrize("dims", [(200, 392), (392, 200), (4096, 4096)])
def test_a_handful_of_rows_in_every_call_form(lens, dims):
    """Calls of at most 16 rows take the weight-streaming kernels in every form: forward with the
    pre-adapter output, input-major weight, IA3 on the input, the privacy flow's epilogue, per-client
    buffers (also one buffer for input and output); input gradient, full and base-only, with the
    pre-adapter gradient, through either weight layout and from per-client buffers.  Every adapter kind,
    ranks 1..128, K with a remainder, widths that are not multiples of the column blocks."""
    d_in, d_out = dims
    big = d_in * d_out > 1 << 20
    if big and len(lens) not in (1, 6):
        pytest.skip("the real layer width runs two of the row mixes")
    kinds = [L, I, N, L, 3, I, L, 3]
    p = make_problem(400 + len(lens) + d_in, d_in, d_out, lens, kinds, [1, 128, 24, 8, 100] if not big else [16, 8, 64])
    off, T, S = p["off"], p["T"], len(p["ads"])
    assert 0 < T <= 16
    oads = oracle_ads(p["ads"])
    h = gh.handle()
    Y0r, Yr = oracle.forward(off, oads, p["X"], p["W"], p["bias"])
    _, Yc = oracle.forward(off, oads, p["X"], p["W"], p["bias"], client_bf16=True)   # IA3 on the input: x * l as the client's bf16 tensor
    kind_of_row = np.array([p["ads"][int(np.searchsorted(off, t, side="right") - 1)].kind for t in range(T)])
    plain_in = np.flatnonzero(kind_of_row != 3)       # rows of input-scaling segments hold the product of the scaled input in Ybase
    for conv1d in (False, True):
        Y, Yb = gh.forward(off, p["ads"], p["X"], p["W"], p["bias"], want_base=True, conv1d=conv1d)
        assert_close_client(gh.bf16_to_f64(Y), Yr, Yc, f"small Y conv1d={conv1d}")
        assert_close(gh.bf16_to_f64(Yb)[plain_in], Y0r[plain_in], f"small Ybase conv1d={conv1d}", out_bf16=True)
        if (kind_of_row == 3).any():
            assert_close_client(gh.bf16_to_f64(Yb)[kind_of_row == 3], Yr[kind_of_row == 3], Yc[kind_of_row == 3], f"small Ybase of IA3_IN rows conv1d={conv1d}")
        for base_only in (False, True):
            dX = gh.backward_input(off, p["ads"], p["dY"], p["W"], base_only=base_only, conv1d=conv1d)
            check_dx(gh.bf16_to_f64(dX), off, oads, p["dY"], p["W"], f"small dX conv1d={conv1d} base_only={base_only}", base_only=base_only)
    # the pre-adapter input gradient next to the full one
    dev = gh.upload_adapters(p["ads"], d_in, d_out, grads=False)
    b = sb.Batch(d_in, d_out, off, dev.descs)
    gd, Wd, bd, Xd = gh.to_dev(p["dY"]), gh.to_dev(p["W"]), gh.to_dev(p["bias"]), gh.to_dev(p["X"])
    dX = torch.full((T, d_in), float("nan"), device="cuda", dtype=torch.bfloat16)
    G = torch.full((T, d_in), float("nan"), device="cuda", dtype=torch.bfloat16)
    sb.symb_base_linear_bwd_input_ex(h, b, gd, Wd, dX, G, sb.SYMB_BWD_FULL, gh.workspace(b, sb.SYMB_OP_BWD_INPUT))
    torch.cuda.synchronize()
    check_dx(gh.bf16_to_f64(dX), off, oads, p["dY"], p["W"], "small dX (with dXbase)")
    Gr = oracle.backward_input(off, oads, p["dY"], p["W"], base_only=True)
    keep = np.flatnonzero(kind_of_row != I)
    if len(keep):
        assert_close(gh.bf16_to_f64(G)[keep], Gr[keep], "small dXbase", out_bf16=True)
    # the denoised forward: a stored noise effect per segment (broadcast and per token) taken off in the epilogue
    rng = np.random.default_rng(9)
    neff = [None if i % 3 == 2 or off[i + 1] == off[i] else
            synth.f32_to_bf16_bits(rng.standard_normal((1 if i % 2 else int(off[i + 1] - off[i]), d_out)).astype(np.float32))
            for i in range(S)]
    Yd = torch.full((T, d_out), float("nan"), device="cuda", dtype=torch.bfloat16)
    sb.symb_base_linear_fwd_denoise(h, b, Xd, Wd, bd, [gh.to_dev(n) for n in neff], Yd, gh.workspace(b, sb.SYMB_OP_FWD))
    torch.cuda.synchronize()
    assert_close_client(gh.bf16_to_f64(Yd), oracle.forward_denoise(off, oads, p["X"], p["W"], p["bias"], neff),
                        oracle.forward_denoise(off, oads, p["X"], p["W"], p["bias"], neff, client_bf16=True), "small denoised Y")
    # per-client buffers (no IA3 on the input in that form): separate output buffers, then one buffer for both
    q = make_problem(500 + len(lens) + d_in, d_in, d_out, lens, [L, I, N, L, I, L, N, L], [1, 128, 24, 8, 100] if not big else [16, 8, 64])
    qads = oracle_ads(q["ads"])
    qdev = gh.upload_adapters(q["ads"], d_in, d_out, grads=False)
    qb = sb.Batch(d_in, d_out, off, qdev.descs)
    qW, qbias = gh.to_dev(q["W"]), gh.to_dev(q["bias"])
    wmax = max(d_in, d_out)
    bufs = [torch.full((max(int(off[i + 1] - off[i]), 1) * wmax + 8 * (i + 1),), float("nan"), device="cuda", dtype=torch.bfloat16) for i in range(S)]
    arena = torch.cat(bufs)                                   # one arena: the 4 GiB window rule
    views, cur = [], 0
    for i in range(S):
        n = int(off[i + 1] - off[i])
        views.append(arena[cur:cur + n * wmax] if n else None)
        cur += bufs[i].numel()

    def view(i, width):
        n = int(off[i + 1] - off[i])
        return views[i][:n * width].view(n, width) if n else None

    def gather(width):
        out = np.zeros((T, width))
        for i in range(S):
            if views[i] is not None:
                out[off[i]:off[i + 1]] = gh.bf16_to_f64(view(i, width))
        return out

    _, qYr = oracle.forward(off, qads, q["X"], q["W"], q["bias"])
    for i in range(S):
        if views[i] is not None:
            view(i, d_in).copy_(gh.to_dev(np.ascontiguousarray(q["X"][off[i]:off[i + 1]])))
    outs = [torch.full((int(off[i + 1] - off[i]), d_out), float("nan"), device="cuda", dtype=torch.bfloat16) if off[i + 1] > off[i] else None for i in range(S)]
    sb.symb_base_linear_fwd_seg(h, qb, [view(i, d_in) for i in range(S)], qW, qbias, outs, gh.workspace(qb, sb.SYMB_OP_FWD))
    torch.cuda.synchronize()
    got = np.zeros((T, d_out))
    for i in range(S):
        if outs[i] is not None:
            got[off[i]:off[i + 1]] = gh.bf16_to_f64(outs[i])
    assert_close(got, qYr, "small per-segment Y", out_bf16=True)
    sb.symb_base_linear_fwd_seg(h, qb, [view(i, d_in) for i in range(S)], qW, qbias, [view(i, d_out) for i in range(S)],
                                gh.workspace(qb, sb.SYMB_OP_FWD_INPLACE))
    torch.cuda.synchronize()
    assert_close(gather(d_out), qYr, "small in-place Y", out_bf16=True)
    for i in range(S):
        if views[i] is not None:
            views[i].fill_(float("nan"))
            view(i, d_out).copy_(gh.to_dev(np.ascontiguousarray(q["dY"][off[i]:off[i + 1]])))
    sb.symb_base_linear_bwd_input_seg(h, qb, [view(i, d_out) for i in range(S)], qW, [view(i, d_in) for i in range(S)],
                                      sb.SYMB_BWD_FULL, gh.workspace(qb, sb.SYMB_OP_BWD_INPUT_INPLACE))
    torch.cuda.synchronize()
    check_dx(gather(d_in), off, qads, q["dY"], q["W"], "small in-place dX")


@pytest.mark.parametrize("case", [
    dict(seed=91, d_in=264, d_out=392, lens=[150, 1, 70, 0, 33], kinds=[L, I, L, L, N], ranks=[8, 16, 5, 3]),
    # segments summed in runs of 1024 tokens, 1100 columns (five column blocks: a full group and a group of one)
    dict(seed=92, d_in=136, d_out=1096, lens=[1700, 3, 2100], kinds=[L, L, L], ranks=[16, 1, 12]),
    # 256x256 tiles in the input gradient
    dict(seed=93, d_in=6208, d_out=136, lens=[700, 5, 795], kinds=[L, N, L], ranks=[16, 8]),
    # layers wide enough for the one-pass dB + dH kernel (at least 64 column blocks of 256): ragged token counts,
    # one-token and empty segments, a last group of one column block with 8 columns, ranks 1..16
    dict(seed=94, d_in=72, d_out=16648, lens=[150, 1, 70, 0, 33], kinds=[L, L, L, L, N], ranks=[8, 16, 5, 3]),
    # ... and segments summed in runs of 1024 tokens
    dict(seed=95, d_in=40, d_out=16384, lens=[1700, 40, 1537], kinds=[L, L, L], ranks=[16, 1, 12]),
])
def test_gradient_call_first_then_the_input_gradient_takes_its_dh(case):
    """symb_adapter_grad leaves dH in the workspace and symb_base_linear_bwd_input with SYMB_BWD_REUSE_DH
    takes it from there; on wide layers with ranks up to 16 the gradient call forms dB and dH in one pass
    over dY.  Gradients and dX against the oracle; dB bit-identical to the two-pass route; accumulation adds."""
    c = dict(case)
    p = make_problem(c.pop("seed"), c.pop("d_in"), c.pop("d_out"), c.pop("lens"), c.pop("kinds"), c.pop("ranks"))
    off, d_in, d_out, T = p["off"], p["d_in"], p["d_out"], p["T"]
    oads = oracle_ads(p["ads"])
    h = gh.handle()
    Xd, dYd, Wd = gh.to_dev(p["X"]), gh.to_dev(p["dY"]), gh.to_dev(p["W"])
    Y0r, _ = oracle.forward(off, oads, p["X"], p["W"], p["bias"])
    Yb = gh.to_dev(synth.f32_to_bf16_bits(Y0r.astype(np.float32)))
    dev = gh.upload_adapters(p["ads"], d_in, d_out, grads=True)
    b = sb.Batch(d_in, d_out, off, dev.descs)
    ws = torch.empty(max(sb.symb_workspace_bytes(b, op) for op in (sb.SYMB_OP_FWD, sb.SYMB_OP_BWD_INPUT, sb.SYMB_OP_ADAPTER_GRAD)),
                     device="cuda", dtype=torch.uint8)
    ws.fill_(0x7f)
    dX = torch.full((T, d_in), float("nan"), device="cuda", dtype=torch.bfloat16)
    sb.symb_adapter_grad(h, b, Xd, dYd, Yb, sb.SYMB_GRAD_OVERWRITE, ws)
    sb.symb_base_linear_bwd_input(h, b, dYd, Wd, dX, sb.SYMB_BWD_FULL | sb.SYMB_BWD_REUSE_DH, ws)
    torch.cuda.synchronize()
    check_dx(gh.bf16_to_f64(dX), off, oads, p["dY"], p["W"], "dX from the gradient call's dH")
    for i, a in enumerate(p["ads"]):
        if a.kind == L and off[i + 1] > off[i]:
            dAr, dBr = oracle.lora_grad(off, oads, p["X"], p["dY"], i)
            assert_close(dev.descs[i].dA.cpu().numpy(), dAr, f"one-pass dA[{i}]")
            assert_close(dev.descs[i].dB.cpu().numpy(), dBr, f"one-pass dB[{i}]")
    # two-pass route: the input gradient first, the gradient call takes its dH
    two = gh.upload_adapters(p["ads"], d_in, d_out, grads=True)
    b2 = sb.Batch(d_in, d_out, off, two.descs)
    sb.symb_base_linear_bwd_input(h, b2, dYd, Wd, dX, sb.SYMB_BWD_FULL, ws)
    sb.symb_adapter_grad(h, b2, Xd, dYd, Yb, sb.SYMB_GRAD_OVERWRITE | sb.SYMB_GRAD_REUSE_DH, ws)
    torch.cuda.synchronize()
    for d1, d2 in zip(dev.descs, two.descs):
        if d1.dB is not None:
            assert torch.equal(d1.dB, d2.dB), "dB must not depend on the route"
    # accumulate on top of the first result
    once = [(d.dA.clone() if d.dA is not None else None, d.dB.clone() if d.dB is not None else None) for d in dev.descs]
    sb.symb_adapter_grad(h, b, Xd, dYd, Yb, sb.SYMB_GRAD_ACCUMULATE, ws)
    torch.cuda.synchronize()
    for (a1, b1), d in zip(once, dev.descs):
        if a1 is not None:
            assert torch.equal(d.dA, a1 + a1)
        if b1 is not None:
            assert torch.equal(d.dB, b1 + b1)
    # the flag is refused where it makes no sense
    with pytest.raises(sb.SymbError) as e:
        sb.symb_base_linear_bwd_input(h, b, dYd, Wd, dX, sb.SYMB_BWD_BASE_ONLY | sb.SYMB_BWD_REUSE_DH, ws)
    assert e.value.status == sb.SYMB_ERR_INVALID_ARG


@pytest.mark.parametrize("case", [
    # the 128x128 tile: about 60 segments per row tile
    dict(seed=101, S=2000, d_in=264, d_out=392),
    # the 256x256 tile in the forward (one LoRA step fetched while another multiplies), about 110 segments per row tile
    dict(seed=102, S=1000, d_in=136, d_out=6208),
])
def test_thousands_of_clients_of_a_few_tokens_each(case):
    """A decode-heavy batch (Sec. 3.7: many inference clients, a token or a few each, batched per layer):
    thousands of segments of 0..9 rows with every adapter kind and ranks 3..16, each with buffers of its
    own, so that every row tile holds dozens of segments.  Everything against the oracle in full."""
    rng = np.random.default_rng(case["seed"])
    lens = [int(x) for x in rng.choice([0, 1, 1, 1, 1, 2, 3, 9], case["S"])]
    p = make_problem(case["seed"], case["d_in"], case["d_out"], lens, [L, L, I, N, L], [4, 8, 16, 3])
    print(f"[many clients] S={case['S']} T={p['T']} {case['d_in']}->{case['d_out']}", flush=True)
    check_all(p, f"{case['S']} clients")


def test_more_segments_than_the_descriptor_slot_holds_are_refused():
    """The per-call descriptors of a batch must fit one 2 MiB slot of the descriptor ring: a batch of
    40000 segments is refused with SYMB_ERR_UNSUPPORTED before anything is launched, and the handle
    keeps working."""
    h = gh.handle()
    S = 40000
    off = np.arange(S + 1, dtype=np.int32)
    b = sb.Batch(64, 64, off, [sb.Adapter() for _ in range(S)])
    X = torch.zeros((S, 64), device="cuda", dtype=torch.bfloat16)
    W = torch.zeros((64, 64), device="cuda", dtype=torch.bfloat16)
    Y = torch.full((S, 64), float("nan"), device="cuda", dtype=torch.bfloat16)
    ws = torch.empty(max(1, sb.symb_workspace_bytes(b, sb.SYMB_OP_FWD)), device="cuda", dtype=torch.uint8)
    with pytest.raises(sb.SymbError) as e:
        sb.symb_base_linear_fwd(h, b, X, W, None, Y, None, ws)
    assert e.value.status == sb.SYMB_ERR_UNSUPPORTED and "capacity" in str(e.value)
    torch.cuda.synchronize()
    assert torch.isnan(Y.float()).all(), "a refused call must leave its output untouched"
    p = make_problem(7, 64, 72, [5, 3], [L, N], [8])
    check_all(p, "after a refused call")


def test_descriptor_ring_wraps_under_a_changing_mix_of_batches():
    """Batches differ from call to call (Sec. 3.7: whoever is queued when a layer runs); the 32-slot
    descriptor ring serves more distinct batches than it has slots.  48 batches (every tile split over K
    ranges: their arrival counters live with the descriptors), 400 calls in random order: each call gives
    the bits of that batch's first call, whether its descriptors were still in place, had been evicted
    and were sent again, or were never seen; a sample of the batches is held to the oracle."""
    h = sb.symb_create(0)
    try:
        rng = np.random.default_rng(11)
        d_in, d_out = 1032, 264
        probs = []
        for k in range(48):
            S = int(rng.integers(1, 5))
            lens = [int(x) for x in rng.choice([1, 3, 17, 40, 64], size=S)]
            kinds = [int(x) for x in rng.choice([L, L, I, N], size=S)]
            p = make_problem(600 + k, d_in, d_out, lens, kinds, [int(x) for x in rng.choice([4, 8, 16, 40], size=S)])
            dev = gh.upload_adapters(p["ads"], d_in, d_out, grads=False)
            p["dev"], p["batch"] = dev, sb.Batch(d_in, d_out, p["off"], dev.descs)
            p["Xd"], p["Wd"], p["bd"] = gh.to_dev(p["X"]), gh.to_dev(p["W"]), gh.to_dev(p["bias"])
            p["Y"] = torch.empty((p["T"], d_out), device="cuda", dtype=torch.bfloat16)
            p["ws"] = gh.workspace(p["batch"], sb.SYMB_OP_FWD)
            p["first"] = None
            probs.append(p)
        order = [int(x) for x in rng.integers(0, len(probs), 400)]
        order[:8] = [0, 1, 0, 1, 2, 0, 1, 2]                   # immediate repeats: descriptors in place
        for n, k in enumerate(order):
            p = probs[k]
            p["Y"].fill_(float("nan"))
            sb.symb_base_linear_fwd(h, p["batch"], p["Xd"], p["Wd"], p["bd"], p["Y"], None, p["ws"], gh.stream_ptr())
            if n % 7 == 0:
                torch.cuda.synchronize()                       # some calls overlap the next one's host work, some do not
            bits = p["Y"].view(torch.int16).clone()
            if p["first"] is None:
                p["first"] = bits
            else:
                assert torch.equal(bits, p["first"]), f"call {n} (batch {k}) differs from that batch's first call"
        torch.cuda.synchronize()
        sent, in_place = sb.symb_debug_descriptor_stats(h)
        assert sent + in_place == len(order) and in_place > 0 and sent > len(probs), (sent, in_place)
        for k in (0, 5, 23, 47):
            p = probs[k]
            _, Yr = oracle.forward(p["off"], oracle_ads(p["ads"]), p["X"], p["W"], p["bias"])
            assert_close(gh.bf16_to_f64(p["first"].view(torch.bfloat16)), Yr, f"ring batch {k} Y", out_bf16=True)
    finally:
        torch.cuda.synchronize()
        sb.symb_destroy(h)


def test_two_streams_share_one_handle():
    """Calls of one host thread on two streams (both at the default priority) through one handle: each
    stream has its own buffers and workspace, the descriptor ring is shared (a slot is found in place only
    by the stream that filled it, and a slot another stream still reads is waited for before it is
    overwritten).  Forward and input gradient of three batches, interleaved over the streams for 40 rounds
    with more distinct descriptor blobs than half the ring: every result has the bits of the same call made
    alone on the default stream."""
    h = sb.symb_create(0)
    try:
        d_in, d_out = 1032, 520
        probs = []
        for k, lens in enumerate([[700, 5, 60], [33, 1, 200, 90], [130]]):
            p = make_problem(700 + k, d_in, d_out, lens, [L, I, N, L], [16, 8, 40])
            dev = gh.upload_adapters(p["ads"], d_in, d_out, grads=False)
            p["dev"], p["batch"] = dev, sb.Batch(d_in, d_out, p["off"], dev.descs)
            p["Xd"], p["Wd"], p["bd"], p["gd"] = gh.to_dev(p["X"]), gh.to_dev(p["W"]), gh.to_dev(p["bias"]), gh.to_dev(p["dY"])
            nws = max(sb.symb_workspace_bytes(p["batch"], op) for op in (sb.SYMB_OP_FWD, sb.SYMB_OP_BWD_INPUT))
            p["buf"] = {}
            for tag in ("alone", "s1", "s2"):
                p["buf"][tag] = (torch.full((p["T"], d_out), float("nan"), device="cuda", dtype=torch.bfloat16),
                                 torch.full((p["T"], d_in), float("nan"), device="cuda", dtype=torch.bfloat16),
                                 torch.empty(nws, device="cuda", dtype=torch.uint8))
            probs.append(p)

        def call(p, tag, stream_ptr):
            Y, dX, ws = p["buf"][tag]
            sb.symb_base_linear_fwd(h, p["batch"], p["Xd"], p["Wd"], p["bd"], Y, None, ws, stream_ptr)
            sb.symb_base_linear_bwd_input(h, p["batch"], p["gd"], p["Wd"], dX, sb.SYMB_BWD_FULL, ws, stream_ptr)

        for p in probs:
            call(p, "alone", gh.stream_ptr())
        torch.cuda.synchronize()
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        rng = np.random.default_rng(3)
        for rnd in range(40):
            a, b = (int(x) for x in rng.integers(0, 3, 2))
            call(probs[a], "s1", s1.cuda_stream)
            call(probs[b], "s2", s2.cuda_stream)
            if rnd % 5 == 4:
                torch.cuda.synchronize()
                for p in probs:
                    for tag in ("s1", "s2"):
                        Y, dX, _ = p["buf"][tag]
                        if not torch.isnan(Y[0, 0].float()):
                            assert torch.equal(Y.view(torch.int16), p["buf"]["alone"][0].view(torch.int16)), (rnd, tag)
                            assert torch.equal(dX.view(torch.int16), p["buf"]["alone"][1].view(torch.int16)), (rnd, tag)
                            Y.fill_(float("nan")); dX.fill_(float("nan"))
                torch.cuda.synchronize()
        p = probs[0]
        oads = oracle_ads(p["ads"])
        _, Yr = oracle.forward(p["off"], oads, p["X"], p["W"], p["bias"])
        assert_close(gh.bf16_to_f64(p["buf"]["alone"][0]), Yr, "two streams: Y", out_bf16=True)
        check_dx(gh.bf16_to_f64(p["buf"]["alone"][1]), p["off"], oads, p["dY"], p["W"], "two streams: dX")
    finally:
        torch.cuda.synchronize()
        sb.symb_destroy(h)
