"""symb_base_linear_fwd_static (the forward whose workspace is a file-scope device array, for
callers that cannot allocate) against symb_base_linear_fwd on the same inputs, through the C ABI:
two calls in a row on one handle, the second with a smaller batch, so that whatever the first call
left in the shared array is there when the second runs.  The two entry points launch the same
kernels, so the outputs must agree bit for bit; the first call is also held to the oracle's bar."""
import gc

import numpy as np
import pytest
import torch

import oracle
import synth
from helpers import assert_close

pytestmark = pytest.mark.gpu

L, I, N = oracle.LORA, oracle.IA3, oracle.NONE


def _problem(seed, d_in, d_out, lens, kinds, ranks, bias):
    import gpu_harness as gh
    rng = np.random.default_rng(seed)
    off = np.zeros(len(lens) + 1, dtype=np.int32)
    off[1:] = np.cumsum(lens)
    nb = lambda shape, std, mean=0.0: synth.f32_to_bf16_bits((mean + std * rng.standard_normal(shape)).astype(np.float32))
    ads = []
    for i in range(len(lens)):
        k = kinds[i % len(kinds)]
        if k == L:
            r = ranks[i % len(ranks)]
            ads.append(gh.HostAdapter(k, r, 16.0 / r, nb((r, d_in), d_in ** -0.5), nb((d_out, r), r ** -0.5)))
        elif k == I:
            ads.append(gh.HostAdapter(k, 0, 0.0, nb((d_out,), 0.1, 1.0)))
        else:
            ads.append(gh.HostAdapter())
    return dict(off=off, T=int(off[-1]), d_in=d_in, d_out=d_out, ads=ads, X=nb((int(off[-1]), d_in), 1.0),
                W=nb((d_out, d_in), d_in ** -0.5), bias=nb((d_out,), 0.5) if bias else None)


def _both(h, p, want_base):
    import gpu_harness as gh
    from paper_2507_03220_amd import binding as sb
    dev = gh.upload_adapters(p["ads"], p["d_in"], p["d_out"], grads=False)
    batch = sb.Batch(p["d_in"], p["d_out"], p["off"], dev.descs)
    Xd, Wd, bd = gh.to_dev(p["X"]), gh.to_dev(p["W"]), gh.to_dev(p["bias"])
    mk = lambda: torch.full((p["T"], p["d_out"]), float("nan"), device="cuda", dtype=torch.bfloat16)
    Y1, Y2 = mk(), mk()
    B1, B2 = (mk(), mk()) if want_base else (None, None)
    # the existing entry point, given a workspace as large as the static array (same split decisions)
    ws = torch.empty(sb.SYMB_STATIC_SCRATCH_BYTES, device="cuda", dtype=torch.uint8)
    sb.symb_base_linear_fwd(h, batch, Xd, Wd, bd, Y1, B1, ws, gh.stream_ptr())
    torch.cuda.synchronize()
    # Allocation events are counted, not bytes held: after other tests the collector may free their tensors
    # at any moment, which lowers the bytes held (and can only raise the device's free memory).
    events = lambda: torch.cuda.memory_stats().get("allocation.all.allocated", 0)
    gc.collect()
    free_before, events_before = torch.cuda.mem_get_info()[0], events()
    sb.symb_base_linear_fwd_static(h, batch, Xd, Wd, bd, Y2, B2, gh.stream_ptr())
    torch.cuda.synchronize()
    # nothing was allocated on the device, by torch or behind its back
    assert events() == events_before and torch.cuda.mem_get_info()[0] >= free_before
    return Y1, Y2, B1, B2


def test_static_forward_matches_the_workspace_forward_twice_in_a_row():
    import gpu_harness as gh
    from paper_2507_03220_amd import binding as sb
    sb.lib()
    h = sb.symb_create(0)
    try:
        # first call: 256x256 tiles, last round of 266 tiles split over K ranges (partial tiles in the array too)
        big = _problem(301, 2056, 33800, [120, 1, 99, 80], [L, N, L, L], [16, 8, 40], bias=False)
        print(f"[no-alloc] first call T={big['T']} {big['d_in']}->{big['d_out']}", flush=True)
        Y1, Y2, _, _ = _both(h, big, want_base=False)
        assert torch.equal(Y1.view(torch.int16), Y2.view(torch.int16)), "static forward differs from the workspace forward"
        _, Yr = oracle.forward(big["off"], [oracle.Adapter(a.kind, a.rank, a.scale, a.A, a.B) for a in big["ads"]],
                               big["X"], big["W"], None)
        assert_close(gh.bf16_to_f64(Y2), Yr, "static forward Y", out_bf16=True)
        # second call, smaller, other kinds and a pre-adapter output: the array still holds the first call's bytes
        small = _problem(302, 320, 264, [130, 1, 0, 77, 1, 40], [L, I, L, N, L, I], [8, 16, 5, 24], bias=True)
        print(f"[no-alloc] second call T={small['T']} {small['d_in']}->{small['d_out']}", flush=True)
        Y1, Y2, B1, B2 = _both(h, small, want_base=True)
        assert torch.equal(Y1.view(torch.int16), Y2.view(torch.int16))
        assert torch.equal(B1.view(torch.int16), B2.view(torch.int16))
        Y0r, Yr = oracle.forward(small["off"], [oracle.Adapter(a.kind, a.rank, a.scale, a.A, a.B) for a in small["ads"]],
                                 small["X"], small["W"], small["bias"])
        assert_close(gh.bf16_to_f64(Y2), Yr, "static forward Y (second call)", out_bf16=True)
        assert_close(gh.bf16_to_f64(B2), Y0r, "static forward Ybase (second call)", out_bf16=True)
        # a batch beyond the array is refused before anything is enqueued
        huge = sb.Batch(64, 64, [0, 200000], [sb.Adapter(sb.SYMB_ADAPTER_LORA, 128, 1.0, Y1, Y1)])
        with pytest.raises(sb.SymbError) as e:
            sb.symb_base_linear_fwd_static(h, huge, Y1, Y1, None, Y1, None, gh.stream_ptr())
        assert e.value.status == sb.SYMB_ERR_WORKSPACE_TOO_SMALL
    finally:
        torch.cuda.synchronize()
        sb.symb_destroy(h)
