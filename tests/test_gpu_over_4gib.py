"""Tensors of more than 4 GiB (more than 2^31 elements): a 32-bit byte offset or element index anywhere
in the path would wrap inside them.  Two shapes with T = 60000 rows, one whose output side is 36864 wide
(Y, Ybase and dY are 4.4 GB each) and one whose input side is (X and dX are): forward, input gradient
both ways of getting dH, and the gradients of a long LoRA segment (walked in runs), of a LoRA segment
that straddles the 4 GiB mark (row 58254) and of an IA3 segment that lies wholly beyond it.

The activations are drawn on the device (seeded torch generator) and only the rows the oracle needs
come back to the host.  Every forward / input-gradient row depends on its own input row and on its
segment's adapter only, so the oracle computes the sampled rows as a batch of their own (same segments,
each shrunk to its sampled rows); the parameter gradients sum over a segment's tokens, so the three
fine-tuning segments are downloaded whole and compared in full.  Same bar as everywhere (helpers.py)."""
import numpy as np
import pytest
import torch

import oracle
import synth
from helpers import assert_close, check_dx

pytestmark = pytest.mark.gpu

L, I, N = oracle.LORA, oracle.IA3, oracle.NONE
T = 60000
LENS = [46000, 10000, 2400, 1000, 600]          # offsets 0, 46000, 56000, 58400, 59400, 60000
KINDS = [N, L, L, I, N]
RANKS = [0, 16, 8, 0, 0]
FINETUNE = [False, True, True, True, False]      # every LoRA segment wants its gradients: the input gradient may take dH
WIDE = 36864                                     # 2^32 bytes / (36864 * 2) = row 58254.2: inside segment 2


def _bits(rng, shape, std, mean=0.0):
    return synth.f32_to_bf16_bits((mean + std * rng.standard_normal(shape)).astype(np.float32))


def _device_normal(rows, width, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    out = torch.empty((rows, width), device="cuda", dtype=torch.bfloat16)
    for r0 in range(0, rows, 8192):              # in blocks: no fp32 copy of the whole tensor
        n = min(8192, rows - r0)
        out[r0:r0 + n] = torch.randn((n, width), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    return out


def _host_bits(t):
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def _f64(t):
    return t.to(torch.float32).cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("d_in,d_out", [(256, WIDE), (WIDE, 256)], ids=["wide_output", "wide_input"])
def test_rows_beyond_the_4_gib_mark(d_in, d_out):
    import gpu_harness as gh
    from paper_2507_03220_amd import binding as sb
    sb.lib()
    h = gh.handle()
    tag = f"over 4 GiB {d_in}->{d_out}"
    rng = np.random.default_rng(4242 + d_in)
    off = np.zeros(len(LENS) + 1, dtype=np.int32)
    off[1:] = np.cumsum(LENS)
    assert int(off[-1]) == T and T * WIDE * 2 > (1 << 32) and T * WIDE > (1 << 31)
    mark = (1 << 32) // (WIDE * 2)
    assert off[2] < mark < off[3] and off[3] > mark

    ads = []
    for k, r, ft in zip(KINDS, RANKS, FINETUNE):
        if k == L:
            ads.append(gh.HostAdapter(k, r, 16.0 / r, _bits(rng, (r, d_in), d_in ** -0.5), _bits(rng, (d_out, r), r ** -0.5), want_grad=ft))
        elif k == I:
            ads.append(gh.HostAdapter(k, 0, 0.0, _bits(rng, (d_out,), 0.1, 1.0), want_grad=ft))
        else:
            ads.append(gh.HostAdapter(want_grad=False))
    oads = [oracle.Adapter(a.kind, a.rank, a.scale, a.A, a.B) for a in ads]
    W = _bits(rng, (d_out, d_in), d_in ** -0.5)
    Wd = gh.to_dev(W)
    print(f"[{tag}] drawing X and dY on the device", flush=True)
    Xd = _device_normal(T, d_in, 11)
    dYd = _device_normal(T, d_out, 12)

    # sampled rows: ends of every segment, seeded rows inside, and the rows around the 4 GiB mark
    rows = set(range(mark - 4, mark + 6))
    for i in range(len(LENS)):
        lo, hi = int(off[i]), int(off[i + 1])
        rows.update([lo, lo + 1, hi - 2, hi - 1])
        rows.update(int(x) for x in rng.integers(lo, hi, 6))
    rows = np.array(sorted(rows), dtype=np.int64)
    coff = np.searchsorted(rows, off).astype(np.int32)           # the same segments, shrunk to their sampled rows
    ridx = torch.from_numpy(rows).cuda()
    Xc, dYc = _host_bits(Xd.index_select(0, ridx)), _host_bits(dYd.index_select(0, ridx))

    dev = gh.upload_adapters(ads, d_in, d_out, grads=True)
    batch = sb.Batch(d_in, d_out, off, dev.descs)
    s = gh.stream_ptr()

    # ---- forward, with the pre-adapter output
    print(f"[{tag}] forward", flush=True)
    Y = torch.full((T, d_out), float("nan"), device="cuda", dtype=torch.bfloat16)
    Yb = torch.full((T, d_out), float("nan"), device="cuda", dtype=torch.bfloat16)
    ws = gh.workspace(batch, sb.SYMB_OP_FWD)
    sb.symb_base_linear_fwd(h, batch, Xd, Wd, None, Y, Yb, ws, s)
    torch.cuda.synchronize()
    Y0r, Yr = oracle.forward(coff, oads, Xc, W, None)
    assert_close(_f64(Y.index_select(0, ridx)), Yr, f"{tag} Y", out_bf16=True)
    assert_close(_f64(Yb.index_select(0, ridx)), Y0r, f"{tag} Ybase", out_bf16=True)
    assert not torch.isnan(Y[-1].float()).any() and not torch.isnan(Y[mark].float()).any()
    del Y, ws

    # ---- the fine-tuning segments, whole: what the gradient calls are compared with
    one = lambda n: np.array([0, n], dtype=np.int32)
    lora_ref = {}
    for q in (1, 2):
        lo, hi = int(off[q]), int(off[q + 1])
        lora_ref[q] = oracle.lora_grad(one(hi - lo), [oads[q]], _host_bits(Xd[lo:hi]), _host_bits(dYd[lo:hi]), 0)
    lo3, hi3 = int(off[3]), int(off[4])
    X3, dY3 = _host_bits(Xd[lo3:hi3]), _host_bits(dYd[lo3:hi3])
    Y0_3, _ = oracle.forward(one(hi3 - lo3), [oads[3]], X3, W, None)
    Y0_3_bits = synth.f32_to_bf16_bits(Y0_3.astype(np.float32))    # the base output the client kept, in bf16
    dl_ref = oracle.ia3_grad(one(hi3 - lo3), [oads[3]], X3, dY3, W, None, 0, Y0_saved=Y0_3_bits)
    Yb.zero_()
    Yb[lo3:hi3] = gh.to_dev(Y0_3_bits)

    def check_grads(route):
        for q, (dA_ref, dB_ref) in lora_ref.items():
            assert_close(dev.descs[q].dA.cpu().numpy(), dA_ref, f"{tag} dA[{q}] ({route})")
            assert_close(dev.descs[q].dB.cpu().numpy(), dB_ref, f"{tag} dB[{q}] ({route})")
        assert_close(dev.descs[3].dA.cpu().numpy(), dl_ref, f"{tag} dl ({route})")
        for d in (dev.descs[1].dA, dev.descs[1].dB, dev.descs[2].dA, dev.descs[2].dB, dev.descs[3].dA):
            d.fill_(float("nan"))

    # ---- gradient call first (dB and dH in one pass over dY where the layer is wide enough), then the
    # input gradient taking its dH; one workspace for both, as the runner lays it out
    print(f"[{tag}] gradients, then the input gradient", flush=True)
    nws = max(sb.symb_workspace_bytes(batch, sb.SYMB_OP_ADAPTER_GRAD), sb.symb_workspace_bytes(batch, sb.SYMB_OP_BWD_INPUT))
    ws = torch.empty(nws, device="cuda", dtype=torch.uint8)
    sb.symb_adapter_grad(h, batch, Xd, dYd, Yb, sb.SYMB_GRAD_OVERWRITE, ws, s)
    torch.cuda.synchronize()
    check_grads("gradients first")
    dX = torch.full((T, d_in), float("nan"), device="cuda", dtype=torch.bfloat16)
    sb.symb_base_linear_bwd_input(h, batch, dYd, Wd, dX, sb.SYMB_BWD_FULL | sb.SYMB_BWD_REUSE_DH, ws, s)
    torch.cuda.synchronize()
    check_dx(_f64(dX.index_select(0, ridx)), coff, oads, dYc, W, f"{tag} dX (dH taken over)")

    # ---- the other order: the input gradient computes dH, the gradient call takes it
    print(f"[{tag}] input gradient, then the gradients", flush=True)
    dX.fill_(float("nan"))
    sb.symb_base_linear_bwd_input(h, batch, dYd, Wd, dX, sb.SYMB_BWD_FULL, ws, s)
    torch.cuda.synchronize()
    check_dx(_f64(dX.index_select(0, ridx)), coff, oads, dYc, W, f"{tag} dX")
    assert not torch.isnan(dX[-1].float()).any() and not torch.isnan(dX[mark].float()).any()
    sb.symb_adapter_grad(h, batch, Xd, dYd, Yb, sb.SYMB_GRAD_OVERWRITE | sb.SYMB_GRAD_REUSE_DH, ws, s)
    torch.cuda.synchronize()
    check_grads("input gradient first")
    del dX, ws, Yb, Xd, dYd
    torch.cuda.empty_cache()
