"""Host-side checks of libsymb.so that need no GPU: every declared symbol is exported,
argument validation, the segment planner and the row->segment map (bit-exact against
the oracle's map).  No compute entry point is called here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
from paper_2507_03220_amd import binding as sb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def _built():
    from paper_2507_03220_amd import build
    build.build(force=False)


def _declared_symbols():
    text = ""
    inc = os.path.join(ROOT, "include")
    for f in sorted(os.listdir(inc)):
        if f.endswith(".h"):
            text += open(os.path.join(inc, f)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(symb_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared_symbols()
    assert set(names) == set(sb.EXPORTS), names
    l = sb.lib()
    for n in names:
        assert getattr(l, n) is not None


def test_status_strings():
    l = sb.lib()
    assert l.symb_status_string(0) == b"SYMB_OK"
    assert l.symb_status_string(2) == b"SYMB_ERR_BAD_SEGMENTS"


def _batch(off, ads=None, d_in=64, d_out=64):
    ads = ads if ads is not None else [sb.Adapter() for _ in range(len(off) - 1)]
    return sb.Batch(d_in, d_out, off, ads)


def test_validation_rejects_bad_batches():
    assert sb.symb_validate_batch(_batch([0, 4, 9])) == sb.SYMB_OK
    assert sb.symb_validate_batch(_batch([0, 0, 0])) == sb.SYMB_OK          # empty segments are legal
    assert sb.symb_validate_batch(_batch([0])) == sb.SYMB_OK                # no segments at all
    assert sb.symb_validate_batch(_batch([1, 4])) == sb.SYMB_ERR_BAD_SEGMENTS
    assert sb.symb_validate_batch(_batch([0, 5, 3])) == sb.SYMB_ERR_BAD_SEGMENTS
    assert sb.symb_validate_batch(_batch([0, 4], d_in=0)) == sb.SYMB_ERR_INVALID_ARG
    assert sb.symb_validate_batch(_batch([0, 4], d_out=12)) == sb.SYMB_ERR_INVALID_ARG   # not a multiple of 8
    fake = 0x1000  # an aligned, never dereferenced address: validation is host-only
    lora = lambda **kw: sb.Adapter(**{**dict(kind=sb.SYMB_ADAPTER_LORA, rank=8, scale=2.0, A=fake, B=fake), **kw})
    assert sb.symb_validate_batch(_batch([0, 4], [lora()])) == sb.SYMB_OK
    assert sb.symb_validate_batch(_batch([0, 4], [lora(rank=0)])) == sb.SYMB_ERR_INVALID_ARG
    assert sb.symb_validate_batch(_batch([0, 4], [lora(A=None)])) == sb.SYMB_ERR_INVALID_ARG
    assert sb.symb_validate_batch(_batch([0, 4], [lora(B=None)])) == sb.SYMB_ERR_INVALID_ARG
    assert sb.symb_validate_batch(_batch([0, 4], [lora(A=fake + 2)])) == sb.SYMB_ERR_INVALID_ARG
    assert sb.symb_validate_batch(_batch([0, 4], [lora(rank=sb.SYMB_MAX_RANK + 1)])) == sb.SYMB_ERR_UNSUPPORTED
    assert sb.symb_validate_batch(_batch([0, 4], [lora(rank=5, B=fake + 2)])) == sb.SYMB_OK   # odd rank: 2-byte B
    assert sb.symb_validate_batch(_batch([0, 4], [sb.Adapter(kind=7)])) == sb.SYMB_ERR_INVALID_ARG
    assert sb.symb_validate_batch(_batch([0, 4], [sb.Adapter(kind=sb.SYMB_ADAPTER_IA3)])) == sb.SYMB_ERR_INVALID_ARG
    assert sb.symb_validate_batch(_batch([0, 4], [sb.Adapter(kind=sb.SYMB_ADAPTER_IA3, A=fake)])) == sb.SYMB_OK
    assert sb.symb_validate_batch(_batch([0, 4], [sb.Adapter(kind=sb.SYMB_ADAPTER_IA3_IN, A=fake)])) == sb.SYMB_OK
    assert sb.symb_validate_batch(_batch([0, 4], [sb.Adapter(kind=sb.SYMB_ADAPTER_IA3_IN)])) == sb.SYMB_ERR_INVALID_ARG
    assert b"IA3 input scaling" in sb.lib().symb_last_error(None)


@pytest.mark.parametrize("seed", range(6))
def test_row_segment_map_is_bit_exact_vs_oracle(seed):
    rng = np.random.default_rng(seed)
    S = int(rng.integers(1, 70))
    lens = rng.choice([0, 1, 1, 2, 3, 17, 64, 255, 256, 257, 1000], size=S)
    off = np.zeros(S + 1, dtype=np.int32)
    off[1:] = np.cumsum(lens)
    got = sb.symb_debug_row_segment_map(_batch(off))
    np.testing.assert_array_equal(got, oracle.row_segment_map(off))


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("tile_m", [16, 128, 256])
def test_row_tile_plan_matches_oracle_map(seed, tile_m):
    rng = np.random.default_rng(100 + seed)
    S = int(rng.integers(1, 70))
    lens = rng.choice([0, 0, 1, 1, 2, 3, 17, 64, 255, 256, 257, 1000], size=S)
    off = np.zeros(S + 1, dtype=np.int32)
    off[1:] = np.cumsum(lens)
    lo, hi = sb.symb_plan_row_tiles(_batch(off), tile_m)
    seg = oracle.row_segment_map(off)
    T = int(off[-1])
    assert len(lo) == (T + tile_m - 1) // tile_m
    for u in range(len(lo)):
        rows = seg[u * tile_m:min(T, (u + 1) * tile_m)]
        assert lo[u] == rows.min() and hi[u] == rows.max()


def test_workspace_bytes_formula():
    fake = 0x1000
    ads = [sb.Adapter(sb.SYMB_ADAPTER_LORA, 5, 1.0, fake, fake, fake, fake), sb.Adapter(),
           sb.Adapter(sb.SYMB_ADAPTER_IA3, 0, 0.0, fake), sb.Adapter(sb.SYMB_ADAPTER_LORA, 40, 1.0, fake, fake)]
    b = sb.Batch(64, 128, [0, 10, 20, 30, 100], ads)
    T, rp = 100, 2 * 48                               # pitch = 2 * (max rank rounded up to 16)
    up = lambda n: (n + 255) // 256 * 256
    packed = (16 + 48) * 128 * 2
    assert sb.symb_workspace_bytes(b, sb.SYMB_OP_FWD) == up(T * rp * 2)
    # Hs (left alone by the input-gradient call), dH, packed B^T, IA3-scaled dY
    assert sb.symb_workspace_bytes(b, sb.SYMB_OP_BWD_INPUT) == 2 * up(T * rp * 2) + up(packed) + up(T * 128 * 2)
    assert sb.symb_workspace_bytes(b, sb.SYMB_OP_ADAPTER_GRAD) == 2 * up(T * rp * 2) + up(packed)   # Hs, dH, packed B^T
    # input-major (Conv1D) weight: forward also packs B^T (at the offset the other operations use), the
    # input gradient also packs A^T (5*64 and 40*64 elements, each rounded up to 8)
    c = sb.Batch(64, 128, [0, 10, 20, 30, 100], ads, sb.SYMB_WEIGHT_CONV1D)
    assert sb.symb_workspace_bytes(c, sb.SYMB_OP_FWD) == 2 * up(T * rp * 2) + up(packed)
    assert sb.symb_workspace_bytes(c, sb.SYMB_OP_BWD_INPUT) == 2 * up(T * rp * 2) + up(packed) + up(T * 128 * 2) + up((5 * 64 + 40 * 64) * 2)
    assert sb.symb_workspace_bytes(c, sb.SYMB_OP_ADAPTER_GRAD) == 2 * up(T * rp * 2) + up(packed)
    none = sb.Batch(64, 128, [0, 100], [sb.Adapter()])
    for op in (sb.SYMB_OP_FWD, sb.SYMB_OP_BWD_INPUT, sb.SYMB_OP_ADAPTER_GRAD):
        assert sb.symb_workspace_bytes(none, op) == 0


def test_workspace_includes_the_runs_of_long_segments_gradients():
    # LoRA gradients of a segment of more than 1536 tokens are summed in runs of 1024 tokens, each run an
    # fp32 array of the gradient's size in the workspace; dB's runs and dA's share the place
    fake = 0x1000
    up = lambda n: (n + 255) // 256 * 256
    ads = [sb.Adapter(sb.SYMB_ADAPTER_LORA, 5, 1.0, fake, fake, fake, fake),      # 2100 tokens: 3 runs
           sb.Adapter(sb.SYMB_ADAPTER_LORA, 40, 1.0, fake, fake, fake, fake),     # 1536 tokens: stays whole
           sb.Adapter(sb.SYMB_ADAPTER_LORA, 8, 1.0, fake, fake)]                  # 1700 tokens, no gradients wanted
    b = sb.Batch(64, 128, [0, 2100, 3636, 5336], ads)
    T, rp = 5336, 2 * 48
    base = 2 * up(T * rp * 2) + up((16 + 48 + 16) * 128 * 2)                     # Hs, dH, packed B^T
    assert sb.symb_workspace_bytes(b, sb.SYMB_OP_ADAPTER_GRAD) == base + up(3 * 5 * 128 * 4)
    assert sb.symb_workspace_bytes(b, sb.SYMB_OP_FWD) == up(T * rp * 2)


def test_workspace_includes_partial_tiles_of_a_k_split():
    # 378 rows on a 4096 x 4096 layer: 3 x 32 = 96 tiles of 128 x 128 for 256 CUs; every tile is computed
    # by 320 // 96 = 3 workgroups, one per K range, each leaving a 64 KiB fp32 partial tile
    none = sb.Batch(4096, 4096, [0, 378], [sb.Adapter()])
    assert sb.symb_workspace_bytes(none, sb.SYMB_OP_FWD) == 96 * 3 * 128 * 128 * 4
    assert sb.symb_workspace_bytes(none, sb.SYMB_OP_BWD_INPUT) == 96 * 3 * 128 * 128 * 4
    assert sb.symb_workspace_bytes(none, sb.SYMB_OP_ADAPTER_GRAD) == 0
    # K = 448 = 7 stages of 64: too short to split; 1500 rows: 12 x 32 = 384 tiles, enough workgroups
    assert sb.symb_workspace_bytes(sb.Batch(448, 4096, [0, 378], [sb.Adapter()]), sb.SYMB_OP_FWD) == 0
    assert sb.symb_workspace_bytes(sb.Batch(4096, 4096, [0, 1500], [sb.Adapter()]), sb.SYMB_OP_FWD) == 0
    # 20480 rows: 80 x 16 tiles of 256 x 256, 160 per XCD = 5 full rounds of its 32 CUs: no split
    assert sb.symb_workspace_bytes(sb.Batch(4096, 4096, [0, 20480], [sb.Adapter()]), sb.SYMB_OP_FWD) == 0
    # 9049 rows: 36 x 16 = 576 tiles, 72 per XCD: the last 8 of them would be a round of their own and are
    # split over 3 K ranges each (24 workgroups on the XCD's 32 CUs; a fourth part would save less than it costs
    # to add up): 8 XCDs x 8 tiles x 3 partial tiles of 256 KiB
    assert sb.symb_workspace_bytes(sb.Batch(4096, 4096, [0, 9049], [sb.Adapter()]), sb.SYMB_OP_FWD) == 8 * 8 * 3 * 256 * 256 * 4
    # 20480 rows on 4608 -> 2048: 640 tiles, 80 per XCD, the last 16 split in two
    assert sb.symb_workspace_bytes(sb.Batch(4608, 2048, [0, 20480], [sb.Adapter()]), sb.SYMB_OP_FWD) == 8 * 16 * 2 * 256 * 256 * 4
    # ... 1440 tiles, 180 per XCD, a last round of 20 tiles: in three parts they are 60 workgroups, two passes of
    # a third of a tile's time each.  Worth it on the long inner dimension (input gradient of 36864 -> 4608:
    # 576 stages per tile); on 4096 stages of work the sum of the partial tiles would eat the gain
    assert sb.symb_workspace_bytes(sb.Batch(36864, 4608, [0, 20480], [sb.Adapter()]), sb.SYMB_OP_FWD) == 8 * 20 * 3 * 256 * 256 * 4
    assert sb.symb_workspace_bytes(sb.Batch(4096, 4608, [0, 20480], [sb.Adapter()]), sb.SYMB_OP_FWD) == 0


def test_unknown_weight_layout_is_rejected():
    b = sb.Batch(64, 64, [0, 4], [sb.Adapter()], weight_layout=7)
    assert sb.lib().symb_validate_batch(b.ref()) == sb.SYMB_ERR_INVALID_ARG


def test_compute_entry_points_fail_cleanly_without_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(sb.SymbError) as e:
        sb.symb_create(0)
    assert e.value.status == sb.SYMB_ERR_DEVICE
    with pytest.raises(sb.SymbError) as e:
        sb.symb_base_linear_fwd(None, _batch([0, 4]), 0x1000, 0x1000, None, 0x1000)
    assert e.value.status == sb.SYMB_ERR_INVALID_ARG      # null handle, nothing launched
