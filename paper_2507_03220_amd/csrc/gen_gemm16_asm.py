#!/usr/bin/env python3
"""Writes gemm16_asm.hpp: the assembly of the 256x256 base GEMM built on v_mfma_f32_16x16x32_bf16.

Run `python gen_gemm16_asm.py` after changing the schedule; the output is committed, the build
does not run this script.

Why this instruction: the chip is power-limited, and with N(0,1) operands the 16x16x32 form
sustains 12 % more flops than the 32x32x16 form (it touches each accumulator once per 32 k
instead of once per 16 k).  Why everything that touches an accumulator is assembly: a wavefront
owns 128x128 of C as 8x8 blocks of 16x16, 4 registers each, i.e. all 256 accumulation registers,
and the instruction writes 4-register blocks.  An inline-assembly operand cannot name part of a
register tuple, and 64 four-register operands are more than the compiler copes with, so the
accumulators are not C++ objects at all: block (i, j) lives in a[4(8i+j) : 4(8i+j)+3], every
template names these registers literally, and the compiler-generated code in between never
touches an accumulation register (a CPU test checks the generated assembly for that).

Lane layout of the instruction, issued as (weight fragment, activation fragment): an operand
lane l holds row l%16 and eight of the 32 k of its 16x32 fragment; which eight does not matter as
long as both operands agree (the instruction multiplies register element e of lane group l/16 of
one operand with the same element of the same lane group of the other).  Here lane group g holds
k = 8(g/2) + 4(g%2) + 0..3 and the same + 16: every 16-byte fragment quad is filled by two 8-byte
LDS reads (a wavefront alone on its SIMD issues in order, and a 16-byte read holds up the next
16-cycle MFMA where an 8-byte read does not), and with this choice the 32 lanes the LDS serves per
clock read both halves of 16 different 16-byte chunks, i.e. all 64 banks once.  The result lane
holds C[m = 16i + l%16][n = 16j + 4(l/16) + e], e = 0..3: four consecutive columns of one row.

Main loop, per 64-k stage P (ring of three A and two B units of 32 KiB in LDS): two 32-k steps of 64 MFMAs each, fragment sets F0/F1 alternating.
  step 0: MFMAs on F0 while the step-1 fragments of stage P are read into F1; the eight loads
          of A(P+2) go out, one per eight MFMAs; then wait for this wavefront's loads of stage
          P+1, barrier (stage P+1 complete for everybody, both units of stage P free);
  step 1: MFMAs on F1 while the step-0 fragments of stage P+1 are read into F0; the eight loads
          of B(P+2) go out during the first 16 MFMAs.
The last two stages run copies of the body without loads.
"""
import os

VT = 116                      # address temporaries v116..v127
S_GA, S_GB = 80, 82
S_CNT, S_ACUR, S_ANXT, S_ANN, S_BCUR, S_BNXT, S_T0, S_T1 = range(84, 92)

# The compiler does not look inside an assembly statement: whatever it places right after one
# must not meet a matrix instruction that is still writing its result.
MFMA_DRAIN = ["s_nop 15", "s_nop 7"]


def configure(nb):
    """Sets the tile-dependent constants: nb = 16x16 blocks per wavefront and dimension (8: 256x256
    tile of the workgroup, 4: 128x128)."""
    global VTOP, NB, F, UNIT, A_BASES, B_BASES, C_PITCH, NPITCH, VA, VB, AV, BV, GA, GB, STRIDE_B, KF, SWA, BLOCKS
    NB = nb
    VTOP = 128 + 16 * nb                        # one past the last VGPR the templates use (256 / 192)
    F = {0: 128, 1: 128 + 8 * nb}               # first VGPR of fragment set 0 / 1 (A: nb x 4 regs, then B: nb x 4 regs)
    UNIT = 4096 * nb                            # one operand's 64-k stage: 32 nb rows x 128 bytes
    A_BASES = (0, UNIT, 2 * UNIT)
    B_BASES = (3 * UNIT, 4 * UNIT)
    C_PITCH = 64 * nb + 16                      # bytes per row of the staged bf16 output tile
    NPITCH = 64 * nb                            # bytes per k-row of an N-contiguous weight unit
    # operand numbers of the main loop
    VA = (0, 1, 2, 3)                           # A fragment lane offsets: 32-k step 0 first / second read, step 1 first / second read
    VB = tuple(range(4, 4 + max(4, nb)))        # K-contiguous W: as VA in VB[0..3]; N-contiguous W: one per 16-column block
    AV = tuple(range(VB[-1] + 1, VB[-1] + 1 + nb))   # global byte offsets of this lane's nb A loads
    BV = tuple(range(AV[-1] + 1, AV[-1] + 1 + nb))   # global byte offsets of this lane's nb B loads
    GA, GB, STRIDE_B, KF, SWA = (BV[-1] + 1 + x for x in range(5))
    BLOCKS = [(i, j) for i in range(nb) for j in range(nb)]


def acc(i, j):
    b = 4 * (NB * i + j)
    return f"a[{b}:{b + 3}]"


def fa(s, i):
    b = F[s] + 4 * i
    return f"v[{b}:{b + 3}]"


def fb(s, j):
    b = F[s] + 4 * NB + 4 * j
    return f"v[{b}:{b + 3}]"


def fb_half(s, j, h):
    b = F[s] + 4 * NB + 4 * j + 2 * h
    return f"v[{b}:{b + 1}]"


def mfma(s, i, j):
    return f"v_mfma_f32_16x16x32_bf16 {acc(i, j)}, {fb(s, j)}, {fa(s, i)}, {acc(i, j)}"


def frag_reads(nn, dst, sa, sb, ks, va=None, vb=None):
    """The LDS reads that fill fragment set `dst` with 32-k step `ks` of the stage whose A / B units
    start at SGPR `sa` / `sb` (or, with va / vb given, at those address operands).  A list of slots:
    each read, preceded by the address add it needs.  A fragment register quad is filled by two
    8-byte reads with an address each (see the lane layout above)."""
    slots = []
    for q in range(2):
        if va is None:
            addr = f"v{VT + q}"
            pre = [f"v_add_u32 {addr}, s{sa}, %{VA[2 * ks + q]}"]
        else:
            addr, pre = va[q], []
        for i in range(NB):
            b = F[dst] + 4 * i + 2 * q
            slots.append((pre if i == 0 else []) + [f"ds_read_b64 v[{b}:{b + 1}], {addr} offset:{2048 * i}"])
    if not nn:
        for q in range(2):
            if vb is None:
                addr = f"v{VT + 2 + q}"
                pre = [f"v_add_u32 {addr}, s{sb}, %{VB[2 * ks + q]}"]
            else:
                addr, pre = vb[q], []
            for j in range(NB):
                slots.append((pre if j == 0 else []) + [f"ds_read_b64 {fb_half(dst, j, q)}, {addr} offset:{2048 * j}"])
    else:
        for j in range(NB):
            if vb is None:
                addr = f"v{VT + 2 + j}"
                pre = [f"v_add_u32 {addr}, s{sb}, %{VB[j]}"]
            else:
                addr, pre = vb[j], []
            for q in range(2):
                slots.append((pre if q == 0 else []) +
                             [f"ds_read_b64_tr_b16 {fb_half(dst, j, q)}, {addr} offset:{32 * NPITCH * ks + 16 * NPITCH * q}"])
    return slots


def unit_loads(sdst, which, js):
    """Per load two slots: the LDS destination into m0, then the load itself (the instruction that
    sits between them covers the wait state an m0 write needs).  s{T0} holds unit + wavefront base."""
    V, G = (AV, S_GA) if which == "A" else (BV, S_GB)
    return [f"s_add_u32 s{S_T0}, s{sdst}, %{SWA}"], \
           [([f"s_add_u32 m0, s{S_T0}, {1024 * j}"], [f"global_load_lds_dwordx4 %{V[j]}, s[{G}:{G + 1}]"]) for j in js]


def unit_loads_flat(sdst, which, js):
    pre, pairs = unit_loads(sdst, which, js)
    out = list(pre)
    for a, b in pairs:
        out += a + ["s_nop 0"] + b
    return out


def advance(which, cond=None):
    G, step = (S_GA, "128") if which == "A" else (S_GB, f"%{STRIDE_B}")
    if cond is None:
        pre = [f"s_mov_b32 s{S_T1}, {step}"] if which == "B" else []
        src = f"s{S_T1}" if which == "B" else step
        return pre + [f"s_add_u32 s{G}, s{G}, {src}", f"s_addc_u32 s{G + 1}, s{G + 1}, 0"]
    return [f"s_cmp_gt_u32 %{KF}, {cond}",
            f"s_cselect_b32 s{S_T1}, {step}, 0",
            f"s_add_u32 s{G}, s{G}, s{S_T1}", f"s_addc_u32 s{G + 1}, s{G + 1}, 0"]


def weave(mf, reads, pairs, first, every):
    """One MFMA, then one other instruction (plus the address add a read may carry): load number j
    puts its m0 write after MFMA first + every*j and the load after the next MFMA; the reads take
    the free places from the start."""
    if len(reads) + 2 * len(pairs) > len(mf):
        # small tile: more other instructions than MFMAs.  Groups (a read with its address add, or a
        # load with its m0 write and the wait state between them) are dealt evenly over the MFMAs,
        # a load after every fourth read.
        groups, rd = [], list(reads)
        ld = [a + ["s_nop 0"] + b for a, b in pairs]
        while rd or ld:
            groups += rd[:4]
            rd = rd[4:]
            if ld:
                groups.append(ld.pop(0))
        out, g = [], 0
        for k, m in enumerate(mf):
            out.append(m)
            upto = (k + 1) * len(groups) // len(mf)
            while g < upto:
                out += groups[g]
                g += 1
        return out
    slots = [None] * len(mf)
    for j, (a, b) in enumerate(pairs):
        slots[first + every * j] = a
        slots[first + every * j + 1] = b
    free = [k for k, s in enumerate(slots) if s is None]
    assert len(reads) <= len(free)
    for k, r in zip(free, reads):
        slots[k] = r
    out = []
    for m, s in zip(mf, slots):
        out.append(m)
        out += s or []
    return out


def rotate():
    return [f"s_mov_b32 s{S_T0}, s{S_ACUR}", f"s_mov_b32 s{S_ACUR}, s{S_ANXT}", f"s_mov_b32 s{S_ANXT}, s{S_ANN}",
            f"s_mov_b32 s{S_ANN}, s{S_T0}",
            f"s_mov_b32 s{S_T0}, s{S_BCUR}", f"s_mov_b32 s{S_BCUR}, s{S_BNXT}", f"s_mov_b32 s{S_BNXT}, s{S_T0}"]


def body(nn, loads_on, last):
    L = []
    # step 0
    reads = frag_reads(nn, 1, S_ACUR, S_BCUR, 1)
    pre, pairs = unit_loads(S_ANN, "A", range(NB)) if loads_on else ([], [])
    L += pre
    L += weave([mfma(0, i, j) for i, j in BLOCKS], reads, pairs, 2, 7)
    if loads_on:
        L += advance("A")
    if last:
        L += ["s_waitcnt lgkmcnt(0)"]
    else:
        L += [f"s_waitcnt vmcnt({NB if loads_on else 0}) lgkmcnt(0)", "s_barrier"]
    # step 1
    reads = [] if last else frag_reads(nn, 0, S_ANXT, S_BNXT, 0)
    pre, pairs = unit_loads(S_BCUR, "B", range(NB)) if loads_on else ([], [])
    L += pre
    L += weave([mfma(1, i, j) for i, j in BLOCKS], reads, pairs, 1, 4)
    if loads_on:
        L += advance("B")
    if not last:
        L += ["s_waitcnt lgkmcnt(0)"]
    return L


def build(nn):
    L = []
    L += [f"s_mov_b64 s[{S_GA}:{S_GA + 1}], %{GA}", f"s_mov_b64 s[{S_GB}:{S_GB + 1}], %{GB}",
          f"s_sub_u32 s{S_CNT}, %{KF}, 2",
          f"s_mov_b32 s{S_ACUR}, {A_BASES[0]}", f"s_mov_b32 s{S_ANXT}, {A_BASES[1]}", f"s_mov_b32 s{S_ANN}, {A_BASES[2]}",
          f"s_mov_b32 s{S_BCUR}, {B_BASES[0]}", f"s_mov_b32 s{S_BNXT}, {B_BASES[1]}"]
    for n, (sa, sb) in enumerate(((S_ACUR, S_BCUR), (S_ANXT, S_BNXT))):
        for which, sd in (("A", sa), ("B", sb)):
            L += unit_loads_flat(sd, which, range(NB))
            L += advance(which, cond=1) if n == 0 else advance(which)
    L += build_zero()                                  # while the first two stages are on their way
    L += [f"s_waitcnt vmcnt({2 * NB})", "s_barrier"]
    for r in frag_reads(nn, 0, S_ACUR, S_BCUR, 0):
        L += r
    L += ["s_waitcnt lgkmcnt(0)"]
    L += [f"s_cmp_lt_u32 %{KF}, 3", "s_cbranch_scc1 2f"]
    L.append("1:")
    L += body(nn, True, False)
    L += rotate()
    L += [f"s_sub_u32 s{S_CNT}, s{S_CNT}, 1", f"s_cmp_lg_u32 s{S_CNT}, 0", "s_cbranch_scc1 1b"]
    L.append("2:")
    L += [f"s_cmp_lt_u32 %{KF}, 2", "s_cbranch_scc1 3f"]
    L += body(nn, False, False)
    L += rotate()
    L.append("3:")
    L += body(nn, False, True)
    L.append("s_waitcnt vmcnt(0)")
    L += MFMA_DRAIN
    return L


def build_kstep32(nn):
    """One 32-wide k-step on a register-staged 64-k tile (K remainder, LoRA term): read the
    fragments, wait, MFMAs.  Operands: %0, %1 A fragment addresses (first / second read); B
    addresses %2, %3 (K-contiguous W) or one per 16-column block from %2 on (N-contiguous W), the
    32-k half already in them; last operand: SGPR mask of this wavefront's 16-row blocks -- a block
    whose bit is clear holds only zero rows of the activation-side tile (rows of other segments in a
    LoRA step), so its reads and MFMAs are skipped."""
    mask = f"%{2 + NB}" if nn else "%4"
    L = [f"s_cmp_eq_u32 {mask}, 0", "s_cbranch_scc1 19f"]
    reads = frag_reads(nn, 0, None, None, 0, va=["%0", "%1"], vb=[f"%{2 + j}" for j in range(NB)])
    a_reads, b_reads = reads[:2 * NB], reads[2 * NB:]   # A: q-major (NB blocks of read 0, then NB of read 1)
    for r in b_reads:
        L += r
    for i in range(NB):
        L += [f"s_bitcmp1_b32 {mask}, {i}", f"s_cbranch_scc0 {20 + i}f"]
        L += a_reads[i] + a_reads[NB + i]
        L.append(f"{20 + i}:")
    L.append("s_waitcnt lgkmcnt(0)")
    for i in range(NB):
        L += [f"s_bitcmp1_b32 {mask}, {i}", f"s_cbranch_scc0 {30 + i}f"]
        L += [mfma(0, i, j) for j in range(NB)]
        L.append(f"{30 + i}:")
    L += MFMA_DRAIN
    L.append("19:")
    return L


def build_zero():
    return [f"v_accvgpr_write_b32 a{n}, 0" for n in range(4 * NB * NB)] + ["s_nop 3"]


def build_stage_out():
    """The whole wavefront tile, rounded to bf16, into the LDS staging tile.  %0: LDS byte address of
    this lane's (m = l%16, n = 4(l/16)) inside the wavefront's part of the tile."""
    L = []
    for n, (i, j) in enumerate(BLOCKS):
        t = 128 + (n % 8) * 6
        b = 4 * (NB * i + j)
        for e in range(4):
            L.append(f"v_accvgpr_read_b32 v{t + e}, a{b + e}")
        L.append(f"v_cvt_pk_bf16_f32 v{t + 4}, v{t}, v{t + 1}")
        L.append(f"v_cvt_pk_bf16_f32 v{t + 5}, v{t + 2}, v{t + 3}")
        L.append(f"ds_write_b64 %0, v[{t + 4}:{t + 5}] offset:{i * 16 * C_PITCH + j * 32}")
    L.append("s_waitcnt lgkmcnt(0)")
    return L


def build_store_partial():
    """All accumulators as fp32 to global memory in register order: block b of a wavefront is 1 KiB,
    16 bytes per lane.  %0: byte offset of this lane's 16 bytes of block 0 inside the partial tile
    (wave * NB * NB KiB + lane * 16); %1: 64-bit base of the partial tile (SGPR pair)."""
    L = [f"v_mov_b32 v{VT}, %0"]
    for b in range(NB * NB):
        L.append(f"global_store_dwordx4 v{VT}, a[{4 * b}:{4 * b + 3}], %1 offset:{(b % 4) * 1024}")
        if b % 4 == 3 and b != NB * NB - 1:
            L.append(f"v_add_u32 v{VT}, 4096, v{VT}")
    L.append("s_waitcnt vmcnt(0)")
    return L


def emit(name, lines):
    out = [f"#define {name} \\"]
    for l in lines:
        out.append(f'    "{l}\\n\\t" \\')
    out.append('    ""')
    return "\n".join(out)


def section(prefix):
    """The templates of the configured tile under the macro prefix `prefix`."""
    vclob = ", ".join(f'"v{r}"' for r in range(VT, VTOP))
    aclob = ", ".join(f'"a{r}"' for r in range(4 * NB * NB))
    return f"""// ---- {32 * NB}x{32 * NB} tile: a wavefront owns {NB}x{NB} blocks, block (i, j) in a[4({NB}i+j) : 4({NB}i+j)+3].
// Main loop operands: %0-%3 A fragment lane offsets inside an A unit (32-k step 0 first / second
// read, step 1 first / second read); %{VB[0]}-%{VB[-1]} B fragment lane offsets inside a B unit (K-contiguous W:
// as for A in %4-%7; N-contiguous W: one per 16-column block); %{AV[0]}-%{AV[-1]} / %{BV[0]}-%{BV[-1]} global byte offsets
// of this lane's {NB} A / {NB} B loads per stage; %{GA},%{GB} global base of the A / B stage (64-bit SGPR);
// %{STRIDE_B} byte stride of B between stages; %{KF} number of 64-k stages (>= 1); %{SWA} LDS byte address of the
// dynamic segment + this wavefront's first load inside a unit (wave * {1024 * NB}).  LDS: units of
// {UNIT // 1024} KiB, A at unit 0/1/2, B at unit 3/4.  Fixed registers: s80-s91, v{VT}-v{VTOP - 1} (fragment sets at
// v{F[0]} and v{F[1]}), a0-a{4 * NB * NB - 1}.
{emit(prefix + "_LOOP_NT", build(False))}

{emit(prefix + "_LOOP_NN", build(True))}

{emit(prefix + "_KSTEP32_NT", build_kstep32(False))}

{emit(prefix + "_KSTEP32_NN", build_kstep32(True))}

{emit(prefix + "_ZERO", build_zero())}

{emit(prefix + "_STAGE_OUT", build_stage_out())}

{emit(prefix + "_STORE_PARTIAL", build_store_partial())}

#define {prefix}_VCLOBBERS {vclob}
#define {prefix}_ACLOBBERS {aclob}
"""


def main():
    here = os.path.dirname(os.path.abspath(__file__))
    sclob = ", ".join(f'"s{r}"' for r in range(80, 92))
    configure(8)
    big = section("SYMB_GEMM16")
    configure(4)
    small = section("SYMB_GEMM16S")
    text = f"""// GENERATED by gen_gemm16_asm.py -- do not edit by hand.
// Assembly of the 4-wavefront base GEMM on v_mfma_f32_16x16x32_bf16 for gfx950, for a 256x256 tile
// (macros SYMB_GEMM16_*) and a 128x128 tile (SYMB_GEMM16S_*).  The accumulators are not operands:
// every template names the accumulation registers literally.  The main loop zeroes the
// accumulators itself (after issuing its first loads); *_ZERO is for a K extent without a single
// full stage.
#pragma once
{big}
{small}
#define SYMB_GEMM16_SCLOBBERS {sclob}
"""
    with open(os.path.join(here, "gemm16_asm.hpp"), "w") as f:
        f.write(text)


if __name__ == "__main__":
    main()
