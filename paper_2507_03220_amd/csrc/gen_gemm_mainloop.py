#!/usr/bin/env python3
"""Writes gemm_mainloop_asm.hpp: the gfx950 main loop of the 256x256 base GEMM as two
inline-assembly templates (W read K-contiguous / N-contiguous).

Run `python gen_gemm_mainloop.py` after changing the schedule; the output is committed,
the build does not run this script.

Why assembly: with 4 wavefronts per workgroup each wavefront owns 128x128 of C
(16 accumulator blocks = all 256 accumulation registers).  Left to the compiler this
configuration shuffles accumulators between register files inside the loop.  Here the
accumulators are pinned ("+a" operands), the two fragment sets live in fixed registers,
and every LDS read and global->LDS load is placed by hand between the MFMAs.

Per iteration (one 32-k stage of a 4-deep LDS ring):
  k-step 0: 16 MFMAs on fragment set F0 while the k-step-1 fragments of this stage
            are read into F1;
  wait for this wavefront's loads of the next stage, barrier (next stage complete for
            everybody, this stage free);
  k-step 1: 16 MFMAs on F1 while the next stage's k-step-0 fragments are read into F0
            and the loads that refill this stage's buffer are issued.
"""
import os

F = {0: 192, 1: 224}          # first VGPR of fragment set 0 / 1 (A: 4x4 regs, then B: 4x4 regs)
VT = 180                      # address temporaries v180..v187
S_GA, S_GB, S_CNT, S_CUR, S_NXT, S_ADVA, S_T0, S_T1, S_T2, S_ADVB, S_WB, S_PRV = 80, 82, 84, 85, 86, 87, 88, 89, 90, 91, 92, 93
STAGE_BYTES = 32768
RING_MASK = 4 * STAGE_BYTES - 1
A_STAGE = 16384

# operand numbers
ACC0 = 0
VA = (16, 17)                 # A fragment lane offsets for k-step 0 / 1
VB = (18, 19, 20, 21)         # NT: B lane offsets k-step 0 / 1 (20, 21 unused); NN: per n-block offsets
AV = (22, 23, 24, 25)         # global byte offsets of this lane's 4 A loads
BV = (26, 27, 28, 29)         # global byte offsets of this lane's 4 B loads
GA, GB, STRIDE_B, KF, SWA = 30, 31, 32, 33, 34


def fa(s, i):
    b = F[s] + 4 * i
    return f"v[{b}:{b + 3}]"


def fb(s, j):
    b = F[s] + 16 + 4 * j
    return f"v[{b}:{b + 3}]"


def fb_half(s, j, h):
    b = F[s] + 16 + 4 * j + 2 * h
    return f"v[{b}:{b + 1}]"


def mfma(s, i, j):
    return f"v_mfma_f32_32x32x16_bf16 %{ACC0 + 4 * i + j}, {fb(s, j)}, {fa(s, i)}, %{ACC0 + 4 * i + j}"


def frag_reads(nn, dst, sbase, ks):
    """Address setup + the LDS reads that fill fragment set `dst` from the stage at SGPR `sbase`."""
    setup, reads = [], []
    setup.append(f"v_add_u32 v{VT}, s{sbase}, %{VA[ks]}")
    for i in range(4):
        reads.append(f"ds_read_b128 {fa(dst, i)}, v{VT} offset:{2048 * i}")
    if not nn:
        setup.append(f"v_add_u32 v{VT + 1}, s{sbase}, %{VB[ks]}")
        for j in range(4):
            reads.append(f"ds_read_b128 {fb(dst, j)}, v{VT + 1} offset:{2048 * j}")
    else:
        for j in range(4):
            setup.append(f"v_add_u32 v{VT + 1 + j}, s{sbase}, %{VB[j]}")
        for j in range(4):
            for h in range(2):
                reads.append(f"ds_read_b64_tr_b16 {fb_half(dst, j, h)}, v{VT + 1 + j} offset:{8192 * ks + 2048 * h}")
    return setup, reads


def half_issue(sdst, which):
    """Four global->LDS loads (the A or the B half of one stage) into the buffer at SGPR `sdst`,
    then the clamped advance of that operand's global base pointer."""
    loads = []
    if which == "A":
        for j in range(4):
            pre = f"s_add_u32 m0, s{sdst}, %{SWA}" if j == 0 else "s_add_u32 m0, m0, 0x400"
            loads.append([pre, "s_nop 0", f"global_load_lds_dwordx4 %{AV[j]}, s[{S_GA}:{S_GA + 1}]"])
        adv = [f"s_cmp_lg_u32 s{S_ADVA}, 0",
               f"s_cselect_b32 s{S_T0}, 64, 0",
               f"s_cselect_b32 s{S_T2}, 1, 0",
               f"s_add_u32 s{S_GA}, s{S_GA}, s{S_T0}", f"s_addc_u32 s{S_GA + 1}, s{S_GA + 1}, 0",
               f"s_sub_u32 s{S_ADVA}, s{S_ADVA}, s{S_T2}"]
    else:
        for j in range(4):
            pre = f"s_add_u32 m0, s{sdst}, s{S_WB}" if j == 0 else "s_add_u32 m0, m0, 0x400"
            loads.append([pre, "s_nop 0", f"global_load_lds_dwordx4 %{BV[j]}, s[{S_GB}:{S_GB + 1}]"])
        adv = [f"s_cmp_lg_u32 s{S_ADVB}, 0",
               f"s_cselect_b32 s{S_T1}, %{STRIDE_B}, 0",
               f"s_cselect_b32 s{S_T2}, 1, 0",
               f"s_add_u32 s{S_GB}, s{S_GB}, s{S_T1}", f"s_addc_u32 s{S_GB + 1}, s{S_GB + 1}, 0",
               f"s_sub_u32 s{S_ADVB}, s{S_ADVB}, s{S_T2}"]
    return loads, adv


def spread(mf, reads, loads):
    """Reads go one (or two) per MFMA from the start; loads go one per 4 MFMAs so the vector
    memory queue never backs up into the MFMA stream."""
    out = []
    per = 2 if len(reads) > 8 else 1
    r = list(reads)
    ld = list(loads)
    for k, m in enumerate(mf):
        out.append(m)
        for _ in range(per):
            if r:
                out.append(r.pop(0))
        if ld and k % 4 == 3:
            out.extend(ld.pop(0))
    assert not r and not ld
    return out


def interleave(mf, others):
    """One `other` group after each MFMA until they run out, then the remaining MFMAs."""
    out = []
    for k, m in enumerate(mf):
        out.append(m)
        if k < len(others):
            o = others[k]
            out.extend(o if isinstance(o, list) else [o])
    for o in others[len(mf):]:
        out.extend(o if isinstance(o, list) else [o])
    return out


def build(nn, no_loads=False, no_reads=False):
    """Load issue order: A(0) B(0) A(1) B(1) A(2) B(2) A(3) in the prologue; iteration t issues
    B(t+3) during k-step 0 (buffer freed by the previous barrier) and A(t+4) during k-step 1
    (buffer freed by this iteration's barrier).  At iteration t's wait, stage t+1 must have
    landed; four younger half-stages (16 loads) may still be in flight."""
    L = []
    L += [f"s_mov_b64 s[{S_GA}:{S_GA + 1}], %{GA}", f"s_mov_b64 s[{S_GB}:{S_GB + 1}], %{GB}",
          f"s_mov_b32 s{S_CNT}, %{KF}", f"s_sub_u32 s{S_ADVA}, %{KF}, 1", f"s_sub_u32 s{S_ADVB}, %{KF}, 1",
          f"s_add_u32 s{S_WB}, %{SWA}, {A_STAGE}", f"s_mov_b32 s{S_CUR}, 0"]
    for t in range(4):
        L.append(f"s_mov_b32 s{S_NXT}, {t * STAGE_BYTES}")
        for which in ("A", "B") if t < 3 else ("A",):
            loads, adv = half_issue(S_NXT, which)
            for g in loads:
                L += g
            L += adv
    # s_prv: the buffer freed by the previous barrier (stage t+3 goes there); starts at stage 3's buffer
    L += [f"s_mov_b32 s{S_NXT}, {STAGE_BYTES}", f"s_mov_b32 s{S_PRV}, {3 * STAGE_BYTES}", "s_waitcnt vmcnt(20)", "s_barrier"]
    setup, reads = frag_reads(nn, 0, S_CUR, 0)
    L += setup + reads + ["s_waitcnt lgkmcnt(0)"]
    # ---- loop
    L.append("1:")
    setup, reads = frag_reads(nn, 1, S_CUR, 1)
    loads, adv = half_issue(S_PRV, "B")
    if no_reads:
        reads = []
    if no_loads:
        loads = []
    L += setup
    mf = [mfma(0, i, j) for i in range(4) for j in range(4)]
    L += spread(mf, reads, loads)
    L += adv
    L += ["s_waitcnt vmcnt(16) lgkmcnt(0)", "s_barrier"]
    setup, reads = frag_reads(nn, 0, S_NXT, 0)
    loads, adv = half_issue(S_CUR, "A")
    if no_reads:
        reads = []
    if no_loads:
        loads = []
    L += setup
    mf = [mfma(1, i, j) for i in range(4) for j in range(4)]
    L += spread(mf, reads, loads)
    L += adv
    L += ["s_waitcnt lgkmcnt(0)",
          f"s_mov_b32 s{S_PRV}, s{S_CUR}",
          f"s_mov_b32 s{S_CUR}, s{S_NXT}",
          f"s_add_u32 s{S_NXT}, s{S_NXT}, {STAGE_BYTES}",
          f"s_and_b32 s{S_NXT}, s{S_NXT}, {RING_MASK}",
          f"s_sub_u32 s{S_CNT}, s{S_CNT}, 1",
          f"s_cmp_lg_u32 s{S_CNT}, 0",
          "s_cbranch_scc1 1b",
          "s_waitcnt vmcnt(0)"]
    return L


def build_kstep64(nn):
    """One 16-wide k-step on a register-staged 64-k tile (K remainder, LoRA term): read the
    eight fragments, wait, 16 MFMAs.  Operands: %0-%15 accumulators, %16 A fragment address,
    %17 (K-contiguous W) or %17-%20 (N-contiguous W, one per 32-column block) B addresses."""
    L = []
    for i in range(4):
        L.append(f"ds_read_b128 {fa(0, i)}, %16 offset:{4096 * i}")
    if not nn:
        for j in range(4):
            L.append(f"ds_read_b128 {fb(0, j)}, %17 offset:{4096 * j}")
    else:
        for j in range(4):
            for h in range(2):
                L.append(f"ds_read_b64_tr_b16 {fb_half(0, j, h)}, %{17 + j} offset:{2048 * h}")
    L.append("s_waitcnt lgkmcnt(0)")
    L += [mfma(0, i, j) for i in range(4) for j in range(4)]
    return L


def emit(name, lines):
    out = [f"#define {name} \\"]
    for l in lines:
        out.append(f'    "{l}\\n\\t" \\')
    out.append('    ""')
    return "\n".join(out)


def main():
    here = os.path.dirname(os.path.abspath(__file__))
    clob = ['"memory"', '"scc"'] + [f'"s{r}"' for r in range(80, 94)] + [f'"v{r}"' for r in range(VT, 256)]
    text = f"""// GENERATED by gen_gemm_mainloop.py -- do not edit by hand.
// Main loop of the 256x256 / 4-wavefront base GEMM for gfx950 as inline-assembly templates.
// Operands: %0-%15 accumulators (AGPR, i-major: block (i, j) is %(4i+j)); %16,%17 A fragment
// lane offsets for k-step 0/1; %18-%21 B fragment lane offsets (K-contiguous W: k-step 0/1 in
// %18,%19; N-contiguous W: one per 32-column block); %22-%25 / %26-%29 global byte offsets of
// this lane's four A / four B loads per stage; %30,%31 global base of the A / B stage (64-bit
// SGPR); %32 byte stride of B between stages; %33 number of 32-k stages (>= 1); %34 byte
// offset of this wavefront's first A load inside a stage (wave * 4096).
// Fixed registers: s80-s93, v{VT}-v255 (fragment sets at v{F[0]} and v{F[1]}).
#pragma once
{emit("SYMB_GEMM_LOOP_NT", build(False))}

{emit("SYMB_GEMM_LOOP_NN", build(True))}

{emit("SYMB_GEMM_KSTEP64_NT", build_kstep64(False))}

{emit("SYMB_GEMM_KSTEP64_NN", build_kstep64(True))}

#ifdef SYMB_GEMM_PROBE   // tuning builds only: the same loop without its in-loop global loads / LDS reads
{emit("SYMB_GEMM_LOOP_NT_NOLOAD", build(False, no_loads=True))}

{emit("SYMB_GEMM_LOOP_NT_NOREAD", build(False, no_loads=True, no_reads=True))}
#endif

#define SYMB_GEMM_LOOP_CLOBBERS {", ".join(clob)}
"""
    with open(os.path.join(here, "gemm_mainloop_asm.hpp"), "w") as f:
        f.write(text)


if __name__ == "__main__":
    main()
