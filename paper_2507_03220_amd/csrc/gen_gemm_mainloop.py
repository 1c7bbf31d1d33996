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

Why 64-k stages: the L2 serves one request per channel and clock whatever its size, so a
K-contiguous operand loaded as 64-byte row pieces (32 k) costs twice the L2 cycles of
whole 128-byte lines (64 k); with 256 CUs loading, half-line requests alone saturate the
L2 at about the rate the matrix pipes consume.  A 64-k stage of one operand is a 32 KiB
unit; 160 KiB of LDS hold a ring of three A units and two B units.

Per iteration (one 64-k stage P, four 16-k steps, fragment sets F0/F1 alternating):
  k-step 0,1: MFMAs while the next k-step's fragments are read; the eight loads of
              A(P+2) go out, one per four MFMAs, into the unit freed by the previous barrier;
  k-step 2:   MFMAs while the k-step-3 fragments are read (last reads of stage P); then wait
              for this wavefront's loads of stage P+1, barrier (stage P+1 complete for
              everybody, both units of stage P free);
  k-step 3:   MFMAs while the first fragments of stage P+1 are read; the eight loads of
              B(P+2) go out, one per two MFMAs, into B(P)'s unit.
"""
import os

F = {0: 192, 1: 224}          # first VGPR of fragment set 0 / 1 (A: 4x4 regs, then B: 4x4 regs)
VT = 180                      # address temporaries v180..v187
S_GA, S_GB = 80, 82
S_CNT, S_ACUR, S_ANXT, S_ANN, S_BCUR, S_BNXT, S_T0, S_T1 = range(84, 92)
LOAD_MOD = (" " + os.environ["SYMB_GEN_LOAD_MOD"]) if os.environ.get("SYMB_GEN_LOAD_MOD") else ""   # tuning: cache policy bits
UNIT = 32768                  # one operand's 64-k stage
A_BASES = (0, UNIT, 2 * UNIT)
B_BASES = (3 * UNIT, 4 * UNIT)

# operand numbers
ACC0 = 0
VA = (16, 17, 18, 19)         # A fragment lane offsets, k-step 0..3
VB = (20, 21, 22, 23)         # NT: B lane offsets, k-step 0..3; NN: per 32-column block
AV = tuple(range(24, 32))     # global byte offsets of this lane's 8 A loads
BV = tuple(range(32, 40))     # global byte offsets of this lane's 8 B loads
GA, GB, STRIDE_B, KF, SWA = 40, 41, 42, 43, 44


# The compiler does not look inside an assembly statement: whatever it places right after one
# (a copy out of an accumulation register, say) must not meet a matrix instruction that is still
# writing its result.  Every template therefore ends with more wait states than the longest
# matrix-result hazard needs.
MFMA_DRAIN = ["s_nop 15", "s_nop 7"]


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


def frag_reads(nn, dst, sa, sb, ks):
    """Address setup + the LDS reads that fill fragment set `dst` with k-step `ks` of the stage
    whose A / B units start at SGPR `sa` / `sb`."""
    setup, reads = [], []
    setup.append(f"v_add_u32 v{VT}, s{sa}, %{VA[ks]}")
    for i in range(4):
        reads.append(f"ds_read_b128 {fa(dst, i)}, v{VT} offset:{4096 * i}")
    if not nn:
        setup.append(f"v_add_u32 v{VT + 1}, s{sb}, %{VB[ks]}")
        for j in range(4):
            reads.append(f"ds_read_b128 {fb(dst, j)}, v{VT + 1} offset:{4096 * j}")
    else:
        for j in range(4):
            setup.append(f"v_add_u32 v{VT + 1 + j}, s{sb}, %{VB[j]}")
        for j in range(4):
            for h in range(2):
                reads.append(f"ds_read_b64_tr_b16 {fb_half(dst, j, h)}, v{VT + 1 + j} offset:{8192 * ks + 2048 * h}")
    return setup, reads


def unit_loads(sdst, which, js):
    """global->LDS loads number `js` (of 8) of one operand's 64-k unit into the unit at SGPR `sdst`."""
    V, G = (AV, S_GA) if which == "A" else (BV, S_GB)
    return [[f"s_add_u32 s{S_T0}, s{sdst}, %{SWA}", f"s_add_u32 m0, s{S_T0}, {1024 * j}", "s_nop 0",
             f"global_load_lds_dwordx4 %{V[j]}, s[{G}:{G + 1}]" + LOAD_MOD] for j in js]


def advance(which, cond=None):
    """Moves an operand's global base pointer to its next 64-k stage; with `cond` only if
    KF > cond (the prologue must not run past a one-stage problem)."""
    G, step = (S_GA, "128") if which == "A" else (S_GB, f"%{STRIDE_B}")
    if cond is None:
        pre = [f"s_mov_b32 s{S_T1}, {step}"] if which == "B" else []
        src = f"s{S_T1}" if which == "B" else step
        return pre + [f"s_add_u32 s{G}, s{G}, {src}", f"s_addc_u32 s{G + 1}, s{G + 1}, 0"]
    return [f"s_cmp_gt_u32 %{KF}, {cond}",
            f"s_cselect_b32 s{S_T1}, {step}, 0",
            f"s_add_u32 s{G}, s{G}, s{S_T1}", f"s_addc_u32 s{G + 1}, s{G + 1}, 0"]


def spread(mf, reads, loads, every):
    """Reads go one (or two) per MFMA from the start; loads go one per `every` MFMAs so the
    vector memory queue never backs up into the MFMA stream."""
    out = []
    per = 2 if len(reads) > 8 else 1
    r = list(reads)
    ld = list(loads)
    for k, m in enumerate(mf):
        out.append(m)
        for _ in range(per):
            if r:
                out.append(r.pop(0))
        if ld and k % every == every - 1:
            out.extend(ld.pop(0))
    assert not r and not ld
    return out


def rotate():
    return [f"s_mov_b32 s{S_T0}, s{S_ACUR}", f"s_mov_b32 s{S_ACUR}, s{S_ANXT}", f"s_mov_b32 s{S_ANXT}, s{S_ANN}",
            f"s_mov_b32 s{S_ANN}, s{S_T0}",
            f"s_mov_b32 s{S_T0}, s{S_BCUR}", f"s_mov_b32 s{S_BCUR}, s{S_BNXT}", f"s_mov_b32 s{S_BNXT}, s{S_T0}"]


def body(nn, loads_on, last, no_reads=False):
    """One 64-k stage P.  loads_on: issue A(P+2) and B(P+2) (steady state; the stage exists);
    otherwise nothing younger than stage P+1 is in flight at the wait.  last: no next stage,
    so no wait, no barrier and no fragment reads in k-step 3."""
    L = []
    plan = [  # (MFMA set, fragments to read: (set, A unit, B unit, k-step), loads, one load per .. MFMAs, advance)
        (0, (1, S_ACUR, S_BCUR, 1), unit_loads(S_ANN, "A", range(0, 4)), 4, None),
        (1, (0, S_ACUR, S_BCUR, 2), unit_loads(S_ANN, "A", range(4, 8)), 4, "A"),
        (0, (1, S_ACUR, S_BCUR, 3), [], 4, None),
        (1, (0, S_ANXT, S_BNXT, 0), unit_loads(S_BCUR, "B", range(8)), 2, "B"),
    ]
    for ks, (mset, (dst, sa, sb, rks), loads, every, adv) in enumerate(plan):
        setup, reads = frag_reads(nn, dst, sa, sb, rks)
        if no_reads or (last and ks == 3):
            setup, reads = [], []
        if not loads_on:
            loads, adv = [], None
        L += setup
        L += spread([mfma(mset, i, j) for i in range(4) for j in range(4)], reads, loads, every)
        if adv:
            L += advance(adv)
        if ks == 2 and not last:
            L += [f"s_waitcnt vmcnt({8 if loads_on else 0}) lgkmcnt(0)", "s_barrier"]
        elif not (last and ks == 3):
            L += ["s_waitcnt lgkmcnt(0)"]
    return L


def build(nn, no_loads=False, no_reads=False):
    """Load issue order: A(0) B(0) A(1) B(1) in the prologue; steady iteration P (P <= KF-3)
    issues A(P+2) during k-steps 0-1 and B(P+2) during k-step 3, and at its wait stage P+1 must
    have landed while the eight loads of A(P+2) may still be in flight.  The last two stages run
    a copy of the body without loads, so nothing is fetched twice and nothing is in flight when
    the loop ends."""
    L = []
    L += [f"s_mov_b64 s[{S_GA}:{S_GA + 1}], %{GA}", f"s_mov_b64 s[{S_GB}:{S_GB + 1}], %{GB}",
          f"s_sub_u32 s{S_CNT}, %{KF}, 2",
          f"s_mov_b32 s{S_ACUR}, {A_BASES[0]}", f"s_mov_b32 s{S_ANXT}, {A_BASES[1]}", f"s_mov_b32 s{S_ANN}, {A_BASES[2]}",
          f"s_mov_b32 s{S_BCUR}, {B_BASES[0]}", f"s_mov_b32 s{S_BNXT}, {B_BASES[1]}"]
    # stage 0, then stage 1 (a one-stage problem fetches stage 0 twice; nobody reads the copy)
    for n, (sa, sb) in enumerate(((S_ACUR, S_BCUR), (S_ANXT, S_BNXT))):
        for which, sd in (("A", sa), ("B", sb)):
            for g in unit_loads(sd, which, range(8)):
                L += g
            L += advance(which, cond=1) if n == 0 else advance(which)
    L += ["s_waitcnt vmcnt(16)", "s_barrier"]
    setup, reads = frag_reads(nn, 0, S_ACUR, S_BCUR, 0)
    L += setup + reads + ["s_waitcnt lgkmcnt(0)"]
    L += [f"s_cmp_lt_u32 %{KF}, 3", "s_cbranch_scc1 2f"]
    # ---- steady loop: stages 0 .. KF-3
    L.append("1:")
    L += body(nn, not no_loads, False, no_reads)
    L += rotate()
    L += [f"s_sub_u32 s{S_CNT}, s{S_CNT}, 1", f"s_cmp_lg_u32 s{S_CNT}, 0", "s_cbranch_scc1 1b"]
    # ---- stage KF-2 (if there is one), then stage KF-1
    L.append("2:")
    L += [f"s_cmp_lt_u32 %{KF}, 2", "s_cbranch_scc1 3f"]
    L += body(nn, False, False, no_reads)
    L += rotate()
    L.append("3:")
    L += body(nn, False, True, no_reads)
    L.append("s_waitcnt vmcnt(0)")
    L += MFMA_DRAIN
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
    L += MFMA_DRAIN
    return L


def emit(name, lines):
    out = [f"#define {name} \\"]
    for l in lines:
        out.append(f'    "{l}\\n\\t" \\')
    out.append('    ""')
    return "\n".join(out)


def main():
    here = os.path.dirname(os.path.abspath(__file__))
    clob = ['"memory"', '"scc"'] + [f'"s{r}"' for r in range(80, 92)] + [f'"v{r}"' for r in range(VT, 256)]
    text = f"""// GENERATED by gen_gemm_mainloop.py -- do not edit by hand.
// Main loop of the 256x256 / 4-wavefront base GEMM for gfx950 as inline-assembly templates.
// Operands: %0-%15 accumulators (AGPR, i-major: block (i, j) is %(4i+j)); %16-%19 A fragment
// lane offsets for k-step 0..3 inside an A unit; %20-%23 B fragment lane offsets inside a B unit
// (K-contiguous W: k-step 0..3; N-contiguous W: one per 32-column block); %24-%31 / %32-%39
// global byte offsets of this lane's eight A / eight B loads per stage; %40,%41 global base of
// the A / B stage (64-bit SGPR); %42 byte stride of B between stages; %43 number of 64-k stages
// (>= 1); %44 LDS byte address of the dynamic segment + this wavefront's first load inside a
// unit (wave * 8192).  LDS: A units at 0/32/64 KiB, B units at 96/128 KiB of the segment.
// Fixed registers: s80-s91, v{VT}-v255 (fragment sets at v{F[0]} and v{F[1]}).
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
