"""The 16x16x32 GEMM kernel keeps its accumulators in a0..a255 behind the compiler's back: every
instruction that touches an accumulation register sits inside one of its assembly templates.  This
test compiles the device code to assembly and checks that the compiler-generated code of those
kernels between the templates names no accumulation register and spills nothing that could land in
one.  No GPU needed (hipcc cross-compiles)."""
import os
import re
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2507_03220_amd", "csrc", "symb_api.hip")


@pytest.fixture(scope="module")
def device_asm():
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "symb.s")
        subprocess.check_call([hipcc, "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-Xclang", "-target-feature",
                               "-Xclang", "-packed-fp32-ops", "--cuda-device-only", "-S", "-o", out, SRC],
                              stderr=subprocess.DEVNULL)
        return open(out).read()


def _kernels(text):
    """{mangled name: [(line, inside an assembly template?)]} of the symb_gemm16_kernel instantiations."""
    out, name, inside = {}, None, False
    for raw in text.splitlines():
        s = raw.strip()
        m = re.match(r"^(_ZN4symb18symb_gemm16_kernel\w+):", s)
        if m:
            name, inside = m.group(1), False
            out[name] = []
            continue
        if s.startswith(".Lfunc_end"):
            name = None
        if name is None:
            continue
        if "ASMSTART" in s:
            inside = True
        elif "ASMEND" in s:
            inside = False
        else:
            out[name].append((s.split(";")[0], inside))
    return out


def test_compiler_code_never_touches_accumulation_registers(device_asm):
    ks = _kernels(device_asm)
    assert len(ks) == 8, sorted(ks)               # {256x256, 128x128 tile} x {K-contiguous, N-contiguous weight} x {plain, full epilogue}
    for name, lines in ks.items():
        inside = [c for c, i in lines if i]
        outside = [c for c, i in lines if not i]
        assert sum("v_mfma_f32_16x16x32_bf16" in c for c in inside) > (500 if "ILi8E" in name else 120), name
        offenders = [c for c in outside if re.search(r"\ba\d+\b|\ba\[\d+", c) or "accvgpr" in c or "v_mfma" in c]
        assert not offenders, (name, offenders[:5])


def test_no_kernel_uses_scratch_memory(device_asm):
    # register spills and stack arrays would show as a private segment; every kernel of the library fits its registers
    found = re.findall(r"\.amdhsa_kernel (\S+)(.*?)\.end_amdhsa_kernel", device_asm, re.S)
    assert len(found) >= 20, [n for n, _ in found]
    for name, body in found:
        m = re.search(r"\.amdhsa_private_segment_fixed_size (\d+)", body)
        assert m and int(m.group(1)) == 0, (name, m and m.group(1))
    for name, lines in _kernels(device_asm).items():
        assert not [c for c, _ in lines if "scratch_" in c], name


def test_kernel_descriptors_claim_the_whole_register_file(device_asm):
    # 256x256 tile: 256 architectural + 256 accumulation registers per lane, one wavefront per SIMD;
    # 128x128 tile: 192 + 64, two wavefronts per SIMD (two workgroups of 80 KiB LDS per CU)
    n = 0
    for m in re.finditer(r"\.amdhsa_kernel (_ZN4symb18symb_gemm16_kernel\w+)(.*?)\.end_amdhsa_kernel", device_asm, re.S):
        body, big = m.group(2), "ILi8E" in m.group(1)
        assert re.search(r"\.amdhsa_next_free_vgpr %d\b" % (512 if big else 256), body), m.group(1)
        assert re.search(r"\.amdhsa_accum_offset %d\b" % (256 if big else 192), body), m.group(1)
        n += 1
    assert n == 8


def _regs(operand):
    """VGPR numbers named by an operand like v5 or v[6:9]."""
    m = re.fullmatch(r"v\[(\d+):(\d+)\]", operand)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.fullmatch(r"v(\d+)", operand)
    return {int(m.group(1))} if m else set()


def test_results_of_assembly_issued_loads_are_untouched_until_their_wait(device_asm):
    # The skinny and small-batch kernels request LDS data from assembly statements and wait for
    # it with an s_waitcnt of their own; the compiler does not know the registers are still in flight.
    # Nothing it generates between such a request and the next explicit wait may read or write them
    # (a register copy placed there would copy stale data; requesting the skinny kernel's adapter rows a
    # slice ahead, in registers that lived across the loop edge, produced exactly that).  Checked per
    # straight-line stretch of the generated code: a label ends the stretch.
    checked = 0
    for m in re.finditer(r"^(_ZN4symb(?:18symb_skinny_kernel|19symb_rowgemv_kernel|21symb_lora_grad_kernel)\w+):(.*?)^\.Lfunc_end", device_asm, re.S | re.M):
        pending, inside = set(), False
        for raw in m.group(2).splitlines():
            s = raw.strip().split(";")[0].strip() if "ASM" not in raw else raw.strip()
            if "ASMSTART" in s:
                inside = True
                continue
            if "ASMEND" in s:
                inside = False
                continue
            if s.endswith(":") or re.match(r"^\.LBB\w+:", s):
                pending.clear()
                continue
            if not s or s.startswith("."):
                continue
            op, _, rest = s.partition(" ")
            args = [a.strip() for a in rest.split(",")]
            if inside and (op == "global_load_dwordx4" or op == "ds_read_b128"):
                pending |= _regs(args[0])
                checked += 1
                continue
            if inside and op == "s_waitcnt":
                if "vmcnt" in rest or "lgkmcnt" in rest:
                    pending.clear()
                continue
            touched = set()
            for a in args:
                for tok in re.findall(r"v\[\d+:\d+\]|v\d+", a):
                    touched |= _regs(tok)
            assert not (touched & pending), (m.group(1), s, sorted(touched & pending))
    assert checked > 50
