"""Builds libsymb.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libsymb.so")
SOURCES = [os.path.join(HERE, "csrc", "symb_api.hip"), os.path.join(HERE, "csrc", "symb_batcher.hip")]
DEPS = SOURCES + [os.path.join(HERE, "csrc", f) for f in
                  ("gemm16_kernel.hpp", "gemm16_asm.hpp", "adapter_kernels.hpp", "symb_device.hpp")] + \
    [os.path.join(os.path.dirname(HERE), "include", f) for f in ("symb.h", "symb_batcher.h")]

FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-shared", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall"]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(d) > t for d in DEPS)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compiles every HIP source into paper_2507_03220_amd/libsymb.so."""
    if not force and not stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + f".tmp{os.getpid()}"
    cmd = [hipcc] + FLAGS + ["-o", tmp] + SOURCES
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if err and verbose:
        print(err, file=sys.stderr)
    os.replace(tmp, LIB)
    return LIB


def build_tool(name: str) -> str:
    """Compiles a stand-alone measurement program (measure/<name>.hip: not part of the library; the
    summaries under profiles/ that quote it give the command) into measure/<name>."""
    out = os.path.join(HERE, "measure", name)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    subprocess.check_call([hipcc, "-O3", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
                           "-packed-fp32-ops", "-o", out, os.path.join(HERE, "measure", name + ".hip")],
                          stderr=subprocess.DEVNULL)
    return out


def build_ceiling() -> str:
    """The MFMA ceiling measurement (measure/mfma_ceiling.hip)."""
    return build_tool("mfma_ceiling")


if __name__ == "__main__":
    if "--ceiling" in sys.argv:
        print(build_ceiling())
    elif "--l2-probe" in sys.argv:
        print(build_tool("l2_lds_probe"))
    else:
        print(build(force=True, verbose=True))
