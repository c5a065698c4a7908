"""Builds libperq.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libperq.so")

SOURCES = ["perq_host.cpp", "perq_colabs.hip", "perq_butterfly.hip", "perq_mfma.hip", "perq_api.hip",
           "perq_gemm.hip", "perq_qerr.hip", "perq_npo2.hip", "perq_npo2_12.hip", "perq_npo2_76.hip", "perq_npo2_32.hip"]

# -packed-fp32-ops: keep the compiler from fusing fp32 pairs into packed VALU instructions.
HIP_FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-ffp-contract=off",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             # keep the one-lane ticket atomic of the matrix-core kernel as written: the wave-level
             # rewrite of uniform atomics reads the result back at once and stalls on it
             "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
             "-Wall", "-Wno-unused-command-line-argument"]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", shutil.which("hipcc")):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def build(verbose: bool = False) -> str:
    """Compile every source and link libperq.so; always recompiles."""
    objdir = os.path.join(PKG, "_build")
    os.makedirs(objdir, exist_ok=True)
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(objdir, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc(), *HIP_FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
               "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for src, cmd, pr in procs:
        out, _ = pr.communicate()
        out = "\n".join(l for l in out.splitlines() if "not a recognized feature" not in l)
        if pr.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{' '.join(cmd)}\n{out}")
        if verbose and out.strip():
            print(out)
    link = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    res = subprocess.run(link, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stdout}")
    return LIB


def check_table_reads() -> int:
    """Compiler check for the prepared-form reads of the matrix-core kernel (perq_mfma.hip).

    The kernel issues eight 16-byte loads as instructions, waits for them by count and only then hands
    the eight register tuples back to the compiler (a comment line in the assembly lists them).  Were the
    compiler to move one of the tuples in between, it would copy registers whose data have not arrived.
    This compiles the file to assembly (about three minutes) and checks, for every kernel variant, that
    the tuples handed back are the ones the loads were given.  Returns the number of variants checked;
    raises on a mismatch.  Run after a compiler upgrade: `python -m paper_2601_22347_amd.build --check-table-reads`."""
    import re
    import tempfile
    with tempfile.TemporaryDirectory() as tmp:
        asm = os.path.join(tmp, "perq_mfma.s")
        flags = [f for f in HIP_FLAGS if f != "-fPIC"]
        cmd = [hipcc(), *flags, "--offload-device-only", "-S", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
               "-x", "hip", os.path.join(CSRC, "perq_mfma.hip"), "-o", asm]
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc failed:\n{res.stdout}")
        text = open(asm).read()
    checked = 0
    for m in re.finditer(r"\n(_ZN4perq\S*mfma_kernel\S*): +; @", text):
        body = text[m.end():text.index("s_endpgm", m.end())].split("\n")
        handed = [l for l in body if "table reads have landed in" in l]
        if not handed:
            continue
        loads = [re.search(r"global_load_dwordx4 (v\[\d+:\d+\])", body[i + 1]).group(1)
                 for i, l in enumerate(body[:-1])
                 if "#ASMSTART" in l and re.search(r"global_load_dwordx4 v\[\d+:\d+\], v\[\d+:\d+\], off\s*$", body[i + 1])]
        for l in handed:
            regs = sorted(re.findall(r"v\[\d+:\d+\]", l))
            if len(loads) % 8 != 0 or regs not in (sorted(loads[:8]), sorted(loads[-8:])):
                raise RuntimeError(f"{m.group(1)}: loads into {loads}, handed back {regs}")
            checked += 1
    if checked == 0:
        raise RuntimeError("no kernel variant with the prepared-form reads found")
    return checked


if __name__ == "__main__":
    import sys
    if "--check-table-reads" in sys.argv:
        print(check_table_reads(), "kernel variants checked")
    else:
        print(build(verbose=True))
