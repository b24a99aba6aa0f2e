"""Builds the HIP library in-tree: csrc/*.hip + csrc/attn_api.cpp -> libattn_gfx950.so.

hipcc cross-compiles for gfx950 without a GPU.  Usage: python -m paper_2205_14135_amd.build
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libattn_gfx950.so")
SOURCES = ["attn_fwd.hip", "attn_fwd_pp.hip", "attn_bwd.hip", "attn_bwd_dkv.hip", "attn_bwd_dkv_fr.hip", "attn_bwd_dkv_fr128.hip",
           "attn_bwd_dkv_w64.hip", "attn_probe.hip", "attn_api.cpp"]
# Kernels that keep their accumulators in accumulation registers addressed by name in raw MFMA
# statements: builtin MFMA results must then stay in architectural registers (this option), and the
# generated code is checked (check_pinned_agprs below).
PINNED_AGPR_SOURCES = ["attn_bwd_dkv_w64.hip"]
PINNED_AGPR_FLAGS = ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]
FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-x", "hip",
    # packed fp32 VALU forms are switched off on purpose (they have misbehaved on the test machines)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.sep not in c or os.path.exists(c)):
            return c
    raise RuntimeError("hipcc not found")


def check_pinned_agprs(asm_text: str, src: str) -> None:
    """The compiler must not touch the accumulation registers of a kernel that addresses them by
    name: outside the raw statements (between ASMSTART and ASMEND) no instruction may name an
    AGPR, nothing may be spilled and no scratch memory may be used."""
    def regs(operand):
        m = re.match(r"v\[(\d+):(\d+)\]$", operand)
        if m:
            return set(range(int(m.group(1)), int(m.group(2)) + 1))
        m = re.match(r"v(\d+)$", operand)
        return {int(m.group(1))} if m else set()

    in_raw = False
    recent = []   # (line number, registers written) of the last vector ALU instructions outside raw statements
    for n, line in enumerate(asm_text.splitlines(), 1):
        if "#ASMSTART" in line:
            in_raw = True
        elif "#ASMEND" in line:
            in_raw = False
        elif in_raw:
            # A raw MFMA must not read an architectural register that one of the two instructions in
            # front of it wrote with the vector ALU: the compiler puts no wait states before it.
            m = re.match(r"\s*v_mfma_\S+\s+a\[[^\]]+\],\s*(v\[\d+:\d+\]),\s*(v\[\d+:\d+\]),", line)
            if m:
                need = regs(m.group(1)) | regs(m.group(2))
                for ln, written in recent[-2:]:
                    if need & written:
                        raise RuntimeError(f"{src}: raw MFMA at line {n} reads v{sorted(need & written)} written at line {ln}")
                recent.append((n, set()))
        elif not in_raw:
            code0 = line.split(";")[0].strip()
            if code0 and not code0.startswith(".") and not code0.endswith(":"):
                ops = code0.split(None, 1)
                dst = regs(ops[1].split(",")[0].strip()) if len(ops) > 1 and ops[0].startswith("v_") else set()
                recent.append((n, dst))
                del recent[:-4]
            code = line.split(";")[0]
            if code.lstrip().startswith("."):
                m = re.match(r"\s*\.(vgpr_spill_count|sgpr_spill_count|private_segment_fixed_size):\s*(\d+)", code)
                if m and int(m.group(2)) != 0 and m.group(1) != "sgpr_spill_count":
                    raise RuntimeError(f"{src}: {m.group(1)} = {m.group(2)} (must be 0)")
                continue
            if re.search(r"(^|[^A-Za-z0-9_.])a(\[\d|\d)", code):
                raise RuntimeError(f"{src}: compiler-generated code names an AGPR (line {n}): {line.strip()}")


def _compile(src: str, extra) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    flags = [*FLAGS, *extra]
    if src in PINNED_AGPR_SOURCES:
        flags += PINNED_AGPR_FLAGS
        asm = os.path.join(OBJ, os.path.splitext(src)[0] + ".s")
        r = subprocess.run([_hipcc(), *flags, "--cuda-device-only", "-S", os.path.join(CSRC, src), "-o", asm],
                           capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}\n{r.stderr}")
        check_pinned_agprs(open(asm).read(), src)
    cmd = [_hipcc(), *flags, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}\n{r.stderr}")
    return obj


def build(verbose: bool = False, extra_flags=()) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(lambda s: _compile(s, list(extra_flags)), SOURCES))
    cmd = [_hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", *objs, "-o", LIB]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    # a kernel whose host stub went missing would only show up when the library is loaded
    nm = subprocess.run(["nm", "-u", LIB], capture_output=True, text=True)
    missing = [l.split()[-1] for l in nm.stdout.splitlines() if "attn" in l]
    if missing:
        raise RuntimeError("undefined symbols in the built library: " + ", ".join(missing[:5]))
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True, extra_flags=sys.argv[1:])
