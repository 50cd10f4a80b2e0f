"""Build libcraft.so (HIP kernels + host planner + C ABI) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libcraft.so")

SOURCES = ["planner.cpp", "forward.cpp", "route.hip", "router.hip", "dispatch.hip", "load.hip", "ffn.hip", "ffn_packed.hip", "quant.hip", "probe.hip",
           "combine.hip"]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


# Sources whose matrix instructions are written as asm statements, which the compiler's hazard
# pass does not recognise: their emitted code is checked here instead (check_matrix_operands).
ASM_MFMA_SOURCES = {"ffn_packed.hip"}


def _registers(token: str) -> set:
    token = token.strip().rstrip(",")
    m = re.match(r"^([va])\[(\d+):(\d+)\]$", token)
    if m:
        return {(m.group(1), r) for r in range(int(m.group(2)), int(m.group(3)) + 1)}
    m = re.match(r"^([va])(\d+)$", token)
    return {(m.group(1), int(m.group(2)))} if m else set()


def check_matrix_operands(asm_path: str) -> int:
    """A matrix instruction may read a register that an ordinary vector instruction wrote two
    issue cycles later at the earliest.  For the matrix instructions the compiler emits itself
    it inserts the wait; here every v_mfma of the emitted gfx950 code is checked against the two
    instructions in front of it (an s_nop of two or more cycles in between settles it).  Returns
    the number of matrix instructions checked; raises on a violation."""
    ins = [l.strip() for l in open(asm_path) if l.startswith("\t") and not l.lstrip().startswith((";", "."))]
    checked, bad = 0, []
    for k, t in enumerate(ins):
        if not t.startswith("v_mfma"):
            continue
        checked += 1
        ops = t.split(None, 1)[1].split(";")[0].split(",")
        src = set().union(*[_registers(o) for o in ops[1:]])
        for back in (1, 2):
            if k - back < 0:
                break
            p = ins[k - back]
            if p.startswith("s_nop"):
                if int(p.split()[1]) + 1 >= 2:
                    break
                continue
            if p.startswith("v_") and not p.startswith("v_mfma"):
                if _registers(p.split(None, 1)[1].split(",")[0]) & src:
                    bad.append(f"{p}  ->  {t}")
    # The loads that write LDS directly take their LDS address from M0, set by an asm statement of
    # its own a few instructions earlier: nothing else in this code may touch M0.
    other_m0 = [t for t in ins if re.search(r"\bm0\b", t) and not re.match(r"^s_mov_b32 m0, (s\d+|vcc_lo|vcc_hi|ttmp\d+)$", t.split(";")[0].strip())]
    if other_m0:
        raise RuntimeError(f"{asm_path}: M0 is used outside the row requests, e.g. {other_m0[0]}")
    if bad:
        raise RuntimeError(f"{asm_path}: {len(bad)} matrix instructions read a register written by one of the two "
                           "vector instructions in front of them, e.g.\n  " + "\n  ".join(bad[:5]))
    return checked


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, src + ".o")
    cmd = [_hipcc(), *FLAGS, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
    if src in ASM_MFMA_SOURCES:
        cmd.insert(-2, "-save-temps=obj")
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    if src in ASM_MFMA_SOURCES:
        stem = os.path.join(OBJ, src.rsplit(".", 1)[0])
        n = check_matrix_operands(stem + "-hip-amdgcn-amd-amdhsa-gfx950.s")
        if n == 0:
            raise RuntimeError(f"{src}: no matrix instruction found in the emitted code")
        for f in os.listdir(OBJ):                  # the intermediate files are not kept
            if f.startswith(os.path.basename(stem) + "-") or f.startswith(src + "-"):
                os.remove(os.path.join(OBJ, f))
    return obj


def build(verbose: bool = True) -> str:
    """Compile every source and link the shared library; always recompiles."""
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.check_call(cmd)
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build()
