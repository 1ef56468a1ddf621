"""Compile the HIP library for gfx950 into paper_2211_10526_amd/libcastling_attn.so."""
from __future__ import annotations

import os
import re
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
# translation units (no device code crosses them; several would compile side by side)
UNITS = ["castling_attn.hip"]
LIB = os.path.join(HERE, "libcastling_attn.so")
OBJ_DIR = os.path.join(HERE, "_build")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed fp32 ALU forms are kept out of the generated code on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def sources() -> list[str]:
    return [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC))] + \
        [os.path.join(os.path.dirname(HERE), "include", "castling_attn.h")]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(s) > t for s in sources())


def _compile(hipcc: str, unit: str) -> tuple[int, list[str], list[str]]:
    """One translation unit -> object file; returns (status, log lines, kernels that spill)."""
    obj = os.path.join(OBJ_DIR, unit.replace(".hip", ".o"))
    cmd = [hipcc] + HIPCC_FLAGS + ["-Rpass-analysis=kernel-resource-usage", "-c",
                                   os.path.join(CSRC, unit), "-o", obj]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass does not know the target feature and says so; that is harmless
    lines = [l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l]
    # Kernels here issue global loads whose landing they track themselves; the compiler must
    # never spill such a register while the load is in flight, so no kernel may spill a vector
    # register or use a stack (scalar registers spilled to lanes of a vector register are fine).
    spilled, name = [], ""
    for l in lines:
        if "Function Name:" in l:
            name = l.split("Function Name:")[1].split("[")[0].strip()
        elif "VGPRs Spill:" in l:
            if int(l.split("VGPRs Spill:")[1].split("[")[0].strip()) != 0:
                spilled.append(name)
        elif "Dynamic Stack:" in l and "True" in l:
            spilled.append(name)
    noise = re.compile(r"remark:|-Rpass-analysis|^In file included from|^\s*\d*\s*\|")
    log = [l for l in lines if l.strip() and not noise.search(l)]
    return res.returncode, log, spilled


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=len(UNITS)) as pool:
        results = list(pool.map(lambda u: _compile(hipcc, u), UNITS))
    log = "\n".join(l for _, lines, _ in results for l in lines)
    if any(rc != 0 for rc, _, _ in results):
        raise RuntimeError("hipcc failed:\n" + log)
    spilled = [k for _, _, ks in results for k in ks]
    if spilled:
        if os.path.exists(LIB):
            os.remove(LIB)
        raise RuntimeError("kernels that spill vector registers (not allowed, see build.py):\n  " +
                           "\n  ".join(spilled))
    objs = [os.path.join(OBJ_DIR, u.replace(".hip", ".o")) for u in UNITS]
    res = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB],
                         stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stdout)
    if verbose and log.strip():
        print(log)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
