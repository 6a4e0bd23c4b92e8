"""Builds libmoe355.so (all HIP sources, gfx950) next to this file with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmoe355.so")
SOURCES = ["api.hip", "route.hip", "permute.hip", "ffn.hip", "combine.hip"]
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


# ffn.hip spells out its software pipeline (loads first, LDS reads one k-step ahead of the MFMAs); the
# machine scheduler would fold that back into load-use pairs to save registers, so it is switched off there.
EXTRA = {"ffn.hip": ["-mllvm", "-enable-misched=false", "-Rpass-analysis=kernel-resource-usage"]}
# The MFMA kernels of ffn.hip keep loads in flight in registers the compiler knows nothing about; a
# register spill there could save such a register before its load has landed.  The build refuses it.
NO_SPILL = {"ffn.hip": "ffn_mfma_kernel"}


def _check_no_spill(src: str, remarks: str) -> None:
    current = ""
    for line in remarks.splitlines():
        if "Function Name:" in line:
            current = line.split("Function Name:")[1].strip()
        elif NO_SPILL[src] in current and ("VGPRs Spill:" in line or "SGPRs Spill:" in line):
            n = int(line.split("Spill:")[1].split()[0])
            if n != 0:
                raise RuntimeError(f"{src}: {current} spills {n} registers ({line.strip()}); "
                                   "the hand-counted load waits of this kernel do not allow that")


def _compile(src: str) -> str:
    obj = os.path.join(HERE, "_build", src.replace(".hip", ".o"))
    cmd = [_hipcc(), *FLAGS, *EXTRA.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    if r.returncode == 0 and src in NO_SPILL:
        _check_no_spill(src, r.stderr)
    kept, skip = [], 0
    for l in r.stderr.splitlines():
        if "-Rpass-analysis=kernel-resource-usage" in l:
            skip = 2                                # a remark is followed by the source line and a caret line
        elif skip and (l.lstrip()[:1].isdigit() or l.lstrip().startswith("|")):
            skip -= 1
        elif noise not in l:
            kept.append(l)
            skip = 0
    err = "\n".join(kept)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = False) -> str:
    os.makedirs(os.path.join(HERE, "_build"), exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        objs = list(pool.map(_compile, SOURCES))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
