"""Builds libmoe355.so (all HIP sources, gfx950) next to this file with hipcc."""
from __future__ import annotations

import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmoe355.so")
SOURCES = ["api.hip", "route.hip", "permute.hip", "ffn.hip", "combine.hip", "schedule.hip"]
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
# Its work-queue atomics are issued by one lane whose answer is wanted later (it arrives under other work); the atomic
# optimizer would rewrite them into a wave reduction whose broadcast waits for the answer on the spot.
EXTRA = {"ffn.hip": ["-mllvm", "-enable-misched=false", "-mllvm", "-amdgpu-atomic-optimizer-strategy=None"]}
# The MFMA kernels of ffn.hip keep loads in flight in registers the compiler knows nothing about and count
# the outstanding loads by hand.  Spill code inside such a region could save a register before its load
# has landed, and its own memory operations would be counted as if they were the kernel's.  The source
# brackets those regions with "; pipeline begin" / "; pipeline end"; the build reads the assembly and
# refuses any scratch access between the two or inside an inner loop of these kernels.
NO_SPILL = {"ffn.hip": "ffn_mfma"}


def check_no_spill(asm: str, kernel_pattern: str, what: str = "assembly") -> None:
    """Raises if a kernel whose name contains kernel_pattern touches scratch memory between a
    "; pipeline begin" and the next "; pipeline end", or inside a loop nested in another loop."""
    kernel, inside, inner = None, False, False
    lines = asm.splitlines()
    for n, line in enumerate(lines, 1):
        text = line.strip()
        if line.startswith("_Z") and ":" in line:                       # a function starts
            name = line.split(":")[0]
            kernel = name if kernel_pattern in name else None
            inside = inner = False
        elif text.startswith(".end_amdhsa_kernel") or text.startswith(".Lfunc_end"):
            kernel = None
        if kernel is None:
            continue
        if line.startswith(".LBB") or line.startswith("; %bb."):        # a block: which loop is it in?
            note = line + (lines[n] if n < len(lines) and lines[n].strip().startswith(";") else "")
            inner = "Depth=2" in note or "Depth=3" in note
        if "; pipeline begin" in text:
            inside = True
        elif "; pipeline end" in text:
            inside = False
        elif text.startswith("scratch_") and (inside or inner):
            raise RuntimeError(f"{what}: spill code inside a hand-counted load pipeline of {kernel} (line {n}: {text})")



_VREG = re.compile(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b")


def _vregs(text: str) -> set:
    out = set()
    for lo, hi, one in _VREG.findall(text):
        out |= set(range(int(lo), int(hi) + 1)) if lo else {int(one)}
    return out


def check_loads_in_flight(asm: str, kernel_pattern: str, what: str = "assembly") -> int:
    """The pipelined loops of the named kernels keep loads in flight that the compiler does not know about
    (it sees inline assembly that defines registers).  Whatever it schedules or copies there, no instruction
    may touch a register whose load has not been waited for.  This walks every inner loop that lies between
    "; pipeline begin" and "; pipeline end", twice around (the second round meets the loads the first left in
    flight), keeping the loads in issue order: "s_waitcnt vmcnt(N)" retires all but the youngest N (loads
    return in order), and any other use of a register with a load still pending is an error.  The loops must
    be single blocks.  Returns the number of loops checked."""
    lines = asm.splitlines()
    kernel, inside, checked, n = None, False, 0, 0
    while n < len(lines):
        line = lines[n]
        text = line.strip()
        if line.startswith("_Z") and ":" in line:
            name = line.split(":")[0]
            kernel = name if kernel_pattern in name else None
            inside = False
        elif text.startswith(".end_amdhsa_kernel"):
            kernel = None
        if kernel is not None:
            if "; pipeline begin" in text:
                inside = True
            elif "; pipeline end" in text:
                inside = False
            elif inside and line.startswith(".LBB") and "Depth=2" in (line + (lines[n + 1] if n + 1 < len(lines) else "")):
                label = line.split(":")[0]
                body, m = [], n + 1
                while m < len(lines):
                    t = lines[m].strip()
                    if lines[m].startswith(".LBB") or "; pipeline" in t:
                        raise RuntimeError(f"{what}: the pipelined loop {label} of {kernel} is not a single block (line {m + 1})")
                    if t and not t.startswith(";"):
                        body.append((m + 1, t.split(";")[0].strip()))
                    if t.startswith("s_cbranch") and t.split()[-1] == label:
                        break
                    m += 1
                pending = []                                  # (registers, line) in issue order
                for round_ in range(2):
                    for ln, t in body:
                        op = t.split()[0]
                        if op == "s_waitcnt":
                            got = re.search(r"vmcnt\((\d+)\)", t)
                            if got:
                                keep = int(got.group(1))
                                pending = pending[len(pending) - keep:] if 0 < keep < len(pending) else ([] if keep == 0 else pending)
                            continue
                        used = _vregs(t)
                        for regs, at in pending:
                            if used & regs:
                                raise RuntimeError(f"{what}: {kernel}: line {ln} ({t}) touches v{min(used & regs)}, whose load "
                                                   f"(line {at}) has not been waited for")
                        if op.startswith(("global_load", "buffer_load", "flat_load")):
                            dst = _vregs(t.split(",")[0])
                            pending.append((dst, ln))
                checked += 1
                n = m
        n += 1
    return checked


def check_prologue_in_flight(asm: str, kernel_pattern: str, what: str = "assembly") -> int:
    """The same rule for the code that leads up to each pipelined loop (from "; pipeline begin" to the loop's
    first block, in layout order, across block labels): the loads written as inline assembly are in flight from
    their issue until a "s_waitcnt vmcnt(N)" that leaves at most N younger ones outstanding, and nothing may
    touch their registers before.  Vector memory operations the compiler generated itself in that stretch
    (one wave takes the block's next work item there) are not put on the list: a wave that does not execute
    them has fewer operations outstanding, so counting them would retire hand-issued loads too early.
    Returns the number of stretches checked."""
    lines = asm.splitlines()
    kernel, checked, n = None, 0, 0
    while n < len(lines):
        line = lines[n]
        if line.startswith("_Z") and ":" in line:
            name = line.split(":")[0]
            kernel = name if kernel_pattern in name else None
        elif line.strip().startswith(".end_amdhsa_kernel"):
            kernel = None
        if kernel is not None and "; pipeline begin" in line:
            pending, in_asm, m = [], True, n + 1          # the marker itself is inline assembly
            while m < len(lines):
                raw = lines[m]
                t = raw.strip()
                if "; pipeline end" in t:
                    break
                if raw.startswith(".LBB") and "Depth=2" in (raw + (lines[m + 1] if m + 1 < len(lines) else "")):
                    break
                if "#ASMSTART" in t:
                    in_asm = True
                elif "#ASMEND" in t:
                    in_asm = False
                if t and not t.startswith(";") and not raw.startswith("."):
                    code = t.split(";")[0].strip()
                    op = code.split()[0]
                    if op == "s_waitcnt":
                        got = re.search(r"vmcnt\((\d+)\)", code)
                        if got:
                            keep = int(got.group(1))
                            pending = pending[len(pending) - keep:] if 0 < keep < len(pending) else ([] if keep == 0 else pending)
                    else:
                        used = _vregs(code)
                        for regs, at in pending:
                            if used & regs:
                                raise RuntimeError(f"{what}: {kernel}: line {m + 1} ({code}) touches v{min(used & regs)}, whose "
                                                   f"load (line {at}) has not been waited for")
                        if in_asm and op.startswith(("global_load", "buffer_load", "flat_load")):
                            pending.append((_vregs(code.split(",")[0]), m + 1))
                m += 1
            checked += 1
            n = m
        n += 1
    return checked


def _compile(src: str) -> str:
    obj = os.path.join(HERE, "_build", src.replace(".hip", ".o"))
    cmd = [_hipcc(), *FLAGS, *EXTRA.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    if r.returncode == 0 and src in NO_SPILL:
        asm = os.path.join(HERE, "_build", src.replace(".hip", ".s"))
        ra = subprocess.run([_hipcc(), *FLAGS, *EXTRA.get(src, []), "-S", "--cuda-device-only",
                             os.path.join(CSRC, src), "-o", asm], capture_output=True, text=True)
        if ra.returncode != 0:
            raise RuntimeError(f"hipcc -S failed on {src}:\n{ra.stderr}")
        text = open(asm).read()
        check_no_spill(text, NO_SPILL[src], src)
        if check_loads_in_flight(text, NO_SPILL[src], src) == 0 or check_prologue_in_flight(text, NO_SPILL[src], src) == 0:
            raise RuntimeError(f"{src}: no pipelined loop found to verify (markers missing?)")
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
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
