"""Static check of the compiled main loop of the prefill GEMM (no GPU needed).

The loop's global loads are inline assembly whose completion the compiler does
not track: a register that a load in flight will write must not be read or
written until a wait has guaranteed the load has landed.  Loads complete in
issue order, so `s_waitcnt vmcnt(N)` guarantees every load that has at least N
younger memory operations behind it.  The functions below read the gfx950
listing the build's own flags produce and verify that property instruction by
instruction, and that the loop holds neither register spills nor a full
`vmcnt(0)` wait (the stall the assembly loads exist to avoid).  build() runs
check() on every build, with the compiler and flags of that build, and fails
the build if it trips; the tests call the same functions.
"""
from __future__ import annotations

import os
import re
import subprocess
import tempfile

KERNELS = {
    "fp32 output": "_ZN4fgmp17gemm_mixed_kernelILi2ELi4ELb0ELb0EE",
    "packed output": "_ZN4fgmp17gemm_mixed_kernelILi2ELi4ELb1ELb0EE",
    "gated packed output": "_ZN4fgmp17gemm_mixed_kernelILi2ELi4ELb1ELb1EE",
}


def make_listing(hipcc: str, flags: list[str], src: str) -> list[str]:
    """The device-side assembly listing of `src` under the given build flags, as lines."""
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "listing.s")
        flags = [f for f in flags if f != "-fPIC"]
        res = subprocess.run([hipcc, *flags, "-S", "--cuda-device-only", "-o", out, src], capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"listing of {src} failed:\n{res.stderr}")
        with open(out) as fh:
            return fh.read().split("\n")


def instructions(lines):
    return [l.strip() for l in lines if l.startswith("\t") and not l.strip().startswith((";", "."))]


def kernel_body(lines, prefix):
    start = next(i for i, l in enumerate(lines) if l.startswith(prefix) and ":" in l)
    end = next(i for i in range(start, len(lines)) if "s_endpgm" in lines[i])
    return lines[start:end]


def main_loop(body):
    hdr = next(i for i, l in enumerate(body) if "Inner Loop Header" in l)
    label = body[hdr].split(":")[0]
    back = next(i for i in range(hdr, len(body)) if re.search(r"s_(?:cbranch_\w+|branch)\s+" + re.escape(label) + r"\b", body[i]))
    return body[hdr + 1 : back + 1]


def _regs(text):
    out = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]", text):
        out.update(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in re.finditer(r"\bv(\d+)\b", text):
        out.add(int(m.group(1)))
    return out


def _is_vmem(ins):
    return ins.startswith(("buffer_load", "buffer_store", "global_load", "global_store", "scratch_"))


def violations(ins, cyclic):
    """(number of loads checked, loads whose destination is touched before a wait has made them land)."""
    n = len(ins)
    bad = []
    checked = 0
    for i, s in enumerate(ins):
        if not s.startswith("buffer_load"):
            continue
        dst = _regs(s.split(",")[0])
        younger = 0
        landed = False
        span = range(1, 2 * n) if cyclic else range(1, n - i)
        for step in span:
            t = ins[(i + step) % n] if cyclic else ins[i + step]
            m = re.match(r"s_waitcnt.*vmcnt\((\d+)\)", t)
            if m and int(m.group(1)) <= younger:
                landed = True
            if _regs(t) & dst:
                checked += 1
                if not landed:
                    bad.append((s, t))
                break
            if _is_vmem(t):
                younger += 1
    return checked, bad


def check_kernel(lines, prefix) -> list[str]:
    """Problems found in one kernel of the listing (empty: none)."""
    problems = []
    body = kernel_body(lines, prefix)
    loop = instructions(main_loop(body))
    if sum(s.startswith("v_mfma") for s in loop) != 6 * 32:
        problems.append("the loop body is not one turn of the register rotation (6 K-steps of 32 matrix instructions)")
    checked, bad = violations(loop, cyclic=True)
    if checked < 6 * 6 or bad:
        problems.append(f"main loop: {checked} loads checked, hazards {bad}")
    checked, bad = violations(instructions(body), cyclic=False)   # prologue -> loop -> remainder -> epilogue
    if checked < 60 or bad:
        problems.append(f"whole kernel: {checked} loads checked, hazards {bad}")
    if [s for s in loop if s.startswith("scratch_")]:
        problems.append("register spill inside the main loop")
    waits = [int(m.group(1)) for s in loop for m in [re.match(r"s_waitcnt.*vmcnt\((\d+)\)", s)] if m]
    if not waits or min(waits) < 6:
        problems.append(f"a wait in the main loop drains (nearly) all loads: {waits}")
    return problems


def check(hipcc: str, flags: list[str], src: str) -> None:
    """Raise if any instantiation of the prefill kernel, compiled as the build compiles it, has a hazard."""
    lines = make_listing(hipcc, flags, src)
    found = {}
    for name, prefix in KERNELS.items():
        p = check_kernel(lines, prefix)
        if p:
            found[name] = p
    if found:
        raise RuntimeError(f"prefill kernel listing check failed: {found}")
