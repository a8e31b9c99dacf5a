"""Static checks on the compiled main loop of the prefill GEMM (no GPU needed).

The loop's global loads are inline assembly whose completion the compiler does
not track: a register that a load in flight will write must not be read or
written until a wait has guaranteed the load has landed.  Loads complete in
issue order, so `s_waitcnt vmcnt(N)` guarantees every load that has at least N
younger memory operations behind it.  The checks below read the gfx950 listing
the build's own flags produce and verify that property instruction by
instruction, and that the loop holds neither register spills nor a full
`vmcnt(0)` wait (the stall the assembly loads exist to avoid).
"""
from __future__ import annotations

import os
import re
import shutil
import subprocess

import pytest

from paper_2504_14152_amd import build

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
SRC = os.path.join(build.CSRC, "fgmp_gemm_mixed.hip")
KERNELS = {
    "fp32 output": "_ZN4fgmp17gemm_mixed_kernelILi2ELi4ELb0ELb0EE",
    "packed output": "_ZN4fgmp17gemm_mixed_kernelILi2ELi4ELb1ELb0EE",
    "gated packed output": "_ZN4fgmp17gemm_mixed_kernelILi2ELi4ELb1ELb1EE",
}

pytestmark = pytest.mark.skipif(shutil.which(HIPCC) is None and not os.path.exists(HIPCC), reason="hipcc not available")


@pytest.fixture(scope="module")
def listing(tmp_path_factory):
    out = tmp_path_factory.mktemp("listing") / "fgmp_gemm_mixed.s"
    flags = [f for f in build.FLAGS if f != "-fPIC"]
    res = subprocess.run([HIPCC, *flags, "-S", "--cuda-device-only", "-o", str(out), SRC], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    return out.read_text().split("\n")


def _instructions(lines):
    return [l.strip() for l in lines if l.startswith("\t") and not l.strip().startswith((";", "."))]


def _kernel_body(lines, prefix):
    start = next(i for i, l in enumerate(lines) if l.startswith(prefix) and ":" in l)
    end = next(i for i in range(start, len(lines)) if "s_endpgm" in lines[i])
    return lines[start:end]


def _main_loop(body):
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


def _violations(ins, cyclic):
    """Loads whose destination is touched before a wait has made them land."""
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


@pytest.mark.parametrize("which", sorted(KERNELS))
def test_no_register_of_a_load_in_flight_is_touched(listing, which):
    body = _kernel_body(listing, KERNELS[which])
    loop = _instructions(_main_loop(body))
    assert sum(s.startswith("v_mfma") for s in loop) == 6 * 32, "the loop body is one turn of the register rotation: 6 K-steps"
    checked, bad = _violations(loop, cyclic=True)
    assert checked >= 6 * 6 and not bad, bad
    # prologue -> loop -> remainder -> epilogue, in program order
    checked, bad = _violations(_instructions(body), cyclic=False)
    assert checked >= 60 and not bad, bad


@pytest.mark.parametrize("which", sorted(KERNELS))
def test_loop_has_no_spills_and_no_full_memory_wait(listing, which):
    loop = _instructions(_main_loop(_kernel_body(listing, KERNELS[which])))
    assert not [s for s in loop if s.startswith("scratch_")], "register spill inside the main loop"
    waits = [int(m.group(1)) for s in loop for m in [re.match(r"s_waitcnt.*vmcnt\((\d+)\)", s)] if m]
    assert waits and min(waits) >= 6, waits


def test_checker_catches_a_planted_hazard():
    # a copy of a load's destination before any wait, and one after a sufficient wait
    early = ["buffer_load_dword v5, v1, s[0:3], 0 offen", "v_mov_b32_e32 v6, v5", "s_waitcnt vmcnt(0)"]
    late = ["buffer_load_dword v5, v1, s[0:3], 0 offen", "buffer_load_dword v7, v1, s[0:3], 0 offen", "s_waitcnt vmcnt(1)",
            "v_mov_b32_e32 v6, v5", "s_waitcnt vmcnt(0)", "v_mov_b32_e32 v8, v7"]
    too_weak = ["buffer_load_dword v5, v1, s[0:3], 0 offen", "buffer_load_dword v7, v1, s[0:3], 0 offen", "s_waitcnt vmcnt(1)",
                "v_mov_b32_e32 v8, v7"]
    assert _violations(early, cyclic=False)[1]
    assert _violations(late, cyclic=False) == (2, [])
    assert _violations(too_weak, cyclic=False)[1]
