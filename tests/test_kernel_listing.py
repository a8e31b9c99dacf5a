"""Static checks on the compiled main loop of the prefill GEMM (no GPU needed): no register that a load in
flight will write is touched before a sufficient wait, no spills and no full memory wait inside the loop.
The checker lives in the package (listing_check.py) because every build runs it too."""
from __future__ import annotations

import os
import shutil

import pytest

from paper_2504_14152_amd import build, listing_check as lc

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
SRC = os.path.join(build.CSRC, "fgmp_gemm_mixed.hip")

pytestmark = pytest.mark.skipif(shutil.which(HIPCC) is None and not os.path.exists(HIPCC), reason="hipcc not available")


@pytest.fixture(scope="module")
def listing():
    return lc.make_listing(HIPCC, build.FLAGS, SRC)


@pytest.mark.parametrize("which", sorted(lc.KERNELS))
def test_no_register_of_a_load_in_flight_is_touched(listing, which):
    assert lc.check_kernel(listing, lc.KERNELS[which]) == []


def test_checker_catches_a_planted_hazard():
    # a copy of a load's destination before any wait, and one after a sufficient wait
    early = ["buffer_load_dword v5, v1, s[0:3], 0 offen", "v_mov_b32_e32 v6, v5", "s_waitcnt vmcnt(0)"]
    late = ["buffer_load_dword v5, v1, s[0:3], 0 offen", "buffer_load_dword v7, v1, s[0:3], 0 offen", "s_waitcnt vmcnt(1)",
            "v_mov_b32_e32 v6, v5", "s_waitcnt vmcnt(0)", "v_mov_b32_e32 v8, v7"]
    too_weak = ["buffer_load_dword v5, v1, s[0:3], 0 offen", "buffer_load_dword v7, v1, s[0:3], 0 offen", "s_waitcnt vmcnt(1)",
                "v_mov_b32_e32 v8, v7"]
    assert lc.violations(early, cyclic=False)[1]
    assert lc.violations(late, cyclic=False) == (2, [])
    assert lc.violations(too_weak, cyclic=False)[1]


def test_full_wait_variant_has_only_full_waits_in_the_loop():
    """The build variant that the runtime guard compares with (every hand-counted wait replaced by a full
    one): its main loop waits with vmcnt(0) only, so it cannot be wrong about how many loads are behind."""
    lines = lc.make_listing(HIPCC, build.FLAGS + build.VARIANTS["fullwait"], SRC)
    import re
    for prefix in lc.KERNELS.values():
        loop = lc.instructions(lc.main_loop(lc.kernel_body(lines, prefix)))
        waits = [int(m.group(1)) for s in loop for m in [re.match(r"s_waitcnt.*vmcnt\((\d+)\)", s)] if m]
        assert waits and max(waits) == 0, waits


# ---- the one-launch decode kernel (fgmp_gemm_stream.hip) ----

STREAM_SRC = os.path.join(build.CSRC, "fgmp_gemm_stream.hip")


def _stream_constants():
    import re
    text = open(STREAM_SRC).read()
    val = lambda name: int(re.search(r"constexpr int " + name + r" = (\d+);", text).group(1))
    asserted = {int(t): int(v) for t, v in re.findall(r"st_step_wait\((\d+)\) == (\d+)", text)}
    return dict(R=val("kStRing"), L=val("kStHLead"), M=val("kStMtLoads"), LS=val("kStLsLoads"), H=val("kStHLoads")), asserted


def test_decode_kernel_wait_counts_follow_from_its_issue_order():
    """The waits of the decode kernel's ring are constants that the source derives with closed formulas and
    pins with static_asserts.  Here the issue order is written out load by load -- prologue: masks of the
    first R tiles, their planes L / S, their plane-H entries; step u: plane H of tile u + L (from step
    R - L on), mask of tile u + R, planes L / S of tile u + R -- and the largest number of outstanding loads
    that still guarantees what step t reads (all of tile t; the mask of tile t + L, from step R - L on) is
    found by search.  It must be the asserted number for every step the source names."""
    c, asserted = _stream_constants()
    R, L = c["R"], c["L"]
    seq = [("M", j) for j in range(R) for _ in range(c["M"])]
    seq += [("LS", j) for j in range(R) for _ in range(c["LS"])]
    seq += [("H", j) for j in range(R) for _ in range(c["H"])]
    issued_before_step = {}
    for u in range(4 * R):
        issued_before_step[u] = len(seq)
        if u >= R - L:
            seq += [("H", u + L)] * c["H"]
        seq += [("M", u + R)] * c["M"] + [("LS", u + R)] * c["LS"]
    assert len(asserted) >= 2 * R
    for t, want in sorted(asserted.items()):
        upto = issued_before_step[t]
        last = lambda tag, tile: max(i for i, x in enumerate(seq[:upto]) if x == (tag, tile))
        need = [last("H", t), last("LS", t), last("M", t)]
        if t >= R - L:
            need.append(last("M", t + L))
        assert min(upto - 1 - i for i in need) == want, (t, want)
    # the steady state repeats with the ring
    assert all(asserted[t] == asserted[t + R] for t in asserted if t >= R and t + R in asserted)


def test_decode_kernel_full_wait_variant_counts_nothing():
    """In the variant the GPU test compares with, every wait of the decode kernel is vmcnt(0)."""
    import re
    lines = lc.make_listing(HIPCC, build.FLAGS + build.VARIANTS["fullwait"], STREAM_SRC)
    start = [i for i, l in enumerate(lines) if l.startswith("_ZN4fgmp18gemm_stream_kernel") and ":" in l]
    assert len(start) >= 9
    for i in start:
        end = next(j for j in range(i, len(lines)) if "s_endpgm" in lines[j])
        # (the waits written by hand sit between the assembler's markers; the compiler's own, for loads it
        # tracks itself, are not meant)
        waits = [int(m.group(1)) for k in range(i + 1, end) if "#ASMSTART" in lines[k - 1]
                 for m in [re.search(r"s_waitcnt.*vmcnt\((\d+)\)", lines[k])] if m]
        assert len(waits) >= 20 and max(waits) == 0
