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
