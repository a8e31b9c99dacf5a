"""Build libfgmp.so (HIP, gfx950) in-tree with hipcc, plus two variants of the same sources that only
tests and the benchmark load:
  libfgmp_hooks.so     -DFGMP_MEASUREMENT_HOOKS: the per-launch timing hook of the prefill kernel and the
                       environment switch for the two-pass prefill path (neither is in libfgmp.so)
  libfgmp_fullwait.so  -DFGMP_FULL_WAITS: every hand-counted `s_waitcnt vmcnt(N)` of the assembly loads is
                       `vmcnt(0)`; the runtime guard requires its results to equal libfgmp.so's bit for bit
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

from . import listing_check

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfgmp.so")
SOURCES = ["fgmp_quantize.hip", "fgmp_gemm.hip", "fgmp_gemm_skinny.hip", "fgmp_gemm_stream.hip", "fgmp_gemm_mixed.hip",
           "fgmp_select.hip", "fgmp_api.hip"]
# -ffp-contract=off: the quantizer's FP32 steps are separately rounded.
# packed-fp32-ops is switched off for the device compiler on purpose.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function"]
VARIANTS = {"hooks": ["-DFGMP_MEASUREMENT_HOOKS=1"], "fullwait": ["-DFGMP_FULL_WAITS=1"]}


def lib_path(variant: str | None = None) -> str:
    return LIB if not variant else os.path.join(HERE, f"libfgmp_{variant}.so")


def source_files() -> list[str]:
    """Every file a library is built from (for the staleness check of the binding)."""
    files = [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if f.endswith((".hip", ".hpp"))]
    files.append(os.path.join(os.path.dirname(HERE), "include", "fgmp.h"))
    return files


def is_stale(path: str) -> bool:
    if not os.path.exists(path):
        return True
    t = os.path.getmtime(path)
    return any(os.path.getmtime(f) > t for f in source_files())


def _hipcc() -> str:
    return os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def build_one(variant: str | None = None, verbose: bool = False, extra_flags: list[str] | None = None,
              out: str | None = None) -> str:
    """Compile every source for gfx950 and link one shared library."""
    hipcc = _hipcc()
    out = out or lib_path(variant)
    build_dir = os.path.join(HERE, "_build", os.path.basename(out).replace(".so", ""))
    os.makedirs(build_dir, exist_ok=True)
    flags = FLAGS + (VARIANTS[variant] if variant else []) + (extra_flags or [])

    def compile_one(src: str) -> str:
        obj = os.path.join(build_dir, src.replace(".hip", ".o"))
        cmd = [hipcc, *flags, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, capture_output=True, text=True)
        # the host pass warns that it does not know the packed-fp32 feature: harmless
        err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc failed for {src}:\n{res.stderr}")
        if verbose and err.strip():
            print(err, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", out]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stderr}")
    return out


def build(verbose: bool = False, extra_flags: list[str] | None = None, out: str | None = None,
          variants: bool = True) -> str:
    """Build libfgmp.so (and, unless an explicit output is asked for, its two variants), then check the
    compiled prefill loop of this very compiler and flag set for load/wait hazards."""
    path = build_one(None, verbose, extra_flags, out)
    if out is None and variants:
        for v in VARIANTS:
            build_one(v, verbose, extra_flags)
    listing_check.check(_hipcc(), FLAGS + (extra_flags or []), os.path.join(CSRC, "fgmp_gemm_mixed.hip"))
    return path


if __name__ == "__main__":
    print(build(verbose=True))
