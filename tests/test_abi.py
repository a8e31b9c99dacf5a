"""Host-side checks that need no GPU: the shared library loads, exports every
symbol the public header declares, and rejects bad arguments before launching
anything."""
import ctypes
import os
import re

from paper_2504_14152_amd import build, fgmp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "fgmp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fgmp_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    if not os.path.exists(build.lib_path()):
        build.build()
    lib = ctypes.CDLL(build.lib_path())
    names = _declared_symbols()
    assert {"fgmp_quantize_weights", "fgmp_quantize_activations", "fgmp_gemm", "fgmp_quant_gemm_fused",
            "fgmp_unpack_canonical"} <= set(names)
    for name in names:
        assert hasattr(lib, name), f"{name} declared in fgmp.h but not exported"


def test_sizes_and_host_side_argument_checks():
    assert fgmp.version().endswith("(gfx950)")
    # 8 x 128 tiles: header + 512 B + 64 B + 8 B + 4 B + 512 B per tile, planes 256-byte aligned
    assert fgmp.packed_bytes(8, 128) == 256 + 512 + 256 + 256 + 256 + 512
    assert fgmp.packed_bytes(8, 24) == 0 and fgmp.packed_bytes(0, 16) == 0
    n_blocks = 4096 * 4096 // 16
    # worst case: 8 + 8 B values, the scale-or-index byte, 1 mask bit, 4 B of tile table per 64 blocks
    assert 16.125 * n_blocks <= fgmp.packed_bytes(4096, 4096) <= (17 + 0.125 + 0.0625) * n_blocks + 2048
    assert fgmp.workspace_bytes(4096, 12288, 4096) >= fgmp.packed_bytes(4096, 4096)
    L = fgmp.lib()
    assert L.fgmp_quantize_activations(None, 0, 8, 128, 128, None, 0.0, 1.0, None, 0, None, None) == -1
    # measurement helper: no sink, no work
    assert L.fgmp_selftest_mfma_rate(256, 10, None, None) == -1
    # measurement hook: a lone event is refused, clearing always works
    assert L.fgmp_selftest_time_gemm_kernel(256, None) == -1
    assert L.fgmp_selftest_time_gemm_kernel(None, None) == 0
    assert L.fgmp_gemm(None, 1, None, 1, 16, None, 1, None, 0, None) == -1
    assert L.fgmp_gemm(256, 1, 256, 1, 24, 256, 1, 256, 0, None) == -2
    assert L.fgmp_unpack_canonical(None, 1, 16, None, None, None, None) == -1
    # the entry points added for the score of Eq. 8, clipping, packed output and the global threshold
    assert L.fgmp_quantize_activations_ex(256, 0, 8, 128, 128, 256, 0.0, 1.0, 5, 256, 1 << 20, None, None) == -1
    assert L.fgmp_quantize_weights_ex(None, 0, 8, 128, 128, None, 0, 0.0, 1.0, 1, None, 0, None, None) == -1
    assert L.fgmp_quantize_weights_clip(256, 0, 8, 128, 128, 256, 0, 0.0, 1.0, 256, 1 << 20, None, None, 0, None) == -1
    assert L.fgmp_quantize_weights_clip(256, 0, 8, 24, 24, 256, 0, 0.0, 1.0, 256, 1 << 20, None, 256, 64, None) == -2
    assert L.fgmp_quantize_weights_clip(256, 0, 8, 128, 128, 256, 0, 0.0, 1.0, 256, 1 << 20, None, 256, 63, None) == -4
    assert fgmp.lib().fgmp_workspace_bytes_packed_out(4096, 12288, 4096) >= fgmp.workspace_bytes(4096, 12288, 4096) + 4096 * 12288 * 4
    assert fgmp.lib().fgmp_workspace_bytes_packed_out(64, 24, 128) == 0          # N must be a multiple of 16
    # gated epilogue: groups of 64 weight rows, a second staging area for the gated values, known operators only
    wb = fgmp.lib().fgmp_workspace_bytes_packed_out_ex
    assert wb(64, 96, 128, 1) == 0 and wb(64, 128, 128, 7) == 0
    assert wb(64, 128, 128, 0) == fgmp.lib().fgmp_workspace_bytes_packed_out(64, 128, 128)
    assert wb(64, 128, 128, 1) >= wb(64, 128, 128, 0) + 64 * 64 * 4
    # the one-launch flag changes no size and is no operator of its own
    assert wb(8, 12288, 4096, 0x100) == wb(8, 12288, 4096, 0) and wb(64, 128, 128, 0x101) == wb(64, 128, 128, 1)
    assert wb(64, 128, 128, 0x102) == 0 and wb(64, 128, 128, 0x200) == 0
    # ... and a decode step's workspace has room for its row groups' decision words behind its own scratch
    assert wb(8, 12288, 4096, 0x100) >= fgmp.workspace_bytes(8, 12288, 4096) + 12288 // 16 * 4
    assert L.fgmp_quant_gemm_fused_packed_out_ex(256, 0, 64, 128, 128, 256, 0.0, 1.0, 256, 96, 1, 256, 0.0, 1.0, 256, 1 << 20,
                                                 None, 256, 1 << 30, None) == -2
    assert L.fgmp_quant_gemm_fused_packed_out_ex(256, 0, 64, 128, 128, 256, 0.0, 1.0, 256, 128, 5, 256, 0.0, 1.0, 256, 1 << 20,
                                                 None, 256, 1 << 30, None) == -1
    assert L.fgmp_quant_gemm_fused_packed_out(256, 0, 64, 128, 128, 256, 0.0, 1.0, 256, 24, 256, 0.0, 1.0, 256, 1 << 20,
                                              None, 256, 1 << 20, None) == -2
    assert L.fgmp_quant_gemm_fused_packed_out(256, 0, 64, 128, 128, 256, 0.0, 1.0, 256, 32, 256, 0.0, 0.0, 256, 1 << 20,
                                              None, 256, 1 << 20, None) == -1   # output scale must be positive
    assert L.fgmp_quant_gemm_fused_packed_out(256, 0, 64, 128, 128, 256, 0.0, 1.0, 256, 32, 256, 0.0, 1.0, 256, 16,
                                              None, 256, 1 << 20, None) == -4   # packed output buffer too small
    assert L.fgmp_threshold_for_fraction_multi(None, None, 1, ctypes.c_double(0.1), None, None) == -1
    # the quantizer's traffic model exists in measurement builds only
    assert L.fgmp_selftest_quantizer_traffic(256, 0, 16384, 8192, 8192, 256, 256, 1 << 30, None) == -5


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode != 0 and "one GPU" in res.stderr


def test_workspace_sizes_over_the_row_counts_where_the_paths_change():
    """Host-side planning only: every M from decode sizes through the first prefill tiles gets a workspace,
    whichever kernel the planner picks (row chunks through the weight-streaming kernel, tiles split along
    K, whole tiles), and it never shrinks below what the FP16 copy of X alone needs."""
    L = fgmp.lib()
    for (N, K) in [(12288, 4096), (4096, 4096), (22016, 4096), (4096, 11008), (264, 2048), (57344, 8192)]:
        for M in list(range(1, 300)) + [511, 512, 513, 1024, 4096]:
            ws = int(L.fgmp_workspace_bytes(M, N, K))
            assert ws >= M * K * 2, (M, N, K, ws)
            assert ws < (1 << 34), (M, N, K, ws)
        assert L.fgmp_workspace_bytes(0, N, K) == 0 and L.fgmp_workspace_bytes(8, N, K + 8) == 0

