"""Thin ctypes binding of libfgmp.so (include/fgmp.h): argument marshalling
only.  PyTorch supplies device memory and the current HIP stream; every step
of the path runs in the library's kernels.  There is no fallback: if the
shared library is missing or a call fails, an exception is raised."""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

from . import build as _build

F32, BF16 = 0, 1
_ERRORS = {-1: "INVALID_ARG", -2: "BAD_SHAPE", -3: "BAD_ALIGN", -4: "BUFFER_TOO_SMALL",
           -5: "UNSUPPORTED", -6: "HIP_ERROR"}
_lib = None


class FgmpError(RuntimeError):
    pass


class _PackedInfo(ctypes.Structure):
    _fields_ = [("rows", ctypes.c_int64), ("K", ctypes.c_int64), ("tensor_scale", ctypes.c_float),
                ("compact", ctypes.c_int32), ("n_blocks", ctypes.c_int64),
                ("n_fp8_blocks", ctypes.c_int64), ("bytes_used", ctypes.c_int64)]


def _library_file() -> str:
    """The shared library to load: FGMP_LIB_PATH (a library built elsewhere, or one of the build's
    variants) or the in-tree libfgmp.so.  A missing in-tree library is built; one that is older than
    any of its sources is rebuilt when a compiler is at hand and refused otherwise, so that no test or
    benchmark result can belong to old code without notice."""
    path = os.environ.get("FGMP_LIB_PATH")
    if path:
        if not os.path.exists(path):
            raise FgmpError(f"FGMP_LIB_PATH={path} does not exist")
        return path
    path = _build.lib_path()
    if _build.is_stale(path):
        have_compiler = os.path.exists(os.environ.get("HIPCC", "/opt/rocm/bin/hipcc"))
        if have_compiler:
            _build.build()
        elif not os.path.exists(path):
            raise FgmpError(f"{path} is missing and there is no hipcc to build it")
        else:
            raise FgmpError(f"{path} is older than its sources and there is no hipcc to rebuild it")
    return path


def lib() -> ctypes.CDLL:
    """Load libfgmp.so (see _library_file) and declare its entry points."""
    global _lib
    if _lib is not None:
        return _lib
    _lib = _load(_library_file())
    return _lib


class use_library:
    """Context manager: route this module's calls to another build of the library (a variant from
    build.lib_path(variant)) for the duration of the block.  For tests and measurements."""

    def __init__(self, path: str):
        if not os.path.exists(path):
            raise FgmpError(f"{path} does not exist")
        self._other = _load(path)

    def __enter__(self):
        global _lib
        lib()
        self._saved, _lib = _lib, self._other
        return self._other

    def __exit__(self, *exc):
        global _lib
        _lib = self._saved
        return False


def _load(path: str) -> ctypes.CDLL:
    L = ctypes.CDLL(path)
    vp, i64, f32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
    L.fgmp_version.restype = ctypes.c_char_p
    L.fgmp_version.argtypes = []
    L.fgmp_packed_bytes.restype = sz
    L.fgmp_packed_bytes.argtypes = [i64, i64]
    L.fgmp_workspace_bytes.restype = sz
    L.fgmp_workspace_bytes.argtypes = [i64, i64, i64]
    L.fgmp_quantize_weights.restype = ctypes.c_int
    L.fgmp_quantize_weights.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, i64, f32, f32, vp, sz, vp, vp]
    L.fgmp_quantize_activations.restype = ctypes.c_int
    L.fgmp_quantize_activations.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, f32, f32, vp, sz, vp, vp]
    L.fgmp_quantize_weights_ex.restype = ctypes.c_int
    L.fgmp_quantize_weights_ex.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, i64, f32, f32, ctypes.c_int, vp, sz, vp, vp]
    L.fgmp_quantize_activations_ex.restype = ctypes.c_int
    L.fgmp_quantize_activations_ex.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, f32, f32, ctypes.c_int, vp, sz, vp, vp]
    L.fgmp_quant_gemm_fused_ex.restype = ctypes.c_int
    L.fgmp_quant_gemm_fused_ex.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, f32, f32, ctypes.c_int, vp, i64, vp, i64,
                                           vp, sz, vp]
    L.fgmp_quantize_weights_clip.restype = ctypes.c_int
    L.fgmp_quantize_weights_clip.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, i64, f32, f32, vp, sz, vp, vp, sz, vp]
    L.fgmp_workspace_bytes_packed_out.restype = sz
    L.fgmp_workspace_bytes_packed_out.argtypes = [i64, i64, i64]
    L.fgmp_workspace_bytes_packed_out_ex.restype = sz
    L.fgmp_workspace_bytes_packed_out_ex.argtypes = [i64, i64, i64, ctypes.c_int]
    L.fgmp_quant_gemm_fused_packed_out_ex.restype = ctypes.c_int
    L.fgmp_quant_gemm_fused_packed_out_ex.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, f32, f32, vp, i64, ctypes.c_int,
                                                      vp, f32, f32, vp, sz, vp, vp, sz, vp]
    L.fgmp_quant_gemm_fused_packed_out.restype = ctypes.c_int
    L.fgmp_quant_gemm_fused_packed_out.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, f32, f32, vp, i64, vp, f32, f32,
                                                   vp, sz, vp, vp, sz, vp]
    L.fgmp_gemm.restype = ctypes.c_int
    L.fgmp_gemm.argtypes = [vp, i64, vp, i64, i64, vp, i64, vp, sz, vp]
    L.fgmp_quant_gemm_fused.restype = ctypes.c_int
    L.fgmp_quant_gemm_fused.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, f32, f32, vp, i64, vp, i64,
                                        vp, sz, vp]
    L.fgmp_quant_gemm_fused_static_scratch.restype = ctypes.c_int
    L.fgmp_quant_gemm_fused_static_scratch.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, f32, f32, vp, i64, vp, i64, vp]
    L.fgmp_unpack_canonical.restype = ctypes.c_int
    L.fgmp_unpack_canonical.argtypes = [vp, i64, i64, vp, vp, vp, vp]
    L.fgmp_dequantize_f16.restype = ctypes.c_int
    L.fgmp_dequantize_f16.argtypes = [vp, i64, i64, vp, i64, i64, vp]
    L.fgmp_quantize_dequantize_f16.restype = ctypes.c_int
    L.fgmp_quantize_dequantize_f16.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, f32, f32, vp, i64, i64, vp]
    L.fgmp_packed_info.restype = ctypes.c_int
    L.fgmp_packed_info.argtypes = [vp, ctypes.POINTER(_PackedInfo), vp]
    L.fgmp_threshold_for_fraction.restype = ctypes.c_int
    L.fgmp_threshold_for_fraction.argtypes = [vp, i64, ctypes.c_double, ctypes.POINTER(f32), vp]
    L.fgmp_threshold_for_fraction_multi.restype = ctypes.c_int
    L.fgmp_threshold_for_fraction_multi.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(i64), ctypes.c_int32,
                                                    ctypes.c_double, ctypes.POINTER(f32), vp]
    L.fgmp_selftest_encode_ranges.restype = ctypes.c_int
    L.fgmp_selftest_encode_ranges.argtypes = [ctypes.c_int, vp, vp, vp, vp]
    L.fgmp_selftest_decode_table.restype = ctypes.c_int
    L.fgmp_selftest_decode_table.argtypes = [ctypes.c_int, vp, vp]
    L.fgmp_selftest_mfma_rate.restype = ctypes.c_int
    L.fgmp_selftest_mfma_rate.argtypes = [ctypes.c_int64, ctypes.c_int32, vp, vp]
    L.fgmp_selftest_time_gemm_kernel.restype = ctypes.c_int
    L.fgmp_selftest_time_gemm_kernel.argtypes = [vp, vp]
    L.fgmp_selftest_quantizer_traffic.restype = ctypes.c_int
    L.fgmp_selftest_quantizer_traffic.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, vp, sz, vp]
    return L


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise FgmpError(f"{what} failed: {_ERRORS.get(rc, rc)}")


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise FgmpError(f"unsupported dtype {t.dtype}")


def _ptr(t) -> int | None:
    return None if t is None else t.data_ptr()


def _require_cuda(*tensors) -> None:
    for t in tensors:
        if t is not None and not t.is_cuda:
            raise FgmpError("all tensors must live on the GPU")


@dataclass
class Packed:
    """An opaque packed FGMP tensor in device memory."""
    buf: torch.Tensor   # uint8
    rows: int
    K: int


def version() -> str:
    return lib().fgmp_version().decode()


def packed_bytes(rows: int, K: int) -> int:
    return int(lib().fgmp_packed_bytes(rows, K))


def workspace_bytes(M: int, N: int, K: int) -> int:
    return int(lib().fgmp_workspace_bytes(M, N, K))


def workspace_bytes_packed_out(M: int, N: int, K: int, epilogue: int | None = None) -> int:
    if epilogue is None:
        return int(lib().fgmp_workspace_bytes_packed_out(M, N, K))
    return int(lib().fgmp_workspace_bytes_packed_out_ex(M, N, K, int(epilogue)))


WORKSPACE_CONTROL_BYTES = 65536   # FGMP_WORKSPACE_CONTROL_BYTES


def new_workspace(nbytes: int, device) -> torch.Tensor:
    """A workspace of `nbytes` whose control region (the arrival counters at its start) is zero, as
    the library requires of a workspace's first use; the rest is left uninitialized."""
    ws = torch.empty(int(nbytes), dtype=torch.uint8, device=device)
    ws[:min(int(nbytes), WORKSPACE_CONTROL_BYTES)].zero_()
    return ws


def _alloc_packed(rows: int, K: int, device) -> Packed:
    n = packed_bytes(rows, K)
    if n == 0:
        raise FgmpError("bad packed shape")
    return Packed(torch.empty(n, dtype=torch.uint8, device=device), rows, K)


SCORE_MODES = {"nvfp4_error": 0, "delta": 1}   # fgmp_score_mode_t
EPILOGUE_NONE, EPILOGUE_SILU_GATE, EPILOGUE_ONE_LAUNCH = 0, 1, 0x100   # fgmp_epilogue_t (the last one is a flag)


def quantize_weights(W: torch.Tensor, fisher: torch.Tensor, threshold: float, tensor_scale: float,
                     want_scores: bool = False, out: Packed | None = None, score_mode: str | None = None):
    _require_cuda(W, fisher)
    N, K = W.shape
    ldf = 0 if fisher.dim() == 1 else fisher.stride(0)
    out = out or _alloc_packed(N, K, W.device)
    scores = torch.empty((N, K // 16), dtype=torch.float32, device=W.device) if want_scores else None
    if score_mode is None:
        rc = lib().fgmp_quantize_weights(_ptr(W), _dtype_code(W), N, K, W.stride(0), _ptr(fisher), ldf,
                                         float(threshold), float(tensor_scale), _ptr(out.buf), out.buf.numel(),
                                         _ptr(scores), _stream())
    else:
        rc = lib().fgmp_quantize_weights_ex(_ptr(W), _dtype_code(W), N, K, W.stride(0), _ptr(fisher), ldf,
                                            float(threshold), float(tensor_scale), SCORE_MODES[score_mode],
                                            _ptr(out.buf), out.buf.numel(), _ptr(scores), _stream())
    _check(rc, "fgmp_quantize_weights")
    return (out, scores) if want_scores else out


def quantize_weights_clip(W: torch.Tensor, fisher: torch.Tensor, threshold: float, tensor_scale: float,
                          want_scores: bool = False, out: Packed | None = None):
    """quantize_weights with the block scales chosen by sensitivity-weighted clipping (Eq. 11)."""
    _require_cuda(W, fisher)
    N, K = W.shape
    ldf = 0 if fisher.dim() == 1 else fisher.stride(0)
    out = out or _alloc_packed(N, K, W.device)
    scores = torch.empty((N, K // 16), dtype=torch.float32, device=W.device) if want_scores else None
    ws = torch.empty(N * (K // 16), dtype=torch.uint8, device=W.device)
    rc = lib().fgmp_quantize_weights_clip(_ptr(W), _dtype_code(W), N, K, W.stride(0), _ptr(fisher), ldf,
                                          float(threshold), float(tensor_scale), _ptr(out.buf), out.buf.numel(),
                                          _ptr(scores), _ptr(ws), ws.numel(), _stream())
    _check(rc, "fgmp_quantize_weights_clip")
    return (out, scores) if want_scores else out


def quantize_activations(X: torch.Tensor, fisher_k: torch.Tensor, threshold: float, tensor_scale: float,
                         want_scores: bool = False, out: Packed | None = None, score_mode: str | None = None):
    _require_cuda(X, fisher_k)
    M, K = X.shape
    out = out or _alloc_packed(M, K, X.device)
    scores = torch.empty((M, K // 16), dtype=torch.float32, device=X.device) if want_scores else None
    if score_mode is None:
        rc = lib().fgmp_quantize_activations(_ptr(X), _dtype_code(X), M, K, X.stride(0), _ptr(fisher_k),
                                             float(threshold), float(tensor_scale), _ptr(out.buf),
                                             out.buf.numel(), _ptr(scores), _stream())
    else:
        rc = lib().fgmp_quantize_activations_ex(_ptr(X), _dtype_code(X), M, K, X.stride(0), _ptr(fisher_k),
                                                float(threshold), float(tensor_scale), SCORE_MODES[score_mode],
                                                _ptr(out.buf), out.buf.numel(), _ptr(scores), _stream())
    _check(rc, "fgmp_quantize_activations")
    return (out, scores) if want_scores else out


def gemm(pX: Packed, pW: Packed, out: torch.Tensor | None = None, workspace: torch.Tensor | None = None):
    if pX.K != pW.K:
        raise FgmpError("K mismatch")
    M, N, K = pX.rows, pW.rows, pX.K
    Y = out if out is not None else torch.empty((M, N), dtype=torch.float32, device=pX.buf.device)
    if workspace is None:
        workspace = new_workspace(workspace_bytes(M, N, K), pX.buf.device)
    ws_n = workspace.numel()
    rc = lib().fgmp_gemm(_ptr(pX.buf), M, _ptr(pW.buf), N, K, _ptr(Y), Y.stride(0), _ptr(workspace), ws_n,
                         _stream())
    _check(rc, "fgmp_gemm")
    return Y


def quant_gemm_fused(X: torch.Tensor, fisher_k: torch.Tensor, threshold: float, scale_x: float, pW: Packed,
                     out: torch.Tensor | None = None, workspace: torch.Tensor | None = None,
                     score_mode: str | None = None):
    _require_cuda(X, fisher_k)
    M, K = X.shape
    if K != pW.K:
        raise FgmpError("K mismatch")
    N = pW.rows
    Y = out if out is not None else torch.empty((M, N), dtype=torch.float32, device=X.device)
    if workspace is None:
        workspace = new_workspace(workspace_bytes(M, N, K), X.device)
    if score_mode is None:
        rc = lib().fgmp_quant_gemm_fused(_ptr(X), _dtype_code(X), M, K, X.stride(0), _ptr(fisher_k),
                                         float(threshold), float(scale_x), _ptr(pW.buf), N, _ptr(Y), Y.stride(0),
                                         _ptr(workspace), workspace.numel(), _stream())
    else:
        rc = lib().fgmp_quant_gemm_fused_ex(_ptr(X), _dtype_code(X), M, K, X.stride(0), _ptr(fisher_k),
                                            float(threshold), float(scale_x), SCORE_MODES[score_mode], _ptr(pW.buf),
                                            N, _ptr(Y), Y.stride(0), _ptr(workspace), workspace.numel(), _stream())
    _check(rc, "fgmp_quant_gemm_fused")
    return Y


STATIC_SCRATCH_BYTES = 16 * 1024 * 1024   # FGMP_STATIC_SCRATCH_BYTES


def quant_gemm_fused_static_scratch(X: torch.Tensor, fisher_k: torch.Tensor, threshold: float, scale_x: float,
                                    pW: Packed, out: torch.Tensor) -> torch.Tensor:
    """quant_gemm_fused without a workspace: the library's static scratch array serves (small products
    only).  `out` is required: the binding allocates nothing either."""
    _require_cuda(X, fisher_k, out)
    M, K = X.shape
    if K != pW.K:
        raise FgmpError("K mismatch")
    rc = lib().fgmp_quant_gemm_fused_static_scratch(_ptr(X), _dtype_code(X), M, K, X.stride(0), _ptr(fisher_k),
                                                    float(threshold), float(scale_x), _ptr(pW.buf), pW.rows,
                                                    _ptr(out), out.stride(0), _stream())
    _check(rc, "fgmp_quant_gemm_fused_static_scratch")
    return out


def quant_gemm_fused_packed_out(X: torch.Tensor, fisher_k: torch.Tensor, threshold: float, scale_x: float,
                                pW: Packed, fisher_n: torch.Tensor, threshold_y: float, scale_y: float,
                                want_scores: bool = False, out: Packed | None = None,
                                workspace: torch.Tensor | None = None, epilogue: int | None = None):
    """Fused step whose results are quantized and packed (a packed M x N activation tensor; with
    epilogue=EPILOGUE_SILU_GATE the gated activation of the 32 + 32 row groups of W, M x N/2)."""
    _require_cuda(X, fisher_k, fisher_n)
    M, K = X.shape
    if K != pW.K:
        raise FgmpError("K mismatch")
    N = pW.rows
    n_out = N // 2 if epilogue is not None and (epilogue & 0xFF) == EPILOGUE_SILU_GATE else N
    out = out or _alloc_packed(M, n_out, X.device)
    scores = torch.empty((M, n_out // 16), dtype=torch.float32, device=X.device) if want_scores else None
    if epilogue is None:
        if workspace is None:
            workspace = new_workspace(lib().fgmp_workspace_bytes_packed_out(M, N, K), X.device)
        rc = lib().fgmp_quant_gemm_fused_packed_out(_ptr(X), _dtype_code(X), M, K, X.stride(0), _ptr(fisher_k),
                                                    float(threshold), float(scale_x), _ptr(pW.buf), N, _ptr(fisher_n),
                                                    float(threshold_y), float(scale_y), _ptr(out.buf), out.buf.numel(),
                                                    _ptr(scores), _ptr(workspace), workspace.numel(), _stream())
        _check(rc, "fgmp_quant_gemm_fused_packed_out")
    else:
        if workspace is None:
            workspace = new_workspace(lib().fgmp_workspace_bytes_packed_out_ex(M, N, K, int(epilogue)), X.device)
        rc = lib().fgmp_quant_gemm_fused_packed_out_ex(_ptr(X), _dtype_code(X), M, K, X.stride(0), _ptr(fisher_k),
                                                       float(threshold), float(scale_x), _ptr(pW.buf), N, int(epilogue),
                                                       _ptr(fisher_n), float(threshold_y), float(scale_y), _ptr(out.buf),
                                                       out.buf.numel(), _ptr(scores), _ptr(workspace), workspace.numel(),
                                                       _stream())
        _check(rc, "fgmp_quant_gemm_fused_packed_out_ex")
    return (out, scores) if want_scores else out


def unpack_canonical(p: Packed):
    """(codes [rows,K] u8, scales [rows,K/16] u8, mask [rows,K/16] u8) on the device."""
    dev = p.buf.device
    codes = torch.empty((p.rows, p.K), dtype=torch.uint8, device=dev)
    scales = torch.empty((p.rows, p.K // 16), dtype=torch.uint8, device=dev)
    mask = torch.empty((p.rows, p.K // 16), dtype=torch.uint8, device=dev)
    rc = lib().fgmp_unpack_canonical(_ptr(p.buf), p.rows, p.K, _ptr(codes), _ptr(scales), _ptr(mask), _stream())
    _check(rc, "fgmp_unpack_canonical")
    return codes, scales, mask


def dequantize_f16(p: Packed, out: torch.Tensor | None = None) -> torch.Tensor:
    """Dense FP16 values (without the tensor scale), zero-padded to [rows_out, ld]."""
    ld = -(-p.K // 128) * 128
    if out is None:
        out = torch.empty((-(-p.rows // 8) * 8, ld), dtype=torch.float16, device=p.buf.device)
    rc = lib().fgmp_dequantize_f16(_ptr(p.buf), p.rows, p.K, _ptr(out), out.shape[0], out.stride(0), _stream())
    _check(rc, "fgmp_dequantize_f16")
    return out


def quantize_dequantize_f16(X: torch.Tensor, fisher_k: torch.Tensor, threshold: float, tensor_scale: float,
                            out: torch.Tensor | None = None) -> torch.Tensor:
    """FP16 values of the codes the quantizer selects (without the tensor scale), [rows_out, ld]."""
    _require_cuda(X, fisher_k)
    M, K = X.shape
    if out is None:
        out = torch.empty((-(-M // 8) * 8, -(-K // 128) * 128), dtype=torch.float16, device=X.device)
    rc = lib().fgmp_quantize_dequantize_f16(_ptr(X), _dtype_code(X), M, K, X.stride(0), _ptr(fisher_k),
                                            float(threshold), float(tensor_scale), _ptr(out), out.shape[0],
                                            out.stride(0), _stream())
    _check(rc, "fgmp_quantize_dequantize_f16")
    return out


def packed_info(p: Packed) -> dict:
    info = _PackedInfo()
    _check(lib().fgmp_packed_info(_ptr(p.buf), ctypes.byref(info), _stream()), "fgmp_packed_info")
    return {name: getattr(info, name) for name, _ in _PackedInfo._fields_}


def threshold_for_fraction(scores: torch.Tensor, fraction: float) -> float:
    _require_cuda(scores)
    s = scores.contiguous().view(-1)
    out = ctypes.c_float()
    _check(lib().fgmp_threshold_for_fraction(_ptr(s), s.numel(), float(fraction), ctypes.byref(out), _stream()),
           "fgmp_threshold_for_fraction")
    return float(out.value)


def threshold_for_fraction_multi(score_tensors, fraction: float) -> float:
    """One threshold over several score tensors (a global threshold over layers, Eq. 10)."""
    flat = [t.contiguous().view(-1) for t in score_tensors]
    _require_cuda(*flat)
    n = len(flat)
    ptrs = (ctypes.c_void_p * n)(*[t.data_ptr() for t in flat])
    counts = (ctypes.c_int64 * n)(*[t.numel() for t in flat])
    out = ctypes.c_float()
    _check(lib().fgmp_threshold_for_fraction_multi(ptrs, counts, n, float(fraction), ctypes.byref(out), _stream()),
           "fgmp_threshold_for_fraction_multi")
    return float(out.value)


def selftest_encode_ranges(fmt: int, device="cuda"):
    mn = torch.empty(256, dtype=torch.int32, device=device)
    mx = torch.empty(256, dtype=torch.int32, device=device)
    viol = torch.empty(4, dtype=torch.int32, device=device)
    _check(lib().fgmp_selftest_encode_ranges(fmt, _ptr(mn), _ptr(mx), _ptr(viol), _stream()),
           "fgmp_selftest_encode_ranges")
    torch.cuda.synchronize()
    to_u32 = lambda t: t.cpu().numpy().view("uint32")
    return to_u32(mn), to_u32(mx), int(to_u32(viol)[0])


def selftest_mfma_rate(workgroups: int, iters: int, sink: torch.Tensor) -> None:
    """Launch the pure-MFMA reference loop (the caller times it); sink: workgroups * 256 floats."""
    assert sink.dtype == torch.float32 and sink.numel() >= workgroups * 256
    _check(lib().fgmp_selftest_mfma_rate(int(workgroups), int(iters), _ptr(sink), _stream()), "fgmp_selftest_mfma_rate")


def selftest_time_gemm_kernel(start: "torch.cuda.Event | None", stop: "torch.cuda.Event | None") -> None:
    """Set (or, with None, clear) the pair of timing events the library records around every launch of
    the prefill GEMM kernel.  The events must have been recorded once already (torch creates the HIP
    event on first use)."""
    hs = 0 if start is None else int(start.cuda_event)
    he = 0 if stop is None else int(stop.cuda_event)
    if (start is not None and hs == 0) or (stop is not None and he == 0):
        raise FgmpError("timing events must be recorded once before they are handed to the library")
    _check(lib().fgmp_selftest_time_gemm_kernel(hs or None, he or None), "fgmp_selftest_time_gemm_kernel")


def selftest_quantizer_traffic(X: torch.Tensor, fisher_k: torch.Tensor, out: Packed) -> None:
    """Launch the traffic model of the activation quantizer (measurement builds only; the caller times it)."""
    _require_cuda(X, fisher_k)
    M, K = X.shape
    _check(lib().fgmp_selftest_quantizer_traffic(_ptr(X), _dtype_code(X), M, K, X.stride(0), _ptr(fisher_k), _ptr(out.buf),
                                                 out.buf.numel(), _stream()), "fgmp_selftest_quantizer_traffic")


def selftest_decode_table(fmt: int, device="cuda"):
    out = torch.empty(256, dtype=torch.float32, device=device)
    _check(lib().fgmp_selftest_decode_table(fmt, _ptr(out), _stream()), "fgmp_selftest_decode_table")
    return out.cpu().numpy()
