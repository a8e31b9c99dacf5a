"""The entry point that allocates nothing (fgmp_quant_gemm_fused_static_scratch): called through the C ABI,
its results must equal fgmp_quant_gemm_fused's bit for bit -- on two calls in a row, the second on a smaller
input (the static array keeps the first call's contents), and a product too large for the array is refused
before anything is launched."""
import numpy as np
import pytest
import torch

from paper_2504_14152_amd import fgmp, synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _case(M, K, N, seed):
    x = synth.activations(M, K, seed, 1)
    w = synth.weights(N, K, seed, 2)
    bits = synth.f32_to_bf16_bits(x)
    xd = torch.from_numpy(bits.view(np.int16)).to(DEV).view(torch.bfloat16)
    wd = torch.from_numpy(w).to(DEV)
    fx = torch.from_numpy(synth.fisher_per_channel(K, seed, 3)).to(DEV)
    fw = torch.from_numpy(synth.fisher_per_channel(K, seed, 4)).to(DEV)
    sx = float(synth.default_tensor_scale(synth.bf16_bits_to_f32(bits)))
    sw = float(synth.default_tensor_scale(w))
    _, sxs = fgmp.quantize_activations(xd, fx, np.inf, sx, want_scores=True)
    _, sws = fgmp.quantize_weights(wd, fw, np.inf, sw, want_scores=True)
    Tx, Tw = fgmp.threshold_for_fraction(sxs, 0.1), fgmp.threshold_for_fraction(sws, 0.1)
    return xd, fx, Tx, sx, fgmp.quantize_weights(wd, fw, Tw, sw)


def test_static_scratch_entry_point_matches_the_workspace_one():
    print("static scratch: 32 x 4096 x 4096, then 5 x 1024 x 520", flush=True)
    big = _case(32, 4096, 4096, 61)      # K ranges combined through partial sums and arrival counters
    small = _case(5, 1024, 520, 62)
    for xd, fx, Tx, sx, pW in (big, small):
        M, N = xd.shape[0], pW.rows
        assert fgmp.workspace_bytes(M, N, pW.K) <= fgmp.STATIC_SCRATCH_BYTES
        want = fgmp.quant_gemm_fused(xd, fx, Tx, sx, pW)
        got = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
        before = torch.cuda.memory_allocated()
        fgmp.quant_gemm_fused_static_scratch(xd, fx, Tx, sx, pW, out=got)
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        assert torch.equal(got, want)
    # once more on the first input: the array now holds the smaller call's leftovers
    xd, fx, Tx, sx, pW = big
    want = fgmp.quant_gemm_fused(xd, fx, Tx, sx, pW)
    got = torch.empty_like(want)
    fgmp.quant_gemm_fused_static_scratch(xd, fx, Tx, sx, pW, out=got)
    assert torch.equal(got, want)


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    xd, fx, Tx, sx, pW = _case(8, 256, 72, 63)
    L = fgmp.lib()
    Y = torch.empty((4096, 72), dtype=torch.float32, device=DEV)
    # a prefill-sized product: its workspace exceeds the static array
    assert fgmp.workspace_bytes(4096, 12288, 4096) > fgmp.STATIC_SCRATCH_BYTES
    rc = L.fgmp_quant_gemm_fused_static_scratch(xd.data_ptr(), 1, 4096, 4096, 4096, fx.data_ptr(), 0.0, 1.0,
                                                pW.buf.data_ptr(), 12288, Y.data_ptr(), 12288, None)
    assert rc == -4
    assert L.fgmp_quant_gemm_fused_static_scratch(None, 1, 8, 256, 256, None, 0.0, 1.0, None, 72, None, 72, None) == -1
