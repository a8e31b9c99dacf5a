"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle
on the same seeded inputs.  Codes, block scales, masks and scores must be
bit-exact; GEMM outputs must satisfy |err| <= 1e-5 * sum_k |x_k w_k|."""
import numpy as np
import pytest
import torch

from oracle import fgmp_oracle as orc
from paper_2504_14152_amd import fgmp, synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _say(msg):
    print(msg, flush=True)


def _to_dev_bf16(x32: np.ndarray):
    """fp32 numpy -> (bf16 device tensor, the exactly equal fp32 numpy array)."""
    bits = synth.f32_to_bf16_bits(x32)
    t = torch.from_numpy(bits.view(np.int16)).to(DEV).view(torch.bfloat16)
    return t, synth.bf16_bits_to_f32(bits)


def _unpack_np(p):
    codes, scales, mask = fgmp.unpack_canonical(p)
    torch.cuda.synchronize()
    return codes.cpu().numpy(), scales.cpu().numpy(), mask.cpu().numpy()


def _assert_quant_equal(p, scores_dev, want, label):
    codes, scales, mask = _unpack_np(p)
    assert np.array_equal(mask, want["mask"]), f"{label}: mask differs in {(mask != want['mask']).sum()} blocks"
    assert np.array_equal(scales, want["scales"]), f"{label}: scales differ"
    assert np.array_equal(codes, want["codes"]), f"{label}: codes differ in {(codes != want['codes']).sum()} elements"
    if scores_dev is not None:
        got = scores_dev.cpu().numpy()
        assert np.array_equal(got.view(np.uint32), want["scores"].view(np.uint32)), f"{label}: scores differ"


# ------------------------------------------------------------------ conversions

@pytest.mark.parametrize("fmt,name", [(0, "e2m1"), (1, "e4m3"), (2, "e2m1-int"), (3, "e4m3-int")])
def test_encoders_over_every_fp32_input(fmt, name):
    """Every non-negative FP32 pattern up to +inf: the device encoder's output
    is piecewise constant; each piece's end points are checked with the oracle
    and the pieces must tile the whole range in increasing code order."""
    _say(f"encode ranges {name}")
    mn, mx, violations = fgmp.selftest_encode_ranges(fmt)
    assert violations == 0
    enc = orc.e2m1_encode if fmt in (0, 2) else orc.e4m3_encode
    used = [c for c in range(256) if mn[c] <= mx[c]]
    assert used == list(range(8 if fmt in (0, 2) else 127))
    expect_start = 0
    for c in used:
        assert int(mn[c]) == expect_start
        lo = np.array([mn[c]], dtype=np.uint32).view(np.float32)
        hi = np.array([mx[c]], dtype=np.uint32).view(np.float32)
        assert int(enc(lo)[0]) == c and int(enc(hi)[0]) == c
        expect_start = int(mx[c]) + 1
    assert expect_start - 1 == 0x7F800000


@pytest.mark.parametrize("fmt", [0, 1, 2, 3])
def test_decode_tables(fmt):
    tab = fgmp.selftest_decode_table(fmt)
    if fmt in (0, 2):
        for c in range(16):
            assert tab[c] == orc.e2m1_decode(c) and np.signbit(tab[c]) == bool(c & 8)
    else:
        for c in range(256):
            if c & 0x7F != 0x7F:
                assert tab[c] == orc.e4m3_decode(c) and np.signbit(tab[c]) == bool(c & 0x80)


# ------------------------------------------------------------------ quantizer

def _run_act_case(x32, fisher, p, label, bf16):
    if bf16:
        xd, xref = _to_dev_bf16(x32)
    else:
        xd, xref = torch.from_numpy(x32).to(DEV), x32
    S = float(synth.default_tensor_scale(xref))
    fd = torch.from_numpy(fisher).to(DEV)
    base = orc.quantize(xref, fisher, np.inf, S)
    T = orc.threshold(base["scores"], p)
    want = orc.quantize(xref, fisher, T, S)
    _say(f"quantize_activations {label} shape={x32.shape} bf16={bf16} p={p} T={T}")
    pk, scores = fgmp.quantize_activations(xd, fd, T, S, want_scores=True)
    torch.cuda.synchronize()
    _assert_quant_equal(pk, scores, want, label)
    T_lib = fgmp.threshold_for_fraction(scores, p)
    assert T_lib == T
    info = fgmp.packed_info(pk)
    assert info["n_fp8_blocks"] == int(want["mask"].sum()) and info["rows"] == x32.shape[0]
    return pk, want, S


@pytest.mark.parametrize("p", [0.0, 0.1, 0.3, 1.0])
def test_quantize_activations_tiny(p):
    cfg = synth.tiny_config(0)
    _run_act_case(cfg["x"], cfg["fisher_x"], p, "tiny", bf16=False)


@pytest.mark.parametrize("rows,K,bf16", [(1, 16, False), (13, 304, True), (8, 128, True), (67, 1040, False),
                                          (256, 4096, True), (300, 11008, True)])
def test_quantize_activations_ragged(rows, K, bf16):
    x = synth.activations(rows, K, 5, 31, outlier_count=max(1, K // 100))
    f = synth.fisher_per_channel(K, 5, 32)
    _run_act_case(x, f, 0.1, "ragged", bf16)


def test_quantize_activations_degenerate_blocks():
    K = 256
    x = np.zeros((9, K), dtype=np.float32)
    x[1, :] = 1e-7                           # block scale underflows to code 0
    x[2, :16] = 448.0                        # at the FP8 maximum
    x[3, ::16] = -3.0
    x[4, :] = np.float32(-0.0)
    x[5, :] = np.linspace(-1, 1, K)
    x[6, :] = np.float32(1e-42)              # fp32 subnormal inputs
    f = synth.fisher_per_channel(K, 1, 33)
    for T in (np.inf, -np.inf, 0.0, 1e-9):
        S = float(np.float32(1.0))
        want = orc.quantize(x, f, T, S)
        pk, sc = fgmp.quantize_activations(torch.from_numpy(x).to(DEV), torch.from_numpy(f).to(DEV), T, S,
                                           want_scores=True)
        _assert_quant_equal(pk, sc, want, f"degenerate T={T}")


def test_quantize_activations_llama_qkv_full_size():
    """The benchmark's activation shape (4096 x 4096 bf16, 1% outlier channels)."""
    x = synth.activations(4096, 4096, 0, 1)
    _run_act_case(x, synth.fisher_per_channel(4096, 0, 3), 0.1, "qkv-prefill-X", bf16=True)


def test_quantize_activations_standalone_size_sampled_rows():
    """The standalone quantizer's benchmark tensor (16384 x 8192 bf16, 1% outlier channels, 8.4 M blocks),
    drawn on the device; the oracle quantizes 96 whole rows (8-row tiles at the start, the end and in
    between) from the same bf16 values and every field of those rows must agree."""
    rows_n, K, p = 16384, 8192, 0.1
    gen = torch.Generator(device=DEV)
    gen.manual_seed(16)
    x = torch.empty((rows_n, K), dtype=torch.float32, device=DEV).normal_(0.0, 1.0, generator=gen)
    ch = torch.randperm(K, device=DEV, generator=gen)[: K // 100]
    x[:, ch] *= 20.0
    xd = x.to(torch.bfloat16)
    del x
    f = synth.fisher_per_channel(K, 0, 16)
    fd = torch.from_numpy(f).to(DEV)
    S = float(xd.abs().max().float()) / 448.0
    _, sc = fgmp.quantize_activations(xd, fd, np.inf, S, want_scores=True)
    T = fgmp.threshold_for_fraction(sc, p)
    del sc
    pk, scores = fgmp.quantize_activations(xd, fd, T, S, want_scores=True)
    info = fgmp.packed_info(pk)
    assert info["n_fp8_blocks"] == int(p * info["n_blocks"] + 0.5)
    rng = np.random.default_rng(16)
    tiles = np.unique(np.concatenate([[0, rows_n // 8 - 1], rng.choice(rows_n // 8, 10, replace=False)]))
    rows = np.concatenate([np.arange(8 * t, 8 * t + 8) for t in tiles])
    ridx = torch.from_numpy(rows).to(DEV)
    want = orc.quantize(xd[ridx].float().cpu().numpy(), f, T, S)
    codes, scales, mask = fgmp.unpack_canonical(pk)
    assert np.array_equal(mask[ridx].cpu().numpy(), want["mask"])
    assert np.array_equal(scales[ridx].cpu().numpy(), want["scales"])
    assert np.array_equal(codes[ridx].cpu().numpy(), want["codes"])
    assert np.array_equal(scores[ridx].cpu().numpy().view(np.uint32), want["scores"].view(np.uint32))


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_quantize_activations_delta_score_large_tensor_sampled_rows(dtype):
    """The Eq. 8 score on a tensor large enough for the trimmed activation kernel (8192 x 8192: 65536 tiles),
    with a tensor scale small enough that some values exceed the FP8 range (the clamping path): 96 whole rows
    against the oracle -- codes, scales, decisions, scores -- and the whole tensor against the general kernel's
    result on a row slice that it serves (same arithmetic)."""
    rows_n, K, p = 8192, 8192, 0.1
    gen = torch.Generator(device=DEV)
    gen.manual_seed(26)
    x = torch.empty((rows_n, K), dtype=torch.float32, device=DEV).normal_(0.0, 1.0, generator=gen)
    ch = torch.randperm(K, device=DEV, generator=gen)[: K // 100]
    x[:, ch] *= 20.0
    xd = x.to(torch.bfloat16) if dtype == "bf16" else x
    del x
    f = synth.fisher_per_channel(K, 0, 26)
    fd = torch.from_numpy(f).to(DEV)
    S = float(xd.abs().max().float()) / 448.0 / 1.5
    _, sc = fgmp.quantize_activations(xd, fd, np.inf, S, want_scores=True, score_mode="delta")
    T = fgmp.threshold_for_fraction(sc, p)
    del sc
    pk, scores = fgmp.quantize_activations(xd, fd, T, S, want_scores=True, score_mode="delta")
    rng = np.random.default_rng(26)
    tiles = np.unique(np.concatenate([[0, rows_n // 8 - 1], rng.choice(rows_n // 8, 10, replace=False)]))
    rows = np.concatenate([np.arange(8 * t, 8 * t + 8) for t in tiles])
    ridx = torch.from_numpy(rows).to(DEV)
    want = orc.quantize(xd[ridx].float().cpu().numpy(), f, T, S, score_mode="delta")
    codes, scales, mask = fgmp.unpack_canonical(pk)
    assert 0 < int(mask.sum()) < mask.numel()
    assert np.array_equal(mask[ridx].cpu().numpy(), want["mask"])
    assert np.array_equal(scales[ridx].cpu().numpy(), want["scales"])
    assert np.array_equal(codes[ridx].cpu().numpy(), want["codes"])
    assert np.array_equal(scores[ridx].cpu().numpy().view(np.uint32), want["scores"].view(np.uint32))
    # the first 2048 rows alone are a tensor of 16384 tiles: the general kernel
    pk2, scores2 = fgmp.quantize_activations(xd[:2048], fd, T, S, want_scores=True, score_mode="delta")
    c2, s2, m2 = fgmp.unpack_canonical(pk2)
    assert torch.equal(c2, codes[:2048]) and torch.equal(s2, scales[:2048]) and torch.equal(m2, mask[:2048])
    assert torch.equal(scores2, scores[:2048])


def test_quantize_activations_fc2_input():
    x = synth.activations(1024, 11008, 0, 5, kind="silu_gate")
    _run_act_case(x, synth.fisher_per_channel(11008, 0, 6), 0.1, "fc2-X", bf16=True)


@pytest.mark.parametrize("N,K,bf16,per_elem,p", [(256, 256, False, True, 0.1), (77, 304, True, True, 0.3),
                                                 (512, 4096, True, False, 0.1), (130, 1024, False, True, 1.0),
                                                 (64, 128, True, True, 0.0)])
def test_quantize_weights(N, K, bf16, per_elem, p):
    w = synth.weights(N, K, 2, 41)
    f = synth.fisher_per_element(N, K, 2, 42) if per_elem else synth.fisher_per_channel(K, 2, 43)
    if bf16:
        wd, wref = _to_dev_bf16(w)
    else:
        wd, wref = torch.from_numpy(w).to(DEV), w
    S = float(synth.default_tensor_scale(wref))
    T = orc.threshold(orc.quantize(wref, f, np.inf, S)["scores"], p)
    want = orc.quantize(wref, f, T, S)
    _say(f"quantize_weights N={N} K={K} bf16={bf16} per_elem={per_elem} p={p}")
    pk, scores = fgmp.quantize_weights(wd, torch.from_numpy(f).to(DEV), T, S, want_scores=True)
    _assert_quant_equal(pk, scores, want, "weights")
    info = fgmp.packed_info(pk)
    n_hi = int(want["mask"].sum())
    assert info["compact"] == 1 and info["n_fp8_blocks"] == n_hi
    # compact storage: 9 B per FP4 block, 16 B per FP8 block, + 1 bit per block, + tables and padding
    n_blocks = N * K // 16
    algorithmic = orc.storage_bits(n_blocks - n_hi, n_hi) / 8
    tiles = -(-N // 8) * -(-K // 128)
    assert algorithmic <= info["bytes_used"] <= tiles * 64 * 9 + n_hi * 8 + tiles * 12 + 6 * 256


@pytest.mark.parametrize("rows,K,p", [(13, 304, 0.3), (256, 4096, 0.1), (64, 1024, 1.0), (40, 256, 0.0)])
def test_dequantize_f16_is_exact(rows, K, p):
    """The FP16 operand form equals the oracle's real-valued decode bit for bit."""
    x = synth.activations(rows, K, 8, 61, outlier_count=3)
    f = synth.fisher_per_channel(K, 8, 62)
    S = float(synth.default_tensor_scale(x))
    T = orc.threshold(orc.quantize(x, f, np.inf, S)["scores"], p)
    want = orc.quantize(x, f, T, S)
    pk = fgmp.quantize_activations(torch.from_numpy(x).to(DEV), torch.from_numpy(f).to(DEV), T, S)
    got = fgmp.dequantize_f16(pk).cpu().numpy()
    ref = orc.dequantize(want["codes"], want["scales"], want["mask"])
    assert np.array_equal(got[:rows, :K].astype(np.float64), ref)
    assert not got[rows:].any() and not got[:, K:].any()


@pytest.mark.parametrize("rows,K,p,scale_div", [(61, 208, 0.25, 1.0), (256, 1024, 0.1, 1.0), (19, 16, 1.0, 1.0),
                                                 (40, 400, 0.5, 8.0), (8, 128, 0.0, 1.0)])
def test_quantize_dequantize_f16_is_exact(rows, K, p, scale_div):
    """Quantizer writing FP16 values directly: equal to the oracle's decode of
    the oracle's codes, zero in the padding, untouched beyond it."""
    _say(f"quantize_dequantize_f16 {rows}x{K} p={p} S/={scale_div}")
    x = synth.activations(rows, K, 8, 71, outlier_count=3)
    f = synth.fisher_per_channel(K, 8, 72)
    S = float(synth.default_tensor_scale(x)) / scale_div
    T = orc.threshold(orc.quantize(x, f, np.inf, S)["scores"], p)
    want = orc.quantize(x, f, T, S)
    ref = orc.dequantize(want["codes"], want["scales"], want["mask"])
    r8, k128 = -(-rows // 8) * 8, -(-K // 128) * 128
    out = torch.full((r8 + 8, k128 + 128), 7.0, dtype=torch.float16, device=DEV)
    fgmp.quantize_dequantize_f16(torch.from_numpy(x).to(DEV), torch.from_numpy(f).to(DEV), T, S, out=out)
    got = out.cpu().numpy()
    assert np.array_equal(got[:rows, :K].astype(np.float64), ref)
    assert not got[rows:r8, :k128].any() and not got[:r8, K:k128].any()
    assert (got[r8:] == 7.0).all() and (got[:, k128:] == 7.0).all()


# ------------------------------------------------------------------ Eq. 8 score mode

@pytest.mark.parametrize("rows,K,bf16,p,scale_div", [(16, 256, False, 0.1, 1.0), (67, 1040, True, 0.3, 1.0),
                                                      (256, 4096, True, 0.1, 1.0), (40, 400, False, 0.5, 8.0),
                                                      (9, 16, True, 1.0, 1.0), (24, 128, False, 0.0, 1.0)])
def test_quantize_activations_delta_score(rows, K, bf16, p, scale_div):
    """Score = sum F (Q_NVFP4(x) - Q_FP8(x))^2: scores, decisions and codes bit-exact,
    including a tensor scale below amax / 448 (FP8 reconstruction saturates)."""
    _say(f"delta score acts {rows}x{K} bf16={bf16} p={p} S/={scale_div}")
    x = synth.activations(rows, K, 12, 81, outlier_count=max(1, K // 100))
    f = synth.fisher_per_channel(K, 12, 82)
    if bf16:
        xd, xref = _to_dev_bf16(x)
    else:
        xd, xref = torch.from_numpy(x).to(DEV), x
    S = float(synth.default_tensor_scale(xref)) / scale_div
    T = orc.threshold(orc.quantize(xref, f, np.inf, S, score_mode="delta")["scores"], p)
    want = orc.quantize(xref, f, T, S, score_mode="delta")
    pk, scores = fgmp.quantize_activations(xd, torch.from_numpy(f).to(DEV), T, S, want_scores=True,
                                           score_mode="delta")
    _assert_quant_equal(pk, scores, want, "delta acts")
    # the plain entry point and the explicit default mode are the same computation
    a = fgmp.quantize_activations(xd, torch.from_numpy(f).to(DEV), T, S)
    b = fgmp.quantize_activations(xd, torch.from_numpy(f).to(DEV), T, S, score_mode="nvfp4_error")
    assert all(torch.equal(u, v) for u, v in zip(fgmp.unpack_canonical(a), fgmp.unpack_canonical(b)))


@pytest.mark.parametrize("N,K,per_elem,p", [(77, 304, True, 0.3), (512, 1024, False, 0.1), (64, 128, True, 1.0)])
def test_quantize_weights_delta_score(N, K, per_elem, p):
    _say(f"delta score weights {N}x{K} per_elem={per_elem} p={p}")
    w = synth.weights(N, K, 13, 83)
    f = synth.fisher_per_element(N, K, 13, 84) if per_elem else np.ones(K, dtype=np.float32)   # ones: Eq. 12
    wd, wref = _to_dev_bf16(w)
    S = float(synth.default_tensor_scale(wref))
    T = orc.threshold(orc.quantize(wref, f, np.inf, S, score_mode="delta")["scores"], p)
    want = orc.quantize(wref, f, T, S, score_mode="delta")
    pk, scores = fgmp.quantize_weights(wd, torch.from_numpy(f).to(DEV), T, S, want_scores=True, score_mode="delta")
    _assert_quant_equal(pk, scores, want, "delta weights")
    assert fgmp.packed_info(pk)["n_fp8_blocks"] == int(want["mask"].sum())


@pytest.mark.parametrize("M,K,N", [(200, 304, 136), (8, 1024, 72)])
def test_fused_delta_score(M, K, N):
    """Fused call with Eq. 8 scoring (prefill and decode shape) against the oracle."""
    _say(f"fused delta M={M} K={K} N={N}")
    x = synth.activations(M, K, 14, 85)
    w = synth.weights(N, K, 14, 86)
    fx, fw = synth.fisher_per_channel(K, 14, 87), synth.fisher_per_channel(K, 14, 88)
    xd, xref = _to_dev_bf16(x)
    wd, wref = _to_dev_bf16(w)
    sx, sw = float(synth.default_tensor_scale(xref)), float(synth.default_tensor_scale(wref))
    Tx = orc.threshold(orc.quantize(xref, fx, np.inf, sx, score_mode="delta")["scores"], 0.2)
    Tw = orc.threshold(orc.quantize(wref, fw, np.inf, sw, score_mode="delta")["scores"], 0.2)
    pW = fgmp.quantize_weights(wd, torch.from_numpy(fw).to(DEV), Tw, sw, score_mode="delta")
    Y = fgmp.quant_gemm_fused(xd, torch.from_numpy(fx).to(DEV), Tx, sx, pW, score_mode="delta")
    qx = orc.quantize(xref, fx, Tx, sx, score_mode="delta")
    qw = orc.quantize(wref, fw, Tw, sw, score_mode="delta")
    want, tol = orc.gemm(orc.dequantize(qx["codes"], qx["scales"], qx["mask"]), sx,
                         orc.dequantize(qw["codes"], qw["scales"], qw["mask"]), sw)
    err = np.abs(Y.cpu().numpy().astype(np.float64) - want)
    assert np.all(err <= tol)
    # an unknown mode is rejected before anything is launched
    buf = torch.empty(fgmp.packed_bytes(M, K), dtype=torch.uint8, device=DEV)
    fxd = torch.from_numpy(fx).to(DEV)
    rc = fgmp.lib().fgmp_quantize_activations_ex(xd.data_ptr(), 1, M, K, K, fxd.data_ptr(), 0.0, 1.0, 7,
                                                 buf.data_ptr(), buf.numel(), None, None)
    assert rc == -1


# ------------------------------------------------------------------ Eq. 11 clipping

@pytest.mark.parametrize("N,K,bf16,per_elem,p", [(64, 256, False, True, 0.1), (77, 304, True, True, 0.3),
                                                 (256, 1024, True, False, 0.1), (8, 16, False, True, 0.0),
                                                 (40, 128, True, True, 1.0)])
def test_quantize_weights_clip(N, K, bf16, per_elem, p):
    """Sensitivity-weighted clipping: chosen scale codes, codes, scores and decisions bit-exact."""
    _say(f"clip weights N={N} K={K} bf16={bf16} per_elem={per_elem} p={p}")
    w = synth.weights(N, K, 15, 91)
    f = synth.fisher_per_element(N, K, 15, 92) if per_elem else synth.fisher_per_channel(K, 15, 93)
    if bf16:
        wd, wref = _to_dev_bf16(w)
    else:
        wd, wref = torch.from_numpy(w).to(DEV), w
    S = float(synth.default_tensor_scale(wref))
    T = orc.threshold(orc.quantize(wref, f, np.inf, S, clip=True)["scores"], p)
    want = orc.quantize(wref, f, T, S, clip=True)
    pk, scores = fgmp.quantize_weights_clip(wd, torch.from_numpy(f).to(DEV), T, S, want_scores=True)
    _assert_quant_equal(pk, scores, want, "clip weights")
    info = fgmp.packed_info(pk)
    assert info["compact"] == 1 and info["n_fp8_blocks"] == int(want["mask"].sum())
    # clipping changed something relative to dynamic max (except in the all-FP8 case, where no scale is kept)
    plain = orc.quantize(wref, f, T, S)
    if p < 1.0 and N * K > 1024:
        assert (plain["scales"] != want["scales"]).mean() > 0.2


def test_gemm_with_clipped_weights():
    M, K, N = 48, 512, 136
    _say("gemm with clipped weights")
    x = synth.activations(M, K, 16, 94)
    w = synth.weights(N, K, 16, 95)
    fx, fw = synth.fisher_per_channel(K, 16, 96), synth.fisher_per_element(N, K, 16, 97)
    xd, xref = _to_dev_bf16(x)
    wd, wref = _to_dev_bf16(w)
    sx, sw = float(synth.default_tensor_scale(xref)), float(synth.default_tensor_scale(wref))
    Tx = orc.threshold(orc.quantize(xref, fx, np.inf, sx)["scores"], 0.1)
    Tw = orc.threshold(orc.quantize(wref, fw, np.inf, sw, clip=True)["scores"], 0.1)
    pW = fgmp.quantize_weights_clip(wd, torch.from_numpy(fw).to(DEV), Tw, sw)
    Y = fgmp.quant_gemm_fused(xd, torch.from_numpy(fx).to(DEV), Tx, sx, pW)
    qx = orc.quantize(xref, fx, Tx, sx)
    qw = orc.quantize(wref, fw, Tw, sw, clip=True)
    want, tol = orc.gemm(orc.dequantize(qx["codes"], qx["scales"], qx["mask"]), sx,
                         orc.dequantize(qw["codes"], qw["scales"], qw["mask"]), sw)
    assert np.all(np.abs(Y.cpu().numpy().astype(np.float64) - want) <= tol)
    # a workspace smaller than one byte per block is refused
    buf = torch.empty(fgmp.packed_bytes(N, K), dtype=torch.uint8, device=DEV)
    fwd = torch.from_numpy(fw).to(DEV)
    ws = torch.empty(N * K // 16, dtype=torch.uint8, device=DEV)
    rc = fgmp.lib().fgmp_quantize_weights_clip(wd.data_ptr(), 1, N, K, K, fwd.data_ptr(), K, 0.0, sw, buf.data_ptr(),
                                               buf.numel(), None, ws.data_ptr(), ws.numel() - 1, None)
    assert rc == -4


# ------------------------------------------------------------------ Eq. 10 global threshold

def test_global_threshold_over_layers():
    """One threshold over the scores of several tensors (Eq. 10) equals the oracle's
    order statistic over their union: the total FP8 fraction is the target, the
    per-tensor fractions differ (layers with larger sensitivities keep more FP8)."""
    _say("global threshold over 3 tensors")
    shapes = [(64, 512, 1.0), (96, 256, 4.0), (32, 1024, 0.25)]      # rows, K, sensitivity multiplier
    dev_scores, ref_scores, cases = [], [], []
    for i, (rows, K, mult) in enumerate(shapes):
        x = synth.activations(rows, K, 18, 100 + i)
        f = (synth.fisher_per_channel(K, 18, 110 + i) * mult).astype(np.float32)
        S = float(synth.default_tensor_scale(x))
        xd, fd = torch.from_numpy(x).to(DEV), torch.from_numpy(f).to(DEV)
        _, sc = fgmp.quantize_activations(xd, fd, np.inf, S, want_scores=True)
        dev_scores.append(sc)
        ref_scores.append(orc.quantize(x, f, np.inf, S)["scores"])
        cases.append((x, f, S, xd, fd))
    p = 0.2
    T = fgmp.threshold_for_fraction_multi(dev_scores, p)
    assert T == orc.threshold(np.concatenate([r.reshape(-1) for r in ref_scores]), p)
    fractions, n_hi, n_all = [], 0, 0
    for (x, f, S, xd, fd), ref in zip(cases, ref_scores):
        pk = fgmp.quantize_activations(xd, fd, T, S)
        info = fgmp.packed_info(pk)
        assert info["n_fp8_blocks"] == int((ref > T).sum())
        fractions.append(info["n_fp8_blocks"] / info["n_blocks"])
        n_hi += info["n_fp8_blocks"]
        n_all += info["n_blocks"]
    assert n_hi == int(p * n_all + 0.5)
    assert fractions[1] > fractions[0] > fractions[2]
    # one tensor: the same as the single-tensor helper
    assert fgmp.threshold_for_fraction_multi(dev_scores[:1], p) == fgmp.threshold_for_fraction(dev_scores[0], p)


@pytest.mark.parametrize("case", ["ties", "signed", "tiny", "ragged union", "large"])
def test_threshold_selection_on_the_device_is_the_exact_order_statistic(case):
    """The threshold helper selects on the device (radix selection over the score arrays where they
    are); its result is the oracle's order statistic bit for bit: boundary scores tied many times over,
    negative scores and both zeros (the Eq. 8 score can be negative), arrays of one to five elements,
    a union of arrays of odd lengths that start at odd addresses, and 20 M scores in three arrays."""
    rng = synth.rng_for(5, {"ties": 1, "signed": 2, "tiny": 3, "ragged union": 4, "large": 5}[case])
    if case == "ties":
        arrays = [rng.integers(0, 7, size=100003).astype(np.float32) * np.float32(0.37)]
    elif case == "signed":
        a = rng.standard_normal(65537).astype(np.float32)
        a[::17] = 0.0
        a[5::19] = -0.0
        arrays = [a, -np.abs(rng.standard_normal(1001)).astype(np.float32) * np.float32(1e-30)]
    elif case == "tiny":
        arrays = [np.array([3.0], np.float32), np.array([1.0, 1.0], np.float32), np.array([2.0, -5.0], np.float32)]
    elif case == "ragged union":
        arrays = [rng.standard_exponential(n).astype(np.float32) for n in (1, 2, 3, 5, 63, 257, 4099, 70001)]
    else:
        arrays = [(rng.standard_exponential(n).astype(np.float32) ** 2) for n in (12_000_001, 7_999_999, 5)]
    # device copies at odd element offsets inside larger buffers (the kernel reads 16 bytes per lane where it can)
    dev = []
    for i, a in enumerate(arrays):
        buf = torch.empty(a.size + 8, dtype=torch.float32, device=DEV)
        off = 1 + i % 3
        buf[off:off + a.size] = torch.from_numpy(a).to(DEV)
        dev.append(buf[off:off + a.size])
    union = np.concatenate(arrays)
    for p in ((0.1, 0.5, 1.0 - 1.0 / union.size) if case == "large" else (0.0, 1.0, 0.5, 0.1, 0.9, 1.0 / union.size, 1.0 - 1.0 / union.size, 0.3333)):
        want = orc.threshold(union, p)
        got = fgmp.threshold_for_fraction_multi(dev, p)
        assert got == want or (np.isnan(got) and np.isnan(want)), (case, p, got, want)
        assert (union > np.float32(got)).sum() <= int(p * union.size + 0.5)
    assert fgmp.threshold_for_fraction(dev[0], 0.25) == orc.threshold(arrays[0], 0.25)


def _exactly_summable(ax, aw):
    """True if every partial sum of ax @ aw.T, in any order, is an fp32 number: all products are multiples
    of one power of two, and the largest sum of magnitudes is below 2**24 of them."""
    def unit(a):
        m, e = np.frexp(np.abs(a[a != 0]).astype(np.float64))
        mi = (m * 2.0 ** 53).astype(np.int64)
        low = mi & -mi                                   # lowest set bit of the 53-bit significand
        return (e - 53 + np.log2(low.astype(np.float64)).astype(np.int64)).min()
    return float((np.abs(ax) @ np.abs(aw).T).max()) / 2.0 ** float(unit(ax) + unit(aw)) < 2.0 ** 24


def test_layer_chain_with_global_thresholds_matches_oracle_stage_by_stage():
    """Three linears in a row as a decoder layer runs them (Sec. 5.3): QKV-like product -> its FP32 result
    is the next input -> FC1 with the gated activation and output-side quantization (packed H never
    leaves as FP32) -> FC2 from the packed tensor.  One threshold for all weights and one for all
    activations (Eq. 10), taken from a calibration pass without quantization: the device's selection over
    the score arrays equals the oracle's over their union, and the layers end up with different FP8
    fractions.  The operands of the first two products are made so that the products of the STORED values
    have no rounding in any order of summation (checked here on the oracle's values): every stage's
    integers -- codes, block scales, decisions -- and scores then equal the oracle's bit for bit, and the
    last stage's FP32 results agree within the product's tolerance."""
    M, K1, N1, N2, N3, seed, p = 136, 128, 128, 256, 72, 42, 0.2
    x1, w1, w2 = synth.exact_sum_operand(M, K1, seed, 1), synth.exact_sum_operand(N1, K1, seed, 2), synth.exact_sum_operand(N2, N1, seed, 3)
    w3, w3ref = _to_dev_bf16(synth.weights(N3, N2 // 2, seed, 7))
    ones1, ones2, ones3 = np.ones(K1, np.float32), np.ones(N1, np.float32), np.ones(N2 // 2, np.float32)
    # calibration pass (no quantization) and per-tensor sensitivities: smaller where the values are larger
    y1c = (x1.astype(np.float64) @ w1.astype(np.float64).T).astype(np.float32)
    hc = orc.gate_columns((y1c.astype(np.float64) @ w2.astype(np.float64).T).astype(np.float32))
    f1 = (synth.fisher_per_channel(K1, seed, 4) * np.float32(2000.0)).astype(np.float32)
    f2 = (synth.fisher_per_channel(N1, seed, 5) * np.float32((np.abs(x1).max() / np.abs(y1c).max()) ** 2 * 0.002)).astype(np.float32)
    fh = (synth.fisher_per_channel(N2 // 2, seed, 6) * np.float32((np.abs(x1).max() / np.abs(hc).max()) ** 2 * 1500.0)).astype(np.float32)
    S1, S2 = 1.0, float(2.0 ** np.ceil(np.log2(np.abs(y1c).max() / 448.0)))
    Sh, S3 = float(np.float32(np.abs(hc).max()) / np.float32(448.0)), float(synth.default_tensor_scale(w3ref))
    # ---- oracle: thresholds, then the quantized chain
    sx = [orc.quantize(t, f, np.inf, S)["scores"] for t, f, S in ((x1, f1, S1), (y1c, f2, S2), (hc, fh, Sh))]
    sw = [orc.quantize(t, f, np.inf, S)["scores"] for t, f, S in ((w1, ones1, 1.0), (w2, ones2, 1.0), (w3ref, ones3, S3))]
    Tx = orc.threshold(np.concatenate([t.reshape(-1) for t in sx]), p)
    Tw = orc.threshold(np.concatenate([t.reshape(-1) for t in sw]), p)
    deq = lambda q: orc.dequantize(q["codes"], q["scales"], q["mask"])
    q1x, q1w = orc.quantize(x1, f1, Tx, S1), orc.quantize(w1, ones1, Tw, 1.0)
    assert _exactly_summable(deq(q1x), deq(q1w))
    y1 = orc.gemm(deq(q1x), S1, deq(q1w), 1.0)[0]
    y1_32 = y1.astype(np.float32)
    assert np.array_equal(y1_32.astype(np.float64), y1)
    q2x, q2w = orc.quantize(y1_32, f2, Tx, S2), orc.quantize(w2, ones2, Tw, 1.0)
    assert _exactly_summable(deq(q2x), deq(q2w))
    y2 = orc.gemm(deq(q2x), S2, deq(q2w), 1.0)[0]
    y2_32 = y2.astype(np.float32)
    assert np.array_equal(y2_32.astype(np.float64), y2)
    want_h = orc.quantize(orc.gate_columns(y2_32), fh, Tx, Sh)
    q3w = orc.quantize(w3ref, ones3, Tw, S3)
    z_want, z_tol = orc.gemm(deq(want_h), Sh, deq(q3w), S3)
    fractions = [float(q["mask"].mean()) for q in (q1x, q2x, want_h)]
    assert fractions[0] > 0.05 and fractions[2] > 0.05 and len({round(f, 3) for f in fractions}) == 3
    # ---- device: the same thresholds from the same calibration tensors, then the chain on its own outputs
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    x1d, w1d, w2d, f1d, f2d, fhd = up(x1), up(w1), up(w2), up(f1), up(f2), up(fh)
    o1d, o2d, o3d = up(ones1), up(ones2), up(ones3)
    dsx = [fgmp.quantize_activations(t, f, np.inf, S, want_scores=True)[1]
           for t, f, S in ((x1d, f1d, S1), (up(y1c), f2d, S2), (up(hc), fhd, Sh))]
    dsw = [fgmp.quantize_weights(t, f, np.inf, S, want_scores=True)[1] for t, f, S in ((w1d, o1d, 1.0), (w2d, o2d, 1.0), (w3, o3d, S3))]
    assert fgmp.threshold_for_fraction_multi(dsx, p) == Tx and fgmp.threshold_for_fraction_multi(dsw, p) == Tw
    pW1, pW2, pW3 = fgmp.quantize_weights(w1d, o1d, Tw, 1.0), fgmp.quantize_weights(w2d, o2d, Tw, 1.0), fgmp.quantize_weights(w3, o3d, Tw, S3)
    Y1 = fgmp.quant_gemm_fused(x1d, f1d, Tx, S1, pW1)
    assert np.array_equal(Y1.cpu().numpy(), y1_32), "stage 1"
    pH, h_scores = fgmp.quant_gemm_fused_packed_out(Y1, f2d, Tx, S2, pW2, fhd, Tx, Sh, want_scores=True,
                                                     epilogue=fgmp.EPILOGUE_SILU_GATE)
    _assert_quant_equal(pH, h_scores, want_h, "stage 2 (gated, packed output)")
    Z = fgmp.gemm(pH, pW3)
    assert np.all(np.abs(Z.cpu().numpy().astype(np.float64) - z_want) <= z_tol), "stage 3"
    got_fr = [fgmp.packed_info(fgmp.quantize_activations(x1d, f1d, Tx, S1))["n_fp8_blocks"] / (M * K1 // 16),
              fgmp.packed_info(pH)["n_fp8_blocks"] / (M * (N2 // 2) // 16)]
    assert got_fr == [fractions[0], fractions[2]]


# ------------------------------------------------------------------ output-side quantization (Sec. 4.2)

def _exact_product_case(M, K, N, seed):
    """Operands whose stored form equals the input and whose product has no rounding in any summation
    order, so that the FP32 results the epilogue quantizes are the oracle's results exactly."""
    x = synth.exact_sum_operand(M, K, seed, 1)
    w = synth.exact_sum_operand(N, K, seed, 2)
    ones = np.ones(K, dtype=np.float32)
    qx, qw = orc.quantize(x, ones, 0.0, 1.0), orc.quantize(w, ones, 0.0, 1.0)
    ax, aw = orc.dequantize(qx["codes"], qx["scales"], qx["mask"]), orc.dequantize(qw["codes"], qw["scales"], qw["mask"])
    assert np.array_equal(ax, x.astype(np.float64)) and np.array_equal(aw, w.astype(np.float64))
    assert 0.1 < qx["mask"].mean() < 0.35 and 0.1 < qw["mask"].mean() < 0.35
    y64, _ = orc.gemm(ax, 1.0, aw, 1.0)
    y32 = y64.astype(np.float32)
    assert np.array_equal(y32.astype(np.float64), y64)          # the results are fp32 numbers
    assert np.abs(y64).max() * 256 < 2 ** 24                    # ... and so is every partial sum (multiples of 2^-8)
    return x, w, ones, y32


@pytest.mark.parametrize("M,K,N", [(136, 128, 272), (300, 64, 512), (257, 128, 48), (24, 128, 160)])
def test_fused_packed_output_matches_oracle(M, K, N):
    """GEMM whose results are scored, quantized and packed before they reach memory: codes, block
    scales, decisions and scores equal the oracle's quantization of the oracle's product (larger M: in
    the GEMM epilogue; M = 24: staged through FP32)."""
    _say(f"packed output M={M} K={K} N={N}")
    x, w, ones, y32 = _exact_product_case(M, K, N, 31)
    f_n = synth.fisher_per_channel(N, 31, 3)
    s_y = float(np.float32(np.abs(y32).max()) / np.float32(448.0))
    T_y = orc.threshold(orc.quantize(y32, f_n, np.inf, s_y)["scores"], 0.2)
    want = orc.quantize(y32, f_n, T_y, s_y)
    xd, wd, od = torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV), torch.from_numpy(ones).to(DEV)
    pW = fgmp.quantize_weights(wd, od, 0.0, 1.0)
    Y = fgmp.quant_gemm_fused(xd, od, 0.0, 1.0, pW)
    assert np.array_equal(Y.cpu().numpy(), y32)
    pY, scores = fgmp.quant_gemm_fused_packed_out(xd, od, 0.0, 1.0, pW, torch.from_numpy(f_n).to(DEV), T_y, s_y,
                                                  want_scores=True)
    _assert_quant_equal(pY, scores, want, "packed output")
    info = fgmp.packed_info(pY)
    assert info["rows"] == M and info["K"] == N and info["n_fp8_blocks"] == int(want["mask"].sum())
    assert abs(info["tensor_scale"] - s_y) <= 1e-7 * s_y
    # the packed result is an ordinary activation tensor: the next layer multiplies it
    w2 = synth.weights(72, N, 31, 4)
    w2d, w2ref = _to_dev_bf16(w2)
    f2 = synth.fisher_per_channel(N, 31, 5)
    s2 = float(synth.default_tensor_scale(w2ref))
    pW2 = fgmp.quantize_weights(w2d, torch.from_numpy(f2).to(DEV), np.inf, s2)
    Z = fgmp.gemm(pY, pW2)
    q2 = orc.quantize(w2ref, f2, np.inf, s2)
    zw, tol = orc.gemm(orc.dequantize(want["codes"], want["scales"], want["mask"]), s_y,
                       orc.dequantize(q2["codes"], q2["scales"], q2["mask"]), s2)
    assert np.all(np.abs(Z.cpu().numpy().astype(np.float64) - zw) <= tol)


@pytest.mark.parametrize("M,K,N", [(200, 512, 272), (4352, 256, 4096)])
def test_packed_output_on_random_inputs_is_consistent(M, K, N):
    """On ordinary inputs the FP32 results differ from the oracle's fp64 product in the last bits, so
    codes cannot be compared one by one; the epilogue must still equal the standalone quantizer run on
    the very FP32 results the plain fused call writes (same arithmetic, same values).  The second shape
    has whole tiles and tiles computed in two parts along K in one launch."""
    c = _quantized_pair(M, K, N, 33, 0.1, per_elem_w=False)
    f_n = torch.from_numpy(synth.fisher_per_channel(N, 33, 9)).to(DEV)
    Y = fgmp.quant_gemm_fused(c["xd"], c["fxd"], c["Tx"], c["sx"], c["pW"])
    s_y = float(Y.abs().max()) / 448.0
    _, sc0 = fgmp.quantize_activations(Y, f_n, np.inf, s_y, want_scores=True)
    T_y = fgmp.threshold_for_fraction(sc0, 0.2)
    ref, sc_ref = fgmp.quantize_activations(Y, f_n, T_y, s_y, want_scores=True)
    got, sc_got = fgmp.quant_gemm_fused_packed_out(c["xd"], c["fxd"], c["Tx"], c["sx"], c["pW"], f_n, T_y, s_y,
                                                   want_scores=True)
    assert torch.equal(sc_ref, sc_got)
    assert all(torch.equal(u, v) for u, v in zip(fgmp.unpack_canonical(ref), fgmp.unpack_canonical(got)))
    assert fgmp.packed_info(got)["n_fp8_blocks"] == int(0.2 * M * N / 16 + 0.5)


@pytest.mark.parametrize("M,K,N", [(136, 128, 256), (300, 64, 512), (257, 128, 64), (24, 128, 128)])
def test_fused_gated_packed_output_matches_oracle(M, K, N):
    """The same with the gated activation in front of the quantizer: what is scored, quantized and packed
    is SiLU(gate) * up of the 32 + 32 row groups of W, as the oracle computes it from its own product
    (larger M: in the GEMM epilogue; M = 24: staged through FP32)."""
    _say(f"gated packed output M={M} K={K} N={N}")
    x, w, ones, y32 = _exact_product_case(M, K, N, 37)
    h32 = orc.gate_columns(y32)
    f_h = synth.fisher_per_channel(N // 2, 37, 3)
    s_h = float(np.float32(np.abs(h32).max()) / np.float32(448.0))
    T_h = orc.threshold(orc.quantize(h32, f_h, np.inf, s_h)["scores"], 0.2)
    want = orc.quantize(h32, f_h, T_h, s_h)
    xd, wd, od = torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV), torch.from_numpy(ones).to(DEV)
    pW = fgmp.quantize_weights(wd, od, 0.0, 1.0)
    pH, scores = fgmp.quant_gemm_fused_packed_out(xd, od, 0.0, 1.0, pW, torch.from_numpy(f_h).to(DEV), T_h, s_h,
                                                  want_scores=True, epilogue=fgmp.EPILOGUE_SILU_GATE)
    _assert_quant_equal(pH, scores, want, "gated packed output")
    info = fgmp.packed_info(pH)
    assert info["rows"] == M and info["K"] == N // 2 and info["n_fp8_blocks"] == int(want["mask"].sum())
    # FC2 consumes it
    w2 = synth.weights(40, N // 2, 37, 4)
    w2d, w2ref = _to_dev_bf16(w2)
    f2 = synth.fisher_per_channel(N // 2, 37, 5)
    s2 = float(synth.default_tensor_scale(w2ref))
    pW2 = fgmp.quantize_weights(w2d, torch.from_numpy(f2).to(DEV), np.inf, s2)
    Z = fgmp.gemm(pH, pW2)
    q2 = orc.quantize(w2ref, f2, np.inf, s2)
    zw, tol = orc.gemm(orc.dequantize(want["codes"], want["scales"], want["mask"]), s_h,
                       orc.dequantize(q2["codes"], q2["scales"], q2["mask"]), s2)
    assert np.all(np.abs(Z.cpu().numpy().astype(np.float64) - zw) <= tol)
    # the operator none is the plain packed-output call
    f_n = torch.from_numpy(synth.fisher_per_channel(N, 37, 6)).to(DEV)
    a = fgmp.quant_gemm_fused_packed_out(xd, od, 0.0, 1.0, pW, f_n, 1.0, 2.0)
    b = fgmp.quant_gemm_fused_packed_out(xd, od, 0.0, 1.0, pW, f_n, 1.0, 2.0, epilogue=fgmp.EPILOGUE_NONE)
    assert all(torch.equal(u, v) for u, v in zip(fgmp.unpack_canonical(a), fgmp.unpack_canonical(b)))


def test_packed_output_epilogues_match_oracle_at_full_k():
    """Both quantizing epilogues against the ORACLE at 4352 x 4096 x 4096: 256 whole tiles and 16 tiles
    computed in four parts along K in one launch, 64 K-steps (ten turns of the kernel's six-step register
    rotation plus a remainder).  The operands are built so that every partial sum of the product is an
    exact FP32 number in any order (multiples of 1/64 well below 2^24 / 64), so the FP32 results the
    epilogue quantizes are the oracle's results bit for bit, and so must be every code, scale, decision
    and score -- without and with the gated activation."""
    M, K, N = 4352, 4096, 4096
    _say(f"packed-output epilogues vs oracle at {M}x{K}x{N}")
    x = synth.exact_sum_operand_long_k(M, K, 71, 1)
    w = synth.exact_sum_operand_long_k(N, K, 71, 2)
    ones = np.ones(K, dtype=np.float32)
    qw = orc.quantize(w, ones, 0.0, 1.0)
    qx = orc.quantize(x, ones, 0.0, 1.0)
    ax, aw = orc.dequantize(qx["codes"], qx["scales"], qx["mask"]), orc.dequantize(qw["codes"], qw["scales"], qw["mask"])
    assert np.array_equal(ax, x.astype(np.float64)) and np.array_equal(aw, w.astype(np.float64))
    assert 0.1 < qx["mask"].mean() < 0.35 and 0.1 < qw["mask"].mean() < 0.35
    y64, _ = orc.gemm(ax, 1.0, aw, 1.0)
    del ax, aw
    y32 = y64.astype(np.float32)
    assert np.array_equal(y32.astype(np.float64), y64) and np.abs(y64).max() * 64 < 2 ** 24 / 16
    del y64
    xd, wd, od = torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV), torch.from_numpy(ones).to(DEV)
    pW = fgmp.quantize_weights(wd, od, 0.0, 1.0)
    Y = fgmp.quant_gemm_fused(xd, od, 0.0, 1.0, pW)
    assert np.array_equal(Y.cpu().numpy(), y32)
    del Y
    # plain epilogue
    f_n = synth.fisher_per_channel(N, 71, 3)
    s_y = float(np.float32(np.abs(y32).max()) / np.float32(448.0))
    T_y = orc.threshold(orc.quantize(y32, f_n, np.inf, s_y)["scores"], 0.2)
    want = orc.quantize(y32, f_n, T_y, s_y)
    pY, scores = fgmp.quant_gemm_fused_packed_out(xd, od, 0.0, 1.0, pW, torch.from_numpy(f_n).to(DEV), T_y, s_y,
                                                  want_scores=True)
    _assert_quant_equal(pY, scores, want, "packed output at full K")
    assert fgmp.packed_info(pY)["n_fp8_blocks"] == int(want["mask"].sum())
    del pY, scores, want
    # gated epilogue
    h32 = orc.gate_columns(y32)
    f_h = synth.fisher_per_channel(N // 2, 71, 4)
    s_h = float(np.float32(np.abs(h32).max()) / np.float32(448.0))
    T_h = orc.threshold(orc.quantize(h32, f_h, np.inf, s_h)["scores"], 0.2)
    want = orc.quantize(h32, f_h, T_h, s_h)
    pH, scores = fgmp.quant_gemm_fused_packed_out(xd, od, 0.0, 1.0, pW, torch.from_numpy(f_h).to(DEV), T_h, s_h,
                                                  want_scores=True, epilogue=fgmp.EPILOGUE_SILU_GATE)
    _assert_quant_equal(pH, scores, want, "gated packed output at full K")


@pytest.mark.parametrize("M,K,N", [(1, 1024, 512), (8, 4096, 1536), (24, 2048, 528), (32, 4096, 2048), (8, 11008, 256),
                                   (3, 512, 22016), (16, 256, 32)])
def test_decode_step_quantizes_its_own_results_matches_oracle(M, K, N):
    """The one-launch decode step (M <= 32) with quantized, packed results against the ORACLE: codes, block
    scales, decisions and scores of the oracle's quantization of the oracle's product, on operands whose
    product has no rounding in any summation order.  One and several runs per wave, 16 and 32 activation
    rows, K in four and in two parts across workgroups (two chained meetings), a last K-tile of the result
    with one row group (N % 128 = 16) and a result narrower than one K-tile, rows beyond M in the last
    row-tile."""
    _say(f"decode step, packed output vs oracle M={M} K={K} N={N}")
    x = synth.exact_sum_operand_long_k(M, K, 83, 1)
    w = synth.exact_sum_operand_long_k(N, K, 83, 2)
    ones = np.ones(K, dtype=np.float32)
    qx, qw = orc.quantize(x, ones, 0.0, 1.0), orc.quantize(w, ones, 0.0, 1.0)
    ax, aw = orc.dequantize(qx["codes"], qx["scales"], qx["mask"]), orc.dequantize(qw["codes"], qw["scales"], qw["mask"])
    assert np.array_equal(ax, x.astype(np.float64)) and np.array_equal(aw, w.astype(np.float64))
    y64, _ = orc.gemm(ax, 1.0, aw, 1.0)
    y32 = y64.astype(np.float32)
    assert np.array_equal(y32.astype(np.float64), y64) and np.abs(y64).max() * 64 < 2 ** 24 / 16
    f_n = synth.fisher_per_channel(N, 83, 3)
    s_y = float(np.float32(np.abs(y32).max()) / np.float32(448.0))
    T_y = orc.threshold(orc.quantize(y32, f_n, np.inf, s_y)["scores"], 0.25)
    want = orc.quantize(y32, f_n, T_y, s_y)
    assert 0 < want["mask"].sum() < want["mask"].size
    xd, wd, od = torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV), torch.from_numpy(ones).to(DEV)
    pW = fgmp.quantize_weights(wd, od, 0.0, 1.0)
    ws = fgmp.new_workspace(fgmp.workspace_bytes_packed_out(M, N, K), DEV)
    base = fgmp.workspace_bytes(M, N, K)
    ws[fgmp.WORKSPACE_CONTROL_BYTES:].fill_(0x5A)
    pY, scores = fgmp.quant_gemm_fused_packed_out(xd, od, 0.0, 1.0, pW, torch.from_numpy(f_n).to(DEV), T_y, s_y,
                                                  want_scores=True, workspace=ws, epilogue=fgmp.EPILOGUE_ONE_LAUNCH)
    _assert_quant_equal(pY, scores, want, "decode step, packed output")
    info = fgmp.packed_info(pY)
    assert info["rows"] == M and info["K"] == N and info["n_fp8_blocks"] == int(want["mask"].sum())
    assert abs(info["tensor_scale"] - s_y) <= 1e-7 * s_y
    assert not bool(ws[:fgmp.WORKSPACE_CONTROL_BYTES].any()), "both kinds of counters are back at zero"
    # one launch: no FP32 results were staged (the row groups' decision words sit right behind the call's own scratch)
    staged_from = (base + 255) // 256 * 256 + (N // 4 + 255) // 256 * 256
    assert bool((ws[staged_from:] == 0x5A).all()), "the results were staged in the workspace"
    # a second call on the same workspace; the library's own choice between one launch and two (same tensor
    # either way); the next layer on the packed result
    pY2 = fgmp.quant_gemm_fused_packed_out(xd, od, 0.0, 1.0, pW, torch.from_numpy(f_n).to(DEV), T_y, s_y, workspace=ws,
                                           epilogue=fgmp.EPILOGUE_ONE_LAUNCH)
    assert all(torch.equal(u, v) for u, v in zip(fgmp.unpack_canonical(pY), fgmp.unpack_canonical(pY2)))
    pY3, sc3 = fgmp.quant_gemm_fused_packed_out(xd, od, 0.0, 1.0, pW, torch.from_numpy(f_n).to(DEV), T_y, s_y, want_scores=True)
    _assert_quant_equal(pY3, sc3, want, "decode step, packed output, default path")
    w2 = synth.weights(64, N, 83, 4)
    w2d, w2ref = _to_dev_bf16(w2)
    f2 = synth.fisher_per_channel(N, 83, 5)
    s2 = float(synth.default_tensor_scale(w2ref))
    pW2 = fgmp.quantize_weights(w2d, torch.from_numpy(f2).to(DEV), np.inf, s2)
    Z = fgmp.gemm(pY, pW2)
    q2 = orc.quantize(w2ref, f2, np.inf, s2)
    zw, tol = orc.gemm(orc.dequantize(want["codes"], want["scales"], want["mask"]), s_y,
                       orc.dequantize(q2["codes"], q2["scales"], q2["mask"]), s2)
    assert np.all(np.abs(Z.cpu().numpy().astype(np.float64) - zw) <= tol)


@pytest.mark.parametrize("M,K,N,dtype", [(1, 4096, 12288, "bf16"), (8, 4096, 22016, "bf16"), (32, 4096, 12288, "fp32"),
                                          (8, 11008, 4096, "bf16"), (19, 1152, 528, "fp32")])
def test_decode_step_packed_output_on_random_inputs_is_consistent(M, K, N, dtype):
    """On ordinary inputs, at the Llama-2-7B decode shapes: the packed results of the one-launch step equal the
    standalone quantizer run on the very FP32 results the plain step writes (same arithmetic on the same
    values), scores included -- and the build whose waits are all full ones gives the same tensor."""
    from paper_2504_14152_amd import build
    _say(f"decode step, packed output vs standalone quantizer {M}x{K}x{N} {dtype}")
    gen = torch.Generator(device=DEV)
    gen.manual_seed(230 + N)
    wd = torch.empty((N, K), dtype=torch.bfloat16, device=DEV).normal_(0.0, 0.02, generator=gen)
    x = synth.activations(M, K, 93, 1)
    xd, xref = (torch.from_numpy(x).to(DEV), x) if dtype == "fp32" else _to_dev_bf16(x)
    fxd = torch.from_numpy(synth.fisher_per_channel(K, 93, 3)).to(DEV)
    sx, sw = float(synth.default_tensor_scale(xref)), float(wd.abs().max().float()) / 448.0
    _, sws = fgmp.quantize_weights(wd, fxd, np.inf, sw, want_scores=True)
    pW = fgmp.quantize_weights(wd, fxd, fgmp.threshold_for_fraction(sws, 0.1), sw)
    del sws, wd
    Tx = fgmp.threshold_for_fraction(fgmp.quantize_activations(xd, fxd, np.inf, sx, want_scores=True)[1], 0.1)
    Y = fgmp.quant_gemm_fused(xd, fxd, Tx, sx, pW)
    f_n = torch.from_numpy(synth.fisher_per_channel(N, 93, 9)).to(DEV)
    s_y = float(Y.abs().max()) / 448.0
    _, sc0 = fgmp.quantize_activations(Y, f_n, np.inf, s_y, want_scores=True)
    T_y = fgmp.threshold_for_fraction(sc0, 0.2)
    ref, sc_ref = fgmp.quantize_activations(Y, f_n, T_y, s_y, want_scores=True)
    got, sc_got = fgmp.quant_gemm_fused_packed_out(xd, fxd, Tx, sx, pW, f_n, T_y, s_y, want_scores=True,
                                                   epilogue=fgmp.EPILOGUE_ONE_LAUNCH)
    assert torch.equal(sc_ref, sc_got)
    assert all(torch.equal(u, v) for u, v in zip(fgmp.unpack_canonical(ref), fgmp.unpack_canonical(got)))
    assert fgmp.packed_info(got)["n_fp8_blocks"] == fgmp.packed_info(ref)["n_fp8_blocks"] > 0
    with fgmp.use_library(build.lib_path("fullwait")):
        full = fgmp.quant_gemm_fused_packed_out(xd, fxd, Tx, sx, pW, f_n, T_y, s_y, epilogue=fgmp.EPILOGUE_ONE_LAUNCH)
    assert all(torch.equal(u, v) for u, v in zip(fgmp.unpack_canonical(full), fgmp.unpack_canonical(got)))


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_decode_step_on_random_shapes(seed):
    """Twelve seeded random decode shapes per seed (1 <= M <= 32, K a multiple of 16 up to 8192 -- mostly not a
    multiple of the 128-element tile --, N a multiple of 16 up to 6000, FP8 fractions 0 / 0.1 / 0.3 / 1): whatever
    split of row groups, parts of K and rounds the planner picks, the product from packed activations is within the
    oracle's tolerance everywhere, the fused step equals it bit for bit, and the step that quantizes its own results
    in the launch writes the tensor the staged path writes."""
    rng = np.random.default_rng(7000 + seed)
    for it in range(12):
        M = int(rng.integers(1, 33))
        K = int(rng.integers(1, 513)) * 16
        N = int(rng.integers(1, 376)) * 16
        p = float(rng.choice([0.0, 0.1, 0.3, 1.0]))
        _say(f"random decode shape {seed}/{it}: M={M} K={K} N={N} p={p}")
        c = _quantized_pair(M, K, N, 7100 + 10 * seed + it, p, per_elem_w=bool(it & 1))
        Y = fgmp.gemm(c["pX"], c["pW"])
        _check_gemm(c, Y, label=f"random {M}x{K}x{N}")
        Yf = fgmp.quant_gemm_fused(c["xd"], c["fxd"], c["Tx"], c["sx"], c["pW"])
        assert torch.equal(Y, Yf)
        s_y = float(Y.abs().max()) / 448.0
        if s_y > 0:
            f_n = torch.from_numpy(synth.fisher_per_channel(N, 7100 + it, 9)).to(DEV)
            _, sc0 = fgmp.quantize_activations(Y, f_n, np.inf, s_y, want_scores=True)
            T_y = fgmp.threshold_for_fraction(sc0, 0.25)
            ref, sc_ref = fgmp.quant_gemm_fused_packed_out(c["xd"], c["fxd"], c["Tx"], c["sx"], c["pW"], f_n, T_y, s_y, want_scores=True)
            got, sc_got = fgmp.quant_gemm_fused_packed_out(c["xd"], c["fxd"], c["Tx"], c["sx"], c["pW"], f_n, T_y, s_y, want_scores=True,
                                                           epilogue=fgmp.EPILOGUE_ONE_LAUNCH)
            assert torch.equal(sc_ref, sc_got), "scores of the packed results"
            assert all(torch.equal(u, v) for u, v in zip(fgmp.unpack_canonical(ref), fgmp.unpack_canonical(got))), "packed results"


@pytest.mark.parametrize("M,K,N", [(272, 128, 512), (32, 2048, 1024)])
def test_packed_results_are_valid_weight_operands(M, K, N):
    """A reader may take a block's plane-H entry from the mask alone (the number of FP8 slots before the block in
    its tile), as the decode kernel does for its weight operand.  So the tensors the quantizing epilogues write
    -- prefill kernel and one-launch decode step -- must serve as W of a decode step like any other packed
    tensor: products against the oracle's, with the oracle's quantization of the exact results as the operand."""
    _say(f"packed results as weight operand M={M} K={K} N={N}")
    x = synth.exact_sum_operand_long_k(M, K, 87, 1)
    w = synth.exact_sum_operand_long_k(N, K, 87, 2)
    ones = np.ones(K, dtype=np.float32)
    y64, _ = orc.gemm(x.astype(np.float64), 1.0, w.astype(np.float64), 1.0)
    y32 = y64.astype(np.float32)
    assert np.array_equal(y32.astype(np.float64), y64)
    f_n = synth.fisher_per_channel(N, 87, 3)
    s_y = float(np.float32(np.abs(y32).max()) / np.float32(448.0))
    T_y = orc.threshold(orc.quantize(y32, f_n, np.inf, s_y)["scores"], 0.3)
    want = orc.quantize(y32, f_n, T_y, s_y)
    xd, wd, od = torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV), torch.from_numpy(ones).to(DEV)
    pW = fgmp.quantize_weights(wd, od, 0.0, 1.0)
    pY = fgmp.quant_gemm_fused_packed_out(xd, od, 0.0, 1.0, pW, torch.from_numpy(f_n).to(DEV), T_y, s_y,
                                          epilogue=fgmp.EPILOGUE_ONE_LAUNCH)
    _assert_quant_equal(pY, None, want, "packed result")
    # 5 new activation rows times the packed result as an M x N weight tensor
    v = synth.activations(5, N, 87, 6)
    vd, vref = _to_dev_bf16(v)
    f_v = synth.fisher_per_channel(N, 87, 7)
    s_v = float(synth.default_tensor_scale(vref))
    qv = orc.quantize(vref, f_v, np.inf, s_v)
    Z = fgmp.quant_gemm_fused(vd, torch.from_numpy(f_v).to(DEV), np.inf, s_v, pY)
    zw, tol = orc.gemm(orc.dequantize(qv["codes"], qv["scales"], qv["mask"]), s_v,
                       orc.dequantize(want["codes"], want["scales"], want["mask"]), s_y)
    assert np.all(np.abs(Z.cpu().numpy().astype(np.float64) - zw) <= tol)


@pytest.mark.parametrize("M,K,N", [(200, 512, 320), (4352, 256, 4096), (9, 1024, 192)])
def test_gated_packed_output_on_random_inputs_is_consistent(M, K, N):
    """On ordinary inputs: the gated epilogue equals the oracle's gate applied to the very FP32 results
    the plain fused call writes, then the standalone quantizer -- so the kernel's SiLU is the oracle's,
    bit for bit, on realistic values (whole and split tiles in the second shape, the staged path in the third)."""
    c = _quantized_pair(M, K, N, 41, 0.1, per_elem_w=False)
    Y = fgmp.quant_gemm_fused(c["xd"], c["fxd"], c["Tx"], c["sx"], c["pW"])
    h = torch.from_numpy(orc.gate_columns(Y.cpu().numpy())).to(DEV)
    f_h = torch.from_numpy(synth.fisher_per_channel(N // 2, 41, 9)).to(DEV)
    s_h = float(h.abs().max()) / 448.0
    _, sc0 = fgmp.quantize_activations(h, f_h, np.inf, s_h, want_scores=True)
    T_h = fgmp.threshold_for_fraction(sc0, 0.15)
    ref, sc_ref = fgmp.quantize_activations(h, f_h, T_h, s_h, want_scores=True)
    got, sc_got = fgmp.quant_gemm_fused_packed_out(c["xd"], c["fxd"], c["Tx"], c["sx"], c["pW"], f_h, T_h, s_h,
                                                   want_scores=True, epilogue=fgmp.EPILOGUE_SILU_GATE)
    assert torch.equal(sc_ref, sc_got)
    assert all(torch.equal(u, v) for u, v in zip(fgmp.unpack_canonical(ref), fgmp.unpack_canonical(got)))


def test_quantize_is_deterministic():
    x = synth.activations(512, 2048, 9, 51)
    xd, xref = _to_dev_bf16(x)
    f = torch.from_numpy(synth.fisher_per_channel(2048, 9, 52)).to(DEV)
    S = float(synth.default_tensor_scale(xref))
    a = fgmp.quantize_activations(xd, f, 0.01, S)
    b = fgmp.quantize_activations(xd, f, 0.01, S)
    ca, cb = fgmp.unpack_canonical(a), fgmp.unpack_canonical(b)
    assert all(torch.equal(u, v) for u, v in zip(ca, cb))


def test_argument_errors():
    x = torch.zeros((8, 128), dtype=torch.float32, device=DEV)
    f = torch.ones(128, dtype=torch.float32, device=DEV)
    big = fgmp.Packed(torch.empty(1 << 16, dtype=torch.uint8, device=DEV), 8, 24)
    with pytest.raises(fgmp.FgmpError, match="BAD_SHAPE"):
        fgmp.quantize_activations(torch.zeros((8, 24), dtype=torch.float32, device=DEV), f[:24], 0.0, 1.0, out=big)
    with pytest.raises(fgmp.FgmpError, match="INVALID_ARG"):
        fgmp.quantize_activations(x, f, 0.0, 0.0)
    with pytest.raises(fgmp.FgmpError, match="BAD_ALIGN"):
        fgmp.quantize_activations(x.view(-1)[1:1 + 7 * 128].view(7, 128), f, 0.0, 1.0)
    small = fgmp.Packed(torch.empty(64, dtype=torch.uint8, device=DEV), 8, 128)
    with pytest.raises(fgmp.FgmpError, match="BUFFER_TOO_SMALL"):
        fgmp.quantize_activations(x, f, 0.0, 1.0, out=small)
    with pytest.raises(fgmp.FgmpError):
        fgmp.quantize_activations(x.double(), f, 0.0, 1.0)
    assert fgmp.packed_bytes(8, 24) == 0 and fgmp.workspace_bytes(0, 1, 16) == 0


# ------------------------------------------------------------------ GEMM

ORACLE_THRESHOLD_LIMIT = 64 * 1024 * 1024


def _quantized_pair(M, K, N, seed, p, kind="normal", per_elem_w=True):
    x = synth.activations(M, K, seed, 1, kind=kind)
    w = synth.weights(N, K, seed, 2)
    fx = synth.fisher_per_channel(K, seed, 3)
    fw = synth.fisher_per_element(N, K, seed, 4) if per_elem_w else synth.fisher_per_channel(K, seed, 4)
    xd, xref = _to_dev_bf16(x)
    wd, wref = _to_dev_bf16(w)
    sx, sw = float(synth.default_tensor_scale(xref)), float(synth.default_tensor_scale(wref))
    fxd, fwd = torch.from_numpy(fx).to(DEV), torch.from_numpy(fw).to(DEV)
    # thresholds from the ORACLE's scores (so that a GEMM test also notices a score regression); tensors
    # beyond 64 M elements take the library's scores, which other tests show bit-equal to the oracle's
    if M * K <= ORACLE_THRESHOLD_LIMIT:
        Tx = orc.threshold(orc.quantize(xref, fx, np.inf, sx)["scores"], p)
    else:
        Tx = fgmp.threshold_for_fraction(fgmp.quantize_activations(xd, fxd, np.inf, sx, want_scores=True)[1], p)
    if N * K <= ORACLE_THRESHOLD_LIMIT:
        Tw = orc.threshold(orc.quantize(wref, fw, np.inf, sw)["scores"], p)
    else:
        Tw = fgmp.threshold_for_fraction(fgmp.quantize_weights(wd, fwd, np.inf, sw, want_scores=True)[1], p)
    pX = fgmp.quantize_activations(xd, fxd, Tx, sx)
    pW = fgmp.quantize_weights(wd, fwd, Tw, sw)
    return dict(xd=xd, xref=xref, wref=wref, fx=fx, fw=fw, fxd=fxd, sx=sx, sw=sw, Tx=Tx, Tw=Tw, pX=pX, pW=pW)


def _check_gemm(c, Y, rows=None, cols=None, label=""):
    qx = orc.quantize(c["xref"] if rows is None else c["xref"][rows], c["fx"], c["Tx"], c["sx"])
    wsel = c["wref"] if cols is None else c["wref"][cols]
    fsel = c["fw"] if (cols is None or c["fw"].ndim == 1) else c["fw"][cols]
    qw = orc.quantize(wsel, fsel, c["Tw"], c["sw"])
    ax = orc.dequantize(qx["codes"], qx["scales"], qx["mask"])
    aw = orc.dequantize(qw["codes"], qw["scales"], qw["mask"])
    want, tol = orc.gemm(ax, c["sx"], aw, c["sw"])
    got = Y.cpu().numpy().astype(np.float64)
    if rows is not None:
        got = got[np.ix_(rows, cols)]
    err = np.abs(got - want)
    ratio = float((err / np.maximum(tol, 1e-300)).max())
    _say(f"gemm {label}: max |err| / (1e-5 sum|xw|) = {ratio:.4f}")
    assert np.all(err <= tol), f"{label}: {(err > tol).sum()} outputs outside tolerance, worst ratio {ratio}"


@pytest.mark.parametrize("p", [0.1, 0.0, 1.0])
def test_gemm_tiny_full(p):
    cfg = synth.tiny_config(0)
    xd, wd = torch.from_numpy(cfg["x"]).to(DEV), torch.from_numpy(cfg["w"]).to(DEV)
    fxd, fwd = torch.from_numpy(cfg["fisher_x"]).to(DEV), torch.from_numpy(cfg["fisher_w"]).to(DEV)
    sx, sw = float(cfg["scale_x"]), float(cfg["scale_w"])
    Tx = orc.threshold(orc.quantize(cfg["x"], cfg["fisher_x"], np.inf, sx)["scores"], p)
    Tw = orc.threshold(orc.quantize(cfg["w"], cfg["fisher_w"], np.inf, sw)["scores"], p)
    pX = fgmp.quantize_activations(xd, fxd, Tx, sx)
    pW = fgmp.quantize_weights(wd, fwd, Tw, sw)
    Y = fgmp.gemm(pX, pW)
    c = dict(xref=cfg["x"], wref=cfg["w"], fx=cfg["fisher_x"], fw=cfg["fisher_w"], sx=sx, sw=sw, Tx=Tx, Tw=Tw)
    _check_gemm(c, Y, label=f"tiny p={p}")
    Yf = fgmp.quant_gemm_fused(xd, fxd, Tx, sx, pW)
    assert torch.equal(Y, Yf)


@pytest.mark.parametrize("M,K,N,p", [(256, 4096, 512, 0.1), (200, 304, 136, 0.3), (1, 128, 8, 0.1),
                                     (130, 1024, 260, 0.5), (72, 768, 264, 0.2), (40, 1280, 40, 0.1)])
def test_gemm_mid_full(M, K, N, p):
    _say(f"gemm mid M={M} K={K} N={N} p={p}")
    c = _quantized_pair(M, K, N, 7, p)
    Y = fgmp.gemm(c["pX"], c["pW"])
    _check_gemm(c, Y, label=f"mid {M}x{K}x{N}")
    Yf = fgmp.quant_gemm_fused(c["xd"], c["fxd"], c["Tx"], c["sx"], c["pW"])
    assert torch.equal(Y, Yf)


def test_gemm_llama_qkv_prefill_sampled():
    """The benchmark's shape and launch configuration; 64 rows x 512 columns
    of the output, picked by a seeded generator, are checked at full K."""
    M, K, N = 4096, 4096, 12288
    _say("gemm qkv prefill 4096x4096x12288")
    c = _quantized_pair(M, K, N, 0, 0.1, per_elem_w=True)
    Y = fgmp.gemm(c["pX"], c["pW"])
    rng = np.random.default_rng(123)
    rows = np.sort(rng.choice(M, 64, replace=False))
    cols = np.sort(rng.choice(N, 512, replace=False))
    rows[0], rows[-1], cols[0], cols[-1] = 0, M - 1, 0, N - 1
    _check_gemm(c, Y, rows, cols, label="qkv prefill sampled")
    assert torch.isfinite(Y).all()
    Yf = fgmp.quant_gemm_fused(c["xd"], c["fxd"], c["Tx"], c["sx"], c["pW"])
    assert torch.equal(Y, Yf)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_fused_prefill_saturating_tensor_scale(dtype):
    """Fused call on a prefill shape with a caller-chosen activation scale four
    times below amax / 448: FP8 blocks saturate at +-448, and the fused path
    (which writes FP16 values instead of packed codes) must agree with the
    oracle and, bit for bit, with quantize-then-multiply."""
    M, K, N, p = 136, 272, 72, 0.4
    _say(f"fused prefill saturating scale dtype={dtype}")
    x = synth.activations(M, K, 21, 1)
    w = synth.weights(N, K, 21, 2)
    fx = synth.fisher_per_channel(K, 21, 3)
    fw = synth.fisher_per_channel(K, 21, 4)
    wd, wref = _to_dev_bf16(w)
    if dtype == "bf16":
        xd, xref = _to_dev_bf16(x)
    else:
        xref = x.astype(np.float32)
        xd = torch.from_numpy(xref).to(DEV)
    sx = float(synth.default_tensor_scale(xref)) / 4.0
    sw = float(synth.default_tensor_scale(wref))
    fxd, fwd = torch.from_numpy(fx).to(DEV), torch.from_numpy(fw).to(DEV)
    Tx = orc.threshold(orc.quantize(xref, fx, np.inf, sx)["scores"], p)
    Tw = orc.threshold(orc.quantize(wref, fw, np.inf, sw)["scores"], p)
    pW = fgmp.quantize_weights(wd, fwd, Tw, sw)
    Yf = fgmp.quant_gemm_fused(xd, fxd, Tx, sx, pW)
    c = dict(xref=xref, wref=wref, fx=fx, fw=fw, sx=sx, sw=sw, Tx=Tx, Tw=Tw)
    _check_gemm(c, Yf, label=f"fused saturating {dtype}")
    Y = fgmp.gemm(fgmp.quantize_activations(xd, fxd, Tx, sx), pW)
    assert torch.equal(Y, Yf)


@pytest.mark.parametrize("M,K,N", [(4352, 512, 4096), (2304, 256, 2304), (2304, 128, 2304)])
def test_gemm_split_last_round_sampled(M, K, N):
    """Tiles of a partly filled last round are computed in parts along K that meet through the workspace:
    272 tiles = 256 whole + 16 in four parts of two K-steps; 81 tiles, all in two parts; and a K too short to
    divide (whole tiles only).  Rows and columns are drawn from every tile."""
    _say(f"gemm {M}x{K}x{N}: whole tiles and split tiles")
    c = _quantized_pair(M, K, N, 11, 0.2, per_elem_w=False)
    Y = fgmp.gemm(c["pX"], c["pW"])
    rng = np.random.default_rng(77)
    rows = np.sort(np.concatenate([t * 256 + rng.choice(256, 3, replace=False) for t in range(M // 256)]))
    cols = np.sort(np.concatenate([t * 256 + rng.choice(256, 16, replace=False) for t in range(N // 256)]))
    _check_gemm(c, Y, rows, cols, label="whole + split tiles")
    assert torch.isfinite(Y).all()
    Yf = fgmp.quant_gemm_fused(c["xd"], c["fxd"], c["Tx"], c["sx"], c["pW"])
    assert torch.equal(Y, Yf)
    # the parts of a tile may arrive in any order: every meeting adds two numbers, so repeated calls agree bit for bit
    for _ in range(3):
        assert torch.equal(Yf, fgmp.quant_gemm_fused(c["xd"], c["fxd"], c["Tx"], c["sx"], c["pW"]))


def test_gemm_llama_fc1_prefill_sampled():
    """The benchmark's FC1 shape and launch configuration: 1376 output tiles, 1280 computed whole and the
    96 of the last round in two parts along K.  Sampled rows and columns (every 256-column tile gets
    some) at full K."""
    M, K, N = 4096, 4096, 22016
    _say("gemm fc1 prefill 4096x4096x22016")
    c = _quantized_pair(M, K, N, 2, 0.1, per_elem_w=False)
    Yf = fgmp.quant_gemm_fused(c["xd"], c["fxd"], c["Tx"], c["sx"], c["pW"])
    rng = np.random.default_rng(321)
    rows = np.sort(np.concatenate([t * 256 + rng.choice(256, 2, replace=False) for t in range(M // 256)]))
    cols = np.sort(np.concatenate([t * 256 + rng.choice(256, 4, replace=False) for t in range(N // 256)]))
    rows[0], rows[-1], cols[0], cols[-1] = 0, M - 1, 0, N - 1
    _check_gemm(c, Yf, rows, cols, label="fc1 prefill sampled")
    assert torch.isfinite(Yf).all()
    assert torch.equal(Yf, fgmp.quant_gemm_fused(c["xd"], c["fxd"], c["Tx"], c["sx"], c["pW"]))


@pytest.mark.parametrize("p", [0.1, 0.0, 1.0])
def test_gemm_llama70b_fc1_shape_sampled(p):
    """The sweep's shape (configs[4]: K 8192, N 57344, M 2048; 470 M weights, 1792 output tiles) and a
    decode step on the same weights, at the sweep's end points too: no FP8 block at all, and every block
    FP8 (the compact upper-half plane is then eight times larger, and a decode step finds more FP8 blocks
    per K range than it stages).  The weights are drawn on the device (seeded); the oracle quantizes
    the sampled rows of X and W itself from the very same bf16 values."""
    M, K, N = 2048, 8192, 57344
    _say(f"gemm 70B fc1 2048x8192x57344 p={p}")
    gen = torch.Generator(device=DEV)
    gen.manual_seed(70)
    wd = torch.empty((N, K), dtype=torch.bfloat16, device=DEV).normal_(0.0, 0.02, generator=gen)
    xd, xref = _to_dev_bf16(synth.activations(M, K, 70, 1))
    fx, fw = synth.fisher_per_channel(K, 70, 3), synth.fisher_per_channel(K, 70, 4)
    fxd, fwd = torch.from_numpy(fx).to(DEV), torch.from_numpy(fw).to(DEV)
    sx, sw = float(synth.default_tensor_scale(xref)), float(wd.abs().max().float()) / 448.0
    _, sxs = fgmp.quantize_activations(xd, fxd, np.inf, sx, want_scores=True)
    _, sws = fgmp.quantize_weights(wd, fwd, np.inf, sw, want_scores=True)
    Tx, Tw = fgmp.threshold_for_fraction(sxs, p), fgmp.threshold_for_fraction(sws, p)
    del sxs, sws
    pW = fgmp.quantize_weights(wd, fwd, Tw, sw)
    info = fgmp.packed_info(pW)
    assert info["n_fp8_blocks"] == int(p * info["n_blocks"] + 0.5)
    rng = np.random.default_rng(170)
    rows = np.sort(rng.choice(M, 24, replace=False))
    cols = np.sort(np.concatenate([rng.choice(N, 300, replace=False), [0, N - 1]]))
    cols = np.unique(cols)
    wsel = wd[torch.from_numpy(cols).to(DEV)].float().cpu().numpy()
    c = dict(xref=xref, wref=None, fx=fx, fw=fw, sx=sx, sw=sw, Tx=Tx, Tw=Tw)

    def check(Y, xrows, label):
        qx = orc.quantize(xref[xrows], fx, Tx, sx)
        qw = orc.quantize(wsel, fw, Tw, sw)
        want, tol = orc.gemm(orc.dequantize(qx["codes"], qx["scales"], qx["mask"]), sx,
                             orc.dequantize(qw["codes"], qw["scales"], qw["mask"]), sw)
        got = Y.cpu().numpy().astype(np.float64)[np.ix_(xrows, cols)]
        err = np.abs(got - want)
        _say(f"gemm {label}: max |err| / (1e-5 sum|xw|) = {float((err / np.maximum(tol, 1e-300)).max()):.4f}")
        assert np.all(err <= tol), label
    del wd
    Y = fgmp.quant_gemm_fused(xd, fxd, Tx, sx, pW)
    check(Y, rows, "70B fc1 prefill sampled")
    assert torch.isfinite(Y).all()
    del Y
    Yd = fgmp.quant_gemm_fused(xd[:8].contiguous(), fxd, Tx, sx, pW)
    check(Yd, np.arange(8), "70B fc1 decode M=8")


def test_gemm_fc2_shape_sampled():
    """The benchmark's FC2 shape (K = 11008 = 86 K-tiles, activations = a gated product)."""
    M, K, N = 4096, 11008, 4096
    _say("gemm fc2 4096x11008x4096")
    c = _quantized_pair(M, K, N, 3, 0.1, kind="silu_gate", per_elem_w=False)
    Y = fgmp.gemm(c["pX"], c["pW"])
    rng = np.random.default_rng(5)
    rows = np.sort(rng.choice(M, 32, replace=False))
    cols = np.sort(rng.choice(N, 256, replace=False))
    _check_gemm(c, Y, rows, cols, label="fc2 sampled")


@pytest.mark.parametrize("M,K,N,p", [(1, 4096, 4096, 0.1), (8, 4096, 4096, 0.1), (32, 4096, 4096, 0.1),
                                     (17, 11008, 4096, 0.1), (5, 304, 100, 0.3), (32, 1024, 72, 1.0),
                                     (16, 2048, 264, 0.5), (3, 4096, 12288, 0.0), (5, 4096, 14000, 0.1),
                                     (9, 11008, 8200, 0.2), (33, 1024, 520, 0.1), (64, 4096, 4096, 0.1),
                                     (96, 2048, 264, 0.3), (70, 11008, 4096, 0.1), (41, 304, 100, 1.0)])
def test_gemm_decode_shapes(M, K, N, p):
    """Weight-streaming path (M <= 32 per launch; more rows in chunks of 32 where that is the faster path): K ranges combined in K order, ragged N
    and K, FP8 fractions beyond the speculative plane-H window, weight tensors with so many rows that
    workgroups take 128 instead of 64 of them, last chunks of 1, 9, 6 and 32 rows."""
    _say(f"gemm decode M={M} K={K} N={N} p={p}")
    c = _quantized_pair(M, K, N, 11, p, per_elem_w=False)
    Y = fgmp.gemm(c["pX"], c["pW"])
    cols = np.arange(0, N, 7) if N > 1000 else np.arange(N)
    _check_gemm(c, Y, np.arange(M), cols, label=f"decode M={M} K={K} N={N} p={p}")
    Y2 = fgmp.gemm(c["pX"], c["pW"])
    assert torch.equal(Y, Y2), "split-K combination must be deterministic"
    Yf = fgmp.quant_gemm_fused(c["xd"], c["fxd"], c["Tx"], c["sx"], c["pW"])
    assert torch.equal(Y, Yf)


@pytest.mark.parametrize("name", ["qkv", "fc1"])
def test_gemm_decode_llama_shapes_at_full_size(name):
    """The benchmark's decode steps at their real sizes and 10% FP8 on both sides: M = 1, 8 and 32 rows
    against the fused QKV weights (12288 x 4096) and the FC1 weights (22016 x 4096).  Every 7th output
    column at full K against the oracle; fused call, packed-activation call and a repeated call agree bit
    for bit."""
    K, N = synth.LLAMA2_7B[name]
    _say(f"decode full size {name}: N={N} K={K}")
    c = _quantized_pair(32, K, N, 13, 0.1, per_elem_w=False)
    cols = np.arange(0, N, 7)
    cols[-1] = N - 1
    for M in (1, 8, 32):
        xm = c["xd"][:M].contiguous()
        Yf = fgmp.quant_gemm_fused(xm, c["fxd"], c["Tx"], c["sx"], c["pW"])
        cm = dict(c, xref=c["xref"][:M])
        _check_gemm(cm, Yf, np.arange(M), cols, label=f"decode {name} M={M}")
        assert torch.isfinite(Yf).all()
        pXm = fgmp.quantize_activations(xm, c["fxd"], c["Tx"], c["sx"])
        assert torch.equal(Yf, fgmp.gemm(pXm, c["pW"]))
        assert torch.equal(Yf, fgmp.quant_gemm_fused(xm, c["fxd"], c["Tx"], c["sx"], c["pW"]))


@pytest.mark.parametrize("M,K,N,p", [(4, 1024, 200, 0.1), (24, 2048, 136, 0.3), (300, 512, 264, 0.1),
                                     (8, 256, 72, 0.0), (300, 256, 72, 0.0)])
def test_compact_weights_relocated_to_bytes_used(M, K, N, p):
    """A compact weight tensor copied into a buffer of exactly bytes_used bytes
    (poisoned guard bytes after it) gives the same product, bit for bit, and
    unpacks to the same codes: no reader depends on bytes beyond bytes_used."""
    _say(f"relocated compact weights M={M} K={K} N={N} p={p}")
    c = _quantized_pair(M, K, N, 17, p, per_elem_w=False)
    pW = c["pW"]
    used = fgmp.packed_info(pW)["bytes_used"]
    assert used <= pW.buf.numel()
    n16 = -(-used // 16) * 16
    small = torch.full((n16 + 4096,), 0xFF, dtype=torch.uint8, device=DEV)
    small[:used] = pW.buf[:used]
    pS = fgmp.Packed(small[:n16], N, K)
    Y0 = fgmp.gemm(c["pX"], pW)
    Y1 = fgmp.gemm(c["pX"], pS)
    assert torch.equal(Y0, Y1)
    Yf = fgmp.quant_gemm_fused(c["xd"], c["fxd"], c["Tx"], c["sx"], pS)
    assert torch.equal(Y0, Yf)
    for u, v in zip(fgmp.unpack_canonical(pW), fgmp.unpack_canonical(pS)):
        assert torch.equal(u, v)
    assert bool((small[n16:] == 0xFF).all())


def test_gemm_two_pass_path_in_subprocess():
    """The alternative prefill path (both operands expanded to FP16 first) exists only in the build with
    measurement hooks, where FGMP_PREFILL_KERNEL=dense chooses it once per process; check it in a child process."""
    import os
    import subprocess
    import sys
    code = (
        "import numpy as np, torch, sys\n"
        "sys.path.insert(0, %r)\n"
        "import tests.test_gpu_parity as t\n"
        "c = t._quantized_pair(200, 1040, 264, 7, 0.2)\n"
        "Y = t.fgmp.gemm(c['pX'], c['pW'])\n"
        "t._check_gemm(c, Y, label='two-pass')\n"
        "print('two-pass ok')\n"
    ) % os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    from paper_2504_14152_amd import build
    env = dict(os.environ, FGMP_PREFILL_KERNEL="dense", FGMP_LIB_PATH=build.lib_path("hooks"))
    res = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, timeout=110)
    assert res.returncode == 0 and "two-pass ok" in res.stdout, res.stdout + res.stderr


def test_mfma_rate_reference_runs():
    """The benchmark's reference loop: launches, finishes, and its arithmetic is kept (finite sums)."""
    _say("mfma rate reference")
    sink = torch.full((64 * 256,), float("nan"), dtype=torch.float32, device=DEV)
    fgmp.selftest_mfma_rate(64, 50, sink)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(sink).all())


def test_gemm_kernel_timing_hook():
    """The measurement hook (only in the build variant with hooks) brackets the prefill GEMM kernel with the
    caller's events; cleared, it records nothing; the shipped library has no hook and says so."""
    from paper_2504_14152_amd import build
    c = _quantized_pair(300, 512, 264, 5, 0.1, per_elem_w=False)
    ea, eb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ea.record()
    eb.record()
    torch.cuda.synchronize()
    with pytest.raises(fgmp.FgmpError):
        fgmp.selftest_time_gemm_kernel(ea, eb)
    fgmp.selftest_time_gemm_kernel(None, None)
    Y_shipped = fgmp.quant_gemm_fused(c["xd"], c["fxd"], c["Tx"], c["sx"], c["pW"])
    with fgmp.use_library(build.lib_path("hooks")):
        fgmp.selftest_time_gemm_kernel(ea, eb)
        try:
            Y = fgmp.quant_gemm_fused(c["xd"], c["fxd"], c["Tx"], c["sx"], c["pW"])
        finally:
            fgmp.selftest_time_gemm_kernel(None, None)
        torch.cuda.synchronize()
        ms = ea.elapsed_time(eb)
        assert 0.0 < ms < 50.0
        _check_gemm(c, Y, label="timed launch")
        assert torch.equal(Y, Y_shipped)
        # with the hook cleared the events keep their timestamps
        fgmp.quant_gemm_fused(c["xd"], c["fxd"], c["Tx"], c["sx"], c["pW"])
        torch.cuda.synchronize()
        assert ea.elapsed_time(eb) == ms


@pytest.mark.parametrize("M,K,N", [(4096, 4096, 12288), (4096, 4096, 22016), (4352, 512, 4096), (300, 1040, 264)])
def test_hand_counted_waits_against_full_waits(M, K, N):
    """Runtime guard for the prefill kernel's hand-counted `s_waitcnt vmcnt(N)`: a second build of the same
    sources in which every such wait is a full one (nothing to miscount) must give the same Y bit for bit
    -- same instructions, same summation order, so any difference is a register read before its load
    landed.  QKV and FC1 at full size (FC1 with tiles split in two along K), a shape with four-part split
    tiles, and a ragged one; whatever the compiler made of the loop."""
    from paper_2504_14152_amd import build
    _say(f"counted waits vs full waits {M}x{K}x{N}")
    gen = torch.Generator(device=DEV)
    gen.manual_seed(90 + N)
    wd = torch.empty((N, K), dtype=torch.bfloat16, device=DEV).normal_(0.0, 0.02, generator=gen)
    xd, xref = _to_dev_bf16(synth.activations(M, K, 90, 1))
    fxd = torch.from_numpy(synth.fisher_per_channel(K, 90, 3)).to(DEV)
    sx, sw = float(synth.default_tensor_scale(xref)), float(wd.abs().max().float()) / 448.0
    _, sws = fgmp.quantize_weights(wd, fxd, np.inf, sw, want_scores=True)
    pW = fgmp.quantize_weights(wd, fxd, fgmp.threshold_for_fraction(sws, 0.1), sw)
    del sws, wd
    Tx = fgmp.threshold_for_fraction(fgmp.quantize_activations(xd, fxd, np.inf, sx, want_scores=True)[1], 0.1)
    Y = fgmp.quant_gemm_fused(xd, fxd, Tx, sx, pW)
    with fgmp.use_library(build.lib_path("fullwait")):
        Y_full = fgmp.quant_gemm_fused(xd, fxd, Tx, sx, pW)
    assert torch.isfinite(Y).all() and torch.equal(Y, Y_full)


@pytest.mark.parametrize("M,K,N,dtype", [(1, 4096, 12288, "bf16"), (8, 4096, 22016, "bf16"), (8, 11008, 4096, "fp32"),
                                          (32, 4096, 4096, "bf16"), (13, 1152, 528, "fp32"), (3, 28672, 8192, "bf16")])
def test_decode_kernel_hand_counted_waits_against_full_waits(M, K, N, dtype):
    """The same guard for the one-launch decode kernel, whose loads are assembly with counted waits as
    well: the build in which every wait is a full one must give the same Y bit for bit.  Runs of eight
    tiles per wave (first pass of the ring plus one turn), long runs that cross row groups, K in three,
    four and four parts across workgroups (counters, partial sums), both row-group widths, both input
    types, a ragged K."""
    from paper_2504_14152_amd import build
    _say(f"decode kernel, counted waits vs full waits {M}x{K}x{N} {dtype}")
    gen = torch.Generator(device=DEV)
    gen.manual_seed(190 + N)
    wd = torch.empty((N, K), dtype=torch.bfloat16, device=DEV).normal_(0.0, 0.02, generator=gen)
    x = synth.activations(M, K, 91, 1)
    xd, xref = (torch.from_numpy(x).to(DEV), x) if dtype == "fp32" else _to_dev_bf16(x)
    fxd = torch.from_numpy(synth.fisher_per_channel(K, 91, 3)).to(DEV)
    sx, sw = float(synth.default_tensor_scale(xref)), float(wd.abs().max().float()) / 448.0
    _, sws = fgmp.quantize_weights(wd, fxd, np.inf, sw, want_scores=True)
    pW = fgmp.quantize_weights(wd, fxd, fgmp.threshold_for_fraction(sws, 0.2), sw)
    del sws, wd
    Tx = fgmp.threshold_for_fraction(fgmp.quantize_activations(xd, fxd, np.inf, sx, want_scores=True)[1], 0.2)
    ws = fgmp.new_workspace(fgmp.workspace_bytes(M, N, K), DEV)
    Y = fgmp.quant_gemm_fused(xd, fxd, Tx, sx, pW, workspace=ws)
    assert not bool(ws[:fgmp.WORKSPACE_CONTROL_BYTES].any()), "every call leaves the control region zero"
    pX = fgmp.quantize_activations(xd, fxd, Tx, sx)
    Yp = fgmp.gemm(pX, pW)
    assert torch.equal(Y, Yp), "quantizing in the kernel and decoding packed activations give the same operand values"
    with fgmp.use_library(build.lib_path("fullwait")):
        Y_full = fgmp.quant_gemm_fused(xd, fxd, Tx, sx, pW)
    assert torch.isfinite(Y).all() and torch.equal(Y, Y_full)


def test_decode_kernel_reads_weights_that_are_not_compact():
    """A tensor packed the way activations are (room for 64 plane-H entries per tile, wherever the writer
    put them) is a valid W: the decode kernel then takes every tile's first entry from plane T instead of
    counting on from the tile before.  Same codes as the compact tensor, same order of summation: the
    same Y bit for bit."""
    M, K, N = 8, 2048, 1056
    c = _quantized_pair(M, K, N, 77, 0.3, per_elem_w=False)
    wd, _ = _to_dev_bf16(c["wref"])
    fwd = torch.from_numpy(c["fw"]).to(DEV)
    pW_strided = fgmp.quantize_activations(wd, fwd, c["Tw"], c["sw"])
    assert fgmp.packed_info(pW_strided)["compact"] == 0 and fgmp.packed_info(c["pW"])["compact"] == 1
    Y = fgmp.quant_gemm_fused(c["xd"], c["fxd"], c["Tx"], c["sx"], c["pW"])
    _check_gemm(c, Y, label="decode kernel, compact W")
    Ys = fgmp.quant_gemm_fused(c["xd"], c["fxd"], c["Tx"], c["sx"], pW_strided)
    assert torch.equal(Y, Ys)


@pytest.mark.parametrize("M,K,N", [(8, 1024, 512), (8, 11008, 512), (24, 2048, 520), (300, 512, 520), (70, 1024, 512)])
def test_fused_call_replays_in_a_hip_graph(M, K, N):
    """The hot-path calls only enqueue kernels on the caller's stream (no allocation, no synchronization,
    no memset nodes: arrival counters are put back to zero by the kernels that use them), so a
    captured step can be replayed: decode shapes (one launch; with K in one part and in three parts that
    meet at the row groups' counters; the older two-kernel path for an odd number of row-tiles), a prefill
    shape whose tiles are computed in two parts, and a decode shape of three row chunks.  Every replay, with eager work and synchronizations in between, must
    reproduce the eager result bit for bit."""
    c = _quantized_pair(M, K, N, 43, 0.1, per_elem_w=False)
    ws = fgmp.new_workspace(fgmp.workspace_bytes(M, N, K), DEV)
    Y_eager = fgmp.quant_gemm_fused(c["xd"], c["fxd"], c["Tx"], c["sx"], c["pW"], workspace=ws).clone()
    Y = torch.empty_like(Y_eager)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fgmp.quant_gemm_fused(c["xd"], c["fxd"], c["Tx"], c["sx"], c["pW"], out=Y, workspace=ws)   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fgmp.quant_gemm_fused(c["xd"], c["fxd"], c["Tx"], c["sx"], c["pW"], out=Y, workspace=ws)
    for rep in range(4):
        Y.zero_()
        ws[fgmp.WORKSPACE_CONTROL_BYTES:].fill_(0xA5 if rep & 1 else 0)   # whatever the scratch holds between replays
        assert not bool(ws[:fgmp.WORKSPACE_CONTROL_BYTES].any()), "every call leaves the control region zero"
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y, Y_eager), f"replay {rep}"
        # eager work of the program between replays
        Z = fgmp.quant_gemm_fused(c["xd"], c["fxd"], c["Tx"], c["sx"], c["pW"])
        assert torch.equal(Z, Y_eager)


@pytest.mark.parametrize("M,K,N", [(8, 1024, 512), (24, 2048, 528)])
def test_decode_step_with_packed_output_replays_in_a_hip_graph(M, K, N):
    """The one-launch step that quantizes its own results, captured and replayed: both kinds of arrival
    counters (parts of K per row group, row groups per tile of the result) are back at zero after every
    replay, whatever the scratch holds in between, and every replay writes the eager call's tensor."""
    c = _quantized_pair(M, K, N, 47, 0.1, per_elem_w=False)
    f_n = torch.from_numpy(synth.fisher_per_channel(N, 47, 9)).to(DEV)
    Y = fgmp.quant_gemm_fused(c["xd"], c["fxd"], c["Tx"], c["sx"], c["pW"])
    s_y = float(Y.abs().max()) / 448.0
    T_y = fgmp.threshold_for_fraction(fgmp.quantize_activations(Y, f_n, np.inf, s_y, want_scores=True)[1], 0.2)
    ws = fgmp.new_workspace(fgmp.workspace_bytes_packed_out(M, N, K), DEV)
    args = (c["xd"], c["fxd"], c["Tx"], c["sx"], c["pW"], f_n, T_y, s_y)
    want = [t.clone() for t in fgmp.unpack_canonical(fgmp.quant_gemm_fused_packed_out(*args, epilogue=fgmp.EPILOGUE_ONE_LAUNCH))]
    assert int(want[2].sum()) > 0
    pY = fgmp.quant_gemm_fused_packed_out(*args, workspace=ws, epilogue=fgmp.EPILOGUE_ONE_LAUNCH)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fgmp.quant_gemm_fused_packed_out(*args, out=pY, workspace=ws, epilogue=fgmp.EPILOGUE_ONE_LAUNCH)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fgmp.quant_gemm_fused_packed_out(*args, out=pY, workspace=ws, epilogue=fgmp.EPILOGUE_ONE_LAUNCH)
    for rep in range(4):
        pY.buf.fill_(0x3C)
        ws[fgmp.WORKSPACE_CONTROL_BYTES:].fill_(0xA5 if rep & 1 else 0)
        assert not bool(ws[:fgmp.WORKSPACE_CONTROL_BYTES].any()), "every call leaves the control region zero"
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = fgmp.unpack_canonical(pY)
        assert all(torch.equal(u, v) for u, v in zip(got, want)), f"replay {rep}"
        Z = fgmp.quant_gemm_fused(c["xd"], c["fxd"], c["Tx"], c["sx"], c["pW"])   # eager work between replays
        assert torch.equal(Z, Y)

