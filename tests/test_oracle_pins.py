"""Pins of the CPU oracle against things other than itself: the published
number formats, an independent library cast, closed forms the paper prints,
exact-representability and scaling invariants, fp64 recomputation and
brute force.  CPU only."""
import os

import numpy as np
import pytest
import torch

from oracle import fgmp_oracle as orc
from paper_2504_14152_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if line:
                parts = line.split()
                out[parts[0]] = parts[1:]
    return out


FORMATS = _golden("number_formats.txt")
PAPER = {k: float(v[0]) for k, v in _golden("paper_closed_forms.txt").items()}
E2M1 = [float(v) for v in FORMATS["e2m1_magnitudes"]]


def _torch_e4m3_decode_all():
    return torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float32).numpy()


# ---------------------------------------------------------------- codecs

def test_e2m1_decode_matches_format_table():
    for code in range(16):
        want = E2M1[code & 7] * (-1.0 if code & 8 else 1.0)
        got = orc.e2m1_decode(code)
        assert got == want and np.signbit(got) == bool(code & 8)


def test_e4m3_decode_matches_library_cast():
    ref = _torch_e4m3_decode_all()
    for code in range(256):
        got = orc.e4m3_decode(code)
        if code & 0x7F == 0x7F:
            assert np.isnan(got) and np.isnan(ref[code])
        else:
            assert got == ref[code] and np.signbit(got) == np.signbit(ref[code])
    assert orc.e4m3_decode(0x7E) == float(FORMATS["e4m3_max"][0])
    assert orc.e4m3_decode(0x01) == float(FORMATS["e4m3_min_subnormal"][0])
    assert orc.e4m3_decode(0x08) == float(FORMATS["e4m3_min_normal"][0])


def test_codes_round_trip():
    for code in range(16):
        assert orc.e2m1_encode(np.float32(orc.e2m1_decode(code))) == code
    for code in range(256):
        if code & 0x7F != 0x7F:
            assert orc.e4m3_encode(np.float32(orc.e4m3_decode(code))) == code


def test_e2m1_tie_points_and_neighbours():
    for item in FORMATS["e2m1_ties"]:
        mid, want = (float(v) for v in item.split(":"))
        mid32 = np.float32(mid)
        below = np.nextafter(mid32, np.float32(0))
        above = np.nextafter(mid32, np.float32(100))
        lo = max(v for v in E2M1 if v < mid)
        hi = min(v for v in E2M1 if v > mid)
        for sign in (1.0, -1.0):
            assert orc.e2m1_decode(orc.e2m1_encode(np.float32(sign * mid32))) == sign * want
            assert orc.e2m1_decode(orc.e2m1_encode(np.float32(sign * below))) == sign * lo
            assert orc.e2m1_decode(orc.e2m1_encode(np.float32(sign * above))) == sign * hi


def test_saturation_and_signed_zero():
    assert orc.e2m1_encode(np.float32(1e30)) == 7
    assert orc.e2m1_encode(np.float32(-6.5)) == 15
    assert orc.e2m1_encode(np.float32(-0.0)) == 8
    assert orc.e2m1_encode(np.float32(-1e-30)) == 8
    assert orc.e4m3_encode(np.float32(3e38)) == 0x7E
    assert orc.e4m3_encode(np.float32(-449.0)) == 0xFE
    assert orc.e4m3_encode(np.float32(464.0)) == 0x7E
    assert orc.e4m3_encode(np.float32(-0.0)) == 0x80
    assert orc.e4m3_encode(np.float32(2.0 ** -11)) == 0x00      # tie between 0 and 2^-9 -> even code 0
    assert orc.e4m3_encode(np.float32(3 * 2.0 ** -10)) == 0x02  # tie between codes 1 and 2 -> 2


def test_e4m3_encode_matches_library_cast_in_range():
    rng = np.random.default_rng(7)
    vals = [rng.standard_normal(200000).astype(np.float32) * s for s in (1e-3, 0.05, 1.0, 30.0, 150.0)]
    table = _torch_e4m3_decode_all()[:127]
    mids = ((table[:-1].astype(np.float64) + table[1:].astype(np.float64)) / 2).astype(np.float32)
    vals += [mids, -mids, np.nextafter(mids, np.float32(0)), np.nextafter(mids, np.float32(1e9)), table, -table]
    x = np.concatenate(vals)
    x = x[np.abs(x) <= 448.0]
    want = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = orc.e4m3_encode(x)
    assert np.array_equal(got, want)


def test_encoders_are_monotone_and_nearest():
    rng = np.random.default_rng(11)
    x = np.sort(np.abs(np.concatenate([rng.standard_normal(100000) * 3, rng.uniform(0, 7, 100000)]))).astype(np.float32)
    q = orc.e2m1_encode(x)
    assert np.all(np.diff(q.astype(np.int32)) >= 0)
    err = np.abs(np.array(E2M1)[q].astype(np.float64) - np.minimum(x, 6.0))
    allerr = np.abs(np.array(E2M1)[None, :] - np.minimum(x, 6.0)[:, None].astype(np.float64)).min(axis=1)
    assert np.array_equal(err, allerr)
    y = np.sort(np.abs(rng.standard_normal(200000) * 100)).astype(np.float32)
    c = orc.e4m3_encode(y)
    assert np.all(np.diff(c.astype(np.int32)) >= 0)


# ---------------------------------------------------------------- quantizer

@pytest.mark.parametrize("S", [1.0, 0.5, 2.0 ** -10, 3 * 2.0 ** -7])
def test_nvfp4_exact_values_round_trip(S):
    """Every E2M1 value times every E4M3 block scale times S is reproduced
    exactly, with score 0 (blocks that are already FP4-exact)."""
    scale_codes = np.arange(1, 127, dtype=np.uint8)
    perm = np.array([7, 0, 9, 3, 12, 5, 14, 1, 8, 15, 2, 11, 4, 13, 6, 10])  # all 16 codes, contains +-6
    e2 = np.array([orc.e2m1_decode(int(c)) for c in perm], dtype=np.float64)
    sv = np.array([orc.e4m3_decode(int(c)) for c in scale_codes], dtype=np.float64)
    x64 = e2[None, :] * sv[:, None] * S
    x = x64.astype(np.float32)
    assert np.array_equal(x.astype(np.float64), x64)
    fisher = np.linspace(0.1, 3.0, 16).astype(np.float32)
    out = orc.quantize(x, fisher, np.inf, S)
    assert np.array_equal(out["scales"][:, 0], scale_codes)
    assert np.array_equal(out["codes"], np.broadcast_to(perm, x.shape))
    assert np.all(out["scores"] == 0.0) and np.all(out["mask"] == 0)


def _random_case(rows=64, K=512, seed=3, per_element=False):
    x = synth.activations(rows, K, seed, 21, outlier_count=5)
    f = synth.fisher_per_element(rows, K, seed, 22) if per_element else synth.fisher_per_channel(K, seed, 23)
    return x, f, float(synth.default_tensor_scale(x))


@pytest.mark.parametrize("per_element", [False, True])
def test_score_agrees_with_fp64_definition(per_element):
    """Eq. 6 recomputed in fp64 from the stored NVFP4 encoding."""
    x, f, S = _random_case(per_element=per_element)
    out = orc.quantize(x, f, np.inf, S)
    # the reconstruction is an fp32 value: d = fp32(e4m3 * S), xhat = fp32(e2m1 * d)
    e4 = _torch_e4m3_decode_all().astype(np.float64)
    d32 = (e4[out["scales"]] * np.float64(np.float32(S))).astype(np.float32)
    e2 = np.array(E2M1 + [-v for v in E2M1])[out["codes"]]
    xhat = (e2 * np.repeat(d32, 16, axis=1).astype(np.float64)).astype(np.float32).astype(np.float64)
    err = (x.astype(np.float64) - xhat) ** 2 * (f.astype(np.float64) if per_element else f.astype(np.float64)[None, :])
    want = err.reshape(x.shape[0], -1, 16).sum(axis=2)
    assert np.all(out["scores"] >= 0)
    np.testing.assert_allclose(out["scores"], want, rtol=1e-6, atol=0)
    # and it is close to the exact product e2m1 * e4m3 * S
    exact = orc.dequantize(out["codes"], out["scales"], out["mask"]) * np.float64(np.float32(S))
    np.testing.assert_allclose(xhat, exact, rtol=2e-7, atol=0)
    # reconstruction error is bounded by half the local E2M1 spacing (<= 1.0 * d) inside the range
    d = np.array([orc.e4m3_decode(int(c)) for c in out["scales"].reshape(-1)]).reshape(out["scales"].shape) * S
    assert np.all(np.abs(x.astype(np.float64) - xhat).reshape(x.shape[0], -1, 16).max(axis=2) <= 1.0 * d + 1e-12 + 1e-6 * np.abs(x).reshape(x.shape[0], -1, 16).max(axis=2) + (d == 0) * 1e9)


# ---------------------------------------------------------------- Eq. 8 score ("delta" mode)

def _both_reconstructions(x, f, S):
    """x_hat in NVFP4 and in FP8 for every element, from two runs whose thresholds force each format."""
    lo = orc.quantize(x, f, np.inf, S)           # every block NVFP4
    hi = orc.quantize(x, f, -np.inf, S)          # every block FP8
    assert not lo["mask"].any() and hi["mask"].all()
    # the reconstructions are fp32 values: x4 = fp32(e2m1 * fp32(e4m3 * S)), x8 = fp32(e4m3 * S)
    S64 = np.float64(np.float32(S))
    e4 = _torch_e4m3_decode_all().astype(np.float64)
    d32 = (e4[lo["scales"]] * S64).astype(np.float32).astype(np.float64)
    e2 = np.array(E2M1 + [-v for v in E2M1])[lo["codes"]]
    x4 = (e2 * np.repeat(d32, 16, axis=1)).astype(np.float32).astype(np.float64)
    x8 = (orc.dequantize(hi["codes"], hi["scales"], hi["mask"]) * S64).astype(np.float32).astype(np.float64)
    np.testing.assert_allclose(x4, orc.dequantize(lo["codes"], lo["scales"], lo["mask"]) * S64, rtol=2e-7)
    return x4, x8


@pytest.mark.parametrize("per_element", [False, True])
def test_delta_score_agrees_with_fp64_definition(per_element):
    """Eq. 8: sum F (Q_FP4(v) - Q_FP8(v))^2, recomputed in fp64 from the two
    encodings produced by separate all-FP4 and all-FP8 runs."""
    x, f, S = _random_case(per_element=per_element)
    q4, q8 = _both_reconstructions(x, f, S)
    w = f.astype(np.float64) if per_element else f.astype(np.float64)[None, :]
    want = ((q4 - q8) ** 2 * w).reshape(x.shape[0], -1, 16).sum(axis=2)
    got = orc.quantize(x, f, np.inf, S, score_mode="delta")["scores"]
    assert np.all(got >= 0)
    np.testing.assert_allclose(got, want, rtol=2e-6, atol=0)
    # the two scores differ (otherwise the mode switch does nothing) but are related through the
    # triangle inequality on the block's weighted error vectors: sqrt(I') <= sqrt(I_fp4) + sqrt(I_fp8)
    base = orc.quantize(x, f, np.inf, S)["scores"].astype(np.float64)
    assert not np.array_equal(got, base.astype(np.float32))
    i8 = ((x.astype(np.float64) - q8) ** 2 * w).reshape(x.shape[0], -1, 16).sum(axis=2)
    assert np.all(np.sqrt(want) <= (np.sqrt(base) + np.sqrt(i8)) * (1 + 1e-5) + 1e-30)


def test_delta_score_is_zero_when_both_formats_agree():
    """Values that NVFP4 and FP8 both represent exactly give Q_FP4 = Q_FP8, so
    Eq. 8 is zero while nothing else about the encoding changes."""
    rng = np.random.default_rng(5)
    mags = np.array(E2M1, dtype=np.float32)
    S = 0.5
    x = (rng.choice(mags, size=(8, 64)) * rng.choice([-1.0, 1.0], size=(8, 64))).astype(np.float32)
    x[:, ::16] = 6.0              # every block's maximum is 6: block scale 1/S
    x *= np.float32(S) * 2.0      # e2m1 * (E4M3 scale 2) * S, all exactly FP8-representable after / S
    f = synth.fisher_per_channel(64, 5, 1)
    d = orc.quantize(x, f, 0.0, S, score_mode="delta")
    e = orc.quantize(x, f, 0.0, S)
    assert not d["scores"].any() and not e["scores"].any() and not d["mask"].any()
    for k in ("codes", "scales", "mask"):
        assert np.array_equal(d[k], e[k])


def test_delta_mode_changes_only_scores_and_decisions():
    """At a fixed decision the stored codes do not depend on the score mode;
    with unit weights the score is the plain squared difference (the
    quantization-error policy, Eq. 12); scaling the weights scales it (Eq. 13)."""
    x, f, S = _random_case()
    for T in (np.inf, -np.inf):
        a, b = orc.quantize(x, f, T, S), orc.quantize(x, f, T, S, score_mode="delta")
        for k in ("codes", "scales", "mask"):
            assert np.array_equal(a[k], b[k])
    q4, q8 = _both_reconstructions(x, f, S)
    ones = np.ones(x.shape[1], dtype=np.float32)
    qe = orc.quantize(x, ones, np.inf, S, score_mode="delta")["scores"]
    np.testing.assert_allclose(qe, ((q4 - q8) ** 2).reshape(x.shape[0], -1, 16).sum(axis=2), rtol=2e-6)
    oe = orc.quantize(x, 4.0 * ones, np.inf, S, score_mode="delta")["scores"]
    assert np.array_equal(oe, 4.0 * qe)
    # power-of-two rescaling of the tensor leaves the decisions unchanged
    T = orc.threshold(orc.quantize(x, f, np.inf, S, score_mode="delta")["scores"], 0.2)
    m0 = orc.quantize(x, f, T, S, score_mode="delta")["mask"]
    m1 = orc.quantize(4.0 * x, f, 16.0 * T, 4.0 * S, score_mode="delta")["mask"]
    assert np.array_equal(m0, m1) and abs(m0.mean() - 0.2) < 0.01


# ---------------------------------------------------------------- Eq. 11 clipping

def _nvfp4_error_fp64(xb, fb, d):
    """sum F (x - Q(x))^2 for one block and one scale step d, in fp64, with an
    E2M1 rounding written here from the format table (nearest, ties to the even code)."""
    mags = np.array(E2M1, dtype=np.float64)
    if d == 0.0:
        return float(np.sum(fb * xb * xb))
    r = np.abs(xb) / d
    dist = np.abs(r[:, None] - mags[None, :])
    best = dist.min(axis=1, keepdims=True)
    cand = np.where(dist == best, np.arange(8)[None, :], 99)
    lo = cand.min(axis=1)
    hi = np.where(cand == 99, -1, cand).max(axis=1)
    code = np.where(lo % 2 == 0, lo, hi)          # a tie is between neighbours: take the even one
    xhat = np.sign(xb) * mags[code] * d
    return float(np.sum(fb * (xb - xhat) ** 2))


def test_clipped_scales_minimize_the_weighted_error():
    """Eq. 11 by brute force in fp64 over all 127 E4M3 scale values, on sampled
    blocks: the oracle's error under its chosen scale equals the minimum, and it
    never exceeds the dynamic-max error."""
    w = synth.weights(32, 256, 4, 31)
    f = synth.fisher_per_element(32, 256, 4, 32)
    S = float(synth.default_tensor_scale(w))
    dyn = orc.quantize(w, f, np.inf, S)
    clip = orc.quantize(w, f, np.inf, S, clip=True)
    assert np.all(clip["scores"] <= dyn["scores"])
    assert clip["scores"].sum() < 0.8 * dyn["scores"].sum()        # it does something on Gaussian weights
    e4 = _torch_e4m3_decode_all().astype(np.float64)[:127]
    S64 = np.float64(np.float32(S))
    rng = np.random.default_rng(0)
    for r, b in zip(rng.integers(0, 32, 40), rng.integers(0, 16, 40)):
        xb = w[r, 16 * b:16 * b + 16].astype(np.float64)
        fb = f[r, 16 * b:16 * b + 16].astype(np.float64)
        errs = np.array([_nvfp4_error_fp64(xb, fb, e4[c] * S64) for c in range(127)])
        np.testing.assert_allclose(clip["scores"][r, b], errs.min(), rtol=1e-5)
        # the stored scale reproduces that error, and the stored codes are that scale's quantization
        np.testing.assert_allclose(errs[clip["scales"][r, b]], errs.min(), rtol=1e-5)
        xhat = orc.dequantize(clip["codes"][r:r + 1, 16 * b:16 * b + 16], clip["scales"][r:r + 1, b:b + 1],
                              clip["mask"][r:r + 1, b:b + 1])[0] * S64
        np.testing.assert_allclose(np.sum(fb * (xb - xhat) ** 2), errs.min(), rtol=1e-5)


def test_clipping_trades_an_insensitive_outlier_for_resolution():
    """One large element with a negligible sensitivity next to fifteen small,
    sensitive ones: dynamic max spends the range on the outlier, Eq. 11 does not."""
    x = np.full((1, 16), 0.7, dtype=np.float32)
    x[0, 5] = 12.0
    f = np.ones((1, 16), dtype=np.float32)
    f[0, 5] = 1e-6
    dyn = orc.quantize(x, f, np.inf, 1.0)
    clip = orc.quantize(x, f, np.inf, 1.0, clip=True)
    assert orc.e4m3_decode(int(dyn["scales"][0, 0])) == 2.0            # 12 / 6
    assert clip["scales"][0, 0] < dyn["scales"][0, 0]
    assert clip["scores"][0, 0] < 0.05 * dyn["scores"][0, 0]
    # the outlier saturates at 6 times the clipped scale
    assert clip["codes"][0, 5] == 7
    # an all-zero block keeps scale code 0, a block that dynamic max represents exactly stays exact
    z = orc.quantize(np.zeros((1, 16), np.float32), f, np.inf, 1.0, clip=True)
    assert z["scales"][0, 0] == 0 and z["scores"][0, 0] == 0.0
    exact = (np.array(E2M1 + E2M1, dtype=np.float32) * 0.25)[None, :]
    e = orc.quantize(exact, f, np.inf, 1.0, clip=True)
    assert e["scores"][0, 0] == 0.0


def test_clipping_invariants():
    w = synth.weights(16, 128, 6, 33)
    f = synth.fisher_per_element(16, 128, 6, 34)
    S = float(synth.default_tensor_scale(w))
    a = orc.quantize(w, f, np.inf, S, clip=True)
    b = orc.quantize(w, 4.0 * f, np.inf, S, clip=True)              # weights scaled by a power of two
    c = orc.quantize(2.0 * w, f, np.inf, 2.0 * S, clip=True)        # tensor and its scale scaled together
    for other in (b, c):
        assert np.array_equal(a["codes"], other["codes"]) and np.array_equal(a["scales"], other["scales"])
    assert np.array_equal(b["scores"], 4.0 * a["scores"]) and np.array_equal(c["scores"], 4.0 * a["scores"])
    # the precision decision uses the clipped error: fewer blocks exceed a fixed threshold
    T = orc.threshold(orc.quantize(w, f, np.inf, S)["scores"], 0.3)
    assert orc.quantize(w, f, T, S, clip=True)["mask"].sum() < orc.quantize(w, f, T, S)["mask"].sum()


def test_block_scale_is_dynamic_max():
    """The stored block scale is the E4M3 code nearest to amax / (6 S)."""
    x, f, S = _random_case()
    out = orc.quantize(x, f, np.inf, S)
    amax = np.abs(x).reshape(x.shape[0], -1, 16).max(axis=2).astype(np.float64)
    u = amax / (6.0 * np.float64(np.float32(S)))
    u = u[u <= 448]
    want = torch.from_numpy(u.astype(np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = out["scales"].reshape(-1)[: want.size]
    # fp32 division vs fp64 then cast can differ only exactly at a rounding boundary; allow none here
    assert np.mean(got == want) > 0.999
    assert np.all(np.abs(got.astype(np.int32) - want.astype(np.int32)) <= 1)


def test_mask_is_strict_compare_and_monotone_in_threshold():
    x, f, S = _random_case()
    base = orc.quantize(x, f, np.inf, S)
    scores = base["scores"]
    prev = None
    for p in (0.0, 0.05, 0.1, 0.5, 1.0):
        T = orc.threshold(scores, p)
        out = orc.quantize(x, f, T, S)
        assert np.array_equal(out["scores"], scores)
        assert np.array_equal(out["mask"], (scores > np.float32(T)).astype(np.uint8))
        assert int(out["mask"].sum()) == int(np.floor(p * scores.size + 0.5))
        if prev is not None:
            assert np.all(out["mask"] >= prev)
        prev = out["mask"]
    T = float(np.sort(scores.reshape(-1))[100])
    out = orc.quantize(x, f, T, S)
    assert out["mask"].reshape(-1)[np.argsort(scores.reshape(-1))[100]] == 0  # a tie at T stays FP4


def test_fp8_blocks_are_e4m3_of_scaled_input_and_carry_no_scale():
    x, f, S = _random_case()
    out = orc.quantize(x, f, -np.inf, S)
    assert np.all(out["mask"] == 1) and np.all(out["scales"] == 0)
    r = (x.astype(np.float32) * (np.float32(1.0) / np.float32(S))).astype(np.float32)
    assert np.all(np.abs(r) <= 448.0 * (1 + 1e-6))
    want = torch.from_numpy(np.clip(r, -448, 448)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(out["codes"], want)


def test_power_of_two_rescaling_invariants():
    x, f, S = _random_case()
    T = orc.threshold(orc.quantize(x, f, np.inf, S)["scores"], 0.1)
    ref = orc.quantize(x, f, T, S)
    a = orc.quantize(x, f * np.float32(4), T * 4, S)
    for k in ("codes", "scales", "mask"):
        assert np.array_equal(ref[k], a[k])
    b = orc.quantize(x * np.float32(8), f, T * 64, S * 8)
    for k in ("codes", "scales", "mask"):
        assert np.array_equal(ref[k], b[k])
    assert np.array_equal(b["scores"], ref["scores"] * np.float32(64))


def test_zero_and_underflowing_blocks():
    K = 32
    x = np.zeros((2, K), dtype=np.float32)
    x[1, :16] = np.float32(1e-6) * np.array([1, -1] * 8, dtype=np.float32)
    x[1, 16:] = np.linspace(-1, 1, 16, dtype=np.float32)
    f = np.full(K, 2.0, dtype=np.float32)
    out = orc.quantize(x, f, np.inf, 1.0)
    assert np.all(out["scales"][0] == 0) and np.all(out["codes"][0] == 0) and np.all(out["scores"][0] == 0)
    # amax/(6S) below half the smallest E4M3 subnormal: scale code 0, signed-zero codes, error = x
    assert out["scales"][1, 0] == 0
    assert np.array_equal(out["codes"][1, :16], np.array([0, 8] * 8, dtype=np.uint8))
    np.testing.assert_allclose(out["scores"][1, 0], 16 * 2.0 * 1e-12, rtol=1e-5)


def test_rejects_bad_arguments():
    x = np.ones((1, 16), dtype=np.float32)
    f = np.ones(16, dtype=np.float32)
    with pytest.raises(ValueError):
        orc.quantize(np.full((1, 16), np.nan, dtype=np.float32), f, 0.0, 1.0)
    with pytest.raises(ValueError):
        orc.quantize(x, f, 0.0, 0.0)
    with pytest.raises(ValueError):
        orc.quantize(np.ones((1, 8), dtype=np.float32), np.ones(8, dtype=np.float32), 0.0, 1.0)


# ---------------------------------------------------------------- threshold

@pytest.mark.parametrize("p", [0.0, 0.1, 0.2, 0.3, 0.37, 1.0])
def test_threshold_selects_requested_fraction(p):
    rng = np.random.default_rng(5)
    s = rng.lognormal(size=4097).astype(np.float32)
    T = orc.threshold(s, p)
    assert int((s > np.float32(T)).sum()) == int(np.floor(p * s.size + 0.5))
    if p == 0.0:
        assert T == np.inf
    if p == 1.0:
        assert T == -np.inf


# ---------------------------------------------------------------- product

def _np_decode(out):
    """Independent decode: library cast for E4M3 bytes, the format table for E2M1."""
    e4 = _torch_e4m3_decode_all().astype(np.float64)
    e2 = np.array(E2M1 + [-v for v in E2M1])
    codes, scales, mask = out["codes"], out["scales"], out["mask"]
    rows, K = codes.shape
    m = np.repeat(mask, 16, axis=1).astype(bool)
    s = np.repeat(e4[scales], 16, axis=1)
    return np.where(m, e4[codes], e2[codes & 15] * s)


@pytest.mark.parametrize("p", [1.0, 0.0, 0.1])
def test_gemm_matches_fp64_brute_force_on_tiny(p):
    """p=1 is a plain per-tensor-scaled FP8 GEMM, p=0 a pure NVFP4 GEMM."""
    cfg = synth.tiny_config(0)
    sx, sw = float(cfg["scale_x"]), float(cfg["scale_w"])
    bx = orc.quantize(cfg["x"], cfg["fisher_x"], np.inf, sx)
    bw = orc.quantize(cfg["w"], cfg["fisher_w"], np.inf, sw)
    qx = orc.quantize(cfg["x"], cfg["fisher_x"], orc.threshold(bx["scores"], p), sx)
    qw = orc.quantize(cfg["w"], cfg["fisher_w"], orc.threshold(bw["scores"], p), sw)
    assert int(qx["mask"].sum()) == int(np.floor(p * 256 + 0.5))
    assert int(qw["mask"].sum()) == int(np.floor(p * 4096 + 0.5))
    ax, aw = _np_decode(qx), _np_decode(qw)
    assert np.array_equal(ax, orc.dequantize(qx["codes"], qx["scales"], qx["mask"]))
    assert np.array_equal(aw, orc.dequantize(qw["codes"], qw["scales"], qw["mask"]))
    Y, tol = orc.gemm(ax, sx, aw, sw)
    want = np.float64(np.float32(sx)) * np.float64(np.float32(sw)) * (ax @ aw.T)
    np.testing.assert_allclose(Y, want, rtol=1e-12, atol=1e-300)
    mag = np.float64(np.float32(sx)) * np.float64(np.float32(sw)) * (np.abs(ax) @ np.abs(aw).T)
    np.testing.assert_allclose(tol, 1e-5 * mag, rtol=1e-12)
    # pure-python dot product on a few entries
    for (i, j) in ((0, 0), (3, 17), (15, 255)):
        acc = 0.0
        for k in range(cfg["K"]):
            acc += float(ax[i, k]) * float(aw[j, k])
        assert abs(acc * float(np.float32(sx)) * float(np.float32(sw)) - Y[i, j]) <= 1e-12 * abs(Y[i, j]) + 1e-300
    # the quantized product approximates the unquantized one
    exact = cfg["x"].astype(np.float64) @ cfg["w"].astype(np.float64).T
    rel = np.linalg.norm(Y - exact) / np.linalg.norm(exact)
    assert rel < (0.05 if p == 1.0 else 0.15)
    # every operand and every operand product is an exact fp16 / fp32 number
    assert np.array_equal(ax.astype(np.float16).astype(np.float64), ax)
    assert np.array_equal(aw.astype(np.float16).astype(np.float64), aw)
    prod = ax[:, None, :64] * aw[None, :64, :64]
    assert np.array_equal(prod.astype(np.float32).astype(np.float64), prod)


def test_gemm_row_and_column_sampling():
    cfg = synth.tiny_config(1)
    sx, sw = float(cfg["scale_x"]), float(cfg["scale_w"])
    qx = orc.quantize(cfg["x"], cfg["fisher_x"], 1e-3, sx)
    qw = orc.quantize(cfg["w"], cfg["fisher_w"], 1e-9, sw)
    ax = orc.dequantize(qx["codes"], qx["scales"], qx["mask"])
    aw = orc.dequantize(qw["codes"], qw["scales"], qw["mask"])
    Y, tol = orc.gemm(ax, sx, aw, sw)
    rows, cols = np.array([5, 0, 9]), np.array([200, 3])
    Ys, tols = orc.gemm(ax, sx, aw, sw, rows, cols)
    assert np.array_equal(Ys, Y[np.ix_(rows, cols)]) and np.array_equal(tols, tol[np.ix_(rows, cols)])


# ---------------------------------------------------------------- closed forms the paper prints

# ------------------------------------------------------------------ gated activation in front of the output quantizer

def _ulps(got, want64):
    want32 = np.asarray(want64, dtype=np.float64).astype(np.float32)
    return np.abs(np.asarray(got, dtype=np.float64) - want64) / np.maximum(np.spacing(np.abs(want32)).astype(np.float64), 1e-45)


def test_exponential_steps_against_fp64():
    """The fp32 exponential the gate is defined with: within 1.5 ulp of exp() over its whole range, exact at
    0, clamped outside [-87, 88], never decreasing."""
    x = np.concatenate([np.linspace(-87.0, 88.0, 30001), np.linspace(-1.0, 1.0, 4001)]).astype(np.float32)
    e = np.array([orc.exp_steps(float(v)) for v in x], dtype=np.float64)
    assert _ulps(e, np.exp(x.astype(np.float64))).max() <= 1.5
    assert orc.exp_steps(0.0) == 1.0 and orc.exp_steps(-0.0) == 1.0
    assert orc.exp_steps(1000.0) == orc.exp_steps(88.0) and orc.exp_steps(-1000.0) == orc.exp_steps(-87.0)
    xs = np.sort(x)
    es = np.array([orc.exp_steps(float(v)) for v in xs])
    assert np.all(np.diff(es) >= 0)


def test_silu_mul_against_fp64_definition():
    """h = g / (1 + e^-g) * u: a few ulp from the fp64 value; closed forms at 0 and where e^-g vanishes
    beside 1; SiLU(g) - SiLU(-g) = g; the sign of u carries over."""
    rng = np.random.default_rng(5)
    g = np.concatenate([rng.normal(0, 3, 40000), rng.uniform(-30, 30, 10000), rng.normal(0, 0.05, 5000)]).astype(np.float32)
    u = rng.normal(0, 2, g.size).astype(np.float32)
    h = orc.silu_mul(g, u)
    g64, u64 = g.astype(np.float64), u.astype(np.float64)
    assert _ulps(h, g64 / (1.0 + np.exp(-g64)) * u64).max() <= 4.0
    # g = 0 (either sign) gives a zero; 1 + e^-g is 1 from g = 17 on, so h is the rounded product g u
    assert np.array_equal(orc.silu_mul(np.array([0.0, -0.0], np.float32), np.array([3.0, 3.0], np.float32)), [0.0, -0.0])
    big = np.array([17.0, 20.5, 88.0, 300.0], np.float32)
    assert np.array_equal(orc.silu_mul(big, np.full(4, 1.25, np.float32)), big * np.float32(1.25))
    # far below zero SiLU(g) = g e^g vanishes; the clamp at 87 keeps the result a tiny negative number
    tiny = orc.silu_mul(np.array([-50.0, -100.0], np.float32), np.ones(2, np.float32))
    assert np.all(tiny <= 0) and np.all(np.abs(tiny) < 1e-19)
    # odd-part identity, from the same routine with u = 1
    gp = np.abs(g[:20000])
    one = np.ones_like(gp)
    diff = orc.silu_mul(gp, one).astype(np.float64) - orc.silu_mul(-gp, one).astype(np.float64)
    assert np.all(np.abs(diff - gp) <= 3 * np.spacing(gp))
    assert np.array_equal(orc.silu_mul(g, -u), -h)


def test_exponential_written_two_ways_agrees():
    """The fixed fp32 sequence (range reduction + polynomial) against a structurally different evaluation --
    the C library's fp64 exponential rounded to fp32 once: never more than one unit in the last place apart,
    equal on about nine inputs in ten, equal at the clamps."""
    x = np.concatenate([np.linspace(-87.0, 88.0, 30001), np.linspace(-1.0, 1.0, 4001)]).astype(np.float32)
    a = np.array([orc.exp_steps(float(v)) for v in x], dtype=np.float32)
    b = np.array([orc.exp_rounded_once(float(v)) for v in x], dtype=np.float32)
    # the second form is what it says: the correctly rounded value of the fp64 exponential
    assert np.array_equal(b, np.exp(x.astype(np.float64)).astype(np.float32))
    ulps = np.abs(a.astype(np.float64) - b.astype(np.float64)) / np.spacing(b).astype(np.float64)
    assert ulps.max() <= 1.0
    assert 0.05 <= np.mean(a != b) <= 0.15
    assert orc.exp_rounded_once(500.0) == orc.exp_rounded_once(88.0)
    assert orc.exp_rounded_once(-500.0) == orc.exp_rounded_once(-87.0)


def gate_sample():
    """The seeded sample the gate's two evaluations are compared on: 256 x 4096 gate and up values ~ N(0, 1.6^2)
    (the spread of a Llama-2-7B FC1 product of N(0,1) activations and N(0, 0.02^2) weights over K = 4096 is
    0.02 * sqrt(4096) = 1.28, wider with the outlier channels)."""
    rng = np.random.default_rng([2504, 19])
    g = rng.normal(0, 1.6, (256, 4096)).astype(np.float32)
    u = rng.normal(0, 1.6, (256, 4096)).astype(np.float32)
    return g, u


def test_gate_sequence_against_once_rounded_fp64_value_and_its_effect_on_codes():
    """What "bit-exact" means for the gated epilogue.  h is DEFINED as a fixed fp32 sequence; the mathematically
    exact h rounded to fp32 once (fp64 evaluation) differs from it in about 38% of the elements, by at most
    3 units in the last place -- and that difference changes NO stored code, block scale or precision decision
    on the sample (65536 blocks): quantization to 4 or 8 bits absorbs it unless a value sits within 3 ulp of a
    rounding boundary.  A kernel that followed another correct evaluation of SiLU would therefore produce
    the same packed tensor except in about one block in 10^5 or fewer; the sequence is fixed only to make
    that remainder testable."""
    g, u = gate_sample()
    h_seq = orc.silu_mul(g, u)
    h_ref = orc.silu_mul_rounded_once(g, u)
    g64, u64 = g.astype(np.float64), u.astype(np.float64)
    assert np.array_equal(h_ref, (g64 / (1.0 + np.exp(-g64)) * u64).astype(np.float32))
    differ = h_seq != h_ref
    ulps = np.abs(h_seq.astype(np.float64) - h_ref.astype(np.float64)) / np.spacing(np.abs(h_ref)).astype(np.float64)
    assert ulps.max() <= 3.0
    assert 0.30 <= differ.mean() <= 0.45          # measured 0.381
    # quantize both with the same sensitivities, scale and 10% threshold (calibrated on the sequence's h)
    f = synth.fisher_per_channel(4096, 0, 77)
    S = float(np.abs(h_seq).max() / np.float32(448.0))
    T = orc.threshold(orc.quantize(h_seq, f, np.inf, S)["scores"], 0.1)
    q_seq, q_ref = orc.quantize(h_seq, f, T, S), orc.quantize(h_ref, f, T, S)
    code_blocks = (q_seq["codes"] != q_ref["codes"]).reshape(256, 256, 16).any(axis=2)
    changed = code_blocks | (q_seq["scales"] != q_ref["scales"]) | (q_seq["mask"] != q_ref["mask"])
    assert abs(q_seq["mask"].mean() - 0.1) < 1e-3
    assert changed.mean() <= 1e-4                  # measured 0 of 65536 blocks
    assert (q_seq["mask"] != q_ref["mask"]).sum() <= 2


def test_gate_columns_pairs_rows_of_a_group_of_64():
    """Columns 64q + c and 64q + 32 + c (c < 32) of the product are the gate and up values of hidden unit 32q + c."""
    rng = np.random.default_rng(6)
    y = rng.normal(0, 2, (5, 192)).astype(np.float32)
    h = orc.gate_columns(y)
    assert h.shape == (5, 96)
    for m in range(5):
        for j in (0, 1, 31, 32, 63, 64, 95):
            q, c = divmod(j, 32)
            want = orc.silu_mul(y[m:m + 1, 64 * q + c], y[m:m + 1, 64 * q + 32 + c])[0]
            assert h[m, j] == want
    with pytest.raises(ValueError):
        orc.gate_columns(y[:, :96])


def test_storage_accounting_reproduces_printed_memory_savings():
    J = 1000000
    for frac_fp4, key in ((0.7, "mem_saving_70pct_fp4"), (0.9, "mem_saving_90pct_fp4")):
        n_lo = int(J * frac_fp4)
        bits = orc.storage_bits(n_lo, J - n_lo)
        saving = 1.0 - bits / (J * 16 * 8)
        assert round(saving, 2) == PAPER[key]
    # bytes per block B(p) = (1-p)*9 + p*16 + 1/8
    assert orc.storage_bits(9, 1) / 8 / 10 == pytest.approx(9.825)


def test_operation_counting_reproduces_printed_energy_per_op():
    """One quantized block of 16 outputs follows 16 dot products of length K,
    i.e. 16 * 2K operations; the paper's 0.20 fJ/op fixes "op" = one multiply
    or one add, hence 2*M*N*K operations per GEMM."""
    K = int(PAPER["min_dot_dim_llama2_7b"])
    bs, lanes = int(PAPER["block_size"]), int(PAPER["lanes"])
    per_op_fj = PAPER["ppu_energy_pj_per_block"] * 1e3 / (bs * 2 * K)
    assert round(per_op_fj, 2) == PAPER["ppu_energy_fj_per_op"]
    assert 2 * bs * lanes == PAPER["ops_per_cycle_per_pe"]
    # datapath cycles (M/L)(K/16)(N/P) vs quantizer cycles (M/16)(N/U) balance at P/U = K/L
    M = N = K
    P = PAPER["pes_per_ppu_4k"]
    assert (M / lanes) * (K / 16) * (N / P) == (M / 16) * (N / 1)


def test_division_by_rounded_reciprocal_with_one_correction_is_correctly_rounded(tmp_path):
    """The activation quantizer for large tensors computes amax / (6 S) as a multiply by the rounded
    reciprocal plus one correction with two fused multiply-adds (the general kernel and the oracle divide).
    The two are the same FP32 number for operands inside the normal range: checked here on the host's IEEE
    arithmetic over 3.5 million structured operand pairs (tests/helpers/division_identity.c)."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("gcc not available")
    src = os.path.join(os.path.dirname(os.path.abspath(__file__)), "helpers", "division_identity.c")
    exe = str(tmp_path / "division_identity")
    subprocess.run([gcc, "-O2", "-ffp-contract=off", "-o", exe, src, "-lm"], check=True)
    res = subprocess.run([exe], capture_output=True, text=True)
    assert res.returncode == 0, res.stdout
    assert res.stdout.startswith("0 mismatches of ")
