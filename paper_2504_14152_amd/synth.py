"""Seeded synthetic inputs shaped like the paper's workloads.

Llama-2 linear-layer shapes at 4K context (Sec. 5.3, Sec. 5.4.3) with
Gaussian stimulus (Sec. 4.3) stand in for real activations, weights and Fisher
information, none of which ship with this repository.  This module holds input
generation only -- random draws, outlier channels, bf16 rounding of the
inputs, the default per-tensor scale -- and none of the method's arithmetic,
so that both the HIP path and the CPU oracle can be fed the same bytes.
"""
from __future__ import annotations

import numpy as np

BLOCK = 16

# (K, N) of the four Llama-2-7B linear layers and the 70B FC1 layer.
LLAMA2_7B = {"qkv": (4096, 12288), "o": (4096, 4096), "fc1": (4096, 22016), "fc2": (11008, 4096)}
LLAMA2_70B_FC1 = (8192, 57344)


def rng_for(seed: int, tensor_id: int) -> np.random.Generator:
    """One independent stream per (seed, tensor)."""
    return np.random.default_rng([int(seed), int(tensor_id)])


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest even), returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to fp32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def outlier_channels(K: int, frac: float, rng: np.random.Generator, count: int | None = None) -> np.ndarray:
    n = count if count is not None else max(1, int(K * frac + 0.5))
    return np.sort(rng.choice(K, size=n, replace=False))


def activations(M: int, K: int, seed: int = 0, tensor_id: int = 1, *, kind: str = "normal",
                outlier_frac: float = 0.01, outlier_count: int | None = None,
                outlier_gain: float = 20.0) -> np.ndarray:
    """fp32 M x K activations: N(0,1) with a few input channels scaled up, or
    SiLU(a)*b of two N(0,1) draws (heavy-tailed, the FC2 input)."""
    rng = rng_for(seed, tensor_id)
    if kind == "normal":
        x = rng.standard_normal((M, K), dtype=np.float32)
        ch = outlier_channels(K, outlier_frac, rng, outlier_count)
        x[:, ch] *= np.float32(outlier_gain)
    elif kind == "silu_gate":
        a = rng.standard_normal((M, K), dtype=np.float32)
        b = rng.standard_normal((M, K), dtype=np.float32)
        x = (a / (np.float32(1.0) + np.exp(-a))) * b
    else:
        raise ValueError(kind)
    return x


def weights(N: int, K: int, seed: int = 0, tensor_id: int = 2, std: float = 0.02) -> np.ndarray:
    """fp32 N x K weights ~ N(0, std)."""
    rng = rng_for(seed, tensor_id)
    w = rng.standard_normal((N, K), dtype=np.float32)
    w *= np.float32(std)
    return w


def fisher_per_channel(K: int, seed: int = 0, tensor_id: int = 3) -> np.ndarray:
    """Per-input-channel sensitivities, lognormal(0, 1), fp32."""
    rng = rng_for(seed, tensor_id)
    return np.exp(rng.standard_normal(K, dtype=np.float32)).astype(np.float32)


def fisher_per_element(N: int, K: int, seed: int = 0, tensor_id: int = 4) -> np.ndarray:
    """Per-element sensitivities, lognormal(0, 1), fp32."""
    rng = rng_for(seed, tensor_id)
    return np.exp(rng.standard_normal((N, K), dtype=np.float32)).astype(np.float32)


def default_tensor_scale(x: np.ndarray) -> np.float32:
    """The FP32 per-tensor scale used when none was calibrated: amax / 448,
    so that the largest element maps to the largest E4M3 magnitude."""
    amax = np.float32(np.max(np.abs(x)))
    return np.float32(amax / np.float32(448.0))


def tiny_config(seed: int = 0) -> dict:
    """The small fp32 case: X 16x256 with two outlier channels, W 256x256."""
    M, K, N = 16, 256, 256
    x = activations(M, K, seed, 1, outlier_count=2)
    w = weights(N, K, seed, 2)
    return {"M": M, "K": K, "N": N, "x": x, "w": w,
            "fisher_x": fisher_per_channel(K, seed, 3),
            "fisher_w": fisher_per_element(N, K, seed, 4),
            "scale_x": default_tensor_scale(x), "scale_w": default_tensor_scale(w)}


def exact_sum_operand(rows: int, K: int, seed: int, tensor_id: int, fp8_block_fraction: float = 0.2) -> np.ndarray:
    """A rows x K fp32 tensor made so that a product of two such tensors has no rounding at all for
    K <= 128, whatever the summation order: every value is a multiple of 2**-4 of magnitude <= 12.
    Each 16-element block is scaled by 2**j, j in {-1, 0, 1}; most blocks hold values from the grid
    {0, .5, 1, 1.5, 2, 3, 4, 6} * 2**j with the value 6 * 2**j present, the others multiples of
    2**j / 8 below 2 * 2**j.  (With a tensor scale of 1 the first kind is exactly representable as a
    4-bit block with a power-of-two block scale, the second only as 8-bit floating point.)"""
    rng = rng_for(seed, tensor_id)
    nb = K // 16
    grid4 = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0], dtype=np.float32)
    j = rng.integers(-1, 2, size=(rows, nb, 1)).astype(np.float32)
    sign = rng.choice(np.array([-1.0, 1.0], dtype=np.float32), size=(rows, nb, 16))
    a = grid4[rng.integers(0, 8, size=(rows, nb, 16))]
    pos = rng.integers(0, 16, size=(rows, nb))
    np.put_along_axis(a, pos[..., None], np.float32(6.0), axis=2)
    b = rng.integers(0, 16, size=(rows, nb, 16)).astype(np.float32) / np.float32(8.0)
    b[..., 0] = np.float32(1.875)          # not on the 4-bit grid for any block scale that also fits the rest
    b[..., 1] = np.float32(0.125)
    kind8 = rng.random(size=(rows, nb, 1)) < fp8_block_fraction
    v = np.where(kind8, b, a) * sign * np.exp2(j).astype(np.float32)
    return v.reshape(rows, K).astype(np.float32)



def exact_sum_operand_long_k(rows: int, K: int, seed: int, tensor_id: int, fp8_block_fraction: float = 0.2) -> np.ndarray:
    """Like exact_sum_operand, for long dot products: every value is a multiple of 2**-3 of magnitude <= 3,
    so a product of two such tensors is a sum of multiples of 2**-6 bounded by 9 K -- exact in fp32 in any
    summation order up to K = 2**16 / 9 * 2**2 (|sum| * 64 < 2**24 holds for K <= 29127).  Each block is scaled by
    2**j, j in {-1, 0}; most blocks hold values from {0, .25, .5, .75, 1, 1.5, 2, 3} * 2**j with 3 * 2**j
    present (a 4-bit block with block scale 2**(j-1) when the tensor scale is 1), the others multiples of
    2**j / 4 up to 2.75 * 2**j with 2.75 * 2**j and 0.25 * 2**j present (exact as 8-bit floating point, not as a 4-bit block)."""
    rng = rng_for(seed, tensor_id)
    nb = K // 16
    grid4 = np.array([0.0, 0.25, 0.5, 0.75, 1.0, 1.5, 2.0, 3.0], dtype=np.float32)
    j = rng.integers(-1, 1, size=(rows, nb, 1)).astype(np.float32)
    sign = rng.choice(np.array([-1.0, 1.0], dtype=np.float32), size=(rows, nb, 16))
    a = grid4[rng.integers(0, 8, size=(rows, nb, 16))]
    pos = rng.integers(0, 16, size=(rows, nb))
    np.put_along_axis(a, pos[..., None], np.float32(3.0), axis=2)
    b = rng.integers(0, 12, size=(rows, nb, 16)).astype(np.float32) / np.float32(4.0)
    b[..., 0] = np.float32(2.75)
    b[..., 1] = np.float32(0.25)
    kind8 = rng.random(size=(rows, nb, 1)) < fp8_block_fraction
    v = np.where(kind8, b, a) * sign * np.exp2(j).astype(np.float32)
    return v.reshape(rows, K).astype(np.float32)
