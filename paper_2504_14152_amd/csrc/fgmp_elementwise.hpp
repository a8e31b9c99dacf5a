// Gated activation in front of the output quantizer: h = SiLU(g) * u, SiLU(g) = g / (1 + e^-g), the
// operator between the two MLP products of the Llama models the paper evaluates (the paper's unit
// quantizes results before they are written out, Sec. 4.2; it does not discuss the operator).  The
// quantized codes depend on h to the last bit, so h is a fixed sequence of FP32 operations, each rounded
// on its own (the build disables FMA contraction; FP32 division is correctly rounded):
//   E(x), x clamped to [-87, 88]: n = rint(x * log2(e)); r = (x - n * C1) - n * C2 with C1 + C2 = ln 2
//   (n * C1 exact); p = degree-7 Taylor polynomial of e^r, Horner; E = p * 2^n.
//   h = (g / (1 + E(-g))) * u
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fgmp {

__device__ __forceinline__ float exp_steps(float x)
{
    x = x > 88.0f ? 88.0f : x;
    x = x < -87.0f ? -87.0f : x;
    const float n = __builtin_rintf(x * 1.44269504f);   // nearest, ties to even
    float r = x - n * 0.693359375f;
    r = r - n * -2.12194440e-4f;
    float p = 1.0f / 5040.0f;
    p = p * r + 1.0f / 720.0f;
    p = p * r + 1.0f / 120.0f;
    p = p * r + 1.0f / 24.0f;
    p = p * r + 1.0f / 6.0f;
    p = p * r + 0.5f;
    p = p * r + 1.0f;
    p = p * r + 1.0f;
    const uint32_t two_n = (uint32_t)((int)n + 127) << 23;
    return p * __builtin_bit_cast(float, two_n);
}

__device__ __forceinline__ float silu_mul(float g, float u)
{
    const float d = 1.0f + exp_steps(-g);
    return (g / d) * u;
}

// Weight rows of a gated product come in groups of 64: rows 64 q .. 64 q + 31 are the gate rows of
// hidden units 32 q .. 32 q + 31, rows 64 q + 32 .. 64 q + 63 their up rows (so that a wave of the
// prefill kernel holds a unit's two values in the same lane and register of two accumulator tiles).
constexpr int kGateGroup = 64;

}  // namespace fgmp
