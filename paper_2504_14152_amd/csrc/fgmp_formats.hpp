// Device-side conversions between FP32 and the two storage formats the paper
// uses (Sec. 4): E2M1 (the NVFP4 element type) and OCP E4M3 (FP8 values and
// NVFP4 block scales).  Rounding is to the nearest representable magnitude,
// ties to the even code, saturating at the format maximum (6 / 448); the sign
// bit is copied from the input.  The integer forms below are the reference
// within the library; the gfx950 conversion instructions are used where they
// give identical results for every input.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fgmp {

__device__ __forceinline__ uint32_t f2u(float f) { return __float_as_uint(f); }
__device__ __forceinline__ float u2f(uint32_t u) { return __uint_as_float(u); }

// ---- E4M3: bias 7, 3 mantissa bits, subnormal step 2^-9, max 448 (0x7E) ----

__device__ __forceinline__ uint32_t e4m3_encode_int(float r)
{
    const uint32_t bits = f2u(r);
    const uint32_t a = bits & 0x7FFFFFFFu;
    uint32_t code;
    if (a >= 0x43E00000u) {          // |r| >= 448 (or NaN/Inf): saturate
        code = 0x7Eu;
    } else if (a < 0x3C800000u) {    // |r| < 2^-6: subnormal range, step 2^-9
        // |r| * 2^9 is exact; adding 2^23 rounds it to an integer, ties to even
        float t = u2f(a) * 512.0f + 8388608.0f;
        code = f2u(t) & 0xFu;        // 0..8 (8 = smallest normal)
    } else {
        uint32_t rounded = a + 0x7FFFFu + ((a >> 20) & 1u);  // RNE on the 20 dropped bits
        code = (rounded >> 20) - (120u << 3);                // rebias 127 -> 7
    }
    return code | ((bits >> 24) & 0x80u);
}

__device__ __forceinline__ float e4m3_decode_int(uint32_t code)
{
    const uint32_t e = (code >> 3) & 15u, m = code & 7u;
    float v;
    if (e == 0)
        v = (float)m * 0.001953125f;                 // m * 2^-9
    else
        v = u2f(((e + 120u) << 23) | (m << 20));     // (1 + m/8) * 2^(e-7)
    return (code & 0x80u) ? -v : v;
}

// ---- E2M1: bias 1, 1 mantissa bit, magnitudes 0 .5 1 1.5 2 3 4 6 ----

__device__ __forceinline__ uint32_t e2m1_encode_int(float r)
{
    const uint32_t bits = f2u(r);
    const uint32_t a = bits & 0x7FFFFFFFu;
    uint32_t code;
    if (a >= 0x40C00000u) {          // |r| >= 6 (or NaN/Inf): saturate
        code = 7u;
    } else if (a < 0x3F800000u) {    // |r| < 1: step 0.5
        float t = u2f(a) * 2.0f + 8388608.0f;
        code = f2u(t) & 0x3u;        // 0, 1, 2 (2 = 1.0)
    } else {
        uint32_t rounded = a + 0x1FFFFFu + ((a >> 22) & 1u);  // RNE on the 22 dropped bits
        code = (rounded >> 22) - (126u << 1);                 // rebias 127 -> 1
    }
    return code | ((bits >> 28) & 0x8u);
}

__device__ __forceinline__ float e2m1_decode_int(uint32_t code)
{
    const uint32_t c = code & 7u;
    // codes >= 2 are normal numbers whose FP32 pattern is (c + 252) << 22
    float v = (c >= 2u) ? u2f((c + 252u) << 22) : 0.5f * (float)c;
    return (code & 8u) ? -v : v;
}

// ---- gfx950 conversion instructions (scale operand 1.0) ----
// Measured against the integer forms over every non-NaN FP32 input: the E2M1
// conversion is identical; the E4M3 conversion is identical up to 464 and
// returns NaN (0x7F) instead of saturating above, hence the clamp to +-448.
// In the packed results the first operand lands in the low nibble / byte.

typedef short short2_t __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

// Two FP32 -> two E2M1 codes in the low byte (a in the low nibble).
__device__ __forceinline__ uint32_t e2m1_encode_pair_hw(float a, float b)
{
    return __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(0u, a, b, 1.0f, 0) & 0xFFu;
}

// Two FP32 -> two E4M3 bytes in the low 16 bits (a in the low byte).
__device__ __forceinline__ uint32_t e4m3_encode_pair_hw(float a, float b)
{
    short2_t z = {0, 0};
    a = __builtin_amdgcn_fmed3f(a, -448.0f, 448.0f);
    b = __builtin_amdgcn_fmed3f(b, -448.0f, 448.0f);
    short2_t r = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(z, a, b, 1.0f, false);
    return (uint32_t)(uint16_t)r[0];
}

// Low byte of `packed` holds two E2M1 codes -> two FP32.
__device__ __forceinline__ float2_t e2m1_decode_pair_hw(uint32_t packed)
{
    return __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(packed, 1.0f, 0);
}

// Low 16 bits of `packed` hold two E4M3 bytes -> two FP32.
__device__ __forceinline__ float2_t e4m3_decode_pair_hw(uint32_t packed)
{
    return __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(packed, 1.0f, false);
}

}  // namespace fgmp
