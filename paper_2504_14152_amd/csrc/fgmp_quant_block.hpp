// The arithmetic of one 16-element block, shared by every kernel that quantizes
// (the standalone quantizer, the clipping search, the GEMM epilogue), so that they
// agree bit for bit: block scale, NVFP4 codes, the block's score, FP8 codes.
#pragma once
#include "fgmp_internal.hpp"

namespace fgmp {

template <bool kHW> __device__ __forceinline__ uint32_t enc_e4m3(float r)
{
    if constexpr (kHW) return e4m3_encode_pair_hw(r, 0.0f) & 0xFFu;
    else return e4m3_encode_int(r);
}

// Load 16 consecutive elements as FP32.
__device__ __forceinline__ void load16(const float *src, float (&x)[16])
{
    const float4 *p = reinterpret_cast<const float4 *>(src);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float4 v = p[i];
        x[4 * i + 0] = v.x; x[4 * i + 1] = v.y; x[4 * i + 2] = v.z; x[4 * i + 3] = v.w;
    }
}

// FP8 codes of 16 values (already multiplied by 1/S) as four dwords.
template <bool kHW, bool kClamp> __device__ __forceinline__ void encode_fp8_block(const float (&r)[16], uint32_t (&c)[4])
{
    if constexpr (kHW) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            short2_t acc = {0, 0};
            float a0 = r[4 * j], a1 = r[4 * j + 1], a2 = r[4 * j + 2], a3 = r[4 * j + 3];
            if constexpr (kClamp) {   // the instruction returns NaN instead of saturating beyond 464
                a0 = __builtin_amdgcn_fmed3f(a0, -448.0f, 448.0f);
                a1 = __builtin_amdgcn_fmed3f(a1, -448.0f, 448.0f);
                a2 = __builtin_amdgcn_fmed3f(a2, -448.0f, 448.0f);
                a3 = __builtin_amdgcn_fmed3f(a3, -448.0f, 448.0f);
            }
            acc = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(acc, a0, a1, 1.0f, false);
            acc = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(acc, a2, a3, 1.0f, true);
            c[j] = (uint32_t)(uint16_t)acc[0] | ((uint32_t)(uint16_t)acc[1] << 16);
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            c[j] = e4m3_encode_int(r[4 * j]) | (e4m3_encode_int(r[4 * j + 1]) << 8) |
                   (e4m3_encode_int(r[4 * j + 2]) << 16) | (e4m3_encode_int(r[4 * j + 3]) << 24);
    }
}

// Header of a packed tensor (one thread of the kernel that writes the tensor calls this).
__device__ __forceinline__ void write_header(PackedHeader *hdr, const PackedLayout &l, float S, uint32_t compact)
{
    hdr->magic = kMagic;
    hdr->version = kVersion;
    hdr->rows = l.rows;
    hdr->K = l.K;
    hdr->tensor_scale = S;
    hdr->compact = compact;
    hdr->off_L = l.off_L;
    hdr->off_S = l.off_S;
    hdr->off_M = l.off_M;
    hdr->off_T = l.off_T;
    hdr->off_H = l.off_H;
    hdr->h_entries = (uint64_t)l.n_tiles * kTileSlots;   // a compact tensor's scan overwrites these two
    hdr->bytes_used = l.total_bytes;
}

__device__ __forceinline__ float block_amax(const float (&x)[16])
{
    float amax = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) amax = fmaxf(amax, fabsf(x[i]));
    return amax;
}

struct BlockCodes {
    uint32_t q[2];     // 16 E2M1 nibbles, element 2i in the low nibble of byte i
    uint32_t sc;       // E4M3 block scale code
    float score;       // Eq. 6 (or Eq. 8) of the block
    uint32_t c8[4];    // FP8 codes of the block (only filled in the Eq. 8 mode)
};

// x: the block; f: its sensitivities; S: tensor scale (inv_S = 1/S, S6 = 6 S computed once by the caller).
// sc_given < 0: dynamic-max scale E4M3(amax / (6 S)) (Sec. 3.3); otherwise the scale code to use.
// kDelta: the score is Eq. 8's weighted square of Q_NVFP4(x) - Q_FP8(x) instead of Eq. 6's NVFP4 error;
// clamp8 says whether the FP8 conversion must clamp to +-448 first (decided per wave by the caller).
// Products are two separately rounded multiplies, the sum is a tree over adjacent pairs.
template <bool kHW, bool kDelta>
__device__ __forceinline__ void quantize_block_math(const float (&x)[16], const float (&f)[16], float amax, float S,
                                                    float inv_S, float S6, int sc_given, bool clamp8, BlockCodes &o)
{
    uint32_t sc;
    if (sc_given < 0) sc = enc_e4m3<kHW>(amax / S6);
    else sc = (uint32_t)sc_given;
    const float d = e4m3_decode_int(sc) * S;
    const float inv_d = (sc != 0u) ? 1.0f / d : 0.0f;

    uint32_t c8[4] = {0u, 0u, 0u, 0u};
    if constexpr (kDelta) {
        float r[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) r[i] = x[i] * inv_S;
        if (clamp8) encode_fp8_block<kHW, true>(r, c8);
        else encode_fp8_block<kHW, false>(r, c8);
    }

    uint32_t q[2] = {0u, 0u};
    float t[16];
    if constexpr (kHW) {
        // each conversion fills one byte of the code word in place (the byte selector is an immediate)
#define FGMP_ENC(W, B, I) q[W] = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(q[W], x[I] * inv_d, x[I + 1] * inv_d, 1.0f, B)
        FGMP_ENC(0, 0, 0); FGMP_ENC(0, 1, 2); FGMP_ENC(0, 2, 4); FGMP_ENC(0, 3, 6);
        FGMP_ENC(1, 0, 8); FGMP_ENC(1, 1, 10); FGMP_ENC(1, 2, 12); FGMP_ENC(1, 3, 14);
#undef FGMP_ENC
#define FGMP_ERR(W, B, I)                                                                          \
    {                                                                                              \
        const float2_t v = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(q[W], 1.0f, B);                \
        float e0, e1;                                                                              \
        if constexpr (kDelta) {                                                                    \
            const float2_t v8 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(c8[(I) / 4], 1.0f, ((I) % 4) >= 2); \
            e0 = v[0] * d - v8[0] * S;                                                             \
            e1 = v[1] * d - v8[1] * S;                                                             \
        } else {                                                                                   \
            e0 = x[I] - v[0] * d;                                                                  \
            e1 = x[I + 1] - v[1] * d;                                                              \
        }                                                                                          \
        t[I] = (e0 * e0) * f[I];                                                                   \
        t[I + 1] = (e1 * e1) * f[I + 1];                                                           \
    }
        FGMP_ERR(0, 0, 0) FGMP_ERR(0, 1, 2) FGMP_ERR(0, 2, 4) FGMP_ERR(0, 3, 6)
        FGMP_ERR(1, 0, 8) FGMP_ERR(1, 1, 10) FGMP_ERR(1, 2, 12) FGMP_ERR(1, 3, 14)
#undef FGMP_ERR
    } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const uint32_t c = e2m1_encode_int(x[i] * inv_d);
            q[i >> 3] |= c << (4 * (i & 7));
            float e;
            if constexpr (kDelta) e = e2m1_decode_int(c) * d - e4m3_decode_int((c8[i >> 2] >> (8 * (i & 3))) & 0xFFu) * S;
            else e = x[i] - e2m1_decode_int(c) * d;
            t[i] = (e * e) * f[i];
        }
    }
#pragma unroll
    for (int w = 16; w > 1; w >>= 1)
#pragma unroll
        for (int i = 0; i < w / 2; ++i) t[i] = t[2 * i] + t[2 * i + 1];
    o.q[0] = q[0];
    o.q[1] = q[1];
    o.sc = sc;
    o.score = t[0];
#pragma unroll
    for (int j = 0; j < 4; ++j) o.c8[j] = c8[j];
}

}  // namespace fgmp
