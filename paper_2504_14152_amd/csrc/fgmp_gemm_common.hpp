// Device helpers shared by the prefill GEMM kernels: block decode with the
// gfx950 conversion instructions, tile geometry, XCD-aware tile order and the
// phase-ordering scheduling hint.
#pragma once
#include "fgmp_internal.hpp"

namespace fgmp {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));

constexpr int kNumXcd = 8;

typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------
// partial sums that workgroups on different XCDs exchange
// ---------------------------------------------------------------------------

// 16-byte accesses to a partial-sum buffer that are coherent across XCDs: buffer instructions with
// the sc0 sc1 cache policy (system scope) bypass the per-XCD L2; being ordinary loads and stores,
// the compiler tracks their completion itself.
constexpr int kCoherent = 1 | 16;   // sc0 | sc1
__device__ __forceinline__ void store_coherent16(__amdgpu_buffer_rsrc_t buf, uint32_t byte_off, float4_t v)
{
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, v), buf, (int)byte_off, 0, kCoherent);
}
__device__ __forceinline__ float4_t load_coherent16(__amdgpu_buffer_rsrc_t buf, uint32_t byte_off)
{
    return __builtin_bit_cast(float4_t, __builtin_amdgcn_raw_buffer_load_b128(buf, (int)byte_off, 0, kCoherent));
}

// ---------------------------------------------------------------------------
// packed -> FP16 decode
// ---------------------------------------------------------------------------

// Decode one block to 16 FP16 values with the gfx950 conversion instructions
// (exact for every code; first element in the low nibble / byte).  `lw` is the
// block's plane-L word, `sb` its plane-S byte, `hw` its plane-H entry (only
// used when `hi`).
__device__ __forceinline__ void decode_block(uint2 lw, uint32_t sb, bool hi, uint2 hw, half2_t (&out)[8])
{
    if (hi) {
        out[0] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(lw.x, 1.0f, false);
        out[1] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(lw.x, 1.0f, true);
        out[2] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(lw.y, 1.0f, false);
        out[3] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(lw.y, 1.0f, true);
        out[4] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(hw.x, 1.0f, false);
        out[5] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(hw.x, 1.0f, true);
        out[6] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(hw.y, 1.0f, false);
        out[7] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(hw.y, 1.0f, true);
    } else {
        // the block scale, in both halves (the multiplies read the low half twice)
        const half2_t s1 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(sb, 1.0f, false);
        const half2_t s = half2_t{s1[0], s1[0]};
        out[0] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lw.x, 1.0f, 0) * s;
        out[1] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lw.x, 1.0f, 1) * s;
        out[2] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lw.x, 1.0f, 2) * s;
        out[3] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lw.x, 1.0f, 3) * s;
        out[4] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lw.y, 1.0f, 0) * s;
        out[5] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lw.y, 1.0f, 1) * s;
        out[6] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lw.y, 1.0f, 2) * s;
        out[7] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lw.y, 1.0f, 3) * s;
    }
}

// Decode the block in slot `lane` of `tile`.
__device__ __forceinline__ void decode_slot(const PackedView &v, int64_t tile, int lane, half2_t (&out)[8])
{
    const uint2 lw = v.L[tile * kTileSlots + lane];
    const uint32_t sb = v.S[tile * kTileSlots + lane];
    const bool hi = (v.M[tile] >> lane) & 1ull;
    uint2 hw = make_uint2(0u, 0u);
    if (hi) hw = v.H[(uint64_t)v.T[tile] + sb];
    decode_block(lw, sb, hi, hw, out);
}

constexpr int kBM = 256, kBN = 256, kBK = 64;
constexpr int kRowBytes = kBK * 2;               // 128 B of K per tile row, 8 chunks of 16 B
constexpr int kTileBytes = kBM * kRowBytes;      // 32 KB per operand per stage

// Map the hardware workgroup id `id` (dispatched round-robin over the 8 XCDs) to a
// logical tile id so that each XCD works on a contiguous range of tiles, then
// to (tile_m, tile_n) in groups of 4 M-tiles so that concurrently running
// workgroups share operand tiles in their XCD's L2: the 32 workgroups an XCD
// runs at a time then cover 4 x 8 tiles, i.e. 4 row panels of A and 8 of the
// packed weights per pass over K (groups of 8 fetch a fifth more, groups of 16
// run 4% slower).
__device__ __forceinline__ void tile_coords(int64_t id, int64_t n_tm, int64_t n_tn, int64_t &tm, int64_t &tn)
{
    const int64_t n = n_tm * n_tn;
    const int64_t xcd = id % kNumXcd, idx = id / kNumXcd;
    const int64_t q = n / kNumXcd, rem = n % kNumXcd;
    const int64_t logical = xcd * q + (xcd < rem ? xcd : rem) + idx;
    constexpr int64_t kGroup = 4;
    const int64_t per_group = kGroup * n_tn;
    const int64_t g = logical / per_group;
    const int64_t first_m = g * kGroup;
    const int64_t gsz = (n_tm - first_m < kGroup) ? n_tm - first_m : kGroup;
    const int64_t in_g = logical % per_group;
    tm = first_m + in_g % gsz;
    tn = in_g / gsz;
}

// LDS tile layout: row r of a 256 x 64 operand tile occupies 128 contiguous
// bytes; its 16-byte chunk q (8 halves of K) sits at chunk position
// q ^ ((r >> 1) & 7).  The swizzle is applied on the global side of the direct
// global->LDS loads (a wave's load always fills 1 KB of consecutive LDS).  The
// LDS serves 256 B (64 banks) per cycle, i.e. 16 lanes of a 16-byte read: 16
// consecutive rows reading the same chunk then touch 16 different 16-byte
// bank groups (measured: no bank-conflict cycles; with q ^ (r & 7) half of
// the LDS cycles were conflicts).
typedef __attribute__((address_space(3))) void lds_void_t;
typedef const __attribute__((address_space(1))) void global_void_t;

// Scheduling hint for one pipeline phase: first the 2 * kVmem global->LDS loads
// and the kReads LDS reads that fetch the next phase's fragments, then the
// kMfma MFMAs on the fragments read one phase earlier.  The reads then have a
// whole phase of MFMA time to land, so no MFMA waits on a read just issued.
template <int kReads, int kMfma, int kVmem> __device__ __forceinline__ void order_phase()
{
    if constexpr (kVmem > 0) __builtin_amdgcn_sched_group_barrier(0x020, 2 * kVmem, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, kReads, 0);
    __builtin_amdgcn_sched_group_barrier(0x008, kMfma, 0);
    __builtin_amdgcn_sched_barrier(0);
}

}  // namespace fgmp
