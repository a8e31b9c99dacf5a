// FGMP block scoring, precision decision, encoding and packing (Sec. 3.1,
// Sec. 3.3 "dynamic max", Sec. 4, Sec. 4.2), one 16-element block per lane.
//
// Arithmetic per block (every FP32 step is one separately rounded IEEE
// operation -- this file is compiled with -ffp-contract=off):
//   amax = max|x_i|; u = amax / (6 S); sc = E4M3(u); d = value(sc) * S
//   inv_d = 1 / d (0 when sc == 0); q_i = E2M1(x_i * inv_d); xh_i = value(q_i) * d
//   t_i = ((x_i - xh_i) * (x_i - xh_i)) * F_i                        (Eq. 2, Eq. 6)
//   score = balanced pairwise tree over t_0..t_15 (adjacent pairs first)
//   FP8 iff score > T (Sec. 4.2); FP8 codes c_i = E4M3(x_i * (1 / S))  (Sec. 5.1)
#include <algorithm>

#include "fgmp_internal.hpp"
#include "fgmp_quant_block.hpp"

namespace fgmp {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

struct QuantParams {
    const void *X;
    int64_t ldx, rows, nb;
    const float *fisher;
    int64_t ld_fisher;
    float T, S;
    PackedView out;
    int64_t n_rt, n_kt;
    float *scores;
    int mode;          // kModeStrided / kModeCount / kModeCompact / kModeF16
    int rt_per_wave;
    PackedLayout layout;   // for the header, written by the first launch of a call
    uint32_t compact;
    _Float16 *x16;         // kModeF16: dequantized values (without the tensor scale), [8 n_rt][ld16]
    int64_t ld16;
    uint32_t *zero;        // words cleared by the first workgroup (counters of the kernel that follows)
    int zero_n;
    bool delta;            // Eq. 8 scoring (see quantize_kernel)
    const uint8_t *sc_override;   // block scale codes chosen beforehand (clipping), [rows][nb]; or nullptr: dynamic max
};

// kModeF16 writes, instead of the packed planes, the FP16 value of every stored
// code (exact: an E2M1 value times an E4M3 scale, or an E4M3 value), which is
// what the prefill GEMM consumes; only the header goes to the packed buffer.
enum { kModeStrided = 0, kModeCount = 1, kModeCompact = 2, kModeF16 = 3 };


// Raw (unconverted) 16 input elements of one block: 2 x 16 B of bf16 or 4 x 16 B of fp32.
template <typename Tin> struct RawBlock;
template <> struct RawBlock<uint16_t> { uint4 v[2]; };
template <> struct RawBlock<float> { uint4 v[4]; };

template <typename Tin> __device__ __forceinline__ void load_raw(const Tin *src, RawBlock<Tin> &r)
{
    const uint4 *p = reinterpret_cast<const uint4 *>(src);
#pragma unroll
    for (int i = 0; i < (int)(sizeof(r.v) / sizeof(uint4)); ++i) r.v[i] = p[i];
}

__device__ __forceinline__ void widen(const RawBlock<uint16_t> &r, float (&x)[16])
{
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const uint32_t w[4] = {r.v[i].x, r.v[i].y, r.v[i].z, r.v[i].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {   // bf16 -> fp32 is a 16-bit shift
            x[8 * i + 2 * j + 0] = u2f(w[j] << 16);
            x[8 * i + 2 * j + 1] = u2f(w[j] & 0xFFFF0000u);
        }
    }
}

__device__ __forceinline__ void widen(const RawBlock<float> &r, float (&x)[16])
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        x[4 * i + 0] = u2f(r.v[i].x); x[4 * i + 1] = u2f(r.v[i].y);
        x[4 * i + 2] = u2f(r.v[i].z); x[4 * i + 3] = u2f(r.v[i].w);
    }
}

// grid.x = K-tiles, grid.y = groups of 4 * rt_per_wave row-tiles; 4 waves per
// workgroup work on 4 adjacent row-tiles of the same K-tile at a time, so the
// per-channel sensitivities stay in registers across the loop.  The input of
// the next row-tile is fetched while the current one is processed.
// kDelta: the score is Eq. 8's (weighted square of Q_NVFP4(x) - Q_FP8(x)) instead of Eq. 6's NVFP4 error;
// the FP8 codes are then computed for every block and reused when the block is kept in FP8.
template <typename Tin, bool kPerElem, bool kHW, int kMode, bool kDelta>
__global__ __launch_bounds__(256) void quantize_kernel(QuantParams p)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int64_t kt = blockIdx.x;
    const int64_t kb = kt * kTileBlocks + (lane & 7);
    const bool kvalid = kb < p.nb;
    const int rloc = lane >> 3;
    const Tin *X = static_cast<const Tin *>(p.X);

    float f[16];
    if constexpr (!kPerElem) {
        if (kvalid) load16(p.fisher + kb * kBlock, f);
        else {
#pragma unroll
            for (int i = 0; i < 16; ++i) f[i] = 0.0f;
        }
    }
    const float inv_S = 1.0f / p.S;
    const float S6 = 6.0f * p.S;
    if constexpr (kMode != kModeCompact) {
        if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0 && p.out.hdr != nullptr)
            write_header(p.out.hdr, p.layout, p.S, p.compact);
    }
    if (blockIdx.x == 0 && blockIdx.y == 0)
        for (int i = threadIdx.x; i < p.zero_n; i += 256) p.zero[i] = 0u;

    const int64_t rt0 = (int64_t)blockIdx.y * p.rt_per_wave * 4 + wave;
    // out-of-range lanes read a valid address (their own K-tile's first block of row 0) and are masked
    auto src_of = [&](int64_t rt) -> const Tin * {
        const int64_t row = rt * kTileRows + rloc;
        const bool ok = kvalid && row < p.rows;
        return X + (ok ? row * p.ldx + kb * kBlock : 0);
    };
    if (rt0 >= p.n_rt) return;
    const int64_t left = (p.n_rt - rt0 + 3) / 4;
    const int n_it = (int)(left < p.rt_per_wave ? left : p.rt_per_wave);

    auto process = [&](int64_t rt, const RawBlock<Tin> &raw_in) {
        const int64_t row = rt * kTileRows + rloc;
        const bool valid = kvalid && row < p.rows;

        float x[16];
        widen(raw_in, x);
        if (!valid) {
#pragma unroll
            for (int i = 0; i < 16; ++i) x[i] = 0.0f;
        }
        if constexpr (kPerElem) {
            if (valid) load16(p.fisher + row * p.ld_fisher + kb * kBlock, f);
            else {
#pragma unroll
                for (int i = 0; i < 16; ++i) f[i] = 0.0f;
            }
        }

        // block scale (dynamic max, or chosen beforehand), NVFP4 codes, score; in the Eq. 8 mode also the
        // FP8 codes of every block (values beyond the FP8 range only occur when the caller's S is below
        // amax / 448: then the wave clamps before converting)
        const float amax = block_amax(x);
        bool clamp8 = false;
        if constexpr (kDelta) clamp8 = __ballot(amax * inv_S > 448.0f) != 0ull;
        int sc_given = -1;
        if (p.sc_override != nullptr) sc_given = valid ? (int)p.sc_override[row * p.nb + kb] : 0;
        BlockCodes bc;
        quantize_block_math<kHW, kDelta>(x, f, amax, p.S, inv_S, S6, sc_given, clamp8, bc);
        const uint32_t sc = bc.sc;
        const uint32_t (&q)[2] = bc.q;
        const uint32_t (&c8)[4] = bc.c8;
        const float score = bc.score;

        const bool hi = valid && (score > p.T);
        const uint64_t ballot = __ballot(hi);
        const int64_t tile = rt * p.n_kt + kt;
        if (p.scores != nullptr && valid) p.scores[row * p.nb + kb] = score;

        if constexpr (kMode == kModeCount) {
            if (lane == 0) p.out.T[tile] = (uint32_t)__popcll(ballot);
        } else if constexpr (kMode == kModeF16) {
            static_assert(kHW, "the FP16 output mode uses the conversion instructions");
            half2_t o[8];
            if (hi) {
                uint32_t c[4];
                if constexpr (kDelta) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) c[j] = c8[j];
                } else {
                    float r[16];
#pragma unroll
                    for (int i = 0; i < 16; ++i) r[i] = x[i] * inv_S;
                    if (amax * inv_S > 448.0f) encode_fp8_block<kHW, true>(r, c);
                    else encode_fp8_block<kHW, false>(r, c);
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    o[2 * j] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(c[j], 1.0f, false);
                    o[2 * j + 1] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(c[j], 1.0f, true);
                }
            } else {
                const half2_t s = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(sc | (sc << 8), 1.0f, false);
                o[0] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(q[0], 1.0f, 0) * s;
                o[1] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(q[0], 1.0f, 1) * s;
                o[2] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(q[0], 1.0f, 2) * s;
                o[3] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(q[0], 1.0f, 3) * s;
                o[4] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(q[1], 1.0f, 0) * s;
                o[5] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(q[1], 1.0f, 1) * s;
                o[6] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(q[1], 1.0f, 2) * s;
                o[7] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(q[1], 1.0f, 3) * s;
            }
            // every slot of the tile is written (zeros where the tensor ends), so the GEMM can read whole tiles
            union { half2_t h[8]; uint4 v[2]; } pack;
#pragma unroll
            for (int j = 0; j < 8; ++j) pack.h[j] = o[j];
            uint4 *dst = reinterpret_cast<uint4 *>(p.x16 + (rt * kTileRows + rloc) * p.ld16 +
                                                   (kt * kTileBlocks + (lane & 7)) * kBlock);
            dst[0] = pack.v[0];
            dst[1] = pack.v[1];
        } else {
            const uint32_t prefix = (uint32_t)__popcll(ballot & ((1ull << lane) - 1ull));
            uint32_t hbase;
            if constexpr (kMode == kModeStrided) {
                hbase = (uint32_t)(tile * kTileSlots);
                if (lane == 0) p.out.T[tile] = hbase;
            } else {
                hbase = p.out.T[tile];
            }
            if (lane == 0) p.out.M[tile] = ballot;

            uint2 lword = make_uint2(q[0], q[1]);
            uint32_t sbyte = sc;
            if (ballot != 0ull) {
                // values beyond the FP8 range only occur when the caller's S is below amax / 448
                const bool any_big = __ballot(hi && amax * inv_S > 448.0f) != 0ull;
                if (hi) {
                    uint32_t c[4];
                    if constexpr (kDelta) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) c[j] = c8[j];
                    } else {
                        float r[16];
#pragma unroll
                        for (int i = 0; i < 16; ++i) r[i] = x[i] * inv_S;
                        if (any_big) encode_fp8_block<kHW, true>(r, c);
                        else encode_fp8_block<kHW, false>(r, c);
                    }
                    lword = make_uint2(c[0], c[1]);
                    p.out.H[(uint64_t)hbase + prefix] = make_uint2(c[2], c[3]);
                    sbyte = prefix;
                }
            }
            p.out.L[tile * kTileSlots + lane] = lword;
            p.out.S[tile * kTileSlots + lane] = (uint8_t)sbyte;
        }
    };

    // software pipeline: the next row-tile's input is in flight while this one is processed
    RawBlock<Tin> cur, nxt;
    load_raw(src_of(rt0), cur);
    for (int it = 0; it + 1 < n_it; ++it) {
        load_raw(src_of(rt0 + 4 * (int64_t)(it + 1)), nxt);
        process(rt0 + 4 * (int64_t)it, cur);
        cur = nxt;
    }
    process(rt0 + 4 * (int64_t)(n_it - 1), cur);
}

// ---------------------------------------------------------------------------
// The activation hot path (Sec. 4.2) once more, trimmed: same arithmetic, result for result, as
// quantize_kernel (NVFP4-error score, one sensitivity per channel, dynamic-max scale).
//   * d = value(sc) * S and 1 / d depend only on the scale code: a table of 127 {d, 1/d} pairs per
//     workgroup (LDS) replaces the decode, the multiply and the division of every block;
//   * u = amax / (6 S) is one multiply by the correctly rounded reciprocal r and one correction step,
//     q1 = fma(fma(-q0, 6S, amax), r, q0): the correctly rounded quotient (q0 is within one unit of it and
//     the residual is exact; magnitudes near the ends of the FP32 range, where that fails, take the plain
//     division instead);
//   * input through range-checked buffer loads: rows beyond the tensor read zeros without a select;
//   * a workgroup's eight waves take eight consecutive K-tiles of one row-tile at a time (2 KB of every
//     row, 4 KB of plane L, 512 B of plane S: contiguous), and workgroups that run at the same time cover
//     whole rows; the launch is one resident set of workgroups that stride over the row-tiles, so a wave
//     keeps its K-tile and the sensitivities stay in registers;
//   * the 12 bytes of per-tile words are not stored tile by tile (those small stores alone cost 6% of the
//     run time): the plane-M and plane-T words of eight row-tiles are gathered in LDS and leave as 64- and
//     32-byte pieces;
//   * the FP8 upper halves of the tiles a wave visits are appended to a region of plane H that belongs to
//     the wave (see h_cnt below).
// Tensors up to 4 GB (32-bit offsets).
// ---------------------------------------------------------------------------
constexpr int kQWaves = 8;    // waves per workgroup = consecutive K-tiles
constexpr int kQBatch = 8;    // row-tiles between two writes of the gathered plane-M words
constexpr int64_t kQMinTiles = 65536;   // smaller tensors do not fill the resident set for long enough: general kernel

// kTraffic (measurement builds only): the kernel's loads and stores with next to no arithmetic between them
// -- the plane-L words are input words, a fixed tenth of the slots counts as FP8 -- i.e. what the memory
// system alone takes for this access pattern; the benchmark times it beside the real kernel.
// kDelta: the score of Eq. 8 (the FP8 codes of every block are computed first and reused for the blocks kept in FP8).
template <typename Tin, int kMode, bool kTraffic = false, bool kDelta = false>
__global__ __launch_bounds__(64 * kQWaves) void quantize_act_kernel(QuantParams p, uint32_t x_bytes, uint32_t out_bytes, int n_kg)
{
    static_assert(kMode == kModeStrided || kMode == kModeF16, "one-pass modes only");
    static_assert(!kTraffic || kMode == kModeStrided, "the traffic model writes packed planes");
    constexpr int kVec = (int)(sizeof(RawBlock<Tin>) / sizeof(uint4));   // 16-byte loads per block
    __shared__ float2 tbl[128];                                            // {d, 1/d} by scale code
    __shared__ uint4 m_lds[kQBatch][kQWaves];                              // plane-M word and plane-T entry, [row-tile of the batch][K-tile]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kg = (int)blockIdx.x % n_kg;                 // the grid is a multiple of n_kg: the K group never changes
    const int rt_first = (int)blockIdx.x / n_kg, rt_step = (int)gridDim.x / n_kg;
    const uint32_t kt = (uint32_t)(kg * kQWaves + wave);
    const uint32_t kb = kt * kTileBlocks + (lane & 7);
    const bool kvalid = kb < (uint32_t)p.nb;               // (a whole wave may lie beyond K: it idles but keeps the barriers)
    const int rloc = lane >> 3;
    const float S = p.S, inv_S = 1.0f / S, S6 = 6.0f * S, r_S6 = 1.0f / S6;
    if (tid < 128) {
        const float d = e4m3_decode_int((uint32_t)tid) * S;
        tbl[tid] = make_float2(d, tid != 0 ? 1.0f / d : 0.0f);
    }
    const __amdgpu_buffer_rsrc_t obuf =
        __builtin_amdgcn_make_buffer_rsrc(p.out.hdr, 0, (int)out_bytes, 0x00020000);
    const uint32_t off_L = (uint32_t)p.layout.off_L, off_S = (uint32_t)p.layout.off_S, off_M = (uint32_t)p.layout.off_M,
                   off_T = (uint32_t)p.layout.off_T, off_H = (uint32_t)p.layout.off_H;
    if (blockIdx.x == 0) {
        if (tid == 0 && p.out.hdr != nullptr) write_header(p.out.hdr, p.layout, S, 0u);
        for (int i = tid; i < p.zero_n; i += 64 * kQWaves) p.zero[i] = 0u;
    }
    float f[16];
    if (kvalid) load16(p.fisher + kb * kBlock, f);
    else {
#pragma unroll
        for (int i = 0; i < 16; ++i) f[i] = 0.0f;
    }
    __syncthreads();
    if (rt_first >= (int)p.n_rt) return;
    const int n_it = ((int)p.n_rt - rt_first + rt_step - 1) / rt_step;
    // Plane H: the FP8 upper halves of all the tiles a wave visits go, in visiting order, into one region
    // of the plane that belongs to the wave (64 entries per tile it owns: the worst case), so that the few
    // entries of a tile continue where the previous tile's stopped instead of starting a 512-byte
    // region of their own (those partial-line writes cost 7% of the run time at 10% FP8).  The regions
    // of the waves with the same K-tile follow each other in the order of their first row-tile.
    uint32_t h_cnt;
    {
        const uint32_t q = (uint32_t)p.n_rt / (uint32_t)rt_step, r = (uint32_t)p.n_rt % (uint32_t)rt_step, y = (uint32_t)rt_first;
        h_cnt = (kt * (uint32_t)p.n_rt + y * q + (y < r ? y : r)) * kTileSlots;
    }

    // input: per-lane byte offset of the lane's block in the workgroup's first row-tile, advanced by rt_step
    // row-tiles per iteration; rows beyond the tensor fall outside the buffer and read zeros; lanes
    // beyond K stay parked outside it
    const __amdgpu_buffer_rsrc_t xbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.X), 0, (int)x_bytes, 0x00020000);
    const uint32_t row_bytes = (uint32_t)p.ldx * (uint32_t)sizeof(Tin);
    uint32_t xoff = kvalid ? (uint32_t)(rt_first * kTileRows + rloc) * row_bytes + kb * (uint32_t)(kBlock * sizeof(Tin)) : 0xFFFFFF00u;
    const uint32_t xstep = kvalid ? (uint32_t)rt_step * kTileRows * row_bytes : 0u;
    auto load_block = [&](RawBlock<Tin> &r) {

        // (a load past the last row-tile lies beyond the buffer -- zeros -- or is unused; offsets stay below 2^32
        // for the tensors this kernel accepts plus one step, which the host checks)
#pragma unroll
        for (int i = 0; i < kVec; ++i) {
            const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(xbuf, (int)xoff + 16 * i, 0, 0);
            r.v[i] = make_uint4(v[0], v[1], v[2], v[3]);
        }
        xoff += xstep;
    };

    auto process = [&](int it, const RawBlock<Tin> &raw_in) {
        const int rt = rt_first + it * rt_step;
        if constexpr (kTraffic) {
            uint32_t w[4] = {raw_in.v[0].x ^ raw_in.v[1].z, raw_in.v[0].y ^ raw_in.v[1].w, raw_in.v[0].z ^ raw_in.v[1].x, raw_in.v[0].w ^ raw_in.v[1].y};
            if constexpr (kVec == 4) {
                w[0] ^= raw_in.v[2].x ^ raw_in.v[3].z; w[1] ^= raw_in.v[2].y ^ raw_in.v[3].w;
                w[2] ^= raw_in.v[2].z ^ raw_in.v[3].x; w[3] ^= raw_in.v[2].w ^ raw_in.v[3].y;
            }
            const uint32_t row = (uint32_t)(rt * kTileRows + rloc);
            const bool valid = kvalid && row < (uint32_t)p.rows;
            const uint32_t tile = (uint32_t)rt * (uint32_t)p.n_kt + kt, slot = tile * kTileSlots + lane;
            const bool hi = valid && ((slot * 2654435761u) >> 24) < 26u;
            const uint64_t ballot = __ballot(hi);
            const uint32_t prefix = __builtin_amdgcn_mbcnt_hi((uint32_t)(ballot >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)ballot, 0u));
            if (lane == 0) m_lds[it % kQBatch][wave] = make_uint4((uint32_t)ballot, (uint32_t)(ballot >> 32), h_cnt, 0u);
            if (hi) __builtin_amdgcn_raw_buffer_store_b64(u32x2_t{w[2], w[3]}, obuf, (int)(off_H + (h_cnt + prefix) * 8u), 0, 0);
            if (kt < (uint32_t)p.n_kt) {
                __builtin_amdgcn_raw_buffer_store_b64(u32x2_t{w[0], w[1]}, obuf, (int)(off_L + slot * 8u), 0, 0);
                __builtin_amdgcn_raw_buffer_store_b8((uint8_t)(hi ? prefix : (w[2] & 0x7Fu)), obuf, (int)(off_S + slot), 0, 0);
            }
            h_cnt += (uint32_t)__popcll(ballot);
            return;
        }
        float x[16];
        widen(raw_in, x);
        const float amax = block_amax(x);
        // block scale: correctly rounded amax / (6 S)
        float u = amax * r_S6;
        // (outside [1e-30, 1e30) -- where a residual could lose bits or the product overflow -- the wave
        // divides; zero is exact either way)
        const bool odd_range = (amax < 1e-30f && amax != 0.0f) || !(u < 1e30f);
        if (__builtin_expect(__ballot(odd_range) != 0ull, 0)) u = amax / S6;
        else u = __builtin_fmaf(__builtin_fmaf(-u, S6, amax), r_S6, u);
        const uint32_t sc = e4m3_encode_pair_hw(u, 0.0f) & 0xFFu;
        const float2 dd = tbl[sc];
        const float d = dd.x, inv_d = dd.y;
        // (Eq. 8: the FP8 codes of every block; values beyond the FP8 range only occur when the caller's S is
        // below amax / 448, then the wave clamps before converting -- clamping changes no value in range)
        uint32_t c8[4] = {0u, 0u, 0u, 0u};
        if constexpr (kDelta) {
            float r8[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) r8[i] = x[i] * inv_S;
            if (__ballot(amax * inv_S > 448.0f) != 0ull) encode_fp8_block<true, true>(r8, c8);
            else encode_fp8_block<true, false>(r8, c8);
        }
        uint32_t q[2] = {0u, 0u};
        float t[16];
#define FGMP_ENC(W, B, I) q[W] = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(q[W], x[I] * inv_d, x[I + 1] * inv_d, 1.0f, B)
        FGMP_ENC(0, 0, 0); FGMP_ENC(0, 1, 2); FGMP_ENC(0, 2, 4); FGMP_ENC(0, 3, 6);
        FGMP_ENC(1, 0, 8); FGMP_ENC(1, 1, 10); FGMP_ENC(1, 2, 12); FGMP_ENC(1, 3, 14);
#undef FGMP_ENC
#define FGMP_ERR(W, B, I)                                                                \
    {                                                                                    \
        const float2_t v = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(q[W], 1.0f, B);      \
        float e0, e1;                                                                    \
        if constexpr (kDelta) {                                                          \
            const float2_t v8 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(c8[(I) / 4], 1.0f, ((I) % 4) >= 2); \
            e0 = v[0] * d - v8[0] * S;                                                   \
            e1 = v[1] * d - v8[1] * S;                                                   \
        } else {                                                                         \
            e0 = x[I] - v[0] * d;                                                        \
            e1 = x[I + 1] - v[1] * d;                                                    \
        }                                                                                \
        t[I] = (e0 * e0) * f[I];                                                         \
        t[I + 1] = (e1 * e1) * f[I + 1];                                                 \
    }
        FGMP_ERR(0, 0, 0) FGMP_ERR(0, 1, 2) FGMP_ERR(0, 2, 4) FGMP_ERR(0, 3, 6)
        FGMP_ERR(1, 0, 8) FGMP_ERR(1, 1, 10) FGMP_ERR(1, 2, 12) FGMP_ERR(1, 3, 14)
#undef FGMP_ERR
#pragma unroll
        for (int w = 16; w > 1; w >>= 1)
#pragma unroll
            for (int i = 0; i < w / 2; ++i) t[i] = t[2 * i] + t[2 * i + 1];
        const float score = t[0];
        // (lanes outside the tensor hold zeros: score 0; a negative or -inf threshold must not select them)
        const uint32_t row = (uint32_t)(rt * kTileRows + rloc);
        const bool valid = kvalid && row < (uint32_t)p.rows;
        const bool hi = valid && (score > p.T);
        const uint64_t ballot = __ballot(hi);
        const uint32_t tile = (uint32_t)rt * (uint32_t)p.n_kt + kt;
        if (p.scores != nullptr && valid) p.scores[(int64_t)row * p.nb + kb] = score;

        if constexpr (kMode == kModeF16) {
            half2_t o[8];
            if (hi) {
                uint32_t c[4];
                if constexpr (kDelta) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) c[j] = c8[j];
                } else {
                    float r[16];
#pragma unroll
                    for (int i = 0; i < 16; ++i) r[i] = x[i] * inv_S;
                    if (amax * inv_S > 448.0f) encode_fp8_block<true, true>(r, c);
                    else encode_fp8_block<true, false>(r, c);
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    o[2 * j] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(c[j], 1.0f, false);
                    o[2 * j + 1] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(c[j], 1.0f, true);
                }
            } else {
                const half2_t s = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(sc | (sc << 8), 1.0f, false);
                o[0] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(q[0], 1.0f, 0) * s;
                o[1] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(q[0], 1.0f, 1) * s;
                o[2] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(q[0], 1.0f, 2) * s;
                o[3] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(q[0], 1.0f, 3) * s;
                o[4] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(q[1], 1.0f, 0) * s;
                o[5] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(q[1], 1.0f, 1) * s;
                o[6] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(q[1], 1.0f, 2) * s;
                o[7] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(q[1], 1.0f, 3) * s;
            }
            union { half2_t h[8]; uint4 v[2]; } pack;
#pragma unroll
            for (int j = 0; j < 8; ++j) pack.h[j] = o[j];
            // every slot of the tile is written (zeros where the tensor ends), so the GEMM can read whole tiles
            if (kt < (uint32_t)p.n_kt) {
                uint4 *dst = reinterpret_cast<uint4 *>(p.x16 + (int64_t)row * p.ld16 + (int64_t)kb * kBlock);
                dst[0] = pack.v[0];
                dst[1] = pack.v[1];
            }
        } else {
            const uint32_t prefix = __builtin_amdgcn_mbcnt_hi((uint32_t)(ballot >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)ballot, 0u));
            const uint32_t slot = tile * kTileSlots + lane;
            if (lane == 0) m_lds[it % kQBatch][wave] = make_uint4((uint32_t)ballot, (uint32_t)(ballot >> 32), h_cnt, 0u);
            uint32_t lw0 = q[0], lw1 = q[1], sbyte = sc;
            if (ballot != 0ull) {
                // values beyond the FP8 range only occur when the caller's S is below amax / 448
                const bool any_big = __ballot(hi && amax * inv_S > 448.0f) != 0ull;
                if (hi) {
                    uint32_t c[4];
                    if constexpr (kDelta) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) c[j] = c8[j];
                    } else {
                        float r[16];
#pragma unroll
                        for (int i = 0; i < 16; ++i) r[i] = x[i] * inv_S;
                        if (any_big) encode_fp8_block<true, true>(r, c);
                        else encode_fp8_block<true, false>(r, c);
                    }
                    lw0 = c[0];
                    lw1 = c[1];
                    sbyte = prefix;
                    __builtin_amdgcn_raw_buffer_store_b64(u32x2_t{c[2], c[3]}, obuf, (int)(off_H + (h_cnt + prefix) * 8u), 0, 0);
                }
            }
            if (kt < (uint32_t)p.n_kt) {
                __builtin_amdgcn_raw_buffer_store_b64(u32x2_t{lw0, lw1}, obuf, (int)(off_L + slot * 8u), 0, 0);
                __builtin_amdgcn_raw_buffer_store_b8((uint8_t)sbyte, obuf, (int)(off_S + slot), 0, 0);
            }
            h_cnt += (uint32_t)__popcll(ballot);
        }
    };
    // the gathered plane-M and plane-T words of the last `n` iterations (a batch): 64 and 32 contiguous bytes per row-tile
    auto write_masks = [&](int it_first, int n) {
        if constexpr (kMode == kModeStrided) {
            __syncthreads();
            const int i = tid / kQWaves, w = tid % kQWaves;
            const uint32_t kt_w = (uint32_t)(kg * kQWaves + w);
            if (i < n && kt_w < (uint32_t)p.n_kt) {
                const uint4 m = m_lds[(it_first + i) % kQBatch][w];
                const uint32_t tile = (uint32_t)(rt_first + (it_first + i) * rt_step) * (uint32_t)p.n_kt + kt_w;
                __builtin_amdgcn_raw_buffer_store_b64(u32x2_t{m.x, m.y}, obuf, (int)(off_M + tile * 8u), 0, 0);
                __builtin_amdgcn_raw_buffer_store_b32(m.z, obuf, (int)(off_T + tile * 4u), 0, 0);
            }
            __syncthreads();
        }
    };

    // two row-tiles per turn, each one's input in flight while the other is processed (two register sets
    // that swap roles: no copies)
    RawBlock<Tin> a, b;
    load_block(a);
    int it = 0;
    for (; it + 2 <= n_it; it += 2) {
        load_block(b);
        process(it, a);
        load_block(a);
        process(it + 1, b);
        if ((it + 2) % kQBatch == 0) write_masks(it + 2 - kQBatch, kQBatch);
    }
    if (it < n_it) {
        process(it, a);
        ++it;
    }
    if (it % kQBatch != 0) write_masks(it - it % kQBatch, it % kQBatch);
}

// Sensitivity-weighted clipping (Sec. 3.3, Eq. 11): for every block, the E4M3 scale code (0 .. 0x7E)
// whose NVFP4 quantization has the smallest weighted error -- brute force, candidates in ascending
// order, a later candidate wins only with a strictly smaller error.  One block per lane; the error of
// a candidate is computed exactly as quantize_kernel computes a block's score.  Offline (weights).
template <typename Tin, bool kPerElem, bool kHW>
__global__ __launch_bounds__(256) void clip_scales_kernel(QuantParams p, uint8_t *sc_out)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int64_t kt = blockIdx.x;
    const int64_t kb = kt * kTileBlocks + (lane & 7);
    const int64_t rt = (int64_t)blockIdx.y * 4 + wave;
    const int64_t row = rt * kTileRows + (lane >> 3);
    if (rt >= p.n_rt || kb >= p.nb || row >= p.rows) return;
    const Tin *X = static_cast<const Tin *>(p.X);
    RawBlock<Tin> raw;
    load_raw(X + row * p.ldx + kb * kBlock, raw);
    float x[16], f[16];
    widen(raw, x);
    load16(p.fisher + (kPerElem ? row * p.ld_fisher : 0) + kb * kBlock, f);

    const float amax = block_amax(x);
    const float inv_S = 1.0f / p.S, S6 = 6.0f * p.S;
    auto error_with = [&](uint32_t sc) {
        BlockCodes bc;
        quantize_block_math<kHW, false>(x, f, amax, p.S, inv_S, S6, (int)sc, false, bc);
        return bc.score;
    };
    uint32_t best = 0u;
    float best_err = error_with(0u);
#pragma unroll 1
    for (uint32_t sc = 1u; sc <= 0x7Eu; ++sc) {
        const float err = error_with(sc);
        if (err < best_err) {
            best_err = err;
            best = sc;
        }
    }
    sc_out[row * p.nb + kb] = (uint8_t)best;
}

// Exclusive prefix sum over the per-tile FP8 counts in plane T (one workgroup),
// then the header fields that depend on the total.
__global__ __launch_bounds__(1024) void scan_tiles_kernel(uint32_t *T, int64_t n_tiles, PackedHeader *hdr,
                                                           uint64_t off_H)
{
    __shared__ uint64_t part[1024];
    const int tid = threadIdx.x;
    const int64_t chunk = (n_tiles + 1023) / 1024;
    const int64_t lo = tid * chunk, hi = (lo + chunk < n_tiles) ? lo + chunk : n_tiles;
    uint64_t sum = 0;
    for (int64_t i = lo; i < hi; ++i) sum += T[i];
    part[tid] = sum;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {   // inclusive Hillis-Steele scan
        uint64_t v = (tid >= off) ? part[tid - off] : 0;
        __syncthreads();
        part[tid] += v;
        __syncthreads();
    }
    uint64_t run = part[tid] - sum;
    for (int64_t i = lo; i < hi; ++i) {
        uint32_t c = T[i];
        T[i] = (uint32_t)run;
        run += c;
    }
    if (tid == 1023) {
        hdr->h_entries = part[1023];
        // at least one entry stays readable: kernels that load plane H unconditionally read entry 0
        hdr->bytes_used = off_H + (part[1023] > 0 ? part[1023] : 1) * 8;
    }
}

// One wave per tile, one slot per lane: packed -> canonical arrays.
__global__ __launch_bounds__(256) void unpack_kernel(PackedView v, PackedLayout l, uint8_t *codes,
                                                      uint8_t *scales, uint8_t *mask)
{
    const int lane = threadIdx.x & 63;
    const int64_t tile = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (tile >= l.n_tiles) return;
    const int64_t rt = tile / l.n_kt, kt = tile % l.n_kt;
    const int64_t row = rt * kTileRows + (lane >> 3);
    const int64_t kb = kt * kTileBlocks + (lane & 7);
    if (row >= l.rows || kb >= l.nb) return;
    const bool hi = (v.M[tile] >> lane) & 1ull;
    const uint2 lw = v.L[tile * kTileSlots + lane];
    const uint32_t sb = v.S[tile * kTileSlots + lane];
    uint4 out;
    if (hi) {
        const uint2 hw = v.H[(uint64_t)v.T[tile] + sb];
        out = make_uint4(lw.x, lw.y, hw.x, hw.y);
    } else {
        // spread 16 nibbles to 16 bytes
        uint32_t w[4];
        const uint32_t src[2] = {lw.x, lw.y};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t h = (src[j >> 1] >> (16 * (j & 1))) & 0xFFFFu;  // 4 nibbles
            w[j] = (h & 0xFu) | ((h & 0xF0u) << 4) | ((h & 0xF00u) << 8) | ((h & 0xF000u) << 12);
        }
        out = make_uint4(w[0], w[1], w[2], w[3]);
    }
    if (codes) *reinterpret_cast<uint4 *>(codes + row * l.K + kb * kBlock) = out;
    if (scales) scales[row * l.nb + kb] = hi ? 0 : (uint8_t)sb;
    if (mask) mask[row * l.nb + kb] = hi ? 1 : 0;
}

// ---- host side ----

static int pick_rt_per_wave(int64_t n_rt)
{

    // enough work per wave to amortize the sensitivity loads, enough workgroups to fill 256 CUs
    if (n_rt >= 4096) return 4;
    if (n_rt >= 1024) return 2;
    return 1;
}

template <typename Tin, int kMode>
static void launch_quantize_mode(const QuantParams &p, bool per_elem, dim3 grid, hipStream_t st)
{
    if (p.delta) {
        if (per_elem)
            hipLaunchKernelGGL((quantize_kernel<Tin, true, kUseHwCvt, kMode, true>), grid, dim3(256), 0, st, p);
        else
            hipLaunchKernelGGL((quantize_kernel<Tin, false, kUseHwCvt, kMode, true>), grid, dim3(256), 0, st, p);
    } else {
        if (per_elem)
            hipLaunchKernelGGL((quantize_kernel<Tin, true, kUseHwCvt, kMode, false>), grid, dim3(256), 0, st, p);
        else
            hipLaunchKernelGGL((quantize_kernel<Tin, false, kUseHwCvt, kMode, false>), grid, dim3(256), 0, st, p);
    }
}

template <typename Tin>
static void launch_quantize(const QuantParams &p, bool per_elem, dim3 grid, hipStream_t st)
{
    switch (p.mode) {
    case kModeStrided: launch_quantize_mode<Tin, kModeStrided>(p, per_elem, grid, st); break;
    case kModeCount: launch_quantize_mode<Tin, kModeCount>(p, per_elem, grid, st); break;
    case kModeF16: launch_quantize_mode<Tin, kModeF16>(p, per_elem, grid, st); break;
    default: launch_quantize_mode<Tin, kModeCompact>(p, per_elem, grid, st); break;
    }
}

#ifdef FGMP_MEASUREMENT_HOOKS
// (measurement builds: the next activation tensor that takes the trimmed kernel runs its traffic model instead)
static thread_local bool g_traffic_model = false;
fgmp_status_t quantize_traffic_model(const void *X, fgmp_dtype_t dt, int64_t rows, int64_t K, int64_t ldx, const float *fisher,
                                     void *packed, size_t packed_bytes, hipStream_t st)
{
    if (make_layout(rows, K).n_tiles < kQMinTiles) return FGMP_ERR_UNSUPPORTED;
    g_traffic_model = true;
    const fgmp_status_t rc = quantize_tensor(X, dt, rows, K, ldx, fisher, 0, 0.0f, 1.0f, packed, packed_bytes, nullptr, false, st);
    const bool ran = !g_traffic_model;
    g_traffic_model = false;
    return rc != FGMP_OK ? rc : ran ? FGMP_OK : FGMP_ERR_UNSUPPORTED;
}
#endif

fgmp_status_t quantize_tensor(const void *X, fgmp_dtype_t dt, int64_t rows, int64_t K, int64_t ldx,
                              const float *fisher, int64_t ld_fisher, float T, float S, void *packed,
                              size_t packed_bytes, float *scores, bool compact, hipStream_t st,
                              _Float16 *x16, int64_t ld16, uint32_t *zero, int64_t zero_n, int score_mode,
                              uint8_t *clip_scales)
{
    if (score_mode != FGMP_SCORE_NVFP4_ERROR && score_mode != FGMP_SCORE_DELTA) return FGMP_ERR_INVALID_ARG;
    if (!X || !fisher || (!packed && !x16)) return FGMP_ERR_INVALID_ARG;
    if (rows <= 0 || K <= 0) return FGMP_ERR_INVALID_ARG;
    if (!(S > 0.0f) || !(S < INFINITY) || T != T) return FGMP_ERR_INVALID_ARG;
    if (dt != FGMP_F32 && dt != FGMP_BF16) return FGMP_ERR_UNSUPPORTED;
    if (K % kBlock != 0 || ldx < K || (ld_fisher != 0 && ld_fisher < K)) return FGMP_ERR_BAD_SHAPE;
    if (rows * (K / kBlock) >= (int64_t)1 << 32) return FGMP_ERR_UNSUPPORTED;
    const int64_t esz = (dt == FGMP_F32) ? 4 : 2;
    if (((uintptr_t)X | (uintptr_t)fisher | (uintptr_t)packed | (uintptr_t)scores) % 16 != 0 ||
        (ldx * esz) % 16 != 0 || (ld_fisher * 4) % 16 != 0)
        return FGMP_ERR_BAD_ALIGN;
    const PackedLayout l = make_layout(rows, K);
    if (x16 != nullptr) {
        // FP16 output: the packed buffer only receives the header
        if (compact || !kUseHwCvt) return FGMP_ERR_UNSUPPORTED;
        if (packed && packed_bytes < sizeof(PackedHeader)) return FGMP_ERR_BUFFER_TOO_SMALL;
        if (ld16 < l.n_kt * kTileK || (uintptr_t)x16 % 16 != 0 || (ld16 * 2) % 16 != 0) return FGMP_ERR_BAD_SHAPE;
    } else if (packed_bytes < l.total_bytes) {
        return FGMP_ERR_BUFFER_TOO_SMALL;
    }

    QuantParams p;
    p.X = X; p.ldx = ldx; p.rows = rows; p.nb = l.nb;
    p.fisher = fisher; p.ld_fisher = ld_fisher;
    p.T = T; p.S = S;
    if (packed) p.out = make_view(packed, l);
    else p.out = PackedView{};
    p.n_rt = l.n_rt; p.n_kt = l.n_kt;
    p.scores = scores;
    p.rt_per_wave = pick_rt_per_wave(l.n_rt);
    const int64_t rt_per_wg = 4 * (int64_t)p.rt_per_wave;
    const int64_t gy = (l.n_rt + rt_per_wg - 1) / rt_per_wg;
    if (gy > 65535 || l.n_kt > 0x7FFFFFFF) return FGMP_ERR_UNSUPPORTED;
    const dim3 grid((unsigned)l.n_kt, (unsigned)gy);
    const bool per_elem = ld_fisher != 0;

    p.layout = l;
    p.compact = compact ? 1u : 0u;
    p.x16 = x16; p.ld16 = ld16;
    if (zero_n < 0 || zero_n > 0x7FFFFFFF || (zero_n > 0 && !zero)) return FGMP_ERR_INVALID_ARG;
    p.zero = zero; p.zero_n = (int)zero_n;
    p.delta = score_mode == FGMP_SCORE_DELTA;
    p.sc_override = clip_scales;
    if (clip_scales != nullptr) {
        // clipping is defined with the NVFP4-error score; the scale search runs first, on the same stream
        if (p.delta || x16 != nullptr) return FGMP_ERR_UNSUPPORTED;
        const int64_t gy4 = (l.n_rt + 3) / 4;
        if (gy4 > 65535) return FGMP_ERR_UNSUPPORTED;
        const dim3 cgrid((unsigned)l.n_kt, (unsigned)gy4);
        if (dt == FGMP_F32) {
            if (per_elem) hipLaunchKernelGGL((clip_scales_kernel<float, true, kUseHwCvt>), cgrid, dim3(256), 0, st, p, clip_scales);
            else hipLaunchKernelGGL((clip_scales_kernel<float, false, kUseHwCvt>), cgrid, dim3(256), 0, st, p, clip_scales);
        } else {
            if (per_elem) hipLaunchKernelGGL((clip_scales_kernel<uint16_t, true, kUseHwCvt>), cgrid, dim3(256), 0, st, p, clip_scales);
            else hipLaunchKernelGGL((clip_scales_kernel<uint16_t, false, kUseHwCvt>), cgrid, dim3(256), 0, st, p, clip_scales);
        }
    }
    // The activation hot path (one pass, NVFP4-error score, one sensitivity per channel, dynamic-max
    // scales) runs on the trimmed kernel when its 32-bit offsets and its shortcut division apply.
    const uint64_t x_bytes = (uint64_t)rows * (uint64_t)ldx * (uint64_t)esz;
    // (offsets: the input plus one stride of the resident set past its end must stay below 2^32)
    const bool fast = kUseHwCvt && !compact && !per_elem && clip_scales == nullptr &&
                      x_bytes < 0x7FFFFF00ull && l.total_bytes < 0xFFFFFF00ull && S >= 1e-30f && S <= 1e30f &&
                      l.n_tiles >= kQMinTiles;
    if (fast) {
        p.mode = x16 != nullptr ? kModeF16 : kModeStrided;
        // one resident set of workgroups, a multiple of the number of K groups, with the row-tiles dealt out
        // evenly: two workgroups of eight waves per compute unit.  (The kernel's 85-93 registers let five waves
        // share a SIMD, i.e. two such workgroups a compute unit: a grid of three per compute unit ran its last
        // third as a second round, 72.9 us on 16384 x 8192 against 69.3; one per compute unit 81.6; three that
        // do fit -- the sensitivities moved to LDS, 74 registers -- 74.3: more waves only crowd the memory system.)
        constexpr int64_t kQResident = 512;
        const int64_t n_kg = (l.n_kt + kQWaves - 1) / kQWaves;
        int64_t gy = std::max<int64_t>(1, kQResident / n_kg);
        if (gy > l.n_rt) gy = l.n_rt;
        const int64_t its = (l.n_rt + gy - 1) / gy;
        gy = (l.n_rt + its - 1) / its;
        const dim3 fgrid((unsigned)(n_kg * gy));
        const uint32_t out_bytes = packed ? (uint32_t)(x16 != nullptr ? sizeof(PackedHeader) : l.total_bytes) : 0u;
        if (p.delta) {
            // the Eq. 8 score
            if (x16 != nullptr) {
                if (dt == FGMP_F32) hipLaunchKernelGGL((quantize_act_kernel<float, kModeF16, false, true>), fgrid, dim3(64 * kQWaves), 0, st, p, (uint32_t)x_bytes, out_bytes, (int)n_kg);
                else hipLaunchKernelGGL((quantize_act_kernel<uint16_t, kModeF16, false, true>), fgrid, dim3(64 * kQWaves), 0, st, p, (uint32_t)x_bytes, out_bytes, (int)n_kg);
            } else {
                if (dt == FGMP_F32) hipLaunchKernelGGL((quantize_act_kernel<float, kModeStrided, false, true>), fgrid, dim3(64 * kQWaves), 0, st, p, (uint32_t)x_bytes, out_bytes, (int)n_kg);
                else hipLaunchKernelGGL((quantize_act_kernel<uint16_t, kModeStrided, false, true>), fgrid, dim3(64 * kQWaves), 0, st, p, (uint32_t)x_bytes, out_bytes, (int)n_kg);
            }
        } else if (x16 != nullptr) {
            if (dt == FGMP_F32) hipLaunchKernelGGL((quantize_act_kernel<float, kModeF16>), fgrid, dim3(64 * kQWaves), 0, st, p, (uint32_t)x_bytes, out_bytes, (int)n_kg);
            else hipLaunchKernelGGL((quantize_act_kernel<uint16_t, kModeF16>), fgrid, dim3(64 * kQWaves), 0, st, p, (uint32_t)x_bytes, out_bytes, (int)n_kg);
#ifdef FGMP_MEASUREMENT_HOOKS
        } else if (g_traffic_model) {
            g_traffic_model = false;
            if (dt == FGMP_F32) hipLaunchKernelGGL((quantize_act_kernel<float, kModeStrided, true>), fgrid, dim3(64 * kQWaves), 0, st, p, (uint32_t)x_bytes, out_bytes, (int)n_kg);
            else hipLaunchKernelGGL((quantize_act_kernel<uint16_t, kModeStrided, true>), fgrid, dim3(64 * kQWaves), 0, st, p, (uint32_t)x_bytes, out_bytes, (int)n_kg);
#endif
        } else {
            if (dt == FGMP_F32) hipLaunchKernelGGL((quantize_act_kernel<float, kModeStrided>), fgrid, dim3(64 * kQWaves), 0, st, p, (uint32_t)x_bytes, out_bytes, (int)n_kg);
            else hipLaunchKernelGGL((quantize_act_kernel<uint16_t, kModeStrided>), fgrid, dim3(64 * kQWaves), 0, st, p, (uint32_t)x_bytes, out_bytes, (int)n_kg);
        }
    } else if (x16 != nullptr) {
        p.mode = kModeF16;
        if (dt == FGMP_F32) launch_quantize<float>(p, per_elem, grid, st);
        else launch_quantize<uint16_t>(p, per_elem, grid, st);
    } else if (!compact) {
        p.mode = kModeStrided;
        if (dt == FGMP_F32) launch_quantize<float>(p, per_elem, grid, st);
        else launch_quantize<uint16_t>(p, per_elem, grid, st);
    } else {
        QuantParams pc = p;
        pc.mode = kModeCount;
        pc.scores = nullptr;
        if (dt == FGMP_F32) launch_quantize<float>(pc, per_elem, grid, st);
        else launch_quantize<uint16_t>(pc, per_elem, grid, st);
        hipLaunchKernelGGL(scan_tiles_kernel, dim3(1), dim3(1024), 0, st, p.out.T, l.n_tiles, p.out.hdr,
                           l.off_H);
        p.mode = kModeCompact;
        if (dt == FGMP_F32) launch_quantize<float>(p, per_elem, grid, st);
        else launch_quantize<uint16_t>(p, per_elem, grid, st);
    }
    return hipGetLastError() == hipSuccess ? FGMP_OK : FGMP_ERR_HIP;
}

fgmp_status_t unpack_tensor(const void *packed, int64_t rows, int64_t K, uint8_t *codes, uint8_t *scales,
                            uint8_t *mask, hipStream_t st)
{
    if (!packed || rows <= 0 || K <= 0) return FGMP_ERR_INVALID_ARG;
    if (K % kBlock != 0) return FGMP_ERR_BAD_SHAPE;
    if (((uintptr_t)packed | (uintptr_t)codes) % 16 != 0) return FGMP_ERR_BAD_ALIGN;
    const PackedLayout l = make_layout(rows, K);
    const PackedView v = make_view(const_cast<void *>(packed), l);
    const int64_t nwg = (l.n_tiles + 3) / 4;
    if (nwg > 0x7FFFFFFF) return FGMP_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(unpack_kernel, dim3((unsigned)nwg), dim3(256), 0, st, v, l, codes, scales, mask);
    return hipGetLastError() == hipSuccess ? FGMP_OK : FGMP_ERR_HIP;
}

// ---- conversion self-test kernels ----

template <int kFormat> __device__ __forceinline__ uint32_t selftest_encode(float r)
{
    if constexpr (kFormat == 2) return e2m1_encode_int(r);
    else if constexpr (kFormat == 3) return e4m3_encode_int(r);
    else if constexpr (kFormat == 4) return e2m1_encode_pair_hw(r, 0.0f) & 0xFu;
    else return e4m3_encode_pair_hw(r, 0.0f) & 0xFFu;
}

constexpr uint32_t kLastPattern = 0x7F800000u;   // +INF
constexpr uint32_t kRunLength = 4096;

template <int kFormat>
__global__ __launch_bounds__(256) void encode_ranges_kernel(uint32_t *min_bits, uint32_t *max_bits,
                                                             uint32_t *violations)
{
    const uint64_t first = ((uint64_t)blockIdx.x * 256 + threadIdx.x) * kRunLength;
    if (first > kLastPattern) return;
    uint64_t last = first + kRunLength - 1;
    if (last > kLastPattern) last = kLastPattern;
    uint32_t cur = selftest_encode<kFormat>(u2f((uint32_t)first)) & 0xFFu;
    uint32_t start = (uint32_t)first;
    for (uint64_t b = first + 1; b <= last; ++b) {
        const uint32_t c = selftest_encode<kFormat>(u2f((uint32_t)b)) & 0xFFu;
        if (c != cur) {
            atomicMin(&min_bits[cur], start);
            atomicMax(&max_bits[cur], (uint32_t)(b - 1));
            if (c < cur) atomicAdd(violations, 1u);
            cur = c;
            start = (uint32_t)b;
        }
    }
    atomicMin(&min_bits[cur], start);
    atomicMax(&max_bits[cur], (uint32_t)last);
}

__global__ void init_ranges_kernel(uint32_t *min_bits, uint32_t *max_bits, uint32_t *violations)
{
    min_bits[threadIdx.x] = 0xFFFFFFFFu;
    max_bits[threadIdx.x] = 0u;
    if (threadIdx.x == 0) *violations = 0u;
}

__global__ void decode_table_kernel(int format, float *out)
{
    const uint32_t c = threadIdx.x;
    float v;
    switch (format) {
    case 2: v = e2m1_decode_int(c & 0xFu); break;
    case 3: v = e4m3_decode_int(c); break;
    case 4: v = e2m1_decode_pair_hw(c & 0xFu)[0]; break;
    default: v = e4m3_decode_pair_hw(c)[0]; break;
    }
    out[c] = v;
}

fgmp_status_t selftest_encode_ranges(int format, uint32_t *min_bits, uint32_t *max_bits,
                                     uint32_t *violations, hipStream_t st)
{
    if (!min_bits || !max_bits || !violations) return FGMP_ERR_INVALID_ARG;
    if (format < 0 || format > 5) return FGMP_ERR_INVALID_ARG;
    if (format < 2) format += kUseHwCvt ? 4 : 2;   // the form the quantizer uses
    hipLaunchKernelGGL(init_ranges_kernel, dim3(1), dim3(256), 0, st, min_bits, max_bits, violations);
    const uint64_t n_threads = ((uint64_t)kLastPattern + kRunLength) / kRunLength;
    const dim3 grid((unsigned)((n_threads + 255) / 256));
    switch (format) {
    case 2: hipLaunchKernelGGL((encode_ranges_kernel<2>), grid, dim3(256), 0, st, min_bits, max_bits, violations); break;
    case 3: hipLaunchKernelGGL((encode_ranges_kernel<3>), grid, dim3(256), 0, st, min_bits, max_bits, violations); break;
    case 4: hipLaunchKernelGGL((encode_ranges_kernel<4>), grid, dim3(256), 0, st, min_bits, max_bits, violations); break;
    default: hipLaunchKernelGGL((encode_ranges_kernel<5>), grid, dim3(256), 0, st, min_bits, max_bits, violations); break;
    }
    return hipGetLastError() == hipSuccess ? FGMP_OK : FGMP_ERR_HIP;
}

fgmp_status_t selftest_decode_table(int format, float *out, hipStream_t st)
{
    if (!out || format < 0 || format > 5) return FGMP_ERR_INVALID_ARG;
    if (format < 2) format += kUseHwCvt ? 4 : 2;
    hipLaunchKernelGGL(decode_table_kernel, dim3(1), dim3(256), 0, st, format, out);
    return hipGetLastError() == hipSuccess ? FGMP_OK : FGMP_ERR_HIP;
}

}  // namespace fgmp
