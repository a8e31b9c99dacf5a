// Decode-shape (M <= 32 tokens) step of the FGMP path in ONE launch (Sec. 4.2 followed by Sec. 4.1):
// the few activation rows are scored, quantized and turned into FP16 operand values inside the kernel
// that streams the packed weights from HBM exactly once, decodes them in registers straight into MFMA
// operands and accumulates in FP32.
//
// One workgroup of twelve waves per compute unit (the grid is one resident set).  A workgroup owns a
// contiguous share of the 16-row groups of W and one of P_g parts of K.  Its waves split the work as
// (row group, part of K): a wave streams the K-tiles of its part for one row group after the other
// ("runs"), and the waves that share a row group add their accumulators through LDS at the end of a run
// -- no partial sums go through memory unless K is also split across workgroups (P_g > 1), where the
// last workgroup to arrive at a row group's counter adds the parts in K order and puts the counter back
// to zero.
//
// The activations: every workgroup needs X^ (FP16 values of the stored codes) for its part of K in LDS
// and makes them itself -- no workgroup waits for another.  A thread owns one K-block of the part and up
// to three rows of it (P_g is chosen so that this covers all M rows): it requests them and the block's
// sensitivities BEFORE anything else -- a wave's loads complete in the order they were issued, and
// activation data behind the weight tiles would only count as arrived after all of those -- then the
// first weight tiles, quantizes while those are on their way (score, decision, codes; Sec. 4.2) and
// writes the FP16 values to LDS.  (From packed activations: decoded by all threads before the stream.)
//
// A wave's loads per K-tile (16 weight rows x 128 K), four instructions: the tile's mask word (the same
// for half of the wave), 16 bytes of plane L per lane (1 KB per wave), the lane's two scale bytes, and --
// once the mask has landed -- 16 bytes of plane H from the lane's first FP8 block on (two neighbouring
// entries if both of its blocks are FP8; lanes without one read entry 0).  A block's entry is the tile's
// first entry plus the number of FP8 slots before the block's; the tile's first entry is its plane-T word,
// which in a compact tensor is the previous tile's plus that tile's number of FP8 slots: only the first
// tile of a run loads it (every tile of a tensor that is not compact).  Fewer, wider requests matter: a
// plain read of these bytes with one 16-byte load per lane runs at about 5 TB/s on this chip, the same
// bytes fetched with six requests per tile (mask, plane T, L, S, two plane-H entries) at 3.4 TB/s.
// The prologue asks for the masks of the first four tiles before their planes L / S, so their plane-H
// requests go out while the bulk is still on its way instead of one memory round trip after it.
// A ring of four register sets holds four tiles in flight per wave (48 KB per compute unit -- more only
// blocks the waves that issue them: a compute unit accepts about that much), across the boundaries between
// runs, indexed statically (the loop body is instantiated per ring slot); a tile is decoded and multiplied
// as soon as it has landed.  Tile addresses are a per-lane offset that never changes plus a scalar.
// Nothing in the kernel divides: every divisor is fixed per launch and comes with its multiplier, and the
// arguments' cache lines are requested together at the start.
#include <algorithm>
#include <cstddef>
#include <cstdlib>

#include "fgmp_gemm_common.hpp"
#include "fgmp_quant_block.hpp"

namespace fgmp {

typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

constexpr int kStMaxWaves = 16;              // most waves a workgroup can have (the kernels take the count as a parameter; 12 -- three
                                             // per SIMD, up to 170 vector registers each -- is what the host chooses)
constexpr int kStRing = 4;                   // K-tiles in flight per wave (a compute unit keeps about 32 KB of requests in flight: more only block the waves that issue them)
constexpr int kStEarly = 4;                  // K-tiles whose planes L / S are requested before the activations are dealt with (<= kStRing)
constexpr int kStHLead = 2;                  // plane-H entries are requested this many tiles ahead (steady state)
constexpr int kStXRows = 3;                  // activation rows per thread, at most
constexpr int kStXPad = 8;                   // halves of padding per LDS activation row (16 bytes: rows fall into different banks)
constexpr int kStXCap = 66048;               // halves of LDS for the activations (129 KB)
constexpr uint32_t kStRsrc = 0x00020000;     // raw buffer, 32-bit data format
constexpr uint32_t kStOutside = 0xFFFFFF00u; // a buffer offset beyond every buffer this kernel addresses

// x / d for x < 65536 with one multiply (d < 65536): mul = ceil(2^32 / d)
struct StreamDiv {
    uint32_t d, mul;
    __device__ __forceinline__ uint32_t operator()(uint32_t x) const { return d == 1u ? x : __umulhi(x, mul); }
};
static StreamDiv stream_div(int d) { return StreamDiv{(uint32_t)d, d > 1 ? (uint32_t)(((1ull << 32) + (uint64_t)d - 1) / (uint64_t)d) : 0u}; }

struct StreamArgs {
    // activations: bf16 / fp32 input to be quantized (Sec. 4.2), or a packed tensor to be decoded
    const void *X;
    int64_t ldx;
    const float *fisher;
    float T, S;
    PackedView xv;              // packed source
    PackedLayout xl;
    // packed weights
    const void *w;
    uint32_t off_L, off_S, off_M, off_T, off_H, n_tiles, n_rt;
    int n_kt;
    int64_t w_rows, w_K;
    // result
    float *Y;
    int64_t ldy;
    int M, N, nb_x;             // nb_x: K / 16
    // ... or, quantized and packed, as the next product's activations (Sec. 4.2): a strided M x N tensor
    void *y_packed;
    uint32_t y_bytes, y_off_L, y_off_S, y_off_M, y_off_T, y_off_H;
    int y_n_kt;
    const float *fisher_y;      // N sensitivities (input channels of the next layer)
    float T_y, S_y;
    float *scores_y;            // nullable, M x N / 16
    uint32_t *dec;              // [row group] which of the M blocks it produced are FP8 (bit m), until the tile's mask word is made
    uint32_t *uctr;             // one arrival counter per 8 row groups (= one K-tile of the packed result); zero between calls
    // scratch
    uint32_t *gctr;             // one arrival counter per row group (P_g > 1); zero between calls
    uint32_t x_bytes;           // extent of the input X
    float *partial;             // [row group][part of K][MT][64 lanes] x 16 bytes (P_g > 1)
    uint32_t partial_bytes;
    // plan
    int P_g, n_slots, tiles_gpart, kp_in, tiles_in, gpr, rounds, n_groups;
    int groups_q, groups_r;     // n_groups = groups_q * n_slots + groups_r: the first groups_r slots own one row group more
    int rows_par;               // activation rows the threads cover at a time: kStThreads / (8 tiles_gpart)
    StreamDiv by_P_g, by_kp_in, by_tiles_in, by_gpr, by_pb;   // (every divisor is fixed per launch: no division in the kernel)
#ifdef FGMP_STREAM_TIMING
    unsigned long long *dbg;    // [workgroup][wave][8] time stamps
#endif
};
// (a build with FGMP_STREAM_TIMING -- none of the shipped variants -- records when each wave passes the
// kernel's phases, behind the call's scratch: the tool the phase times quoted in the design notes came from)
#ifdef FGMP_STREAM_TIMING
#define ST_STAMP(i) do { if (lane == 0) a.dbg[((size_t)wg * kStMaxWaves + wave) * 8 + (i)] = wall_clock64(); } while (0)
#else
#define ST_STAMP(i) do { } while (0)
#endif

// FP16 operand values of one activation block (m, kb): quantized from the input exactly as the
// standalone quantizer does (score, decision, codes; Sec. 4.2), or decoded from a packed tensor.
// x, f: the block and its sensitivities (zeros outside the tensor) -> FP16 values of the stored codes
__device__ __forceinline__ void stream_quantize_block(const StreamArgs &a, bool inside, const float (&x)[16], const float (&f)[16],
                                                      float inv_S, float S6, half2_t (&o)[8])
{
    const float amax = block_amax(x);
    BlockCodes bc;
    quantize_block_math<true, false>(x, f, amax, a.S, inv_S, S6, -1, false, bc);
    const bool hi = inside && bc.score > a.T;
    if (hi) {
        float r[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) r[i] = x[i] * inv_S;
        uint32_t c[4];
        if (amax * inv_S > 448.0f) encode_fp8_block<true, true>(r, c);
        else encode_fp8_block<true, false>(r, c);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            o[2 * j] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(c[j], 1.0f, false);
            o[2 * j + 1] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(c[j], 1.0f, true);
        }
    } else {
        const half2_t s = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(bc.sc | (bc.sc << 8), 1.0f, false);
        o[0] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(bc.q[0], 1.0f, 0) * s;
        o[1] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(bc.q[0], 1.0f, 1) * s;
        o[2] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(bc.q[0], 1.0f, 2) * s;
        o[3] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(bc.q[0], 1.0f, 3) * s;
        o[4] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(bc.q[1], 1.0f, 0) * s;
        o[5] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(bc.q[1], 1.0f, 1) * s;
        o[6] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(bc.q[1], 1.0f, 2) * s;
        o[7] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(bc.q[1], 1.0f, 3) * s;
    }
}

template <int kSrc>
__device__ __forceinline__ void stream_x_block(const StreamArgs &a, int m, int kb, float inv_S, float S6, half2_t (&o)[8])
{
    if constexpr (kSrc == 2) {
        const int64_t tile = (int64_t)(m >> 3) * a.xl.n_kt + (kb >> 3);
        if (kb < a.nb_x) decode_slot(a.xv, tile, (m & 7) * kTileBlocks + (kb & 7), o);
        else {
#pragma unroll
            for (int i = 0; i < 8; ++i) o[i] = half2_t{(_Float16)0.0f, (_Float16)0.0f};
        }
    } else {
        float x[16], f[16];
        if (kb < a.nb_x) {
            if constexpr (kSrc == 0) {
                const uint4 *p = reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(a.X) + (int64_t)m * a.ldx + kb * kBlock);
                const uint4 v0 = p[0], v1 = p[1];
                const uint32_t wd[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    x[2 * j] = u2f(wd[j] << 16);
                    x[2 * j + 1] = u2f(wd[j] & 0xFFFF0000u);
                }
            } else {
                load16(static_cast<const float *>(a.X) + (int64_t)m * a.ldx + kb * kBlock, x);
            }
            load16(a.fisher + kb * kBlock, f);
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) x[i] = f[i] = 0.0f;
        }
        stream_quantize_block(a, kb < a.nb_x, x, f, inv_S, S6, o);
    }
}

// One block -> 16 FP16 values (exact for every code; first element in the low nibble / byte): every lane
// takes the 4-bit route, the lanes whose block is FP8 then overwrite the result -- with both kinds in
// nearly every wave, this costs fewer instructions than two exclusive branches.  (The 4-bit route of an
// FP8 block multiplies by whatever its plane-S byte decodes to; nothing of it survives.)
// s: the block scale in both halves
__device__ __forceinline__ void st_decode_block(uint2 lw, half2_t s, bool hi, uint2 hw, half2_t (&out)[8])
{
    out[0] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lw.x, 1.0f, 0) * s;
    out[1] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lw.x, 1.0f, 1) * s;
    out[2] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lw.x, 1.0f, 2) * s;
    out[3] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lw.x, 1.0f, 3) * s;
    out[4] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lw.y, 1.0f, 0) * s;
    out[5] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lw.y, 1.0f, 1) * s;
    out[6] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lw.y, 1.0f, 2) * s;
    out[7] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lw.y, 1.0f, 3) * s;
    if (hi) {
        out[0] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(lw.x, 1.0f, false);
        out[1] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(lw.x, 1.0f, true);
        out[2] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(lw.y, 1.0f, false);
        out[3] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(lw.y, 1.0f, true);
        out[4] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(hw.x, 1.0f, false);
        out[5] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(hw.x, 1.0f, true);
        out[6] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(hw.y, 1.0f, false);
        out[7] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(hw.y, 1.0f, true);
    }
}

struct StreamSlot {
    u32x4_t l;          // plane L: blocks 2g, 2g+1 of this lane's weight row
    uint32_t s;         // plane S: their two bytes
    u32x2_t m;          // plane M: the tile's mask word
    uint32_t t;         // plane T: first plane-H entry of the tile
    u32x4_t up;         // plane H: two consecutive entries -- the second is the entry of the lane's second block where that
                        // is FP8, the first the entry of its first block where that is FP8
    uint32_t bits;      // which of the lane's two blocks are FP8 (from the mask, when the plane-H request is made)
};

// The stream's loads are assembly with hand-counted waits.  Left to the compiler, every wait in the
// loop becomes vmcnt(0): the stores, atomics and barriers that close a run sit on conditional paths
// inside the same loop, and with them in sight the compiler no longer knows how many loads are younger
// than the one it needs.  Loads (and stores) complete in issue order, so a wait only has to count what
// was issued after the load it needs; extra memory operations in between only make it stricter.  The
// destination of a load holds the data only after a later wait that names it; until then the register
// must not be read -- the ring slots are indexed statically, so none is ever copied.
// A build with FGMP_FULL_WAITS waits for every load instead: same instructions, same summation order,
// nothing to miscount -- the library a test compares this one with, bit for bit.
#ifdef FGMP_FULL_WAITS
constexpr int st_pending(int) { return 0; }
#else
constexpr int st_pending(int n) { return n; }
#endif
constexpr int kStMtLoads = 1;     // loads of st_load_m (a plane-T load that may follow it is not counted: a load the
                                  // waits do not know of only makes them stricter)
constexpr int kStLsLoads = 2;     // loads of st_load_ls
constexpr int kStHLoads = 1;      // loads of st_load_h
__device__ __forceinline__ void st_load_m(StreamSlot &s, __amdgpu_buffer_rsrc_t r, uint32_t vM, uint32_t tile)
{
    asm volatile("buffer_load_dwordx2 %0, %1, %2, %3 offen" : "=v"(s.m) : "v"(vM), "s"(r), "s"(tile * 8u));
}
__device__ __forceinline__ void st_load_t(StreamSlot &s, __amdgpu_buffer_rsrc_t r, uint32_t vT, uint32_t tile)
{
    asm volatile("buffer_load_dword %0, %1, %2, %3 offen" : "=v"(s.t) : "v"(vT), "s"(r), "s"(tile * 4u));
}
__device__ __forceinline__ void st_load_ls(StreamSlot &s, __amdgpu_buffer_rsrc_t r, uint32_t vL, uint32_t vS, uint32_t tile)
{
    // (plane L is read once and is most of the traffic: a streaming load -- it does not displace the small planes'
    // lines, which neighbouring tiles share, from the caches; 6-7% on the Llama-2 shapes.  The same hint on the
    // other planes' loads costs what it gains here.)
    asm volatile("buffer_load_dwordx4 %0, %1, %2, %3 offen nt" : "=v"(s.l) : "v"(vL), "s"(r), "s"(tile * (kTileSlots * 8u)));
    asm volatile("buffer_load_ushort %0, %1, %2, %3 offen" : "=v"(s.s) : "v"(vS), "s"(r), "s"(tile * (uint32_t)kTileSlots));
}
__device__ __forceinline__ void st_load_h(StreamSlot &s, __amdgpu_buffer_rsrc_t r, uint32_t off)
{
    asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen" : "=v"(s.up) : "v"(off), "s"(r));
}
// at most kPending loads outstanding; the named registers count as written here
template <int kPending> __device__ __forceinline__ void st_wait_mt(StreamSlot &s)
{
    asm volatile("s_waitcnt vmcnt(%2)" : "+v"(s.m), "+v"(s.t) : "n"(st_pending(kPending)));
}
template <int kPending> __device__ __forceinline__ void st_wait_all(StreamSlot &s)
{
    asm volatile("s_waitcnt vmcnt(%5)" : "+v"(s.l), "+v"(s.s), "+v"(s.m), "+v"(s.t), "+v"(s.up) : "n"(st_pending(kPending)));
}
// the first 32 bytes and bytes 72..87 of the weights' header, through the vector memory path like
// everything else (a scalar load of it would sit in front of the kernel's first instructions)
struct StreamHeader {
    u32x4_t h0, h1, h2;
};
constexpr int kStHeaderLoads = 3;
__device__ __forceinline__ void st_load_header(StreamHeader &h, __amdgpu_buffer_rsrc_t r)
{
    asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen" : "=v"(h.h0) : "v"(0u), "s"(r));
    asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen" : "=v"(h.h1) : "v"(16u), "s"(r));
    asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen" : "=v"(h.h2) : "v"(72u), "s"(r));
}
template <int kPending> __device__ __forceinline__ void st_wait_header(StreamHeader &h)
{
    asm volatile("s_waitcnt vmcnt(%3)" : "+v"(h.h0), "+v"(h.h1), "+v"(h.h2) : "n"(st_pending(kPending)));
}
// raw input of one K-block of up to three activation rows (bf16: 2 x 16 bytes each, fp32: 4) and the
// block's 16 sensitivities
template <int kSrc> struct StreamXRaw {
    static constexpr int kQuads = kSrc == 1 ? 4 : 2;
    u32x4_t f[4];
    u32x4_t x[kStXRows][kQuads];
};
template <int kSrc> constexpr int st_x_loads() { return 4 + kStXRows * StreamXRaw<kSrc>::kQuads; }
template <int kSrc> __device__ __forceinline__ void st_load_x_row(u32x4_t (&x)[StreamXRaw<kSrc>::kQuads], __amdgpu_buffer_rsrc_t xb, uint32_t xoff)
{
    asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen" : "=v"(x[0]) : "v"(xoff), "s"(xb));
    asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen offset:16" : "=v"(x[1]) : "v"(xoff), "s"(xb));
    if constexpr (kSrc == 1) {
        asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen offset:32" : "=v"(x[2]) : "v"(xoff), "s"(xb));
        asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen offset:48" : "=v"(x[3]) : "v"(xoff), "s"(xb));
    }
}
__device__ __forceinline__ void st_load_f(u32x4_t (&f)[4], __amdgpu_buffer_rsrc_t fb, uint32_t foff)
{
    asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen" : "=v"(f[0]) : "v"(foff), "s"(fb));
    asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen offset:16" : "=v"(f[1]) : "v"(foff), "s"(fb));
    asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen offset:32" : "=v"(f[2]) : "v"(foff), "s"(fb));
    asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen offset:48" : "=v"(f[3]) : "v"(foff), "s"(fb));
}
template <int kPending, int kSrc> __device__ __forceinline__ void st_wait_x(StreamXRaw<kSrc> &r)
{
    if constexpr (kSrc == 1)
        asm volatile("s_waitcnt vmcnt(%16)"
                     : "+v"(r.f[0]), "+v"(r.f[1]), "+v"(r.f[2]), "+v"(r.f[3]), "+v"(r.x[0][0]), "+v"(r.x[0][1]), "+v"(r.x[0][2]), "+v"(r.x[0][3]),
                       "+v"(r.x[1][0]), "+v"(r.x[1][1]), "+v"(r.x[1][2]), "+v"(r.x[1][3]), "+v"(r.x[2][0]), "+v"(r.x[2][1]), "+v"(r.x[2][2]), "+v"(r.x[2][3])
                     : "n"(st_pending(kPending)));
    else
        asm volatile("s_waitcnt vmcnt(%10)"
                     : "+v"(r.f[0]), "+v"(r.f[1]), "+v"(r.f[2]), "+v"(r.f[3]), "+v"(r.x[0][0]), "+v"(r.x[0][1]), "+v"(r.x[1][0]), "+v"(r.x[1][1]),
                       "+v"(r.x[2][0]), "+v"(r.x[2][1])
                     : "n"(st_pending(kPending)));
}

// Loads younger than the one a ring step needs.  Issue order: the prologue (mask / plane T of the first
// kStRing tiles, header, their planes L / S, their plane H), then per step u: plane H of tile u + kStHLead
// (from step kStRing - kStHLead on; the prologue covered the first kStRing tiles), mask / plane T of tile
// u + kStRing, planes L / S of tile u + kStRing.
constexpr int kStFirstH = kStRing - kStHLead;
constexpr int st_step_loads(int u) { return (u >= kStFirstH ? kStHLoads : 0) + kStMtLoads + kStLsLoads; }
constexpr int st_steps_loads(int from, int to)   // steps from .. to - 1
{
    int n = 0;
    for (int u = from; u < to; ++u) n += st_step_loads(u);
    return n;
}
// step t needs every load of tile t ...
constexpr int st_behind_tile(int t)
{
    if (t < kStRing) return (kStRing - 1 - t) * kStHLoads + st_steps_loads(0, t);           // its plane H came with the prologue
    return kStMtLoads + kStLsLoads + st_steps_loads(t - kStHLead + 1, t);                   // plane H at step t - kStHLead, before that step's tile loads
}
// ... and, to ask for plane H of tile t + kStHLead (t >= kStFirstH), that tile's mask / plane T, requested
// at step t + kStHLead - kStRing
constexpr int st_behind_mt(int t) { return kStLsLoads + st_steps_loads(t + kStHLead - kStRing + 1, t); }
constexpr int st_step_wait(int t)
{
    const int a = st_behind_tile(t);
    if (t < kStFirstH) return a;
    const int b = st_behind_mt(t);
    return a < b ? a : b;
}
static_assert(kStRing == 4 && kStHLead == 2, "the step lists below are written out for these");
static_assert(st_step_wait(0) == 3 && st_step_wait(1) == 5 && st_step_wait(2) == 5 && st_step_wait(3) == 6, "first pass");
static_assert(st_step_wait(4) == 6 && st_step_wait(5) == 6 && st_step_wait(6) == 6 && st_step_wait(7) == 6, "steady state");
static_assert(st_step_wait(8) == 6 && st_step_wait(9) == 6 && st_step_wait(10) == 6 && st_step_wait(11) == 6, "steady state");

// MT: 16-row groups of X (1: M <= 16, 2: M <= 32).  kXR: rows of X kept in LDS (1, 8, 16 or 32; rows of the
// MFMA operand beyond them alias rows there are -- they only feed output rows that are never stored).
// kSrc: 0 bf16 input, 1 fp32 input, 2 packed activations.
// kPack: the results leave quantized and packed instead of as FP32 (Sec. 4.2: the quantization unit sits behind
// the accumulators).  A 16-column block of one output row is exactly one row group's result, so the wave that
// holds a row group's final sums scores and encodes its M blocks itself (the quantizer's own block arithmetic) and
// writes their plane-L words, scale bytes and scores.  What a block's neighbours decide matters only for the
// tile's mask word and for the place of its FP8 upper half among the tile's plane-H entries: a tile of the
// result spans 8 row groups, which belong to different waves and workgroups.  Each row group leaves its M
// decisions (one word) and its FP8 upper halves (at the block's own slot of the tile's 64-entry region) with
// accesses that are coherent across the chip and bumps the counter of its group of 8; the wave that arrives
// last builds the mask words, moves the entries to their ranks, writes the ranks as the FP8 blocks' plane-S
// bytes and puts the counter back to zero.  Nothing waits for anything.
template <int kStWaves, int MT, int kXR, int kSrc, bool kPack = false>
__global__ __launch_bounds__(64 * kStWaves) void gemm_stream_kernel(StreamArgs a)
{
    constexpr int kStThreads = 64 * kStWaves;
    static_assert(kXR == 1 || kXR == 8 || kXR == 16 * MT, "rows of X in LDS");
    __shared__ __attribute__((aligned(16))) _Float16 xs[kStXCap];
    __shared__ float4_t red[kStWaves][MT][64];
    __shared__ uint32_t hw[4];   // what the kernel needs of the weights' header

    // The arguments span several cache lines, and the code below reads them where it needs them: one
    // scalar load per line, up front and all in flight together, instead of one memory round trip each.
    {
        typedef const uint32_t __attribute__((address_space(4))) *const_words_t;
        const_words_t ka = (const_words_t)__builtin_amdgcn_kernarg_segment_ptr();
        uint32_t touch = 0;
#pragma unroll
        for (size_t off = 0; off < sizeof(StreamArgs); off += 64) touch ^= ka[off / 4];
        asm volatile("" ::"s"(touch));
    }
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wg = (int)blockIdx.x;
    const int slot = (int)a.by_P_g((uint32_t)wg), kp_g = wg - slot * a.P_g;
    const int g_first = slot * a.groups_q + (slot < a.groups_r ? slot : a.groups_r);
    const int g_end = g_first + a.groups_q + (slot < a.groups_r ? 1 : 0);
    const int kt_part0 = kp_g * a.tiles_gpart;
    const int kt_part1 = kt_part0 + a.tiles_gpart < a.n_kt ? kt_part0 + a.tiles_gpart : a.n_kt;
    const int xrow = a.tiles_gpart * kTileK + kStXPad;      // halves per LDS row
    ST_STAMP(0);

    // ---- this wave's part of the work: K-tiles [kt_b, kt_b + nt) of the row groups
    // g_first + gsub, g_first + gsub + gpr, ... (one "run" per round of the workgroup)
    const int gsub = (int)a.by_kp_in((uint32_t)wave), kpi = wave - gsub * a.kp_in;
    const int kt_b = kt_part0 + kpi * a.tiles_in;
    const int nt = (kt_b + a.tiles_in < kt_part1 ? kt_b + a.tiles_in : kt_part1) - kt_b;   // <= 0: no tiles
    int n_runs = 0;
    if (nt > 0 && gsub < a.gpr && g_first + gsub < g_end) n_runs = (int)a.by_gpr((uint32_t)(g_end - g_first - gsub + a.gpr - 1));
    const int total = n_runs * (nt > 0 ? nt : 0);
    // waves of a row group that have tiles in this part of K (the last part may be shorter than the others)
    const int kp_eff = (int)a.by_tiles_in((uint32_t)(kt_part1 - kt_part0 + a.tiles_in - 1));

    // ---- weight addressing: lane (nl = lane % 16, g = lane / 16) owns blocks 2g, 2g+1 of weight row nl
    // of the group; rows 0-7 are the group's first row-tile, rows 8-15 its second, n_kt tiles further (the
    // tensor has an even number of row-tiles).  A tile's loads: these per-lane offsets plus a scalar.
    const int nl = lane & 15, g = lane >> 4;
    const uint32_t sel = (uint32_t)(nl >> 3);
    const uint32_t slot0 = (uint32_t)(nl & 7) * kTileBlocks + 2u * g;   // slot of the lane's first block in its tile
    // the mask bits of slots below slot0 (slot0 is even: both of the lane's blocks are in the same mask word)
    const bool upper = slot0 >= 32u;
    const uint32_t sh = slot0 & 31u;
    const uint32_t below_lo = upper ? 0xFFFFFFFFu : (1u << sh) - 1u, below_hi = upper ? (1u << sh) - 1u : 0u;
    const uint32_t second = sel * (uint32_t)a.n_kt;
    const uint32_t vL = a.off_L + (slot0 + second * kTileSlots) * 8u, vS = a.off_S + slot0 + second * kTileSlots;
    const uint32_t vM = a.off_M + second * 8u, vT = a.off_T + second * 4u;

    // the wave's tiles in the order it multiplies them: index of the first row-tile's tile, and whether
    // there is one (past the last tile the same loads are issued -- the waits count them -- through a
    // buffer of no bytes: they return zeros without touching memory, and so does the plane-H request they
    // lead to)
    int cur = 2 * (g_first + gsub) * a.n_kt + kt_b, cur_c = 0, left = total;
    const int run_skip = 2 * a.gpr * a.n_kt - (nt - 1);
    auto next_tile = [&](uint32_t &t, uint32_t &bytes, bool &first) {
        t = (uint32_t)cur;
        bytes = left > 0 ? a.off_H : 0u;
        first = cur_c == 0;
        --left;
        if (++cur_c == nt) {
            cur_c = 0;
            cur += run_skip;
        } else {
            ++cur;
        }
    };
    auto wbuf_of = [&](uint32_t bytes) { return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.w), 0, (int)bytes, kStRsrc); };
    const __amdgpu_buffer_rsrc_t wbuf = wbuf_of(a.off_H);

    StreamSlot ring[kStRing];

    // ---- activations -> FP16 values in LDS
    const float inv_S = 1.0f / a.S, S6 = 6.0f * a.S;
    auto store_block_lds = [&](int m, int kbl, const half2_t (&o)[8]) {
        union { half2_t h[8]; uint4 v[2]; } pack;
#pragma unroll
        for (int j = 0; j < 8; ++j) pack.h[j] = o[j];
        uint4 *dst = reinterpret_cast<uint4 *>(&xs[m * xrow + kbl * kBlock]);
        dst[0] = pack.v[0];
        dst[1] = pack.v[1];
    };
    // bf16 / fp32 input: the thread's K-block of the part and its rows my_r, my_r + rows_par, ...
    constexpr bool x_early = kSrc != 2;
    constexpr int kXs = kSrc == 2 ? 0 : kSrc;
    StreamXRaw<kXs> xraw;
    // (the mapping is the same in every part of K: in a shorter last part some threads own a block beyond it,
    // which is beyond K as well -- zeros)
    const int pb = a.tiles_gpart * kTileBlocks;
    const int rows_par = a.rows_par;                      // rows the threads cover at a time (the plan keeps it >= M / 3)
    const int my_r = (int)a.by_pb((uint32_t)tid), my_kbl = tid - my_r * pb;
    const int my_kb = kt_part0 * kTileBlocks + my_kbl;
    const bool my_active = my_r < rows_par;
    // The weights' header (bytes 0..31, 72..87) is read by the first wave alone, for all -- thousands of
    // waves asking for the same two cache lines is a queue at one memory channel -- and it is that wave's
    // oldest request (a request that a wave leaves out must be older than everything its waits count).
    StreamHeader hdr;
    if (wave == 0) st_load_header(hdr, wbuf);
    if constexpr (x_early) {
        constexpr uint32_t esz = kSrc == 1 ? 4u : 2u;
        const __amdgpu_buffer_rsrc_t xb = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.X), 0, (int)a.x_bytes, kStRsrc);
        const __amdgpu_buffer_rsrc_t fb = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.fisher), 0, a.nb_x * kBlock * 4, kStRsrc);
        const bool inside = my_active && my_kb < a.nb_x;
        // (these are the oldest loads of the wave: a wave without a row, or without a second or third one,
        // leaves them out -- the waits only count what is issued AFTER a load)
        const int wave_r = (int)a.by_pb((uint32_t)(wave * 64));   // lowest my_r in this wave
#pragma unroll
        for (int j = 0; j < kStXRows; ++j) {
            const int m = my_r + j * rows_par;
            if (wave_r + j * rows_par < a.M && wave_r < rows_par) {
                if (j == 0) st_load_f(xraw.f, fb, inside ? (uint32_t)my_kb * (kBlock * 4u) : kStOutside);
                st_load_x_row<kXs>(xraw.x[j], xb, inside && m < a.M ? (uint32_t)m * (uint32_t)a.ldx * esz + (uint32_t)my_kb * (kBlock * esz) : kStOutside);
            }
        }
    } else {
        // packed activations: decoded by everyone, before the stream
        for (int m = my_r; m < a.M; m += rows_par) {
            if (!my_active) break;
            half2_t o[8];
            stream_x_block<2>(a, m, my_kb, inv_S, S6, o);
            store_block_lds(m, my_kbl, o);
        }
    }

    // ---- prologue of the weight stream
    uint32_t pt[kStRing], pbytes[kStRing];
#pragma unroll
    for (int j = 0; j < kStRing; ++j) {
        bool first;
        next_tile(pt[j], pbytes[j], first);
        st_load_m(ring[j], wbuf_of(pbytes[j]), vM, pt[j]);
        st_load_t(ring[j], wbuf_of(pbytes[j]), vT, pt[j]);   // (of all the first tiles: what kind of tensor this is, is not known yet)
    }
#pragma unroll
    for (int j = 0; j < kStEarly; ++j) st_load_ls(ring[j], wbuf_of(pbytes[j]), vL, vS, pt[j]);
    ST_STAMP(1);
    if constexpr (x_early) {
        st_wait_x<kStRing * kStMtLoads + kStEarly * kStLsLoads, kXs>(xraw);
        float f[16];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) f[4 * i + e] = u2f(xraw.f[i][e]);
#pragma unroll
        for (int j = 0; j < kStXRows; ++j) {
            const int m = my_r + j * rows_par;
            if (my_active && m < a.M) {
                float x[16];
                if constexpr (kSrc == 1) {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
#pragma unroll
                        for (int e = 0; e < 4; ++e) x[4 * i + e] = u2f(xraw.x[j][i][e]);
                } else {
#pragma unroll
                    for (int i = 0; i < 2; ++i)
#pragma unroll
                        for (int e = 0; e < 4; ++e) {   // bf16 -> fp32 is a 16-bit shift
                            x[8 * i + 2 * e] = u2f(xraw.x[j][i][e] << 16);
                            x[8 * i + 2 * e + 1] = u2f(xraw.x[j][i][e] & 0xFFFF0000u);
                        }
                }
                half2_t o[8];
                // (a block beyond K inside the part's last tile: zeros came back, zeros go to LDS)
                stream_quantize_block(a, my_kb < a.nb_x, x, f, inv_S, S6, o);
                store_block_lds(m, my_kbl, o);
            }
        }
    }
    if (wave == 0) {
        st_wait_header<kStRing * kStMtLoads + kStEarly * kStLsLoads>(hdr);
        auto hdr_u64 = [](uint32_t lo, uint32_t hi) { return ((uint64_t)hi << 32) | lo; };
        const bool ok = hdr.h0[0] == kMagic && hdr_u64(hdr.h0[2], hdr.h0[3]) == (uint64_t)a.w_rows && hdr_u64(hdr.h1[0], hdr.h1[1]) == (uint64_t)a.w_K;
        if (lane == 0) {
            hw[0] = ok ? 1u : 0u;
            hw[1] = hdr.h1[2];                 // tensor scale
            hw[2] = hdr.h1[3];                 // compact?
            hw[3] = ok ? hdr.h2[2] : 0u;       // bytes in use: plane H ends there (a compact tensor may live in a buffer of exactly that size)
        }
    }
    // X^ and the header words are complete when every wave has passed here (LDS stores done; the loads stay in flight)
    __builtin_amdgcn_s_waitcnt(0xC07F);
    __builtin_amdgcn_s_barrier();
    ST_STAMP(2);
#pragma unroll
    for (int j = kStEarly; j < kStRing; ++j) st_load_ls(ring[j], wbuf_of(pbytes[j]), vL, vS, pt[j]);

    auto word = [](uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); };
    const bool w_ok = word(hw[0]) != 0u;
    const float w_scale = __builtin_bit_cast(float, word(hw[1]));
    // compact tensors store the tiles' plane-H entries back to back in tile order: within a run, a tile's
    // first entry follows from the tile before it, and only the first tile of a run needs its plane-T word
    const bool every_t = word(hw[2]) == 0u;
    const uint32_t w_used = word(hw[3]);
    const __amdgpu_buffer_rsrc_t hbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.w), 0, (int)w_used, kStRsrc);
    // (every lane loads: lanes without an FP8 block read entry 0, which every tensor with an FP8 block has;
    // the indices are range-checked against the tensor's bytes_used, so no content of the small planes can
    // lead outside)
    uint32_t t_next = 0;   // (per lane: of its own row-tile) first entry of the next tile in line for its plane-H request
    int h_c = 0;           // that tile's place in its run
    auto issue_h = [&](StreamSlot &s) {
        const uint32_t bits = ((upper ? s.m[1] : s.m[0]) >> sh) & 3u;
        const uint32_t t0 = (h_c == 0 || every_t) ? s.t : t_next;
        t_next = t0 + (uint32_t)__builtin_popcount(s.m[0]) + (uint32_t)__builtin_popcount(s.m[1]);
        if (++h_c == nt) h_c = 0;
        const uint32_t r0 = t0 + (uint32_t)__builtin_popcount(s.m[0] & below_lo) + (uint32_t)__builtin_popcount(s.m[1] & below_hi);
        s.bits = bits;
        // 16 bytes from one entry before the second block's: that entry lands in the upper half whatever the
        // first block is, and the first block's, where it is FP8, is the one before it (lanes without FP8 blocks
        // read neighbouring entries they do not use; at the very start the 8 bytes in front of the plane)
        st_load_h(s, hbuf, a.off_H - 8u + (r0 + (bits & 1u)) * 8u);
    };
    auto issue_tile = [&](StreamSlot &s) {
        uint32_t t, bytes;
        bool first;
        next_tile(t, bytes, first);
        const __amdgpu_buffer_rsrc_t r = wbuf_of(bytes);
        st_load_m(s, r, vM, t);
        if (first || every_t) st_load_t(s, r, vT, t);
        st_load_ls(s, r, vL, vS, t);
    };
    // (the masks were requested first: they are here long before planes L / S)
#define ST_H(J) st_wait_mt<kStRing * kStLsLoads + (J) * kStHLoads>(ring[J]); issue_h(ring[J]);
    ST_H(0) ST_H(1) ST_H(2) ST_H(3)
#undef ST_H
    ST_STAMP(3);

    // ---- the products
    // (two accumulators per 16 rows of X: consecutive matrix instructions do not wait for each other)
    float4_t acc[MT], acc2[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) acc[i] = acc2[i] = float4_t{0.0f, 0.0f, 0.0f, 0.0f};
    bool x_ok = true;
    float x_scale = a.S;
    if constexpr (kSrc == 2) {
        x_ok = a.xv.hdr->magic == kMagic && a.xv.hdr->rows == a.xl.rows && a.xv.hdr->K == a.xl.K;
        x_scale = a.xv.hdr->tensor_scale;
    }
    const float ss = (w_ok && x_ok) ? x_scale * w_scale : 0.0f;
    float *const Y = a.Y;
    const int64_t ldy = a.ldy;
    const int M = a.M, N = a.N;
    const _Float16 *xrow_p = &xs[(nl % kXR) * xrow + 32 * g];
    int con_run = 0, con_c = 0;   // tile being multiplied
    int runs_closed = 0;

    // v[mt][r] = the final sum of Y[m = 16 mt + 4 g + r][n = 16 grp + nl] before the tensor scales
    auto emit = [&](const float4_t (&v)[MT], int grp) {
        if constexpr (!kPack) {
            const int64_t n = (int64_t)grp * 16 + nl;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int m = mt * 16 + 4 * g + r;
                    if (m < M && n < N) Y[m * ldy + n] = v[mt][r] * ss;
                }
        } else {
            // lane m takes the 16 results of output row m: through this wave's own slice of the reduction
            // buffer (nobody else reads it here; LDS serves one wave's accesses in order)
            float *tb = reinterpret_cast<float *>(&red[wave][0][0]);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int r = 0; r < 4; ++r) tb[(mt * 16 + 4 * g + r) * 16 + nl] = v[mt][r] * ss;
            const int m = lane;
            const bool valid = m < M, in_tile = m < ((M + kTileRows - 1) & ~(kTileRows - 1));
            float x[16], f[16];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float4_t t4 = *reinterpret_cast<const float4_t *>(&tb[(m & (16 * MT - 1)) * 16 + 4 * i]);
#pragma unroll
                for (int e = 0; e < 4; ++e) x[4 * i + e] = valid ? t4[e] : 0.0f;
            }
            // (the group's 16 sensitivities are the same for every lane: scalar loads, which the counted
            // vector-memory waits of the stream do not see)
            typedef const float __attribute__((address_space(4))) *const_floats_t;
            const_floats_t fy = (const_floats_t)(a.fisher_y + (size_t)grp * kBlock);
#pragma unroll
            for (int i = 0; i < 16; ++i) f[i] = valid ? fy[i] : 0.0f;
            const float inv_Sy = 1.0f / a.S_y, S6y = 6.0f * a.S_y;
            BlockCodes bc;
            quantize_block_math<true, false>(x, f, block_amax(x), a.S_y, inv_Sy, S6y, -1, false, bc);
            const bool hi = valid && bc.score > a.T_y;
            const uint32_t decisions = (uint32_t)__ballot(hi);
            const int y_nb = N / kBlock;
            if (a.scores_y != nullptr && valid) a.scores_y[(int64_t)m * y_nb + grp] = bc.score;
            const int unit = grp >> 3;
            const __amdgpu_buffer_rsrc_t ybuf = __builtin_amdgcn_make_buffer_rsrc(a.y_packed, 0, (int)a.y_bytes, kStRsrc);
            const __amdgpu_buffer_rsrc_t dbuf = __builtin_amdgcn_make_buffer_rsrc(a.dec, 0, a.n_groups * 4, kStRsrc);
            if (in_tile) {
                const uint32_t at = ((uint32_t)(m >> 3) * (uint32_t)a.y_n_kt + (uint32_t)unit) * kTileSlots + (uint32_t)(m & 7) * kTileBlocks + (uint32_t)(grp & 7);
                u32x2_t lword = u32x2_t{bc.q[0], bc.q[1]};
                if (hi) {
                    float rr[16];
#pragma unroll
                    for (int e = 0; e < 16; ++e) rr[e] = x[e] * inv_Sy;
                    uint32_t c[4];
                    encode_fp8_block<true, true>(rr, c);
                    lword = u32x2_t{c[0], c[1]};
                    __builtin_amdgcn_raw_buffer_store_b64(u32x2_t{c[2], c[3]}, ybuf, (int)(a.y_off_H + at * 8u), 0, kCoherent);
                } else {
                    __builtin_amdgcn_raw_buffer_store_b8((uint8_t)bc.sc, ybuf, (int)(a.y_off_S + at), 0, 0);
                }
                __builtin_amdgcn_raw_buffer_store_b64(lword, ybuf, (int)(a.y_off_L + at * 8u), 0, 0);
            }
            if (lane == 0) __builtin_amdgcn_raw_buffer_store_b32(decisions, dbuf, grp * 4, 0, kCoherent);
            __builtin_amdgcn_s_waitcnt(0);
            uint32_t before = 0;
            if (lane == 0) before = __hip_atomic_fetch_add(&a.uctr[unit], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            before = (uint32_t)__builtin_amdgcn_readfirstlane((int)before);
            const int expected = a.n_groups - 8 * unit < 8 ? a.n_groups - 8 * unit : 8;
            if (before == (uint32_t)(expected - 1)) {
                // all row groups of this K-tile of the result have left their decisions and entries: lane = slot
                const int gq = 8 * unit + (lane & 7);
                const uint32_t d = __builtin_amdgcn_raw_buffer_load_b32(dbuf, gq < a.n_groups ? gq * 4 : (int)kStOutside, 0, kCoherent);
                for (int rt = 0; rt * kTileRows < M; ++rt) {
                    const bool fp8 = (d >> (rt * kTileRows + (lane >> 3))) & 1u;
                    const uint64_t mask = __ballot(fp8);
                    const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
                    const uint32_t tile = (uint32_t)rt * (uint32_t)a.y_n_kt + (uint32_t)unit, at = tile * kTileSlots + lane;
                    // (every entry is in a register before the first one is stored: a store waits for its
                    // data, i.e. for the load instruction as a whole.  Asking for all 64 entries together with
                    // the decisions -- one round trip instead of two -- measured slower, 16.4 against 15.3 us.)
                    const u32x2_t e = __builtin_amdgcn_raw_buffer_load_b64(ybuf, fp8 ? (int)(a.y_off_H + at * 8u) : (int)kStOutside, 0, kCoherent);
                    if (fp8) {
                        __builtin_amdgcn_raw_buffer_store_b64(e, ybuf, (int)(a.y_off_H + (tile * kTileSlots + rank) * 8u), 0, kCoherent);
                        __builtin_amdgcn_raw_buffer_store_b8((uint8_t)rank, ybuf, (int)(a.y_off_S + at), 0, 0);
                    }
                    if (gq >= a.n_groups) {   // K-blocks of the tile beyond N: FP4 zeros
                        __builtin_amdgcn_raw_buffer_store_b64(u32x2_t{0u, 0u}, ybuf, (int)(a.y_off_L + at * 8u), 0, 0);
                        __builtin_amdgcn_raw_buffer_store_b8((uint8_t)0, ybuf, (int)(a.y_off_S + at), 0, 0);
                    }
                    if (lane == 0) {
                        __builtin_amdgcn_raw_buffer_store_b64(u32x2_t{(uint32_t)mask, (uint32_t)(mask >> 32)}, ybuf, (int)(a.y_off_M + tile * 8u), 0, 0);
                        __builtin_amdgcn_raw_buffer_store_b32(tile * kTileSlots, ybuf, (int)(a.y_off_T + tile * 4u), 0, 0);
                    }
                }
                if (lane == 0) {
                    __hip_atomic_store(&a.uctr[unit], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (unit == 0) write_header(static_cast<PackedHeader *>(a.y_packed), make_layout(M, N), a.S_y, 0u);
                }
            }
        }
    };
    // acc[mt][r] = Y[m = 16 mt + 4 g + r][n = 16 grp + nl] (partial over this wave's K-tiles)
    auto close_run = [&](int grp) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt] += acc2[mt];
        if (a.kp_in > 1) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) red[wave][mt][lane] = acc[mt];
            __builtin_amdgcn_s_waitcnt(0xC07F);   // LDS stores done; the weight loads in flight stay in flight
            __builtin_amdgcn_s_barrier();
            if (kpi == 0) {
                for (int p = 1; p < kp_eff; ++p) {   // in K order
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) acc[mt] += red[wave + p][mt][lane];
                }
            }
            __builtin_amdgcn_s_waitcnt(0xC07F);
            __builtin_amdgcn_s_barrier();
        }
        if (kpi == 0) {
            bool final_sums = a.P_g == 1;
            if (!final_sums) {
                // K is also split across workgroups: this part goes to memory (accesses that are
                // coherent across the chip); whoever arrives last at the group's counter adds the parts
                // in K order -- the result does not depend on who that is -- and clears the counter
                const __amdgpu_buffer_rsrc_t pbuf = __builtin_amdgcn_make_buffer_rsrc(a.partial, 0, (int)a.partial_bytes, kStRsrc);
                const uint32_t base = (uint32_t)grp * (uint32_t)a.P_g * (MT * 1024u) + lane * 16u;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) store_coherent16(pbuf, base + (uint32_t)kp_g * (MT * 1024u) + mt * 1024u, acc[mt]);
                __builtin_amdgcn_s_waitcnt(0);
                uint32_t before = 0;
                if (lane == 0) before = __hip_atomic_fetch_add(&a.gctr[grp], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                before = (uint32_t)__builtin_amdgcn_readfirstlane((int)before);
                if (before == (uint32_t)(a.P_g - 1)) {
                    float4_t sum[MT];
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) sum[mt] = float4_t{0.0f, 0.0f, 0.0f, 0.0f};
                    for (int p = 0; p < a.P_g; ++p) {
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt) sum[mt] += load_coherent16(pbuf, base + (uint32_t)p * (MT * 1024u) + mt * 1024u);
                    }
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) acc[mt] = sum[mt];
                    final_sums = true;
                    if (lane == 0) __hip_atomic_store(&a.gctr[grp], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
            if (final_sums) emit(acc, grp);
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt] = acc2[mt] = float4_t{0.0f, 0.0f, 0.0f, 0.0f};
        ++runs_closed;
    };
    // one K-tile: decode (b[4 j + i] = halves 2i, 2i+1 of MFMA j's B operand; MFMA j reduces over the K
    // elements 32 g + 8 j .. + 7 of the tile), multiply, and close the run after its last tile
    // (the activation operands of a tile are asked for before the wait for the tile: the LDS answers meanwhile)
    auto read_a = [&](half8_t (&af)[4][MT]) {
        if constexpr (MT == 1) {
            const _Float16 *xc = xrow_p + (kt_b - kt_part0 + con_c) * kTileK;
#pragma unroll
            for (int j = 0; j < 4; ++j) af[j][0] = *reinterpret_cast<const half8_t *>(xc + 8 * j);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    auto consume = [&](StreamSlot &s, half8_t (&af)[4][MT]) {
        const _Float16 *xc = xrow_p + (kt_b - kt_part0 + con_c) * kTileK;
        half2_t b[16];
        const uint32_t bits = s.bits;
        // (one conversion decodes both scale bytes)
        const half2_t s01 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(s.s, 1.0f, false);
        st_decode_block(make_uint2(s.l[0], s.l[1]), half2_t{s01[0], s01[0]}, bits & 1u, make_uint2(s.up[0], s.up[1]), reinterpret_cast<half2_t(&)[8]>(b[0]));
        st_decode_block(make_uint2(s.l[2], s.l[3]), half2_t{s01[1], s01[1]}, bits & 2u, make_uint2(s.up[2], s.up[3]),
                        reinterpret_cast<half2_t(&)[8]>(b[8]));
        const half8_t *bv = reinterpret_cast<const half8_t *>(b);
        // the slot's registers are free from here on: its next tile is requested before the products, not after
        issue_tile(s);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                if constexpr (MT != 1) af[j][mt] = *reinterpret_cast<const half8_t *>(xc + mt * 16 * xrow + 8 * j);
                if (j % 2 == 0) acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(af[j][mt], bv[j], acc[mt], 0, 0, 0);
                else acc2[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(af[j][mt], bv[j], acc2[mt], 0, 0, 0);
            }
        }
        if (++con_c >= nt) {
            close_run(g_first + gsub + con_run * a.gpr);
            con_c = 0;
            ++con_run;
        }
    };

    if (total > 0) {
        // the first eight steps (their plane H came with the prologue), then the steady state
#define ST_STEP(J, T)                                                                 \
    if ((T) < total) {                                                                \
        if constexpr ((T) >= kStFirstH) st_wait_mt<st_step_wait(T)>(ring[((J) + kStHLead) % kStRing]); \
        half8_t af[4][MT];                                                            \
        read_a(af);                                                                   \
        st_wait_all<st_step_wait(T)>(ring[J]);                                        \
        if constexpr ((T) >= kStFirstH) issue_h(ring[((J) + kStHLead) % kStRing]);     \
        consume(ring[J], af);                                                         \
    }
        ST_STEP(0, 0) ST_STEP(1, 1) ST_STEP(2, 2) ST_STEP(3, 3)
        ST_STAMP(4);
        for (int base = kStRing; base < total; base += kStRing) {
#define ST_LOOP_STEP(J)                                                    \
    if (base + (J) < total) {                                              \
        st_wait_mt<st_step_wait(kStRing + (J))>(ring[((J) + kStHLead) % kStRing]); \
        half8_t af[4][MT];                                                 \
        read_a(af);                                                        \
        st_wait_all<st_step_wait(kStRing + (J))>(ring[J]);                 \
        issue_h(ring[((J) + kStHLead) % kStRing]);                         \
        consume(ring[J], af);                                              \
    }
            ST_LOOP_STEP(0) ST_LOOP_STEP(1) ST_LOOP_STEP(2) ST_LOOP_STEP(3)
#undef ST_LOOP_STEP
        }
#undef ST_STEP
    }
    ST_STAMP(5);
    // every register a load may still write stays reserved until all loads have landed
#pragma unroll
    for (int j = 0; j < kStRing; ++j) st_wait_all<0>(ring[j]);
    ST_STAMP(6);
    // rounds this wave had no row group in: it still meets the others at the barriers
    if (a.kp_in > 1) {
        for (int r = runs_closed; r < a.rounds; ++r) {
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_s_barrier();
        }
    }
    ST_STAMP(7);
}

// ---- host side ----

struct StreamPlan {
    bool ok;
    int waves, mt, xr, P_g, n_slots, tiles_gpart, kp_in, tiles_in, gpr, rounds, n_groups, grid;
    size_t total;   // scratch: the partial sums
    uint32_t partial_bytes;
};

constexpr int kStCus = 256;

static StreamPlan stream_plan(int64_t M, int64_t N, int64_t K)
{
    StreamPlan p{};
    const PackedLayout lw = make_layout(N, K);
    constexpr uint64_t kLimit = 0xFFFFFF00ull;   // buffer loads address the packed weights with 32-bit offsets
    if (M < 1 || M > 32 || lw.total_bytes >= kLimit) return p;
    if (lw.n_rt % 2 != 0) return p;   // (a row group is two row-tiles)
    p.mt = M <= 16 ? 1 : 2;
    p.waves = 12;   // (measured: 8 and 16 waves per workgroup both run 5-15% slower on the Llama-2 shapes)
    const int kStThreads = 64 * p.waves, kStWaves = p.waves;
    p.xr = M == 1 ? 1 : M <= 8 ? 8 : 16 * p.mt;   // (one token: a single row, whatever K -- no part of K goes to another workgroup for the LDS's sake)
    const int n_kt = (int)lw.n_kt;
    // parts of K across workgroups: as few as let a part's rows fit the LDS and let every thread do with
    // one K-block of at most kStXRows rows
    int max_tiles = (kStXCap / p.xr - kStXPad) / kTileK;
    const int rows_par = (int)((M + kStXRows - 1) / kStXRows);           // rows the threads must cover at a time
    max_tiles = std::min(max_tiles, kStThreads / rows_par / kTileBlocks);
    if (max_tiles < 1) return p;
    p.P_g = (n_kt + max_tiles - 1) / max_tiles;
    p.tiles_gpart = (n_kt + p.P_g - 1) / p.P_g;
    p.P_g = (n_kt + p.tiles_gpart - 1) / p.tiles_gpart;
    if (p.P_g > 16) return p;
    p.n_slots = kStCus / p.P_g;
    p.grid = p.n_slots * p.P_g;
    p.n_groups = (int)((N + 15) / 16);
    if ((int64_t)p.n_groups * p.P_g * p.mt * 1024 >= (int64_t)kLimit) return p;
    const int groups_cu = (p.n_groups + p.n_slots - 1) / p.n_slots;
    // waves = (row groups of a round) x (parts of K inside the workgroup): the split with the fewest
    // K-tiles per wave over all rounds
    int best_cost = 0x7FFFFFFF;
    for (int kp = 1; kp <= kStWaves; ++kp) {
        if (kStWaves % kp != 0) continue;
        const int gpr = kStWaves / kp;
        const int use_gpr = groups_cu < gpr ? groups_cu : gpr;
        const int rounds = (groups_cu + use_gpr - 1) / use_gpr;
        const int tiles_in = (p.tiles_gpart + kp - 1) / kp;
        const int cost = rounds * tiles_in * 8 + (kp > 1 ? rounds * 3 : 0);
        if (cost < best_cost) {
            best_cost = cost;
            p.kp_in = kp;
            p.gpr = use_gpr;
            p.rounds = rounds;
            p.tiles_in = tiles_in;
        }
    }
    // the row groups' counters live in the zeroed control region at the start of every workspace
    if (p.P_g > 1 && (size_t)p.n_groups * 4 > kWsCtrlRegion) return p;
    p.partial_bytes = p.P_g > 1 ? (uint32_t)((size_t)p.n_groups * p.P_g * p.mt * 1024) : 0u;
    p.total = (size_t)align_up(p.partial_bytes, 256);
    p.ok = true;
    return p;
}

bool gemm_stream_applies(int64_t M, int64_t N, int64_t K) { return kUseHwCvt && stream_plan(M, N, K).ok; }

// Scratch bytes of a call (beyond the control region); the kernel must apply.
size_t gemm_stream_scratch_bytes(int64_t M, int64_t N, int64_t K)
{
    const StreamPlan p = stream_plan(M, N, K);
#ifdef FGMP_STREAM_TIMING
    return p.ok && kUseHwCvt ? p.total + (size_t)kStCus * kStMaxWaves * 64 : 0;
#else
    return p.ok && kUseHwCvt ? p.total : 0;
#endif
}

template <int kSrc, bool kPack = false> static void launch_stream(const StreamPlan &p, const StreamArgs &a, hipStream_t st)
{
    const dim3 grid((unsigned)p.grid), block((unsigned)(64 * p.waves));
    if (p.xr == 1) hipLaunchKernelGGL((gemm_stream_kernel<12, 1, 1, kSrc, kPack>), grid, block, 0, st, a);
    else if (p.mt == 1 && p.xr == 8) hipLaunchKernelGGL((gemm_stream_kernel<12, 1, 8, kSrc, kPack>), grid, block, 0, st, a);
    else if (p.mt == 1) hipLaunchKernelGGL((gemm_stream_kernel<12, 1, 16, kSrc, kPack>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((gemm_stream_kernel<12, 2, 32, kSrc, kPack>), grid, block, 0, st, a);
}

// Whether the one-launch step can also quantize and pack its results (`po` without a gate): the counters of
// both meetings -- parts of K per row group, row groups per K-tile of the result -- share the control region.
constexpr int kStUnitCtr0 = 14336;   // first word of the second kind
bool gemm_stream_packs(int64_t M, int64_t N, int64_t K)
{
    const StreamPlan p = stream_plan(M, N, K);
    return kUseHwCvt && p.ok && N % kBlock == 0 && p.n_groups <= kStUnitCtr0 &&
           (size_t)(kStUnitCtr0 + (p.n_groups + 7) / 8) * 4 <= kWsCtrlRegion;
}
// (Whether it pays: a row group's epilogue ends in a chain of memory round trips -- its stores acknowledged, the
// counter, for the last of eight the others' decisions and entries -- while the other workgroups still stream at
// full rate: 4-5 us that nothing overlaps with, against ~3 us for launching the standalone quantizer on staged
// FP32 results.  Llama-2-7B linears, one launch / two launches inside a HIP graph, us: QKV 15.5 / 14.0 at M = 1,
// 17.7 / 16.3 at M = 8, 22.6 / 20.3 at M = 32; FC1 20.6 / 19.5, 23.0 / 21.7, 36.9 / 29.3 -- where waves close
// several row groups or parts of K meet first, every epilogue also drains the wave's loads in flight.  So the
// library stages by default and quantizes in the launch on request.)
// scratch of such a call: the partial sums, then one word of decisions per row group
size_t gemm_stream_pack_scratch_bytes(int64_t M, int64_t N, int64_t K)
{
    return gemm_stream_scratch_bytes(M, N, K) + (size_t)align_up((uint64_t)((N + 15) / 16) * 4, 256);
}

// src: 0 bf16 X, 1 fp32 X (quantized in the kernel with fisher / T / S), 2 packed X.
// ctrl: the workspace's control region (kWsCtrlRegion bytes, zero between calls); scratch: gemm_stream_scratch_bytes.
fgmp_status_t gemm_stream(int src, const void *X, int64_t ldx, const float *fisher, float T, float S, const void *packed_X,
                          int64_t M, const void *packed_W, int64_t N, int64_t K, float *Y, int64_t ldy, void *ctrl,
                          void *scratch, hipStream_t st, const PackOut *po)
{
    const StreamPlan p = stream_plan(M, N, K);
    if (!p.ok || !kUseHwCvt) return FGMP_ERR_UNSUPPORTED;
    if (po != nullptr && (po->gate || src == 2 || !gemm_stream_packs(M, N, K))) return FGMP_ERR_UNSUPPORTED;
    const PackedLayout lw = make_layout(N, K);
    StreamArgs a{};
    a.X = X; a.ldx = ldx; a.fisher = fisher; a.T = T; a.S = S;
    if (src == 2) {
        a.xl = make_layout(M, K);
        a.xv = make_view(const_cast<void *>(packed_X), a.xl);
    }
    a.w = packed_W;
    a.off_L = (uint32_t)lw.off_L; a.off_S = (uint32_t)lw.off_S; a.off_M = (uint32_t)lw.off_M;
    a.off_T = (uint32_t)lw.off_T; a.off_H = (uint32_t)lw.off_H;
    a.n_tiles = (uint32_t)lw.n_tiles; a.n_rt = (uint32_t)lw.n_rt; a.n_kt = (int)lw.n_kt;
    a.w_rows = N; a.w_K = K;
    a.Y = Y; a.ldy = ldy; a.M = (int)M; a.N = (int)N; a.nb_x = (int)(K / kBlock);
    if (po != nullptr) {
        a.y_packed = po->out.hdr;
        a.y_bytes = (uint32_t)po->layout.total_bytes;
        a.y_off_L = (uint32_t)po->layout.off_L; a.y_off_S = (uint32_t)po->layout.off_S; a.y_off_M = (uint32_t)po->layout.off_M;
        a.y_off_T = (uint32_t)po->layout.off_T; a.y_off_H = (uint32_t)po->layout.off_H;
        a.y_n_kt = (int)po->layout.n_kt;
        a.fisher_y = po->fisher; a.T_y = po->T; a.S_y = po->S; a.scores_y = po->scores;
        a.dec = reinterpret_cast<uint32_t *>(static_cast<char *>(scratch) + p.total);
        a.uctr = static_cast<uint32_t *>(ctrl) + kStUnitCtr0;
    }
    a.gctr = static_cast<uint32_t *>(ctrl);
    a.partial = static_cast<float *>(scratch);
    a.partial_bytes = p.partial_bytes;
    a.x_bytes = src == 2 ? 0u : (uint32_t)((uint64_t)M * (uint64_t)ldx * (src == 1 ? 4u : 2u));
    a.P_g = p.P_g; a.n_slots = p.n_slots; a.tiles_gpart = p.tiles_gpart; a.kp_in = p.kp_in;
    a.tiles_in = p.tiles_in; a.gpr = p.gpr; a.rounds = p.rounds; a.n_groups = p.n_groups;
    a.groups_q = p.n_groups / p.n_slots; a.groups_r = p.n_groups % p.n_slots;
    a.rows_par = 64 * p.waves / (p.tiles_gpart * kTileBlocks);
    a.by_P_g = stream_div(p.P_g); a.by_kp_in = stream_div(p.kp_in); a.by_tiles_in = stream_div(p.tiles_in);
    a.by_gpr = stream_div(p.gpr); a.by_pb = stream_div(p.tiles_gpart * kTileBlocks);
#ifdef FGMP_STREAM_TIMING
    a.dbg = reinterpret_cast<unsigned long long *>(static_cast<char *>(scratch) + p.total);
#endif
    if (po != nullptr) {
        if (src == 0) launch_stream<0, true>(p, a, st);
        else launch_stream<1, true>(p, a, st);
    } else if (src == 0) launch_stream<0>(p, a, st);
    else if (src == 1) launch_stream<1>(p, a, st);
    else launch_stream<2>(p, a, st);
    return hipGetLastError() == hipSuccess ? FGMP_OK : FGMP_ERR_HIP;
}

}  // namespace fgmp
