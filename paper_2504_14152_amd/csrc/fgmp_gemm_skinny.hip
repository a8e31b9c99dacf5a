// Decode-shape (M <= 32 tokens per launch) block-mixed-precision GEMM (Sec. 4.1): the
// packed weights are streamed from HBM exactly once and decoded in registers
// straight into MFMA operands; the few activation rows sit in LDS as FP16.
//
// Work split: a workgroup owns 16 weight rows per wave (4 waves, or 8 when X has
// more than 16 rows) and a range of at most 8 K-tiles (1024 K elements).  K
// ranges are combined deterministically, per wave: every wave stores its
// partial tile, and the last one to arrive adds the partials in K order and
// writes Y.
//
// Lane (nl = lane % 16, g = lane / 16) of a wave reads, per K-tile of 128, the
// 16 bytes that hold blocks 2g and 2g+1 of weight row nl -- a wave's load is
// 1 KB of consecutive plane-L bytes -- and decodes them into the B operands of
// four 16x16x32 MFMAs; MFMA j therefore reduces over the K elements
// 32 g + 8 j .. 32 g + 8 j + 7 (g = 0..3) of the tile, and the A operand is
// read from LDS with the same assignment.  Only plane L is streamed tile by
// tile; the small planes of a wave's 2 x 8 tiles -- scale bytes, mask words and
// the FP8 blocks' upper halves (plane H, contiguous for consecutive K-tiles of
// a compact tensor) -- are fetched in bulk at the start, with full-width loads,
// and parked in LDS, where each lane picks its bytes per tile.
//
// A call lasts 10-30 us, so what matters is the chain of dependent steps a wave
// goes through (per-wave time stamps: about a third each for start-up -- kernel
// arguments, first loads, the plane-T -> plane-H dependency --, the K-tile loop,
// and the split-K hand-over), not instruction count alone.  Every access to the
// packed tensors is a buffer load whose per-lane offset is computed once and
// whose per-K-tile displacement is a scalar offset.  The buffer range check
// also makes every load safe without a select: tiles past the K range or rows
// past the tensor read other tiles' bytes or zeros, and their results are
// never stored.
#include <cstddef>

#include "fgmp_gemm_common.hpp"

namespace fgmp {

typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

// K-tiles per workgroup and plane-H entries staged per row-tile and K range (FP8 blocks beyond fetch
// their entry directly).  Sized by LDS: every workgroup of a launch should be resident at once (4 per
// CU with 4 waves and up to 8 rows of X -- as many as the waves' 120 vector registers allow --, 3 with
// 9..16 rows, 2 per CU with 8 waves and 17..32 rows).
constexpr int skinny_max_cols(int mt) { return mt == 1 ? 8 : 7; }
constexpr int skinny_h_window(int mt) { return mt == 1 ? 192 : 64; }
constexpr int kSkPrefetch = 4;    // plane-L K-tiles in flight per wave (2..4 measure alike, 8 is slower)
constexpr int kSkXPad = 8;        // halves of padding per LDS activation row

constexpr int kSkSumPass = 4;     // partial tiles summed per pass (their loads are in flight together)
constexpr int kSkMaxSplit = 16;   // most K ranges per row group the planner asks for

constexpr uint32_t kRsrcFlags = 0x00020000;   // raw buffer, 32-bit data format

__device__ __forceinline__ uint4 ld128(__amdgpu_buffer_rsrc_t b, uint32_t off, uint32_t soff = 0)
{
    const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(b, (int)off, (int)soff, 0);
    return make_uint4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ uint2 ld64(__amdgpu_buffer_rsrc_t b, uint32_t off)
{
    const u32x2_t v = __builtin_amdgcn_raw_buffer_load_b64(b, (int)off, 0, 0);
    return make_uint2(v[0], v[1]);
}
__device__ __forceinline__ uint32_t ld32(__amdgpu_buffer_rsrc_t b, uint32_t off)
{
    return __builtin_amdgcn_raw_buffer_load_b32(b, (int)off, 0, 0);
}
__device__ __forceinline__ uint32_t ld16(__amdgpu_buffer_rsrc_t b, uint32_t off, uint32_t soff = 0)
{
    return (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(b, (int)off, (int)soff, 0);
}
__device__ __forceinline__ uint32_t ld8(__amdgpu_buffer_rsrc_t b, uint32_t off)
{
    return (uint32_t)__builtin_amdgcn_raw_buffer_load_b8(b, (int)off, 0, 0);
}

static_assert(offsetof(PackedHeader, magic) == 0 && offsetof(PackedHeader, rows) == 8 && offsetof(PackedHeader, K) == 16 &&
                  offsetof(PackedHeader, tensor_scale) == 24 && offsetof(PackedHeader, h_entries) == 72 &&
                  offsetof(PackedHeader, bytes_used) == 80,
              "the kernel reads these header fields by byte offset");

struct SkinnyStage {
    uint4 l;       // blocks 2g, 2g+1 of this lane's row
};

struct SkinnyArgs {
    const void *w;            // packed weights (header first)
    const PackedHeader *xh;   // header of the activations (tensor scale, shape check)
    const _Float16 *x16;      // activations as FP16 values, [>= 16 MT rows][ld16]
    float *Y;
    float *partial;
    uint32_t *counters;       // one per (row group, wave), zeroed by the kernel that prepares x16
    int64_t ld16, ldy, M, N;
    int64_t w_rows, w_K, x_rows, x_K;                          // the shapes the headers must state
    uint32_t off_L, off_S, off_M, off_T, off_H, n_tiles;       // layout of the packed weights
    uint32_t partial_bytes;
    int n_kt, cols_per_wg, ksplit;
};

// kWaves waves per workgroup, 16 weight rows each; they share the activations in LDS.
// kXR: activation rows kept in LDS (8 when M <= 8, else all 16 MT): rows of the MFMA operand beyond them
// alias the rows there are -- they only feed output rows that are never stored -- and the smaller
// workgroup lets one more of them be resident per compute unit.
template <int MT, int kWaves, int kXR>
__global__ __launch_bounds__(64 * kWaves) void gemm_skinny_kernel(SkinnyArgs a)
{
    constexpr int kRows = 16 * kWaves;   // weight rows per workgroup
    constexpr int kSkMaxCols = skinny_max_cols(MT), kSkHWin = skinny_h_window(MT);
    constexpr int kXRow = kSkMaxCols * kTileK + kSkXPad;
    static_assert(kXR == 16 * MT || (MT == 1 && kXR == 8), "rows of X in LDS");
    __shared__ __attribute__((aligned(1024))) _Float16 xs[kXR][kXRow];
    // per wave (sel = which of its two row-tiles):
    __shared__ uint2 m_lds[kWaves][16];                       // mask words, [sel][K-tile]
    __shared__ uint32_t t_lds[kWaves][16];                    // plane-H offsets relative to the K range's first, [sel][K-tile]
    __shared__ __attribute__((aligned(16))) uint8_t s_lds[kWaves][2][8 * kTileSlots];   // plane S, [sel][K-tile][slot] (always 8 tiles' worth is loaded)
    __shared__ __attribute__((aligned(16))) uint2 h_lds[kWaves][2][kSkHWin];                     // plane H window, [sel][entry]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ksplit = a.ksplit;
    const int64_t rg = blockIdx.x / ksplit;
    const int ks = blockIdx.x % ksplit;
    const int c0 = ks * a.cols_per_wg;
    const int ncols = (a.n_kt - c0 < a.cols_per_wg) ? a.n_kt - c0 : a.cols_per_wg;

    // Planes L, S, M, T have fixed extents; plane H ends where the header says (a compact tensor may
    // live in a buffer of exactly bytes_used bytes).
    const __amdgpu_buffer_rsrc_t wbuf =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.w), 0, (int)a.off_H, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t xhbuf =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<PackedHeader *>(a.xh), 0, (int)kHeaderBytes, kRsrcFlags);
    const int nl = lane & 15, g = lane >> 4;
    const uint32_t rtA = (uint32_t)rg * (kRows / kTileRows) + wave * 2;   // the wave's two row-tiles: rtA, rtA + 1
    const int my_sel = nl >> 3;                        // which of the two this lane's weight row is in
    const int slot0 = (nl & 7) * kTileBlocks + 2 * g;  // slots of blocks 2g, 2g+1 within the tile
    const uint32_t tile0 = (rtA + my_sel) * a.n_kt + c0;
    const uint32_t voff_L = a.off_L + (tile0 * kTileSlots + slot0) * 8u;
    // Per-tile words (mask, plane-H offset) of the wave's 2 x 8 tiles, one tile per lane (lanes 0-15);
    // lanes 16, 17 fetch the plane-H offset of the tile after the K range, i.e. where its entries end.
    const int w_sel = (lane >> 3) & 1;
    const uint32_t w_tile = (rtA + w_sel) * a.n_kt + c0 + (lane & 7);
    const uint32_t end_tile = (rtA + (lane & 1)) * a.n_kt + c0 + ncols;
    const uint32_t t_tile = lane < 16 ? w_tile : end_tile;
    const uint32_t s_tile0 = (rtA + (lane >> 5)) * a.n_kt + c0;
    const char *xg = reinterpret_cast<const char *>(a.x16) + (int64_t)c0 * (kTileK * 2);
    const int64_t x_row_bytes = a.ld16 * 2;
    const int x_load_rows = __builtin_amdgcn_readfirstlane((int)a.M);
    // everything above only needs the kernel arguments; no load below waits for more than those
    __builtin_amdgcn_sched_barrier(0);

    // ---- activations: the M rows there are, (ncols * 128) halves each, straight into LDS; one wave-load
    // fills 1 KB = half a row of 8 K-tiles.  The other rows of the 16 MT stay as the LDS happens to be:
    // they only feed output rows that are never stored (every workgroup re-reads its slice of X from
    // the L2; at M = 1 that is 2 KB instead of 32).  Chunks past the K range re-read the row's first
    // chunk (never used).
    // Written as assembly: while a global->LDS load that the compiler knows of is pending, it turns
    // every wait for an ordinary load into vmcnt(0), and the start-up below lives on exact waits (the
    // plane-H window can be requested as soon as the plane-T words are here, with the plane-L ring
    // still in flight).  Loads complete in issue order and these are the first, so every later wait
    // for a loaded register also covers them.
#pragma unroll
    for (int u = 0; u < 2 * kXR / kWaves; ++u) {
        const int id = wave + kWaves * u, r = id >> 1, h = id & 1;
        const int chunk = h * 64 + lane;
        const int src_chunk = chunk < ncols * (kTileK / 8) ? chunk : 0;
        // (a row of fewer than 8 K-tiles ends inside the second wave-load: the lanes beyond it stay out)
        if (chunk < kSkMaxCols * (kTileK / 8) && r < x_load_rows) {
            const uint32_t dst = (uint32_t)(uintptr_t)(lds_void_t *)&xs[r][h * 512];   // M0: the wave's LDS destination
            const uint32_t voff = (uint32_t)(r * x_row_bytes + src_chunk * 16);
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(dst), "v"(voff), "s"(xg) : "memory");
        }
    }
    __builtin_amdgcn_sched_barrier(0);   // keep these loads ahead of all others (see the barrier below)

    // ---- weights: the small planes of the 2 x 8 tiles in bulk, the headers, then the plane-L stream.
    // The headers come through the vector memory path like everything else (every lane reads the same
    // bytes), so that no wait for an earlier load also waits for them.
    const uint2 mvec = ld64(wbuf, a.off_M + w_tile * 8u);
    uint32_t tvec = ld32(wbuf, a.off_T + t_tile * 4u);
    // plane S: 512 contiguous bytes per row-tile, one 16-byte load per lane
    const uint4 svec = ld128(wbuf, a.off_S + s_tile0 * kTileSlots + (lane & 31) * 16u);
    const uint4 wh0 = ld128(wbuf, 0), wh1 = ld128(wbuf, 16), wh2 = ld128(wbuf, 72);   // see PackedHeader
    const uint4 xh0 = ld128(xhbuf, 0), xh1 = ld128(xhbuf, 16);

    auto issue_l = [&](int c, SkinnyStage &st) {
        // the K-tile displacement is uniform: it travels in the scalar offset, not through the vector ALU
        st.l = ld128(wbuf, voff_L, (uint32_t)(kTileSlots * 8) * c);
    };
    // The first half of the plane-L ring goes out now; the second half follows the plane-H window loads
    // below, which depend on the plane-T words: every workgroup of the launch starts at the same time, and
    // behind the whole ring (4 KB per wave, 12 MB over the chip) those loads would wait a microsecond longer.
    SkinnyStage ring[kSkPrefetch];
    static_assert(kSkPrefetch == 4, "two stages before, two after the plane-H window loads");
    issue_l(0, ring[0]);
    issue_l(1, ring[1]);

    // header fields: magic at byte 0, rows at 8, K at 16, tensor_scale at 24, h_entries at 72, bytes_used at 80
    auto hdr_ok = [](const uint4 &h0, const uint4 &h1, int64_t rows, int64_t K) {
        return h0.x == kMagic && (((uint64_t)h0.w << 32) | h0.z) == (uint64_t)rows &&
               (((uint64_t)h1.y << 32) | h1.x) == (uint64_t)K;
    };
    const bool w_ok = hdr_ok(wh0, wh1, a.w_rows, a.w_K);
    const bool x_ok = hdr_ok(xh0, xh1, a.x_rows, a.x_K);
    const float w_scale = __builtin_bit_cast(float, wh1.z), x_scale = __builtin_bit_cast(float, xh1.z);
    const uint32_t w_h_entries = wh2.x;
    const uint32_t w_used = w_ok ? (uint32_t)__builtin_amdgcn_readfirstlane((int)wh2.z) : 0u;
    const __amdgpu_buffer_rsrc_t hbuf =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.w), 0, (int)w_used, kRsrcFlags);

    // Plane H: the entries of the K range's tiles of one row-tile are contiguous, from the first tile's
    // offset to the offset of the tile after the range (the plane's end for the tensor's last tile).
    if (lane >= 16 && end_tile >= a.n_tiles) tvec = w_h_entries;
    const uint32_t startA = __builtin_amdgcn_readlane(tvec, 0), startB = __builtin_amdgcn_readlane(tvec, 8);
    const uint32_t endA = __builtin_amdgcn_readlane(tvec, 16), endB = __builtin_amdgcn_readlane(tvec, 17);
    const uint32_t needA = endA - startA, needB = endB - startB;       // entries (garbage rows: any value)
    // any FP8 block of this wave beyond the staged window?  (then those blocks fetch their entry directly)
    const bool any_far = needA > (uint32_t)kSkHWin || needB > (uint32_t)kSkHWin;
    if (lane < 16) {
        m_lds[wave][lane] = mvec;
        t_lds[wave][lane] = tvec - (w_sel ? startB : startA);
    }
    *reinterpret_cast<uint4 *>(&s_lds[wave][lane >> 5][(lane & 31) * 16]) = svec;
    // (written and read by the same wave, LDS operations of a wave execute in order: no barrier needed)
    {
        // 128 entries (1 KB) per wave-load and row-tile; as many loads as the fuller row-tile needs
        const uint32_t need = needA > needB ? needA : needB;
        const uint32_t my_start = (lane >> 5) ? startB : startA;   // lanes 0-31: row-tile A, 32-63: row-tile B
        // the first 64 entries per row-tile unconditionally (nearly always all that is needed; a load
        // the compiler knows to be issued gets an exact wait, which leaves the two plane-L loads
        // behind it in flight), the rest only if the range holds more
        const uint32_t e = 2u * (lane & 31);
        const uint4 hv0 = ld128(hbuf, a.off_H + (my_start + e) * 8u);
        issue_l(2, ring[2]);
        issue_l(3, ring[3]);
        *reinterpret_cast<uint4 *>(&h_lds[wave][lane >> 5][e]) = hv0;
        // (load and store in one branch: a load left pending at the end of a branch would make every
        // later wait a full one)
#pragma unroll
        for (int u = 1; u < kSkHWin / 64; ++u) {
            if ((uint32_t)(64 * u) < need) {
                const uint4 hv = ld128(hbuf, a.off_H + (my_start + 64u * u + e) * 8u);
                *reinterpret_cast<uint4 *>(&h_lds[wave][lane >> 5][64u * u + e]) = hv;
            }
        }
    }
    const uint8_t *m_byte = reinterpret_cast<const uint8_t *>(&m_lds[wave][my_sel * 8]) + (nl & 7);
    const uint16_t *s_pair = reinterpret_cast<const uint16_t *>(&s_lds[wave][my_sel][slot0]);
    const uint32_t *t_rel = &t_lds[wave][my_sel * 8];
    const uint2 *h_win = &h_lds[wave][my_sel][0];

    // Everything a tile's decode looks up -- mask byte, scale-or-index bytes, the tile's offset into the
    // plane-H window and, through those, the upper halves of its FP8 blocks -- is fetched from LDS for
    // all K-tiles of the range at once, before the loop: two rounds of independent reads instead of a
    // chain of dependent LDS round trips inside every tile.  (Tiles past the range read other bytes of
    // the wave's LDS, or zeros beyond it; they are never consumed.)
    uint32_t mb[kSkMaxCols], sv[kSkMaxCols], tr[kSkMaxCols];
#pragma unroll
    for (int c = 0; c < kSkMaxCols; ++c) {
        mb[c] = m_byte[c * 8];
        sv[c] = s_pair[c * (kTileSlots / 2)];
        tr[c] = t_rel[c];
    }
    uint2 up_a[kSkMaxCols], up_b[kSkMaxCols];
#pragma unroll
    for (int c = 0; c < kSkMaxCols; ++c) {
        const uint32_t e0 = tr[c] + (sv[c] & 0xFFu), e1 = tr[c] + (sv[c] >> 8);
        up_a[c] = h_win[e0 < (uint32_t)kSkHWin ? e0 : 0u];
        up_b[c] = h_win[e1 < (uint32_t)kSkHWin ? e1 : 0u];
    }

    // The activation loads were issued before the per-tile words that the code above has waited for,
    // and loads complete in order: this wave's have landed, and after the barrier every wave's.  A bare
    // barrier: the usual one first waits for every outstanding load, and the plane-L ring should stay
    // in flight across it.  (Everything else in LDS is private to the wave that wrote it.)
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0)
    __builtin_amdgcn_s_barrier();

    float4_t acc[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) acc[i] = float4_t{0.0f, 0.0f, 0.0f, 0.0f};

    const _Float16 *xrow = &xs[nl % kXR][32 * g];
    auto consume = [&](int c, const SkinnyStage &st, uint32_t mbyte, uint32_t svc, uint32_t trel, uint2 up0, uint2 up1) {
        const uint32_t mbits = mbyte >> (2 * g);   // bits 0, 1: blocks 2g, 2g+1 are FP8
        const uint32_t s0 = svc & 0xFFu, s1 = svc >> 8;
        const bool hi0 = mbits & 1u, hi1 = mbits & 2u;
        // K ranges with more FP8 blocks than the window holds: fetch directly.  Rare; the wait sits
        // inside the branch so that the common path keeps counting only its own prefetches.
        if (any_far) {
            const uint32_t e0 = trel + s0, e1 = trel + s1;   // entry = tile's offset in the window + index byte
            const uint32_t my_start = my_sel ? startB : startA;
            if (hi0 && e0 >= (uint32_t)kSkHWin) up0 = ld64(hbuf, a.off_H + (my_start + e0) * 8u);
            if (hi1 && e1 >= (uint32_t)kSkHWin) up1 = ld64(hbuf, a.off_H + (my_start + e1) * 8u);
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
        }
        half2_t b[16];   // b[4 j + i]: halves 2i, 2i+1 of MFMA j's operand
        decode_block(make_uint2(st.l.x, st.l.y), s0, hi0, up0, reinterpret_cast<half2_t(&)[8]>(b[0]));
        decode_block(make_uint2(st.l.z, st.l.w), s1, hi1, up1, reinterpret_cast<half2_t(&)[8]>(b[8]));
        const half8_t *bv = reinterpret_cast<const half8_t *>(b);
        const _Float16 *xc = xrow + c * kTileK;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const half8_t af = *reinterpret_cast<const half8_t *>(xc + mt * 16 * kXRow + 8 * j);
                acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(af, bv[j], acc[mt], 0, 0, 0);
            }
        }
    };
    // One pass over the range's tiles, instantiated per tile: the plane-L ring and the looked-up words
    // are indexed statically (a ring stage's registers are the targets of loads in flight and must not
    // be copied).  Tiles past the K range load other bytes of the buffer (or zeros) that are never
    // consumed.
#pragma unroll
    for (int c = 0; c < kSkMaxCols; ++c) {
        if (c < ncols) consume(c, ring[c % kSkPrefetch], mb[c], sv[c], tr[c], up_a[c], up_b[c]);
        if (c + kSkPrefetch < kSkMaxCols) issue_l(c + kSkPrefetch, ring[c % kSkPrefetch]);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // drain the plane-L loads of tiles past the K range

    float *const Y = a.Y;
    const int64_t ldy = a.ldy, M = a.M, N = a.N;
    // acc[mt][r] = partial Y[m = 16 mt + 4 (lane / 16) + r][n = 64 rg + 16 wave + lane % 16]
    // operands whose headers do not match the call's shapes count as zeros
    const bool ok = w_ok && x_ok;
    const float ss = x_scale * w_scale;
    const int64_t n = rg * kRows + wave * 16 + nl;
    if (ksplit == 1) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int64_t m = mt * 16 + 4 * g + r;
                if (m < M && n < N) Y[m * ldy + n] = ok ? acc[mt][r] * ss : 0.0f;
            }
        return;
    }
    // K ranges are combined per wave (16 weight rows), without workgroup barriers.  Partial layout:
    // [workgroup][wave][mt][lane] vectors of 16 bytes, a lane's four accumulators of one MFMA tile.
    // Partials and counters cross XCDs: they are written and read with system-coherent vector
    // accesses (sc0 sc1), which bypass the per-XCD L2; a wave's stores are complete before it bumps
    // the counter, so the wave that observes the last arrival reads complete partials.  It adds them
    // in K order -- the result does not depend on which wave came last.
    constexpr uint32_t kWaveBytes = 64 * 16 * MT;                 // one wave's partial
    const __amdgpu_buffer_rsrc_t pbuf =
        __builtin_amdgcn_make_buffer_rsrc(a.partial, 0, (int)a.partial_bytes, kRsrcFlags);
    const uint32_t mine = ((uint32_t)blockIdx.x * kWaves + wave) * kWaveBytes + lane * 16u;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) store_coherent16(pbuf, mine + mt * 1024u, acc[mt]);
    __builtin_amdgcn_s_waitcnt(0);
    uint32_t before = 0;
    if (lane == 0)
        before = __hip_atomic_fetch_add(&a.counters[rg * kWaves + wave], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    before = __builtin_amdgcn_readfirstlane(before);
    if (before != (uint32_t)(ksplit - 1)) return;
    const uint32_t first = ((uint32_t)(rg * ksplit) * kWaves + wave) * kWaveBytes + lane * 16u;
    float4_t sum[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) sum[mt] = float4_t{0.0f, 0.0f, 0.0f, 0.0f};
    for (int k0 = 0; k0 < ksplit; k0 += kSkSumPass) {
        float4_t part[kSkSumPass][MT];
#pragma unroll
        for (int k = 0; k < kSkSumPass; ++k) {
            const int kk = k0 + k < ksplit ? k0 + k : ksplit - 1;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                part[k][mt] = load_coherent16(pbuf, first + (uint32_t)kk * (kWaves * kWaveBytes) + mt * 1024u);
        }
#pragma unroll
        for (int k = 0; k < kSkSumPass; ++k)
            if (k0 + k < ksplit) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) sum[mt] += part[k][mt];
            }
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int64_t m = mt * 16 + 4 * g + r;
            if (m < M && n < N) Y[m * ldy + n] = ok ? sum[mt][r] * ss : 0.0f;
        }
}

// ---- host side ----

struct SkinnyPlan {
    int mt, waves, cols_per_wg, ksplit;
    int64_t row_groups;
    size_t off_partial, off_counters, total;
};

static SkinnyPlan skinny_plan(int64_t M, int64_t N, int64_t K)
{
    SkinnyPlan p;
    const PackedLayout lw = make_layout(N, K);
    p.mt = M <= 16 ? 1 : 2;
    // 17..32 rows of X need twice the LDS per workgroup: 8 waves share it, so that every workgroup of
    // the launch is still resident at once.  Every workgroup re-reads its K range of X: with very long
    // K, 16 waves -- twice the weight rows per workgroup, half that traffic -- pay off (FC2, K = 11008,
    // M = 32: 23.7 -> 21.1 us); otherwise they only make the workgroups fewer and longer (O projection,
    // K = 4096: 15.0 -> 16.3 us; a 57344 x 8192 tensor: 128 -> 131 us).
    p.waves = p.mt == 1 ? 4 : (lw.n_kt > 64 ? 16 : 8);
    const int64_t rows_per_wg = 16 * p.waves;
    p.row_groups = (N + rows_per_wg - 1) / rows_per_wg;
    // At least one workgroup per CU, each with as many K-tiles as its LDS holds: further splitting of K
    // only shortens a workgroup's stream below its start-up latency and lengthens the sum over K ranges
    // (Llama-2-7B O projection, N = K = 4096, M = 8: 13.2 us with 256 workgroups of 8 K-tiles, 17.0 us
    // with 704 of 3); more workgroups than are resident at once pay the start-up twice.
    const int64_t target_wgs = p.mt == 1 ? 256 : 128;
    int64_t want = (target_wgs + p.row_groups - 1) / p.row_groups;
    const int max_cols = skinny_max_cols(p.mt);
    const int64_t need = (lw.n_kt + max_cols - 1) / max_cols;
    if (want < need) want = need;
    if (want > kSkMaxSplit) want = kSkMaxSplit;
    if (want < need) want = need;   // long K: more ranges than one summing pass, still correct
    if (want > lw.n_kt) want = lw.n_kt;
    p.cols_per_wg = (int)((lw.n_kt + want - 1) / want);
    p.ksplit = (int)((lw.n_kt + p.cols_per_wg - 1) / p.cols_per_wg);
    p.off_partial = 0;
    p.off_counters = (size_t)align_up((uint64_t)p.row_groups * p.ksplit * (16 * p.mt) * rows_per_wg * 4, 256);
    p.total = p.off_counters + (size_t)align_up((uint64_t)p.row_groups * p.waves * sizeof(uint32_t), 256);
    return p;
}

// More than 32 rows (up to kSkinnyMaxRows) may run as chunks of 32 rows, one launch each, on the same
// stream: the weights of the later chunks come from the Infinity Cache, and a few such passes are
// faster than the 256-row MFMA tiles of the prefill kernel, whose time hardly depends on M below 256
// (Llama-2-7B, microseconds per fused step at M = 33 / 64 / 96 in chunks against the prefill kernel at
// M = 96 .. 256: QKV 31 / 35 / 49 against 44 .. 56, O 22 / 24 / 34 against 43 .. 49, FC2 35 / 39 / 55
// against 82 .. 85, FC1 47 / 55 / 78 against 64).  Workspace: the chunks' partial sums one after the other, then all of their
// counters, contiguous, so that one clearing pass covers them.
constexpr int64_t kSkChunkRows = 32;
static_assert(kSkinnyMaxRows % kSkChunkRows == 0, "whole chunks");
constexpr int kSkMaxChunks = (int)(kSkinnyMaxRows / kSkChunkRows);

struct SkinnyChunks {
    int n;
    SkinnyPlan plan[kSkMaxChunks];
    int64_t rows[kSkMaxChunks];
    size_t off_partial[kSkMaxChunks], off_counters[kSkMaxChunks], counters_begin, n_counters, total;
};

static SkinnyChunks skinny_chunks(int64_t M, int64_t N, int64_t K)
{
    SkinnyChunks c;
    c.n = (int)((M + kSkChunkRows - 1) / kSkChunkRows);
    size_t off = 0;
    for (int i = 0; i < c.n; ++i) {
        c.rows[i] = M - i * kSkChunkRows < kSkChunkRows ? M - i * kSkChunkRows : kSkChunkRows;
        c.plan[i] = skinny_plan(c.rows[i], N, K);
        c.off_partial[i] = off;
        off += c.plan[i].off_counters - c.plan[i].off_partial;   // the chunk's partial sums
    }
    c.counters_begin = off;
    c.n_counters = 0;
    for (int i = 0; i < c.n; ++i) {
        c.off_counters[i] = off;
        const size_t bytes = c.plan[i].total - c.plan[i].off_counters;
        off += bytes;
        c.n_counters += bytes / sizeof(uint32_t);
    }
    c.total = off;
    return c;
}

size_t gemm_skinny_workspace_bytes(int64_t M, int64_t N, int64_t K) { return skinny_chunks(M, N, K).total; }

// Whether n chunks beat the prefill kernel, from a cost model fitted to the measurements above (times in
// microseconds).  One 32-row pass: a fixed 8 us plus the packed weights at 2.5 TB/s; later passes cost
// 0.65 of that while the weights fit the Infinity Cache.  Prefill kernel below 257 rows: one tile per
// 256 weight rows, two workgroups per tile when that fills at most half the chip (the longer one takes
// 9/16 of the K-steps), four when at most a quarter (and a second meeting), 1.45 us per K-step of 64,
// rounds of 256 workgroups.
static bool chunks_beat_prefill_kernel(int64_t n_chunks, int64_t N, int64_t K)
{
    const double w_bytes = 0.62 * (double)N * (double)K;
    const double pass = 8.0 + w_bytes / 2.5e6;
    const double t_chunks = 5.0 + pass * (1.0 + (w_bytes < 200e6 ? 0.65 : 1.0) * (double)(n_chunks - 1));
    const int64_t tiles = (N + 255) / 256, nk = (K + 127) / 128 * 2;
    const int64_t tail = tiles % 256;
    const int parts = tail <= 64 && nk >= 8 ? 4 : (tail <= 128 && nk >= 4 ? 2 : 1);
    const int64_t units = parts * tiles;
    const double steps = parts == 4 ? (double)nk / 4.0 : (parts == 2 ? (double)nk * 9.0 / 16.0 : (double)nk);
    const double t_prefill = (parts == 4 ? 16.0 : 10.0) + (double)((units + 255) / 256) * steps * 1.45;
    return t_chunks < t_prefill;
}

bool gemm_skinny_applies(int64_t M, int64_t N, int64_t K)
{
    // buffer loads address the packed tensors with 32-bit offsets
    constexpr uint64_t kLimit = 0xFFFFFF00ull;
    if (M > kSkinnyMaxRows || make_layout(N, K).total_bytes >= kLimit || make_layout(M, K).total_bytes >= kLimit)
        return false;
    const int64_t n_chunks = (M + kSkChunkRows - 1) / kSkChunkRows;
    return n_chunks == 1 || chunks_beat_prefill_kernel(n_chunks, N, K);
}

int64_t gemm_skinny_x16_rows(int64_t M)
{
    return M <= 16 ? 16 : (M + kSkChunkRows - 1) / kSkChunkRows * kSkChunkRows;
}

// The arrival counters of a call must be zero when the kernels start: the caller clears
// gemm_skinny_counters(...) words in the kernel that prepares x16 (same stream).
SkinnyCounters gemm_skinny_counters(int64_t M, int64_t N, int64_t K, void *workspace)
{
    const SkinnyChunks c = skinny_chunks(M, N, K);
    return SkinnyCounters{reinterpret_cast<uint32_t *>(static_cast<char *>(workspace) + c.counters_begin),
                          (int64_t)c.n_counters};
}

fgmp_status_t gemm_skinny(const PackedHeader *xh, const PackedLayout &lx, const _Float16 *x16, int64_t ld16,
                          const void *w, const PackedLayout &lw, int64_t M, int64_t N, int64_t K, float *Y,
                          int64_t ldy, void *workspace, hipStream_t st)
{
    if (!gemm_skinny_applies(M, N, K)) return FGMP_ERR_UNSUPPORTED;
    const SkinnyChunks ch = skinny_chunks(M, N, K);
    char *ws = static_cast<char *>(workspace);
    if (!xh || !x16 || ld16 < lx.n_kt * kTileK || (uintptr_t)x16 % 16 != 0 || (ld16 * 2) % 16 != 0)
        return FGMP_ERR_BAD_SHAPE;
    for (int i = 0; i < ch.n; ++i) {
        const SkinnyPlan &p = ch.plan[i];
        if (p.row_groups * p.ksplit > 0x7FFFFFFF || p.off_counters - p.off_partial > 0x7FFFFFFFu)
            return FGMP_ERR_UNSUPPORTED;
    }
    for (int i = 0; i < ch.n; ++i) {
        const SkinnyPlan &p = ch.plan[i];
        const int64_t rows = ch.rows[i];
        SkinnyArgs a;
        a.w = w; a.xh = xh;
        a.x16 = x16 + i * kSkChunkRows * ld16; a.ld16 = ld16;
        a.w_rows = lw.rows; a.w_K = lw.K; a.x_rows = lx.rows; a.x_K = lx.K;
        a.off_L = (uint32_t)lw.off_L; a.off_S = (uint32_t)lw.off_S; a.off_M = (uint32_t)lw.off_M;
        a.off_T = (uint32_t)lw.off_T; a.off_H = (uint32_t)lw.off_H; a.n_tiles = (uint32_t)lw.n_tiles;
        a.n_kt = (int)lw.n_kt;
        a.cols_per_wg = p.cols_per_wg; a.ksplit = p.ksplit;
        a.partial = reinterpret_cast<float *>(ws + ch.off_partial[i]);
        a.partial_bytes = (uint32_t)(p.off_counters - p.off_partial);
        a.counters = reinterpret_cast<uint32_t *>(ws + ch.off_counters[i]);
        a.Y = Y + i * kSkChunkRows * ldy; a.ldy = ldy; a.M = rows; a.N = N;
        const dim3 grid((unsigned)(p.row_groups * p.ksplit));
        if (p.mt == 1 && rows <= 8) hipLaunchKernelGGL((gemm_skinny_kernel<1, 4, 8>), grid, dim3(256), 0, st, a);
        else if (p.mt == 1) hipLaunchKernelGGL((gemm_skinny_kernel<1, 4, 16>), grid, dim3(256), 0, st, a);
        else if (p.waves == 8) hipLaunchKernelGGL((gemm_skinny_kernel<2, 8, 32>), grid, dim3(512), 0, st, a);
        else hipLaunchKernelGGL((gemm_skinny_kernel<2, 16, 32>), grid, dim3(1024), 0, st, a);
        if (hipGetLastError() != hipSuccess) return FGMP_ERR_HIP;
    }
    return FGMP_OK;
}

}  // namespace fgmp
