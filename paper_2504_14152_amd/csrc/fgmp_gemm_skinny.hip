// Decode-shape (M <= 32 tokens) block-mixed-precision GEMM (Sec. 4.1): the
// packed weights are streamed from HBM exactly once and decoded in registers
// straight into MFMA operands; the few activation rows sit in LDS as FP16.
//
// Work split: a workgroup owns 64 weight rows (4 waves x 16 rows) and a range
// of at most 8 K-tiles (1024 K elements).  K ranges of one row group are
// combined deterministically: every workgroup stores its partial tile, and the
// last one to arrive adds the partials in K order and writes Y.
//
// Lane (nl = lane % 16, g = lane / 16) of a wave reads, per K-tile of 128, the
// 16 bytes that hold blocks 2g and 2g+1 of weight row nl -- a wave's load is
// 1 KB of consecutive plane-L bytes -- and decodes them into the B operands of
// four 16x16x32 MFMAs; MFMA j therefore reduces over the K elements
// 32 g + 8 j .. 32 g + 8 j + 7 (g = 0..3) of the tile, and the A operand is
// read from LDS with the same assignment.  The FP8 blocks' upper halves (plane
// H) of a tile are fetched speculatively, 32 entries per tile per wave, and
// handed to the lane that needs them with ds_bpermute.
#include <atomic>
#include <chrono>
#include <random>

#include "fgmp_gemm_common.hpp"

namespace fgmp {

typedef float float4_t __attribute__((ext_vector_type(4)));

constexpr int kSkRows = 64;       // weight rows per workgroup
constexpr int kSkMaxCols = 8;     // K-tiles per workgroup
constexpr int kSkPrefetch = 4;    // K-tiles in flight per wave
constexpr int kSkXPad = 8;        // halves of padding per LDS activation row
constexpr int kSkSpec = 32;       // plane-H entries fetched speculatively per tile

constexpr int kSkSumPass = 4;     // partial tiles summed per pass (their loads are in flight together)
constexpr int kSkMaxSplit = 16;   // most K ranges per row group the planner asks for

// 16-byte accesses to the partial-sum buffer that are coherent across XCDs: buffer instructions with
// the sc0 sc1 cache policy (system scope) bypass the per-XCD L2; being ordinary loads and stores,
// the compiler tracks their completion itself.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
constexpr int kCoherent = 1 | 16;   // sc0 | sc1
__device__ __forceinline__ void store_coherent16(__amdgpu_buffer_rsrc_t buf, uint32_t byte_off, float4_t v)
{
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, v), buf, (int)byte_off, 0, kCoherent);
}
__device__ __forceinline__ float4_t load_coherent16(__amdgpu_buffer_rsrc_t buf, uint32_t byte_off)
{
    return __builtin_bit_cast(float4_t, __builtin_amdgcn_raw_buffer_load_b128(buf, (int)byte_off, 0, kCoherent));
}

// Arrival counter of a row group that needs no clearing between calls: the word holds
// (epoch << 8) | count, and a value left by an earlier call (or never initialised) carries a
// different 56-bit epoch and is treated as zero.  Returns how many workgroups arrived before.
__device__ __forceinline__ uint32_t arrive(unsigned long long *ctr, unsigned long long epoch)
{
    unsigned long long old = __hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (;;) {
        const bool same = (old >> 8) == epoch;
        const unsigned long long want = same ? old + 1 : ((epoch << 8) | 1ull);
        if (__hip_atomic_compare_exchange_strong(ctr, &old, want, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_AGENT))
            return same ? (uint32_t)(old & 0xFFull) : 0u;
    }
}

struct SkinnyStage {
    uint4 l;       // blocks 2g, 2g+1 of this lane's row
    uint32_t s;    // their two scale-or-index bytes
    uint2 h;       // speculative plane-H entry (lane & 31) of tile (lane >> 5)
};

template <int MT>
__global__ __launch_bounds__(256) void gemm_skinny_kernel(PackedView W, PackedLayout lw, PackedView X,
                                                           PackedLayout lx, int cols_per_wg, int ksplit,
                                                           float *partial, uint32_t partial_bytes,
                                                           unsigned long long *counters, unsigned long long epoch,
                                                           float *Y, int64_t ldy, int64_t M, int64_t N)
{
    constexpr int kXRow = kSkMaxCols * kTileK + kSkXPad;
    __shared__ __attribute__((aligned(16))) _Float16 xs[16 * MT][kXRow];
    __shared__ uint32_t arrival;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t rg = blockIdx.x / ksplit;
    const int ks = blockIdx.x % ksplit;
    const int64_t c0 = (int64_t)ks * cols_per_wg;
    const int ncols = (int)((lw.n_kt - c0 < cols_per_wg) ? lw.n_kt - c0 : cols_per_wg);
    // The header is only used to zero the result of a mismatched operand; no load
    // address depends on it, so the stream starts without waiting for this load.
    const PackedHeader wh = *W.hdr;
    const PackedHeader xh = *X.hdr;

    const int nl = lane & 15, g = lane >> 4;
    const int64_t rtA = rg * (kSkRows / kTileRows) + wave * 2;   // the wave's two row-tiles: rtA, rtA + 1
    const int my_sel = nl >> 3;                        // which of the two this lane's weight row is in
    const int64_t my_rt = rtA + my_sel;
    const bool row_ok = my_rt < lw.n_rt;
    const int slot0 = (nl & 7) * kTileBlocks + 2 * g;  // slots of blocks 2g, 2g+1 within the tile
    const int spec_sel = lane >> 5, spec_e = lane & 31;
    const bool spec_ok = rtA + spec_sel < lw.n_rt;

    // Loads are unconditional (indices clamped into the buffer, results masked at
    // use) so that the number of loads in flight is known at compile time and a
    // consume step waits only for its own K-tile, not for the prefetches behind
    // it.  Everything whose address does not depend on another load goes first.
    const int64_t rt_ld = row_ok ? my_rt : 0;
    const int64_t spec_rt_ld = spec_ok ? rtA + spec_sel : 0;
    const uint64_t h_last = (uint64_t)lw.n_tiles * kTileSlots - 1;
    uint64_t mcol[kSkMaxCols];   // mask word of the lane's own tile, per K-tile
    uint32_t tcol[kSkMaxCols];   // plane-H offset of the lane's speculative tile, per K-tile
#pragma unroll
    for (int c = 0; c < kSkMaxCols; ++c) {
        const int cc = c < ncols ? c : ncols - 1;
        mcol[c] = W.M[rt_ld * lw.n_kt + c0 + cc];
        tcol[c] = W.T[spec_rt_ld * lw.n_kt + c0 + cc];
    }
    auto issue_ls = [&](int c, SkinnyStage &st) {
        const int cc = c < ncols ? c : ncols - 1;
        const int64_t tile = rt_ld * lw.n_kt + c0 + cc;
        st.l = *reinterpret_cast<const uint4 *>(&W.L[tile * kTileSlots + slot0]);
        st.s = *reinterpret_cast<const uint16_t *>(&W.S[tile * kTileSlots + slot0]);
    };
    auto issue_h = [&](int c, SkinnyStage &st) {
        const uint64_t hidx = (uint64_t)tcol[c] + spec_e;
        st.h = W.H[hidx < h_last ? hidx : h_last];
    };
    SkinnyStage ring[kSkPrefetch];
#pragma unroll
    for (int p = 0; p < kSkPrefetch; ++p) issue_ls(p, ring[p]);

    // activations of this K range: packed tiles (8 rows x 128 K, one block per lane) decoded straight
    // into LDS; 2 MT row-tiles x ncols K-tiles, spread over the 4 waves
    {
#pragma unroll
        for (int p = 0; p < kSkPrefetch; ++p) issue_h(p, ring[p]);
        const bool x_ok = xh.magic == kMagic && xh.rows == lx.rows && xh.K == lx.K;
        const int n_xt = 2 * MT * ncols;
        for (int i = wave; i < n_xt; i += 4) {
            const int xrt = i / ncols, xc = i % ncols;
            half2_t vals[8];
            if (xrt < lx.n_rt && x_ok) {
                decode_slot(X, (int64_t)xrt * lx.n_kt + c0 + xc, lane, vals);
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) vals[j] = half2_t{(_Float16)0.0f, (_Float16)0.0f};
            }
            const uint32_t *w = reinterpret_cast<const uint32_t *>(vals);
            uint4 *dst = reinterpret_cast<uint4 *>(&xs[xrt * kTileRows + (lane >> 3)][xc * kTileK + (lane & 7) * kBlock]);
            dst[0] = make_uint4(w[0], w[1], w[2], w[3]);
            dst[1] = make_uint4(w[4], w[5], w[6], w[7]);
        }
    }
    __syncthreads();

    float4_t acc[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) acc[i] = float4_t{0.0f, 0.0f, 0.0f, 0.0f};

    auto consume = [&](int c, const SkinnyStage &st) {
        if (c >= ncols) return;
        const uint64_t m = row_ok ? mcol[c] : 0ull;
        const uint4 lv = row_ok ? st.l : make_uint4(0, 0, 0, 0);
        const uint32_t sv = row_ok ? st.s : 0u;
        const uint32_t s0 = sv & 0xFFu, s1 = (sv >> 8) & 0xFFu;
        const bool hi0 = (m >> slot0) & 1ull, hi1 = (m >> (slot0 + 1)) & 1ull;
        // upper halves of FP8 blocks: entry s of the lane's tile sits in lane 32 * my_sel + s
        uint2 up0, up1;
        {
            const int a0 = (my_sel * kSkSpec + (int)(s0 & (kSkSpec - 1))) << 2;
            const int a1 = (my_sel * kSkSpec + (int)(s1 & (kSkSpec - 1))) << 2;
            up0.x = __builtin_amdgcn_ds_bpermute(a0, st.h.x);
            up0.y = __builtin_amdgcn_ds_bpermute(a0, st.h.y);
            up1.x = __builtin_amdgcn_ds_bpermute(a1, st.h.x);
            up1.y = __builtin_amdgcn_ds_bpermute(a1, st.h.y);
            // Tiles with more FP8 blocks than the speculative window: fetch directly.
            // Rare; the wait sits inside the branch so that the common path keeps
            // counting only its own prefetches.
            const bool far0 = hi0 && s0 >= (uint32_t)kSkSpec, far1 = hi1 && s1 >= (uint32_t)kSkSpec;
            if (__builtin_amdgcn_ballot_w64(far0 || far1) != 0ull) {
                const uint32_t tA = __builtin_amdgcn_readlane(tcol[c], 0), tB = __builtin_amdgcn_readlane(tcol[c], 32);
                const uint64_t my_t = my_sel ? tB : tA;
                if (far0) up0 = W.H[my_t + s0];
                if (far1) up1 = W.H[my_t + s1];
                __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
            }
        }
        half2_t b[16];   // b[4 j + i]: halves 2i, 2i+1 of MFMA j's operand
        if (hi0) {
            b[0] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(lv.x, 1.0f, false);
            b[1] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(lv.x, 1.0f, true);
            b[2] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(lv.y, 1.0f, false);
            b[3] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(lv.y, 1.0f, true);
            b[4] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(up0.x, 1.0f, false);
            b[5] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(up0.x, 1.0f, true);
            b[6] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(up0.y, 1.0f, false);
            b[7] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(up0.y, 1.0f, true);
        } else {
            const half2_t s = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(s0 | (s0 << 8), 1.0f, false);
            b[0] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lv.x, 1.0f, 0) * s;
            b[1] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lv.x, 1.0f, 1) * s;
            b[2] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lv.x, 1.0f, 2) * s;
            b[3] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lv.x, 1.0f, 3) * s;
            b[4] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lv.y, 1.0f, 0) * s;
            b[5] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lv.y, 1.0f, 1) * s;
            b[6] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lv.y, 1.0f, 2) * s;
            b[7] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lv.y, 1.0f, 3) * s;
        }
        if (hi1) {
            b[8] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(lv.z, 1.0f, false);
            b[9] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(lv.z, 1.0f, true);
            b[10] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(lv.w, 1.0f, false);
            b[11] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(lv.w, 1.0f, true);
            b[12] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(up1.x, 1.0f, false);
            b[13] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(up1.x, 1.0f, true);
            b[14] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(up1.y, 1.0f, false);
            b[15] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(up1.y, 1.0f, true);
        } else {
            const half2_t s = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(s1 | (s1 << 8), 1.0f, false);
            b[8] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lv.z, 1.0f, 0) * s;
            b[9] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lv.z, 1.0f, 1) * s;
            b[10] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lv.z, 1.0f, 2) * s;
            b[11] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lv.z, 1.0f, 3) * s;
            b[12] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lv.w, 1.0f, 0) * s;
            b[13] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lv.w, 1.0f, 1) * s;
            b[14] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lv.w, 1.0f, 2) * s;
            b[15] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(lv.w, 1.0f, 3) * s;
        }
        const half8_t *bv = reinterpret_cast<const half8_t *>(b);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const half8_t a = *reinterpret_cast<const half8_t *>(&xs[mt * 16 + nl][c * kTileK + 32 * g + 8 * j]);
                acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, bv[j], acc[mt], 0, 0, 0);
            }
        }
    };

#pragma unroll
    for (int c = 0; c < kSkMaxCols; ++c) {
        consume(c, ring[c % kSkPrefetch]);
        if (c + kSkPrefetch < kSkMaxCols) {
            issue_ls(c + kSkPrefetch, ring[c % kSkPrefetch]);
            issue_h(c + kSkPrefetch, ring[c % kSkPrefetch]);
        }
    }

    // acc[mt][r] = partial Y[m = 16 mt + 4 (lane / 16) + r][n = 64 rg + 16 wave + lane % 16]
    const bool w_ok = wh.magic == kMagic && wh.rows == lw.rows && wh.K == lw.K;
    const float ss = w_ok ? xh.tensor_scale * wh.tensor_scale : 0.0f;
    const int n_local = wave * 16 + nl;
    if (ksplit == 1) {
        const int64_t n = rg * kSkRows + n_local;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int64_t m = mt * 16 + 4 * g + r;
                if (m < M && n < N) Y[m * ldy + n] = acc[mt][r] * ss;
            }
        return;
    }
    // Partial tile layout: [n_local (64)][m (16 MT)], so a lane's four accumulators of one MFMA tile
    // (rows 4g .. 4g+3 of column n_local) are 16 contiguous bytes.  Partials and the arrival counter
    // cross XCDs: they are written and read with system-coherent vector accesses (sc0 sc1), which
    // bypass the per-XCD L2, and the stores are waited for before the counter is bumped, so no cache
    // write-back or invalidate is needed.
    constexpr uint32_t kTileBytes32 = kSkRows * (16 * MT) * 4;   // bytes of one partial tile
    const __amdgpu_buffer_rsrc_t pbuf =
        __builtin_amdgcn_make_buffer_rsrc(partial, 0, (int)partial_bytes, 0x00020000);
    const uint32_t mine = (uint32_t)blockIdx.x * kTileBytes32;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
        store_coherent16(pbuf, mine + (uint32_t)(n_local * (16 * MT) + mt * 16 + 4 * g) * 4u, acc[mt]);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (tid == 0) arrival = arrive(&counters[rg], epoch);
    __syncthreads();
    if (arrival != (uint32_t)(ksplit - 1)) return;
    // last workgroup of this row group: add the partials in K order, 4 rows of one column per thread
    const uint32_t first = (uint32_t)(rg * ksplit) * kTileBytes32;
    constexpr int kVecs = kSkRows * (16 * MT) / 4;   // 16-byte vectors per partial tile
    for (int i = tid; i < kVecs; i += 256) {
        float4_t sum = float4_t{0.0f, 0.0f, 0.0f, 0.0f};
        for (int k0 = 0; k0 < ksplit; k0 += kSkSumPass) {
            float4_t part[kSkSumPass];
#pragma unroll
            for (int k = 0; k < kSkSumPass; ++k) {
                const int kk = k0 + k < ksplit ? k0 + k : ksplit - 1;
                part[k] = load_coherent16(pbuf, first + (uint32_t)kk * kTileBytes32 + (uint32_t)i * 16u);
            }
#pragma unroll
            for (int k = 0; k < kSkSumPass; ++k)
                if (k0 + k < ksplit) sum += part[k];
        }
        const int64_t n = rg * kSkRows + i / (4 * MT);
        const int64_t m0 = (i % (4 * MT)) * 4;
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (m0 + r < M && n < N) Y[(m0 + r) * ldy + n] = sum[r] * ss;
    }
}

// ---- host side ----

struct SkinnyPlan {
    int mt, cols_per_wg, ksplit;
    int64_t row_groups;
    size_t off_partial, off_counters, total;
};

static SkinnyPlan skinny_plan(int64_t M, int64_t N, int64_t K)
{
    SkinnyPlan p;
    const PackedLayout lw = make_layout(N, K);
    p.mt = M <= 16 ? 1 : 2;
    p.row_groups = (N + kSkRows - 1) / kSkRows;
    // about three workgroups per CU, at most 8 K-tiles each
    int64_t want = (768 + p.row_groups - 1) / p.row_groups;
    int max_cols = kSkMaxCols;
    const int64_t need = (lw.n_kt + max_cols - 1) / max_cols;
    if (want < need) want = need;
    if (want > kSkMaxSplit) want = kSkMaxSplit;
    if (want < need) want = need;   // long K: more ranges than one summing pass, still correct
    if (want > lw.n_kt) want = lw.n_kt;
    p.cols_per_wg = (int)((lw.n_kt + want - 1) / want);
    p.ksplit = (int)((lw.n_kt + p.cols_per_wg - 1) / p.cols_per_wg);
    p.off_partial = 0;
    p.off_counters = (size_t)align_up((uint64_t)p.row_groups * p.ksplit * (16 * p.mt) * kSkRows * 4, 256);
    p.total = p.off_counters + (size_t)align_up((uint64_t)p.row_groups * 8, 256);
    return p;
}

size_t gemm_skinny_workspace_bytes(int64_t M, int64_t N, int64_t K) { return skinny_plan(M, N, K).total; }

// A fresh 56-bit tag per call for the arrival counters (see arrive()).
static unsigned long long next_epoch()
{
    static std::atomic<unsigned long long> counter{[] {
        std::random_device rd;
        return ((unsigned long long)rd() << 32) ^ rd() ^ (unsigned long long)std::chrono::steady_clock::now().time_since_epoch().count();
    }()};
    return counter.fetch_add(1) & ((1ull << 56) - 1);
}

fgmp_status_t gemm_skinny(const PackedView &X, const PackedLayout &lx, const PackedView &W, const PackedLayout &lw,
                          int64_t M, int64_t N, int64_t K, float *Y, int64_t ldy, void *workspace, hipStream_t st)
{
    const SkinnyPlan p = skinny_plan(M, N, K);
    char *ws = static_cast<char *>(workspace);
    float *partial = reinterpret_cast<float *>(ws + p.off_partial);
    unsigned long long *counters = reinterpret_cast<unsigned long long *>(ws + p.off_counters);
    const size_t partial_bytes = p.off_counters - p.off_partial;
    if (p.row_groups * p.ksplit > 0x7FFFFFFF || partial_bytes > 0x7FFFFFFFu || p.ksplit > 255)
        return FGMP_ERR_UNSUPPORTED;
    const unsigned long long epoch = next_epoch();
    const dim3 grid((unsigned)(p.row_groups * p.ksplit));
    if (p.mt == 1)
        hipLaunchKernelGGL((gemm_skinny_kernel<1>), grid, dim3(256), 0, st, W, lw, X, lx, p.cols_per_wg, p.ksplit,
                           partial, (uint32_t)partial_bytes, counters, epoch, Y, ldy, M, N);
    else
        hipLaunchKernelGGL((gemm_skinny_kernel<2>), grid, dim3(256), 0, st, W, lw, X, lx, p.cols_per_wg, p.ksplit,
                           partial, (uint32_t)partial_bytes, counters, epoch, Y, ldy, M, N);
    return hipGetLastError() == hipSuccess ? FGMP_OK : FGMP_ERR_HIP;
}

}  // namespace fgmp
