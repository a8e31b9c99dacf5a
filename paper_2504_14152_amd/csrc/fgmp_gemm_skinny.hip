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
#include "fgmp_internal.hpp"

namespace fgmp {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));

constexpr int kSkRows = 64;       // weight rows per workgroup
constexpr int kSkMaxCols = 8;     // K-tiles per workgroup
constexpr int kSkPrefetch = 4;    // K-tiles in flight per wave
constexpr int kSkXPad = 8;        // halves of padding per LDS activation row
constexpr int kSkSpec = 32;       // plane-H entries fetched speculatively per tile

struct SkinnyStage {
    uint4 l;       // blocks 2g, 2g+1 of this lane's row
    uint32_t s;    // their two scale-or-index bytes
    uint2 h;       // speculative plane-H entry (lane & 31) of tile (lane >> 5)
};

template <int MT>
__global__ __launch_bounds__(256) void gemm_skinny_kernel(PackedView W, PackedLayout lw, const _Float16 *Xh,
                                                           int64_t ldx, int cols_per_wg, int ksplit,
                                                           float *partial, uint32_t *counters, float *Y,
                                                           int64_t ldy, int64_t M, int64_t N,
                                                           const PackedHeader *hx)
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
    const float sx = hx->tensor_scale;

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

    // activations of this K range -> LDS through registers (all loads first)
    {
        constexpr int kChunksPerRow = kSkMaxCols * (kTileK / 8);   // 128 chunks of 16 B
        constexpr int kIters = 16 * MT * kChunksPerRow / 256;
        uint4 xr[kIters];
#pragma unroll
        for (int it = 0; it < kIters; ++it) {
            const int i = tid + 256 * it, m = i / kChunksPerRow, ch = i % kChunksPerRow;
            const int chc = ch < ncols * (kTileK / 8) ? ch : 0;
            xr[it] = *reinterpret_cast<const uint4 *>(Xh + (int64_t)m * ldx + c0 * kTileK + chc * 8);
        }
#pragma unroll
        for (int p = 0; p < kSkPrefetch; ++p) issue_h(p, ring[p]);
#pragma unroll
        for (int it = 0; it < kIters; ++it) {
            const int i = tid + 256 * it, m = i / kChunksPerRow, ch = i % kChunksPerRow;
            if (ch < ncols * (kTileK / 8)) *reinterpret_cast<uint4 *>(&xs[m][ch * 8]) = xr[it];
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
    const float ss = w_ok ? sx * wh.tensor_scale : 0.0f;
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
    float *mine = partial + ((int64_t)blockIdx.x * (16 * MT)) * kSkRows;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 4; ++r)
            __hip_atomic_store(&mine[(mt * 16 + 4 * g + r) * kSkRows + n_local], acc[mt][r], __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
    // Partials and the arrival counter are written and read with agent-scope
    // atomics, which bypass the per-XCD caches; waiting for the stores to
    // complete before the counter is bumped orders them without a cache
    // write-back.
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (tid == 0)
        arrival = __hip_atomic_fetch_add(&counters[rg], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (arrival != (uint32_t)(ksplit - 1)) return;
    // last workgroup of this row group: add the partials in K order
    const float *first = partial + (rg * ksplit * (16 * MT)) * kSkRows;
    for (int i = tid; i < 16 * MT * kSkRows; i += 256) {
        const int64_t m = i / kSkRows, n = rg * kSkRows + i % kSkRows;
        float sum = 0.0f;
        for (int k = 0; k < ksplit; ++k)
            sum += __hip_atomic_load(&first[(int64_t)k * (16 * MT) * kSkRows + i], __ATOMIC_RELAXED,
                                     __HIP_MEMORY_SCOPE_AGENT);
        if (m < M && n < N) Y[m * ldy + n] = sum * ss;
    }
}

// ---- host side ----

struct SkinnyPlan {
    int mt, cols_per_wg, ksplit;
    int64_t row_groups, ldx;
    size_t off_x, off_partial, off_counters, total;
};

static SkinnyPlan skinny_plan(int64_t M, int64_t N, int64_t K)
{
    SkinnyPlan p;
    const PackedLayout lw = make_layout(N, K);
    p.mt = M <= 16 ? 1 : 2;
    p.row_groups = (N + kSkRows - 1) / kSkRows;
    p.ldx = lw.n_kt * kTileK;
    // about three workgroups per CU, at most 8 K-tiles each
    int64_t want = (768 + p.row_groups - 1) / p.row_groups;
    const int64_t need = (lw.n_kt + kSkMaxCols - 1) / kSkMaxCols;
    if (want < need) want = need;
    if (want > lw.n_kt) want = lw.n_kt;
    p.cols_per_wg = (int)((lw.n_kt + want - 1) / want);
    p.ksplit = (int)((lw.n_kt + p.cols_per_wg - 1) / p.cols_per_wg);
    p.off_x = 0;
    p.off_partial = (size_t)align_up((uint64_t)(16 * p.mt) * p.ldx * 2, 256);
    p.off_counters = p.off_partial +
                     (size_t)align_up((uint64_t)p.row_groups * p.ksplit * (16 * p.mt) * kSkRows * 4, 256);
    p.total = p.off_counters + (size_t)align_up((uint64_t)p.row_groups * 4, 256);
    return p;
}

size_t gemm_skinny_workspace_bytes(int64_t M, int64_t N, int64_t K) { return skinny_plan(M, N, K).total; }

fgmp_status_t gemm_skinny(const PackedView &X, const PackedLayout &lx, const PackedView &W, const PackedLayout &lw,
                          int64_t M, int64_t N, int64_t K, float *Y, int64_t ldy, void *workspace, hipStream_t st)
{
    const SkinnyPlan p = skinny_plan(M, N, K);
    char *ws = static_cast<char *>(workspace);
    _Float16 *xh = reinterpret_cast<_Float16 *>(ws + p.off_x);
    float *partial = reinterpret_cast<float *>(ws + p.off_partial);
    uint32_t *counters = reinterpret_cast<uint32_t *>(ws + p.off_counters);
    if (p.row_groups * p.ksplit > 0x7FFFFFFF) return FGMP_ERR_UNSUPPORTED;
    const int64_t n_rt_pad = (16 * p.mt) / kTileRows;
    // one launch decodes the activations and clears the arrival counters
    const DecodeJob jx = make_decode_job(X, lx, xh, p.ldx, n_rt_pad);
    const fgmp_status_t rc = launch_decode_f16(jx, nullptr, counters, p.ksplit > 1 ? p.row_groups : 0, st);
    if (rc != FGMP_OK) return rc;
    const dim3 grid((unsigned)(p.row_groups * p.ksplit));
    if (p.mt == 1)
        hipLaunchKernelGGL((gemm_skinny_kernel<1>), grid, dim3(256), 0, st, W, lw, xh, p.ldx, p.cols_per_wg,
                           p.ksplit, partial, counters, Y, ldy, M, N, X.hdr);
    else
        hipLaunchKernelGGL((gemm_skinny_kernel<2>), grid, dim3(256), 0, st, W, lw, xh, p.ldx, p.cols_per_wg,
                           p.ksplit, partial, counters, Y, ldy, M, N, X.hdr);
    return hipGetLastError() == hipSuccess ? FGMP_OK : FGMP_ERR_HIP;
}

}  // namespace fgmp
