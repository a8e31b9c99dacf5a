// Prefill GEMM with the weight operand decoded inside the kernel (Sec. 4.1):
// A = activations already expanded to FP16 (small: M x K), fetched by direct
// global->LDS loads; B = packed FGMP weights, read as plane-L/S/M/T/H bytes,
// decoded per block by the workgroup's threads according to the block's
// metadata bit, and written to LDS in the MFMA operand layout.  Compared with
// expanding W to FP16 in memory first, the kernel pulls 0.6 instead of 2 bytes
// per weight through the cache hierarchy and the expansion pass disappears.
//
// Thread t of the 512 owns weight row t / 2 of the 256-row tile and, per
// 64-wide K-step, the two blocks 2 (t % 2), 2 (t % 2) + 1: one 16-byte load
// from plane L, two scale-or-index bytes, the tile's mask word and plane-H
// offset.  Loads run two K-steps ahead in registers (plane-H entries one step
// ahead, since their address needs the mask and index bytes); every load is
// unconditional, so outstanding loads can be counted at compile time.
#include "fgmp_gemm_common.hpp"

namespace fgmp {

struct BRegs {
    uint4 l;       // plane L: two adjacent blocks
    uint32_t s;    // plane S: their two bytes
    uint64_t m;    // plane M word of the tile
    uint32_t t;    // plane T entry of the tile
};

template <int kWM, int kWN>
__global__ __launch_bounds__(kWM *kWN * 64, 1) void gemm_mixed_kernel(const _Float16 *__restrict__ A, int64_t ld,
                                                                       PackedView W, PackedLayout lw, int nk,
                                                                       float *__restrict__ Y, int64_t ldy, int64_t M,
                                                                       int64_t N, int64_t n_tm, int64_t n_tn,
                                                                       const PackedHeader *ha)
{
    constexpr int kWaves = kWM * kWN;
    static_assert(kWaves == 8, "the weight decode assigns two blocks per K-step to each of 512 threads");
    constexpr int TM = kBM / (32 * kWM), TN = kBN / (32 * kWN);
    constexpr int kLoads = 32 / kWaves;
    __shared__ __attribute__((aligned(1024))) char lds[2][2][kTileBytes];   // [stage][operand]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / kWN, wn = wave % kWN;
    int64_t tm, tn;
    tile_coords(n_tm, n_tn, tm, tn);

    // ---- A: direct global -> LDS, chunk swizzle applied on the global side ----
    const int lr = lane >> 3, lc = (lane & 7) ^ (((wave * 8 + lr) >> 1) & 7);
    const char *ga = reinterpret_cast<const char *>(A + (tm * kBM + wave * 8 + lr) * ld) + lc * 16;
    const int64_t row_step = kWaves * 8 * ld * 2;
    auto issue_a = [&](int kt, int stage) {
#pragma unroll
        for (int i = 0; i < kLoads; ++i)
            __builtin_amdgcn_global_load_lds((global_void_t *)(ga + i * row_step + (int64_t)kt * kRowBytes),
                                             (lds_void_t *)&lds[stage][0][(kWaves * i + wave) * 1024], 16, 0, 0);
    };

    // ---- B: packed weights through registers ----
    const int br = tid >> 1, bp = tid & 1;
    const int64_t row_b = tn * kBN + br;
    const bool b_ok = (row_b >> 3) < lw.n_rt;
    const int64_t rt_b = b_ok ? (row_b >> 3) : lw.n_rt - 1;   // rows beyond the tensor read a valid tile, are zeroed
    const int r8 = (int)(row_b & 7);
    const int swz_b = (br >> 1) & 7;
    const int last_kt = nk - 1;
    auto slot_of = [&](int kt) { return r8 * kTileBlocks + (kt & 1) * 4 + 2 * bp; };
    auto load_b = [&](int kt, BRegs &b) {
        kt = kt < last_kt ? kt : last_kt;
        const int64_t tile = rt_b * lw.n_kt + (kt >> 1);
        const int64_t slot = tile * kTileSlots + slot_of(kt);
        b.l = *reinterpret_cast<const uint4 *>(&W.L[slot]);
        b.s = *reinterpret_cast<const uint16_t *>(&W.S[slot]);
        b.m = W.M[tile];
        b.t = W.T[tile];
    };
    auto load_h = [&](int kt, const BRegs &b, uint2 (&h)[2]) {
        kt = kt < last_kt ? kt : last_kt;
        const int s0 = slot_of(kt);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const bool hi = (b.m >> (s0 + j)) & 1ull;
            const uint64_t idx = hi ? (uint64_t)b.t + ((b.s >> (8 * j)) & 0xFFu) : 0ull;
            h[j] = W.H[idx];
        }
    };
    auto decode_store = [&](int kt, const BRegs &b, const uint2 (&h)[2], int stage, int j) {
        kt = kt < last_kt ? kt : last_kt;
        const int s0 = slot_of(kt);
        char *row = &lds[stage][1][br * kRowBytes];
        {
            const bool hi = (b.m >> (s0 + j)) & 1ull;
            const uint32_t w0 = j ? b.l.z : b.l.x, w1 = j ? b.l.w : b.l.y;
            half2_t v[8];
            if (hi) {
                v[0] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w0, 1.0f, false);
                v[1] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w0, 1.0f, true);
                v[2] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w1, 1.0f, false);
                v[3] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w1, 1.0f, true);
                v[4] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(h[j].x, 1.0f, false);
                v[5] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(h[j].x, 1.0f, true);
                v[6] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(h[j].y, 1.0f, false);
                v[7] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(h[j].y, 1.0f, true);
            } else {
                const uint32_t sb = (b.s >> (8 * j)) & 0xFFu;
                const half2_t sc = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(sb | (sb << 8), 1.0f, false);
                v[0] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w0, 1.0f, 0) * sc;
                v[1] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w0, 1.0f, 1) * sc;
                v[2] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w0, 1.0f, 2) * sc;
                v[3] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w0, 1.0f, 3) * sc;
                v[4] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w1, 1.0f, 0) * sc;
                v[5] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w1, 1.0f, 1) * sc;
                v[6] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w1, 1.0f, 2) * sc;
                v[7] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w1, 1.0f, 3) * sc;
            }
            uint32_t o[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) o[i] = b_ok ? __builtin_bit_cast(uint32_t, v[i]) : 0u;
            const int c = 2 * (2 * bp + j);   // the block's two 16-byte chunks within the 128-byte row
            *reinterpret_cast<uint4 *>(row + ((c ^ swz_b) << 4)) = make_uint4(o[0], o[1], o[2], o[3]);
            *reinterpret_cast<uint4 *>(row + (((c + 1) ^ swz_b) << 4)) = make_uint4(o[4], o[5], o[6], o[7]);
        }
    };

    float16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    int frag_off[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
        frag_off[kk] = (lane & 31) * kRowBytes + (((2 * kk + (lane >> 5)) ^ ((lane >> 1) & 7)) << 4);
    auto read_frags = [&](int stage, int kk, half8_t (&a)[TM], half8_t (&b)[TN]) {
        const char *la = &lds[stage][0][wm * (TM * 32) * kRowBytes], *lb = &lds[stage][1][wn * (TN * 32) * kRowBytes];
#pragma unroll
        for (int i = 0; i < TM; ++i) a[i] = *reinterpret_cast<const half8_t *>(la + i * 32 * kRowBytes + frag_off[kk]);
#pragma unroll
        for (int j = 0; j < TN; ++j) b[j] = *reinterpret_cast<const half8_t *>(lb + j * 32 * kRowBytes + frag_off[kk]);
    };
    auto mfma_block = [&](const half8_t (&a)[TM], const half8_t (&b)[TN]) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], acc[i][j], 0, 0, 0);
    };
    constexpr int kReads = TM + TN, kMfma = TM * TN;

    // ---- prologue: K-step 0 decoded into stage 0; K-step 1 ready in registers; K-step 2 in flight ----
    BRegs cur, nxt, far;
    uint2 hcur[2], hnxt[2];
    issue_a(0, 0);
    issue_a(nk > 1 ? 1 : 0, 1);
    load_b(0, cur);
    load_h(0, cur, hcur);
    decode_store(0, cur, hcur, 0, 0);
    decode_store(0, cur, hcur, 0, 1);
    load_b(1, cur);
    load_h(1, cur, hcur);
    load_b(2, nxt);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    half8_t fa[2][TM], fb[2][TN];
    read_frags(0, 0, fa[0], fb[0]);
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0)

    // Iteration kt multiplies K-step kt (stage kt & 1) and, before its barrier,
    // decodes K-step kt + 1 into the other stage; after the barrier that stage is
    // readable and the stage just consumed takes the A loads of K-step kt + 2.
    for (int kt = 0; kt < nk; ++kt) {
        const int st = kt & 1;
        load_b(kt + 3, far);            // 4 register loads ...
        load_h(kt + 2, nxt, hnxt);      // ... + 2: the only loads younger than the A loads at this iteration's barrier
        read_frags(st, 1, fa[1], fb[1]);
        mfma_block(fa[0], fb[0]);
        // fragment reads first, then one weight load per MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, kReads, 0);
#pragma unroll
        for (int g = 0; g < 6; ++g) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, kMfma - 6, 0);
        __builtin_amdgcn_sched_barrier(0);
        decode_store(kt + 1, cur, hcur, st ^ 1, 0);
        decode_store(kt + 1, cur, hcur, st ^ 1, 1);
        read_frags(st, 2, fa[0], fb[0]);
        mfma_block(fa[1], fb[1]);
        // fragment reads first, then the decode arithmetic spread between the MFMAs
        __builtin_amdgcn_sched_group_barrier(0x100, kReads, 0);
#pragma unroll
        for (int g = 0; g < kMfma; ++g) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 10, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x200, 4, 0);
        __builtin_amdgcn_sched_barrier(0);
        read_frags(st, 3, fa[1], fb[1]);
        mfma_block(fa[0], fb[0]);
        order_phase<kReads, kMfma, 0>();
        // LDS traffic of this wave done (lgkmcnt 0) and its A loads landed: they are older than this
        // iteration's six register loads, which may stay in flight (vmcnt 6)
        __builtin_amdgcn_s_waitcnt(0x0076);
        __syncthreads();
        issue_a(kt + 2 < nk ? kt + 2 : nk - 1, st);
        read_frags(st ^ 1, 0, fa[0], fb[0]);
        mfma_block(fa[1], fb[1]);
        order_phase<kReads, kMfma, kLoads / 2>();
        __builtin_amdgcn_s_waitcnt(0xC07F);
        cur = nxt;
        hcur[0] = hnxt[0];
        hcur[1] = hnxt[1];
        nxt = far;
    }
    __builtin_amdgcn_s_waitcnt(0);

    const bool w_ok = W.hdr->magic == kMagic && W.hdr->rows == lw.rows && W.hdr->K == lw.K;
    const float ss = w_ok ? ha->tensor_scale * W.hdr->tensor_scale : 0.0f;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int64_t col = tn * kBN + wn * (TN * 32) + j * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = tm * kBM + wm * (TM * 32) + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (row < M && col < N) Y[row * ldy + col] = acc[i][j][r] * ss;
            }
        }
}

void launch_gemm_mixed(const _Float16 *a16, int64_t ld, const PackedView &W, const PackedLayout &lw, float *Y,
                       int64_t ldy, int64_t M, int64_t N, int64_t n_tm, int64_t n_tn, const PackedHeader *ha,
                       hipStream_t st)
{
    hipLaunchKernelGGL((gemm_mixed_kernel<2, 4>), dim3((unsigned)(n_tm * n_tn)), dim3(512), 0, st, a16, ld, W, lw,
                       (int)(ld / kBK), Y, ldy, M, N, n_tm, n_tn, ha);
}

}  // namespace fgmp
