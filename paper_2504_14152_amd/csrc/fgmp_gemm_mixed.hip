// Prefill GEMM with the weight operand decoded inside the kernel (Sec. 4.1):
// A = activations already expanded to FP16 (small: M x K), fetched by direct
// global->LDS loads; B = packed FGMP weights, read as plane-L/S/M/T/H bytes,
// decoded per block by the workgroup's threads according to the block's
// metadata bit, and written to LDS in the MFMA operand layout.  Compared with
// expanding W to FP16 in memory first, the kernel pulls 0.6 instead of 2 bytes
// per weight through the cache hierarchy and the expansion pass disappears.
//
// Each pair of the 512 threads owns one weight row of the 256-row tile; a
// thread handles, per 64-wide K-step, the two blocks 2 (t % 2), 2 (t % 2) + 1:
// one 16-byte load from plane L, two scale-or-index bytes, the row's half of
// the tile's mask word and the tile's plane-H offset.  The small fields are
// loaded three K-steps before their blocks are multiplied, plane L and the
// plane-H entries (whose addresses need the small fields) two, and the decode
// into LDS runs one step ahead; every load is unconditional, so outstanding
// loads can be counted at compile time.
//
// All memory loads of the main loop are written as assembly with hand-counted
// waits.  The compiler files a global->LDS load under a different event class
// than an ordinary load and, while both classes are pending, turns every wait
// for a loaded register into vmcnt(0): a full memory round trip in every
// K-step, because a load has always just been issued.  Loads complete in issue
// order, so a wait only has to count the loads issued after the one it needs;
// the register sets rotate by index (the loop body is instantiated for one
// whole turn of the rotation), so a register that a load in flight will write
// is never copied.
//
// One workgroup computes one 256 x 256 output tile over all of K -- except the
// tiles of a last round that fills at most half of the chip: those are
// computed by two (at most a quarter: four) workgroups each, over
// complementary K ranges, which meet pairwise through the workspace after
// their loops (see SplitTail).
#include <type_traits>

#include "fgmp_elementwise.hpp"
#include "fgmp_gemm_common.hpp"
#include "fgmp_quant_block.hpp"

namespace fgmp {

typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

// Per thread and K-step: the plane-L words (needed when the step is decoded) and the small fields
// (needed one step earlier, for the plane-H addresses).
template <int kBPT> struct LRegs {
    u32x4_t l[kBPT / 2];   // plane L: kBPT adjacent blocks
};
struct MetaRegs {
    uint32_t s;            // plane S: the blocks' bytes
    uint32_t m;            // the half of the tile's plane-M word that holds the thread's row
    uint32_t t;            // plane T entry of the tile
};

// Buffer loads (range-checked: out-of-range lanes read zero) with a per-lane byte offset, a uniform
// byte offset and an immediate one.  The destination holds the data only after a later
// wait_loaded<>() that names it; until then the register must not be read.
template <int kImm> __device__ __forceinline__ void load_b128(u32x4_t &d, __amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff)
{
    asm volatile("buffer_load_dwordx4 %0, %1, %2, %3 offen offset:%4" : "=v"(d) : "v"(voff), "s"(r), "s"(soff), "n"(kImm));
}
__device__ __forceinline__ void load_b64(u32x2_t &d, __amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff)
{
    asm volatile("buffer_load_dwordx2 %0, %1, %2, %3 offen" : "=v"(d) : "v"(voff), "s"(r), "s"(soff));
}
__device__ __forceinline__ void load_b32(uint32_t &d, __amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff)
{
    asm volatile("buffer_load_dword %0, %1, %2, %3 offen" : "=v"(d) : "v"(voff), "s"(r), "s"(soff));
}
__device__ __forceinline__ void load_b16(uint32_t &d, __amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff)
{
    asm volatile("buffer_load_ushort %0, %1, %2, %3 offen" : "=v"(d) : "v"(voff), "s"(r), "s"(soff));
}
// Wait until at most kPending loads are outstanding; the named registers count as written here, so
// no use of them can move above the wait.  A build with FGMP_FULL_WAITS waits for every load instead
// (kPending = 0 everywhere): same instructions, same summation order, no counting to get wrong -- the
// library a test compares this one with, bit for bit.
#ifdef FGMP_FULL_WAITS
constexpr int pending(int) { return 0; }
#else
constexpr int pending(int n) { return n; }
#endif
template <int kPending, int kBPT> __device__ __forceinline__ void wait_loaded(LRegs<kBPT> &b)
{
    if constexpr (kBPT == 2) asm volatile("s_waitcnt vmcnt(%1)" : "+v"(b.l[0]) : "n"(pending(kPending)));
    else asm volatile("s_waitcnt vmcnt(%2)" : "+v"(b.l[0]), "+v"(b.l[1]) : "n"(pending(kPending)));
}
template <int kPending> __device__ __forceinline__ void wait_loaded(MetaRegs &b)
{
    asm volatile("s_waitcnt vmcnt(%3)" : "+v"(b.s), "+v"(b.m), "+v"(b.t) : "n"(pending(kPending)));
}
template <int kPending, int kBPT> __device__ __forceinline__ void wait_loaded(u32x2_t (&h)[kBPT])
{
    if constexpr (kBPT == 2) asm volatile("s_waitcnt vmcnt(%2)" : "+v"(h[0]), "+v"(h[1]) : "n"(pending(kPending)));
    else asm volatile("s_waitcnt vmcnt(%4)" : "+v"(h[0]), "+v"(h[1]), "+v"(h[2]), "+v"(h[3]) : "n"(pending(kPending)));
}

// kPackOut: instead of storing FP32 results, the epilogue scores and quantizes them block by block (16
// consecutive output columns) and writes a packed tensor -- the placement of the quantization unit in
// the paper (Sec. 4.2): results are quantized before they leave for memory.  kGate (with kPackOut): the
// weight rows come in groups of 32 gate rows and 32 up rows, and what is quantized is
// SiLU(gate result) * up result, half as many columns.
template <int kWM, int kWN, bool kPackOut, bool kGate>
__global__ __launch_bounds__(kWM *kWN * 64, 1) void gemm_mixed_kernel(const _Float16 *__restrict__ A, int64_t ld,
                                                                       PackedView W, PackedLayout lw, int nk_total,
                                                                       float *__restrict__ Y, int64_t ldy, int64_t M,
                                                                       int64_t N, int64_t n_tm, int64_t n_tn,
                                                                       const PackedHeader *ha, PackOut po, SplitTail sp)
{
    constexpr int kWaves = kWM * kWN;
    static_assert(kWaves == 8 || kWaves == 4, "the weight decode assigns 2 (512 threads) or 4 (256 threads) blocks per K-step to a thread");
    constexpr int kBPT = 16 / kWaves;             // weight blocks per thread and K-step
    constexpr int kBLoads = kBPT / 2 + 3 + kBPT;  // register loads per K-step: plane L, S, M, T, plane H
    typedef LRegs<kBPT> LRegsT;
    constexpr int TM = kBM / (32 * kWM), TN = kBN / (32 * kWN);
    constexpr int kLoads = 32 / kWaves;
    __shared__ __attribute__((aligned(1024))) char lds[2][2][kTileBytes];   // [stage][operand]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / kWN, wn = wave % kWN;
    // Workgroups [0, n_whole) compute one tile each over all of K.  The tiles beyond -- a last, partly
    // filled round of the chip -- are split in n_parts along K: workgroup n_whole + u takes tile
    // n_whole + u % n_split and part u / n_split of its K-steps.
    int64_t tm, tn;
    const int unit = (int)blockIdx.x - sp.n_whole;
    const bool split = unit >= 0;
    const int split_tile = split ? unit % sp.n_split : 0, part = split ? unit / sp.n_split : 0;
    tile_coords(split ? sp.n_whole + split_tile : (int64_t)blockIdx.x, n_tm, n_tn, tm, tn);
    const int kt0 = split ? sp.kt_bound[part] : 0;                          // first K-step of this workgroup
    const int nk = split ? sp.kt_bound[part + 1] - kt0 : nk_total;          // and how many

    // ---- A: direct global -> LDS, chunk swizzle applied on the global side.  The address is a uniform
    // base (tile row, K-step) plus a per-lane 32-bit offset that never changes, so the loop spends no
    // vector instructions on it. ----
    const int lr = lane >> 3, lc = (lane & 7) ^ (((wave * 8 + lr) >> 1) & 7);
    const char *a_tile = reinterpret_cast<const char *>(A + tm * kBM * ld) + (int64_t)kt0 * kRowBytes;
    const uint32_t a_off = (uint32_t)((wave * 8 + lr) * ld * 2 + lc * 16);
    const int64_t a_step = (int64_t)kWaves * 8 * ld * 2;   // load i fetches rows 8 kWaves i + ...
    auto issue_a = [&](int kt, int stage) {
        const char *base = a_tile + (int64_t)kt * kRowBytes;
#pragma unroll
        for (int i = 0; i < kLoads; ++i) {
            // M0 carries the LDS address of the wave's 1 KB destination
            const uint32_t dst = (uint32_t)(uintptr_t)(lds_void_t *)&lds[stage][0][(kWaves * i + wave) * 1024];
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(dst), "v"(a_off), "s"(base + i * a_step)
                         : "memory");
        }
    };

    // ---- B: packed weights through registers.  Buffer loads: the per-thread offset is computed once,
    // the K-step displacement is uniform and travels in the scalar offset (no vector address math in
    // the loop).  Tile indices are clamped into the tensor, so every index read from it is valid. ----
    const __amdgpu_buffer_rsrc_t wbuf =
        __builtin_amdgcn_make_buffer_rsrc(W.hdr, 0, (int)(uint32_t)lw.total_bytes, 0x00020000);
    // weight row and which pair of its blocks.  Lane pairs share a row; rows are dealt so that eight
    // consecutive lanes -- what the LDS takes from a 16-byte write per clock -- hold rows r, r+2, r+4, r+6:
    // with the swizzle below their chunks then fall into eight different 16-byte bank groups (dealing the
    // rows in order gave 20% bank-conflict cycles on these writes).
    const int br = kBPT == 2 ? (tid >> 4) * 8 + 2 * ((tid >> 1) & 3) + ((tid >> 3) & 1) : tid, bp = kBPT == 2 ? tid & 1 : 0;
    const int64_t row_b = tn * kBN + br;
    // rows beyond the tensor read a valid tile; their products only reach output columns that are never stored
    const uint32_t rt_b = (uint32_t)((row_b >> 3) < lw.n_rt ? (row_b >> 3) : lw.n_rt - 1);
    const int r8 = (int)(row_b & 7);
    const int swz_b = (br >> 1) & 7;
    const int last_kt = nk_total - 1 - kt0;   // K-steps count from the workgroup's first one; kt0 is even
    const uint32_t tile_b = rt_b * (uint32_t)lw.n_kt + (uint32_t)(kt0 >> 1);   // first tile of the thread's row-tile in this workgroup's K range
    const uint32_t vL = (uint32_t)lw.off_L + (tile_b * kTileSlots + r8 * kTileBlocks + 2 * bp) * 8u;
    const uint32_t vS = (uint32_t)lw.off_S + tile_b * kTileSlots + r8 * kTileBlocks + 2 * bp;
    const uint32_t vM = (uint32_t)lw.off_M + tile_b * 8u + (r8 < 4 ? 0u : 4u);   // rows 0-3 of a tile: low half of its mask word
    const uint32_t vT = (uint32_t)lw.off_T + tile_b * 4u;
    const uint32_t off_H = (uint32_t)lw.off_H;
    const int m_shift = (r8 & 3) * 8 + 2 * bp;   // bit of the thread's first block of an even K-step in its mask dword
    auto load_l = [&](int kt, LRegsT &b) {
        kt = kt < last_kt ? kt : last_kt;
        const uint32_t t2 = (uint32_t)__builtin_amdgcn_readfirstlane(kt) >> 1, odd = (uint32_t)__builtin_amdgcn_readfirstlane(kt) & 1u;   // K-tile, and which half of its 8 blocks
        load_b128<0>(b.l[0], wbuf, vL, t2 * (kTileSlots * 8) + odd * 32);
        if constexpr (kBPT == 4) load_b128<16>(b.l[kBPT / 2 - 1], wbuf, vL, t2 * (kTileSlots * 8) + odd * 32);
    };
    auto load_meta = [&](int kt, MetaRegs &b) {
        kt = kt < last_kt ? kt : last_kt;
        const uint32_t t2 = (uint32_t)__builtin_amdgcn_readfirstlane(kt) >> 1, odd = (uint32_t)__builtin_amdgcn_readfirstlane(kt) & 1u;
        if constexpr (kBPT == 2) load_b16(b.s, wbuf, vS, t2 * kTileSlots + odd * 4);
        else load_b32(b.s, wbuf, vS, t2 * kTileSlots + odd * 4);
        load_b32(b.m, wbuf, vM, t2 * 8);
        load_b32(b.t, wbuf, vT, t2 * 4);
    };
    // bit j of the result: the thread's block j of K-step kt is FP8
    auto hi_bits = [&](int kt, const MetaRegs &b) {
        kt = kt < last_kt ? kt : last_kt;
        return (b.m >> (m_shift + (kt & 1) * 4)) & ((1u << kBPT) - 1u);
    };
    auto load_h = [&](int kt, const MetaRegs &b, u32x2_t (&h)[kBPT]) {
        const uint32_t bits = hi_bits(kt, b);
#pragma unroll
        for (int j = 0; j < kBPT; ++j) {
            const bool hi = (bits >> j) & 1u;
            const uint32_t idx = hi ? b.t + ((b.s >> (8 * j)) & 0xFFu) : 0u;
            load_b64(h[j], wbuf, off_H + idx * 8u, 0u);
        }
    };
    // LDS destination of the thread's blocks: chunk c of the 128-byte row sits at position c ^ swz_b; the
    // thread's chunks are 4 bp + d (kBPT == 2) or d (kBPT == 4), and XOR-ing d into the address of
    // chunk d = 0 reaches them all, so one address register per stage is enough.
    const uint32_t b_wr0 = (uint32_t)(kTileBytes + br * kRowBytes + ((((kBPT == 2 ? 4 * bp : 0)) ^ swz_b) << 4));
    auto decode_store = [&](int kt, const LRegsT &bl, const MetaRegs &b, const u32x2_t (&h)[kBPT], int stage, int j) {
        const uint32_t bits = hi_bits(kt, b);
        char *base = &lds[0][0][0];
        const uint32_t at = b_wr0 + (uint32_t)stage * (2 * kTileBytes);
        half2_t v[8];
        const u32x4_t &lq = bl.l[j >> 1];
        decode_block((j & 1) ? make_uint2(lq[2], lq[3]) : make_uint2(lq[0], lq[1]), (b.s >> (8 * j)) & 0xFFu,
                     (bits >> j) & 1u, make_uint2(h[j][0], h[j][1]), v);
        const uint32_t *o = reinterpret_cast<const uint32_t *>(v);
        *reinterpret_cast<uint4 *>(base + (at ^ ((2 * j) << 4))) = make_uint4(o[0], o[1], o[2], o[3]);
        *reinterpret_cast<uint4 *>(base + (at ^ ((2 * j + 1) << 4))) = make_uint4(o[4], o[5], o[6], o[7]);
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

    // Register sets by K-step: plane-L words of step k live in lring[k % 2], the small fields in
    // mring[k % 3], plane-H entries in hring[k % 2].  Loads per thread and K-step: kNM (planes S, M, T
    // of step kt + 3), kNL (plane L of step kt + 2), kNH (plane H of step kt + 2), then -- after the
    // barrier -- kLoads global->LDS loads of A.
    constexpr int kNM = 3, kNL = kBPT / 2, kNH = kBPT;
    static_assert(kNM + kNL + kNH == kBLoads, "load count");
    LRegsT lring[2];
    MetaRegs mring[3];
    u32x2_t hring[2][kBPT];

    // ---- prologue: K-step 0 decoded into stage 0; K-step 1 ready in registers; the small fields of
    // K-step 2 in flight ----
    issue_a(0, 0);
    issue_a(nk > 1 ? 1 : 0, 1);
    load_l(0, lring[0]);
    load_meta(0, mring[0]);
    wait_loaded<0>(lring[0]);
    wait_loaded<0>(mring[0]);
    load_h(0, mring[0], hring[0]);
    wait_loaded<0>(hring[0]);
#pragma unroll
    for (int j = 0; j < kBPT; ++j) decode_store(0, lring[0], mring[0], hring[0], 0, j);
    load_l(1, lring[1]);
    load_meta(1, mring[1]);
    wait_loaded<0>(lring[1]);
    wait_loaded<0>(mring[1]);
    load_h(1, mring[1], hring[1]);
    load_meta(2, mring[2]);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    half8_t fa[2][TM], fb[2][TN];
    read_frags(0, 0, fa[0], fb[0]);
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0)

    // Iteration kt multiplies K-step kt (stage kt & 1) and, before its barrier,
    // decodes K-step kt + 1 into the other stage; after the barrier that stage is
    // readable and the stage just consumed takes the A loads of K-step kt + 2.
    // Loads in flight, oldest first, when iteration kt starts: planes S, M, T of step kt + 2 (kNM),
    // plane L and plane H of step kt + 1 (kNL + kNH), A of step kt + 1 (kLoads).
    // (the body is instantiated for kt % 6 = 0..5, so every LDS address in it is a register plus an
    // immediate and every register set is named statically)
    auto k_step = [&](int kt, auto phase_c) {
        constexpr int r = decltype(phase_c)::value, st = r & 1;
        LRegsT &lcur = lring[(r + 1) % 2], &lnxt = lring[r % 2];
        MetaRegs &mcur = mring[(r + 1) % 3], &mnxt = mring[(r + 2) % 3], &mfar = mring[r % 3];
        u32x2_t(&hcur)[kBPT] = hring[(r + 1) % 2], (&hnxt)[kBPT] = hring[r % 2];
        read_frags(st, 1, fa[1], fb[1]);
        load_meta(kt + 3, mfar);
        // everything issued one iteration ago has landed: the small fields of step kt + 2, plane L and
        // plane H of step kt + 1
        wait_loaded<kLoads + kNM>(mnxt);
        wait_loaded<kLoads + kNM>(lcur);
        wait_loaded<kLoads + kNM>(hcur);
        mfma_block(fa[0], fb[0]);
        __builtin_amdgcn_sched_barrier(0);
        // The decode is a stretch of vector arithmetic with no MFMA in it (its FP8 / NVFP4 branches keep
        // the scheduler from interleaving any); the other wave of the SIMD keeps the matrix pipe busy.
#pragma unroll
        for (int j = 0; j < kBPT; ++j) decode_store(kt + 1, lcur, mcur, hcur, st ^ 1, j);
        // the registers of the step just decoded take the loads of step kt + 2
        load_l(kt + 2, lnxt);
        load_h(kt + 2, mnxt, hnxt);
        read_frags(st, 2, fa[0], fb[0]);
        mfma_block(fa[1], fb[1]);
        order_phase<kReads, kMfma, 0>();
        read_frags(st, 3, fa[1], fb[1]);
        mfma_block(fa[0], fb[0]);
        order_phase<kReads, kMfma, 0>();
        // LDS traffic of this wave done (lgkmcnt 0) and its A loads landed: they are older than this
        // iteration's kBLoads register loads, which may stay in flight (vmcnt kBLoads)
        __builtin_amdgcn_s_waitcnt(0x0070 | pending(kBLoads));
        __syncthreads();
        issue_a(kt + 2 < nk ? kt + 2 : nk - 1, st);
        read_frags(st ^ 1, 0, fa[0], fb[0]);
        mfma_block(fa[1], fb[1]);
        order_phase<kReads, kMfma, 0>();
        __builtin_amdgcn_s_waitcnt(0xC07F);
    };
    // whole turns of the rotation, then the 0, 2 or 4 K-steps left (nk is even: the K extent is padded
    // to whole 128-element tiles)
    int kt = 0;
    for (; kt + 6 <= nk; kt += 6) {
        k_step(kt, std::integral_constant<int, 0>{});
        k_step(kt + 1, std::integral_constant<int, 1>{});
        k_step(kt + 2, std::integral_constant<int, 2>{});
        k_step(kt + 3, std::integral_constant<int, 3>{});
        k_step(kt + 4, std::integral_constant<int, 4>{});
        k_step(kt + 5, std::integral_constant<int, 5>{});
    }
    if (kt < nk) {
        k_step(kt, std::integral_constant<int, 0>{});
        k_step(kt + 1, std::integral_constant<int, 1>{});
        if (kt + 2 < nk) {
            k_step(kt + 2, std::integral_constant<int, 2>{});
            k_step(kt + 3, std::integral_constant<int, 3>{});
        }
    }
    // The last iterations load past the K range (clamped, unused): every register a load may still
    // write stays reserved until all loads have landed.
    wait_loaded<0>(lring[0]);
    wait_loaded<0>(lring[1]);
    wait_loaded<0>(mring[0]);
    wait_loaded<0>(mring[1]);
    wait_loaded<0>(mring[2]);
    wait_loaded<0>(hring[0]);
    wait_loaded<0>(hring[1]);
    __builtin_amdgcn_s_waitcnt(0);

    const bool w_ok = W.hdr->magic == kMagic && W.hdr->rows == lw.rows && W.hdr->K == lw.K;
    const float ss = w_ok ? ha->tensor_scale * W.hdr->tensor_scale : 0.0f;
    if (split) {
        // Two workgroups that hold partial sums of the same tile meet (`meet` below).  One that finds the
        // meeting's counter at 1 knows the other's accumulators are in memory, complete: it adds them to
        // its own and goes on.  Otherwise every wave stores its accumulators (16 bytes per lane and
        // store, [slot][wave][register quad][lane]); when all of the workgroup's stores are complete, one
        // thread bumps the counter; if the other arrived meanwhile (both stored), the workgroup that
        // bumped second goes on with the sum, the other one is done.  a + b = b + a exactly, so the result
        // does not depend on the order of arrival.  With two parts the first is the shorter one and is
        // launched first, so it normally is in memory when the second needs it, off the critical path.
        // With four parts, parts 0, 1 and 2, 3 meet first, then the two pair sums: (p0 + p1) + (p2 + p3)
        // whatever the order.  Partials and counters cross XCDs: system-coherent accesses that bypass the
        // per-XCD L2.
        constexpr uint32_t kWaveBytes = TM * TN * 4 * 1024;
        const __amdgpu_buffer_rsrc_t pbuf =
            __builtin_amdgcn_make_buffer_rsrc(sp.partial, 0, (int)sp.partial_bytes, 0x00020000);
        uint32_t *arrived = reinterpret_cast<uint32_t *>(&lds[0][0][0]);   // the operand stages are free now
        // (32-row bands of the tile beyond the tensor's last row are not exchanged: nothing of them is stored)
        auto band_has_rows = [&](int i) { return tm * kBM + wm * (TM * 32) + i * 32 < M; };
        auto meet = [&](int counter, int my_slot, int other_slot) {
            const uint32_t mine = (uint32_t)(my_slot * kWaves + wave) * kWaveBytes + lane * 16u;
            const uint32_t other = (uint32_t)(other_slot * kWaves + wave) * kWaveBytes + lane * 16u;
            __syncthreads();
            if (tid == 0) *arrived = __hip_atomic_load(&sp.counters[counter], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            if (*arrived == 0u) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    if (band_has_rows(i)) {
#pragma unroll
                        for (int j = 0; j < TN; ++j)
#pragma unroll
                            for (int q = 0; q < 4; ++q)
                                store_coherent16(pbuf, mine + ((i * TN + j) * 4 + q) * 1024u,
                                                 float4_t{acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]});
                    }
                __builtin_amdgcn_s_waitcnt(0);
                __syncthreads();   // all stores of the workgroup are complete (and everyone has read *arrived)
                if (tid == 0)
                    *arrived = __hip_atomic_fetch_add(&sp.counters[counter], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __syncthreads();
                if (*arrived == 0u) return false;
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
                if (band_has_rows(i)) {
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const float4_t o = load_coherent16(pbuf, other + ((i * TN + j) * 4 + q) * 1024u);
#pragma unroll
                            for (int e = 0; e < 4; ++e) acc[i][j][4 * q + e] += o[e];
                        }
                }
            return true;
        };
        const bool four = sp.n_parts == 4;
        const int slots = four ? 6 : 2, counters = four ? 3 : 1;   // per tile
        if (!meet(split_tile * counters + (part >> 1), split_tile * slots + part, split_tile * slots + (part ^ 1))) return;
        if (four && !meet(split_tile * counters + 2, split_tile * slots + 4 + (part >> 1),
                          split_tile * slots + 4 + ((part >> 1) ^ 1)))
            return;
    }
    if constexpr (!kPackOut) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int64_t col = tn * kBN + wn * (TN * 32) + j * 32 + (lane & 31);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t row = tm * kBM + wm * (TM * 32) + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    // (streaming stores: the 4 M N bytes of results are not read again here and would only push
                    // operand panels out of the caches: 1.5% on the Llama-2-7B shapes)
                    if (row < M && col < N) __builtin_nontemporal_store(acc[i][j][r] * ss, &Y[row * ldy + col]);
                }
            }
    } else {
        // Each 32 x 32 accumulator tile is transposed through LDS (wave-private, the operand stages are
        // free now) so that a lane owns one output block: (row = lane % 32, 16 columns = lane / 32).  The
        // block goes through the quantizer's arithmetic; codes, scale bytes and FP8 upper halves are
        // written by the lane, the mask words of the 64 packed tiles this workgroup covers are gathered
        // in LDS; the FP8 upper halves go to the block's own slot of the tile's plane-H region first and to
        // their final places once the masks are complete (below).
        constexpr int kTStride = 36;   // floats per transposed row: 16-byte aligned rows, staggered banks
        __syncthreads();
        float *tbuf = reinterpret_cast<float *>(&lds[0][0][0]) + wave * (32 * kTStride);
        unsigned long long *m_lds = reinterpret_cast<unsigned long long *>(&lds[1][1][0]);
        if (tid < 64) m_lds[tid] = 0ull;
        __syncthreads();
        const PackedLayout &ly = po.layout;
        const float inv_Sy = 1.0f / po.S, S6y = 6.0f * po.S;
        const int brow = lane & 31, bblk = lane >> 5;
        // gated: a wave's two accumulator tiles of a row band are the gate and the up values of the same 32
        // hidden units, element by element; the workgroup's 256 weight rows give 128 output columns
        static_assert(!kGate || TN == 2, "a wave must hold one group of 32 gate and 32 up rows");
        constexpr int kOutTiles = kGate ? 1 : TN, kOutBN = kGate ? kBN / 2 : kBN;
        const int64_t n_out = kGate ? N / 2 : N;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < kOutTiles; ++j) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float v;
                    if constexpr (kGate) v = silu_mul(acc[i][0][r] * ss, acc[i][1][r] * ss);
                    else v = acc[i][j][r] * ss;
                    tbuf[(8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)) * kTStride + (lane & 31)] = v;
                }
                float x[16], f[16];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float4 t4 = *reinterpret_cast<const float4 *>(&tbuf[brow * kTStride + 16 * bblk + 4 * v]);
                    x[4 * v] = t4.x; x[4 * v + 1] = t4.y; x[4 * v + 2] = t4.z; x[4 * v + 3] = t4.w;
                }
                const int row_l = wm * (TM * 32) + i * 32 + brow;              // within the workgroup's 256 x 256
                const int col_l = wn * (kOutTiles * 32) + j * 32 + 16 * bblk;   // within the workgroup's output columns
                const int64_t row = tm * kBM + row_l, col0 = tn * kOutBN + col_l;
                const bool valid = row < M && col0 < n_out;
                if (valid) load16(po.fisher + col0, f);
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    x[e] = valid ? x[e] : 0.0f;
                    f[e] = valid ? f[e] : 0.0f;
                }
                const float amax = block_amax(x);
                BlockCodes bc;
                quantize_block_math<true, false>(x, f, amax, po.S, inv_Sy, S6y, -1, false, bc);
                const bool hi = valid && bc.score > po.T;
                if (po.scores != nullptr && valid) po.scores[row * ly.nb + (col0 >> 4)] = bc.score;
                const int64_t rt = row >> 3, kt = col0 >> 7;
                const int slot = (int)(row & 7) * kTileBlocks + (int)((col0 >> 4) & 7);
                if (rt < ly.n_rt && kt < ly.n_kt) {
                    const int64_t at = (rt * ly.n_kt + kt) * kTileSlots + slot;
                    uint2 lword = make_uint2(bc.q[0], bc.q[1]);
                    uint32_t sbyte = bc.sc;
                    if (hi) {
                        float rr[16];
#pragma unroll
                        for (int e = 0; e < 16; ++e) rr[e] = x[e] * inv_Sy;
                        uint32_t c[4];
                        encode_fp8_block<true, true>(rr, c);
                        lword = make_uint2(c[0], c[1]);
                        po.out.H[at] = make_uint2(c[2], c[3]);
                        atomicOr(&m_lds[(row_l >> 3) * 2 + (col_l >> 7)], 1ull << slot);
                    } else {
                        po.out.S[at] = (uint8_t)sbyte;
                    }
                    po.out.L[at] = lword;
                }
            }
        __builtin_amdgcn_s_waitcnt(0);   // this wave's stores have reached the L2
        __syncthreads();
        // A block's plane-H entry belongs at the number of FP8 slots before it in its tile (readers may take
        // that from the mask), and that number is its plane-S byte: known now that the tile's mask word is
        // complete.  One wave per tile, lane = slot, moves the entries from the blocks' own slots (every
        // entry is in a register before the first one is stored again: a store waits for its data, i.e. for
        // the load instruction as a whole).
        for (int q = wave; q < 64; q += kWaves) {
            const int64_t rt = tm * (kBM / kTileRows) + (q >> 1), kt = tn * (kOutBN / kTileK) + (q & 1);
            if (rt < ly.n_rt && kt < ly.n_kt && (q & 1) < kOutBN / kTileK) {
                const unsigned long long mask = m_lds[q];
                const int64_t tile = rt * ly.n_kt + kt;
                if ((mask >> lane) & 1ull) {
                    const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
                    const uint2 e = po.out.H[tile * kTileSlots + lane];
                    po.out.H[tile * kTileSlots + rank] = e;
                    po.out.S[tile * kTileSlots + lane] = (uint8_t)rank;
                }
                if (lane == 0) {
                    po.out.M[tile] = mask;
                    po.out.T[tile] = (uint32_t)(tile * kTileSlots);
                }
            }
        }
        // the header: by the workgroup that completes the first tile of the launch order
        const int first_tile = split ? sp.n_whole + split_tile : (int)blockIdx.x;
        if (first_tile == 0 && tid == 0) write_header(po.out.hdr, ly, po.S, 0u);
    }
}

// A tile keeps a compute unit busy for one "round"; the chip runs kNumCu tiles per round.  When the
// last round is at most half full, its tiles are split along K: two shorter workgroups per tile still
// fit one round, which then takes about half the time (4096 x 22016: 1376 tiles = 5 rounds + 96 tiles;
// 6 rounds become 5.5) -- four when the round is at most a quarter full (small M: a QKV product of
// 256 rows has 48 tiles).  Fuller last rounds, and K ranges too short to divide, are left alone.
constexpr int64_t kNumCu = 256;
constexpr size_t kSplitSlotBytes = (size_t)kBM * kBN * 4;   // the accumulators of one workgroup

static int64_t split_tiles(int64_t n_tiles)
{
    const int64_t tail = n_tiles % kNumCu;
    return tail <= kNumCu / 2 ? tail : 0;
}

size_t gemm_mixed_split_bytes(int64_t n_tiles)
{
    const int64_t n = split_tiles(n_tiles);
    if (n == 0) return 0;
    const bool four = n <= kNumCu / 4;   // (sized for four parts even when K turns out too short for them)
    return (size_t)n * (four ? 6 : 2) * kSplitSlotBytes + (size_t)align_up((uint64_t)n * (four ? 3 : 1) * 4, 256);
}

SplitTail plan_split_tail(int64_t n_tiles, int nk, void *region)
{
    SplitTail sp{};
    const int64_t n = split_tiles(n_tiles);
    if (n == 0 || nk < 4 || region == nullptr) {
        sp.n_whole = (int)n_tiles;
        return sp;
    }
    sp.n_whole = (int)(n_tiles - n);
    sp.n_split = (int)n;
    // K-step pairs are 128-element tiles of the packed layout: every boundary is even
    if (n <= kNumCu / 4 && nk >= 8) {
        sp.n_parts = 4;
        for (int p = 0; p <= 4; ++p) sp.kt_bound[p] = p == 4 ? nk : (nk * p / 4) & ~1;
    } else {
        // somewhat less than half: the first part is done, and in memory, before the second one asks for it
        sp.n_parts = 2;
        sp.kt_bound[0] = 0;
        sp.kt_bound[1] = ((nk * 7 / 16) & ~1) >= 2 ? (nk * 7 / 16) & ~1 : 2;
        sp.kt_bound[2] = nk;
    }
    const bool four = sp.n_parts == 4;
    sp.n_counters = (int)n * (four ? 3 : 1);
    sp.partial_bytes = (uint32_t)((size_t)n * (four ? 6 : 2) * kSplitSlotBytes);
    sp.partial = static_cast<float *>(region);
    sp.counters = reinterpret_cast<uint32_t *>(static_cast<char *>(region) + sp.partial_bytes);
    return sp;
}

// Measurement hook (only in builds with FGMP_MEASUREMENT_HOOKS; the shipped launcher records nothing):
// a pair of events recorded around every launch of the kernel.
#ifdef FGMP_MEASUREMENT_HOOKS
static hipEvent_t g_ev_start = nullptr, g_ev_stop = nullptr;
bool set_gemm_kernel_events(hipEvent_t start, hipEvent_t stop)
{
    g_ev_start = start;
    g_ev_stop = stop;
    return true;
}
#else
bool set_gemm_kernel_events(hipEvent_t, hipEvent_t) { return false; }
#endif

void launch_gemm_mixed(const _Float16 *a16, int64_t ld, const PackedView &W, const PackedLayout &lw, float *Y,
                       int64_t ldy, int64_t M, int64_t N, int64_t n_tm, int64_t n_tn, const PackedHeader *ha,
                       hipStream_t st, const SplitTail &sp, const PackOut *pack_out)
{
#ifdef FGMP_MEASUREMENT_HOOKS
    if (g_ev_start) (void)hipEventRecord(g_ev_start, st);
#endif
    const unsigned grid = (unsigned)(sp.n_whole + sp.n_parts * sp.n_split);
#ifndef FGMP_MIXED_WM
#define FGMP_MIXED_WM 2
#define FGMP_MIXED_WN 4
#endif
    constexpr int kThreads = FGMP_MIXED_WM * FGMP_MIXED_WN * 64;
    if (pack_out != nullptr && pack_out->gate)
        hipLaunchKernelGGL((gemm_mixed_kernel<FGMP_MIXED_WM, FGMP_MIXED_WN, true, true>), dim3(grid),
                           dim3(kThreads), 0, st, a16, ld, W, lw, (int)(ld / kBK), Y, ldy, M, N, n_tm, n_tn, ha,
                           *pack_out, sp);
    else if (pack_out != nullptr)
        hipLaunchKernelGGL((gemm_mixed_kernel<FGMP_MIXED_WM, FGMP_MIXED_WN, true, false>), dim3(grid),
                           dim3(kThreads), 0, st, a16, ld, W, lw, (int)(ld / kBK), Y, ldy, M, N, n_tm, n_tn, ha,
                           *pack_out, sp);
    else
        hipLaunchKernelGGL((gemm_mixed_kernel<FGMP_MIXED_WM, FGMP_MIXED_WN, false, false>), dim3(grid),
                           dim3(kThreads), 0, st, a16, ld, W, lw, (int)(ld / kBK), Y, ldy, M, N, n_tm, n_tn, ha,
                           PackOut{}, sp);
#ifdef FGMP_MEASUREMENT_HOOKS
    if (g_ev_stop) (void)hipEventRecord(g_ev_stop, st);
#endif
}

}  // namespace fgmp
