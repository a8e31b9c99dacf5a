// Block-mixed-precision GEMM Y = S_x S_w (X^ W^^T) over packed FGMP operands
// (Sec. 4.1).  Each 16-element block is decoded according to its metadata
// bit -- FP8 value, or E2M1 value times its E4M3 block scale -- into FP16,
// where both kinds of operand are exactly representable (at most 6
// significant bits, magnitudes 2^-10 .. 2688), multiplied on the matrix
// cores and accumulated in FP32, which is what the paper's four dot-product
// units followed by the FP32 partial-sum adder compute.
//
// Prefill path (M > 32): the activations are expanded to FP16 in the caller's
// workspace by a decode pass (small), and the 256x256x64-tiled MFMA kernel of
// fgmp_gemm_mixed.hip decodes the packed weights itself.  This file holds the
// decode pass, the dispatch, and the alternative two-pass path in which both
// operands are expanded first and a plain FP16 kernel multiplies them.
#include <stdlib.h>

#include <algorithm>

#include "fgmp_elementwise.hpp"
#include "fgmp_gemm_common.hpp"

namespace fgmp {

// One wave per 8 x 128 tile of the zero-padded FP16 matrix out[8 n_rt_pad][ld].
// One launch serves up to two tensors (both GEMM operands) and can clear a
// small array of counters on the side.
__global__ __launch_bounds__(256) void decode_f16_kernel(DecodeJob ja, DecodeJob jb, uint32_t *zero, int64_t zero_n)
{
    const int lane = threadIdx.x & 63;
    int64_t id = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    {
        const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
        if (gid < zero_n) zero[gid] = 0u;
    }
    const bool second = id >= ja.waves;
    if (second) id -= ja.waves;
    const DecodeJob &j = second ? jb : ja;
    if (id >= j.waves) return;
    const PackedLayout &l = j.l;
    const int64_t rt = id / l.n_kt, kt = id % l.n_kt;
    half2_t vals[8];
    // an operand whose header does not describe the shape this launch assumes decodes to zeros
    const bool header_ok = j.v.hdr->magic == kMagic && j.v.hdr->rows == l.rows && j.v.hdr->K == l.K;
    if (rt < l.n_rt && header_ok) {
        decode_slot(j.v, rt * l.n_kt + kt, lane, vals);
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) vals[i] = half2_t{(_Float16)0.0f, (_Float16)0.0f};
    }
    _Float16 *dst = j.out + (rt * kTileRows + (lane >> 3)) * j.ld + kt * kTileK + (lane & 7) * kBlock;
    uint4 *d4 = reinterpret_cast<uint4 *>(dst);
    const uint32_t *w = reinterpret_cast<const uint32_t *>(vals);
    d4[0] = make_uint4(w[0], w[1], w[2], w[3]);
    d4[1] = make_uint4(w[4], w[5], w[6], w[7]);
}

DecodeJob make_decode_job(const PackedView &v, const PackedLayout &l, _Float16 *out, int64_t ld, int64_t n_rt_pad)
{
    DecodeJob j;
    j.v = v;
    j.l = l;
    j.out = out;
    j.ld = ld;
    j.waves = n_rt_pad * l.n_kt;
    return j;
}

fgmp_status_t launch_decode_f16(const DecodeJob &a, const DecodeJob *b, uint32_t *zero, int64_t zero_n,
                                hipStream_t st)
{
    DecodeJob none = a;
    none.waves = 0;
    const DecodeJob &jb = b ? *b : none;
    int64_t blocks = (a.waves + jb.waves + 3) / 4;
    const int64_t zblocks = (zero_n + 255) / 256;
    if (blocks < zblocks) blocks = zblocks;
    if (blocks > 0x7FFFFFFF) return FGMP_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(decode_f16_kernel, dim3((unsigned)blocks), dim3(256), 0, st, a, jb, zero, zero_n);
    return FGMP_OK;
}

// ---------------------------------------------------------------------------
// dense FP16 x FP16 -> FP32 MFMA kernel, A [Mp][ld], B [Np][ld], both K-major
// ---------------------------------------------------------------------------

// kWM x kWN waves per workgroup; each wave owns a (256 / kWM) x (256 / kWN)
// piece of the tile as TM x TN MFMA tiles of 32 x 32.
template <int kWM, int kWN>
__global__ __launch_bounds__(kWM *kWN * 64, 1) void gemm_f16_kernel(const _Float16 *__restrict__ A,
                                                                     const _Float16 *__restrict__ B, int64_t ld,
                                                                     int nk, float *__restrict__ Y, int64_t ldy,
                                                                     int64_t M, int64_t N, int64_t n_tm,
                                                                     int64_t n_tn, const PackedHeader *ha,
                                                                     const PackedHeader *hb)
{
    constexpr int kWaves = kWM * kWN;
    constexpr int TM = kBM / (32 * kWM), TN = kBN / (32 * kWN);
    constexpr int kLoads = 32 / kWaves;          // 1 KB wave-loads per operand per wave per K-step
    __shared__ __attribute__((aligned(1024))) char lds[2][2][kTileBytes];   // [stage][operand]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / kWN, wn = wave % kWN;
    int64_t tm, tn;
    tile_coords(blockIdx.x, n_tm, n_tn, tm, tn);

    // direct global -> LDS: wave-load j (j = kWaves i + wave) fills tile rows 8 j .. 8 j + 7;
    // lane (lr = lane / 8, c = lane % 8) fetches global chunk c ^ swizzle(row) of its row;
    // rows of successive i differ by a multiple of 16, which leaves the swizzle unchanged
    const int lr = lane >> 3, lc = (lane & 7) ^ (((wave * 8 + lr) >> 1) & 7);
    const char *ga = reinterpret_cast<const char *>(A + (tm * kBM + wave * 8 + lr) * ld) + lc * 16;
    const char *gb = reinterpret_cast<const char *>(B + (tn * kBN + wave * 8 + lr) * ld) + lc * 16;
    const int64_t row_step = kWaves * 8 * ld * 2;   // bytes between wave-loads i and i + 1

    auto issue_loads = [&](int kt, int stage) {
#pragma unroll
        for (int i = 0; i < kLoads; ++i) {
            __builtin_amdgcn_global_load_lds((global_void_t *)(ga + i * row_step + (int64_t)kt * kRowBytes),
                                             (lds_void_t *)&lds[stage][0][(kWaves * i + wave) * 1024], 16, 0, 0);
            __builtin_amdgcn_global_load_lds((global_void_t *)(gb + i * row_step + (int64_t)kt * kRowBytes),
                                             (lds_void_t *)&lds[stage][1][(kWaves * i + wave) * 1024], 16, 0, 0);
        }
    };

    float16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // operand fragment of lane: row (lane & 31) of a 32-row group, K chunk 2 kk + (lane >> 5)
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

    // Software pipeline.  LDS holds two K-steps; the fragments of the next
    // 16-wide K slice are read while the MFMAs of the current one run.
    // Before the last slice of a K-step every wave has finished reading the
    // current stage, so that is where the barrier sits: after it the other
    // stage (filled by loads issued one K-step earlier) is visible, and the
    // stage just consumed is refilled with the K-step after next.
    half8_t fa[2][TM], fb[2][TN];
    issue_loads(0, 0);
    issue_loads(nk > 1 ? 1 : 0, 1);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    read_frags(0, 0, fa[0], fb[0]);
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): enter the loop with an empty LDS queue (see its end)
    for (int kt = 0; kt < nk; ++kt) {
        const int st = kt & 1;
        read_frags(st, 1, fa[1], fb[1]);
        mfma_block(fa[0], fb[0]);
        order_phase<kReads, kMfma, 0>();
        read_frags(st, 2, fa[0], fb[0]);
        mfma_block(fa[1], fb[1]);
        order_phase<kReads, kMfma, 0>();
        read_frags(st, 3, fa[1], fb[1]);
        mfma_block(fa[0], fb[0]);
        order_phase<kReads, kMfma, 0>();
        __builtin_amdgcn_s_waitcnt(0);   // own LDS reads done, own global->LDS loads landed
        __syncthreads();
        // the last two iterations reload the final K-step, which nobody reads again
        issue_loads(kt + 2 < nk ? kt + 2 : nk - 1, st);
        read_frags(st ^ 1, 0, fa[0], fb[0]);
        mfma_block(fa[1], fb[1]);
        order_phase<kReads, kMfma, kLoads>();
        // the fragments for the next iteration were requested a phase ago; waiting for them here (LDS
        // counter only) costs nothing and lets the next iteration start with a known-empty LDS queue
        __builtin_amdgcn_s_waitcnt(0xC07F);
    }
    __builtin_amdgcn_s_waitcnt(0);

    // per-tensor scales are applied once, after accumulation
    const float ss = ha->tensor_scale * hb->tensor_scale;
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

#ifndef FGMP_GEMM_WM
#define FGMP_GEMM_WM 2
#define FGMP_GEMM_WN 4
#endif

static inline int64_t round_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

struct GemmWorkspace {
    int64_t ld, Mp, Np;
    size_t off_a, off_b, off_split, total;   // off_split: partial tiles and counters of a split last round
};

static GemmWorkspace gemm_ws_layout(int64_t M, int64_t N, int64_t K)
{
    GemmWorkspace w;
    w.ld = round_up(K, kTileK);
    w.Mp = round_up(M, kBM);
    w.Np = round_up(N, kBN);
    w.off_a = 0;
    w.off_b = (size_t)align_up((uint64_t)w.Mp * w.ld * 2, 256);
    w.off_split = w.off_b + (size_t)align_up((uint64_t)w.Np * w.ld * 2, 256);
    w.total = w.off_split + gemm_mixed_split_bytes((w.Mp / kBM) * (w.Np / kBN));
    return w;
}

// The prefill kernel decodes the weights inside the MFMA kernel.  Builds with FGMP_MEASUREMENT_HOOKS
// (never the shipped library) can select the two-pass path instead -- both operands expanded to FP16
// in the workspace, then a plain FP16 kernel -- with FGMP_PREFILL_KERNEL=dense in the environment.
static bool prefill_decodes_in_kernel()
{
#ifdef FGMP_MEASUREMENT_HOOKS
    static const bool in_kernel = [] {
        const char *e = getenv("FGMP_PREFILL_KERNEL");
        return !(e && e[0] == 'd');
    }();
    return in_kernel;
#else
    return true;
#endif
}

// The MFMA kernel that decodes the weights itself addresses them with 32-bit buffer offsets; larger
// weight tensors take the two-pass path.
static bool mixed_kernel_applies(int64_t N, int64_t K)
{
    return prefill_decodes_in_kernel() && make_layout(N, K).total_bytes < 0xFFFFFF00ull;
}

// FP16 activations of a decode-shape call: gemm_skinny_x16_rows(M) rows
static size_t skinny_x16_bytes(int64_t M, int64_t K)
{
    return (size_t)align_up((uint64_t)gemm_skinny_x16_rows(M) * round_up(K, kTileK) * 2, 256);
}

// (all of these count the bytes behind the control region)
size_t gemm_only_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    const size_t other = gemm_skinny_applies(M, N, K) ? skinny_x16_bytes(M, K) + gemm_skinny_workspace_bytes(M, N, K)
                                                      : gemm_ws_layout(M, N, K).total;
    return std::max(other, gemm_stream_scratch_bytes(M, N, K));
}

size_t gemm_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    // the fused call also keeps the quantized activations here: packed, or header + FP16 values
    return kWsCtrlRegion + (size_t)make_layout(M, K).total_bytes + gemm_only_workspace_bytes(M, N, K);
}

size_t quant_gemm_workspace_need(int64_t M, int64_t N, int64_t K)
{
    if (gemm_stream_applies(M, N, K)) return kWsCtrlRegion + gemm_stream_scratch_bytes(M, N, K);
    return gemm_workspace_bytes(M, N, K);
}

// `skip`: bytes behind the control region that the caller keeps for itself (the fused call's packed activations)
fgmp_status_t gemm_packed(const void *packed_X, int64_t M, const void *packed_W, int64_t N, int64_t K,
                          float *Y, int64_t ldy, void *workspace, size_t workspace_bytes, hipStream_t st, size_t skip)
{
    if (!packed_X || !packed_W || !Y || !workspace) return FGMP_ERR_INVALID_ARG;
    if (M <= 0 || N <= 0 || K <= 0) return FGMP_ERR_INVALID_ARG;
    if (K % kBlock != 0 || ldy < N) return FGMP_ERR_BAD_SHAPE;
    if (((uintptr_t)packed_X | (uintptr_t)packed_W | (uintptr_t)Y | (uintptr_t)workspace) % 16 != 0)
        return FGMP_ERR_BAD_ALIGN;
    if (workspace_bytes < kWsCtrlRegion + skip + gemm_only_workspace_bytes(M, N, K)) return FGMP_ERR_BUFFER_TOO_SMALL;
    const PackedLayout la = make_layout(M, K), lb = make_layout(N, K);
    const PackedView A = make_view(const_cast<void *>(packed_X), la);
    const PackedView B = make_view(const_cast<void *>(packed_W), lb);
    void *const ctrl = workspace;
    workspace = static_cast<char *>(workspace) + kWsCtrlRegion + skip;
    if (gemm_stream_applies(M, N, K))
        return gemm_stream(2, nullptr, 0, nullptr, 0.0f, 1.0f, packed_X, M, packed_W, N, K, Y, ldy, ctrl, workspace, st);
    if (gemm_skinny_applies(M, N, K)) {
        // decode shapes: expand the few activation rows to FP16 once, then stream the weights
        _Float16 *x16 = static_cast<_Float16 *>(workspace);
        const int64_t ld16 = round_up(K, kTileK);
        const DecodeJob jx = make_decode_job(A, la, x16, ld16, gemm_skinny_x16_rows(M) / kTileRows);
        char *sws = static_cast<char *>(workspace) + skinny_x16_bytes(M, K);
        const SkinnyCounters ctr = gemm_skinny_counters(M, N, K, sws);
        const fgmp_status_t rcx = launch_decode_f16(jx, nullptr, ctr.ptr, ctr.n, st);
        if (rcx != FGMP_OK) return rcx;
        return gemm_skinny(A.hdr, la, x16, ld16, packed_W, lb, M, N, K, Y, ldy, sws, st);
    }
    const GemmWorkspace w = gemm_ws_layout(M, N, K);
    if (mixed_kernel_applies(N, K)) {
        // activations expanded to FP16 once (M x K is small); weights decoded inside the MFMA kernel
        _Float16 *x16 = reinterpret_cast<_Float16 *>(static_cast<char *>(workspace) + w.off_a);
        const int64_t tiles_m = w.Mp / kBM, tiles_n = w.Np / kBN;
        if (tiles_m * tiles_n > 0x7FFFFFFF) return FGMP_ERR_UNSUPPORTED;
        const DecodeJob jx = make_decode_job(A, la, x16, w.ld, w.Mp / kTileRows);
        const SplitTail sp = plan_split_tail(tiles_m * tiles_n, (int)(w.ld / kBK), static_cast<char *>(workspace) + w.off_split);
        const fgmp_status_t rcx = launch_decode_f16(jx, nullptr, sp.counters, (int64_t)sp.n_counters, st);
        if (rcx != FGMP_OK) return rcx;
        launch_gemm_mixed(x16, w.ld, B, lb, Y, ldy, M, N, tiles_m, tiles_n, A.hdr, st, sp);
        return hipGetLastError() == hipSuccess ? FGMP_OK : FGMP_ERR_HIP;
    }
    _Float16 *a16 = reinterpret_cast<_Float16 *>(static_cast<char *>(workspace) + w.off_a);
    _Float16 *b16 = reinterpret_cast<_Float16 *>(static_cast<char *>(workspace) + w.off_b);
    const int64_t n_tm = w.Mp / kBM, n_tn = w.Np / kBN;
    if (n_tm * n_tn > 0x7FFFFFFF) return FGMP_ERR_UNSUPPORTED;
    const DecodeJob ja = make_decode_job(A, la, a16, w.ld, w.Mp / kTileRows);
    const DecodeJob jb = make_decode_job(B, lb, b16, w.ld, w.Np / kTileRows);
    const fgmp_status_t rc = launch_decode_f16(ja, &jb, nullptr, 0, st);
    if (rc != FGMP_OK) return rc;
    hipLaunchKernelGGL((gemm_f16_kernel<FGMP_GEMM_WM, FGMP_GEMM_WN>), dim3((unsigned)(n_tm * n_tn)),
                       dim3(FGMP_GEMM_WM * FGMP_GEMM_WN * 64), 0, st, a16, b16, w.ld,
                       (int)(w.ld / kBK), Y, ldy, M, N, n_tm, n_tn, A.hdr, B.hdr);
    return hipGetLastError() == hipSuccess ? FGMP_OK : FGMP_ERR_HIP;
}

// Fused call.  Prefill shapes: the quantizer writes the FP16 values of the codes
// it selects straight into the GEMM's A operand (the packed form of X is never
// materialized; only its header, which carries the tensor scale).  Other shapes
// and the two-pass path go through the packed activations.
fgmp_status_t quant_gemm(const void *X, fgmp_dtype_t dt, int64_t M, int64_t K, int64_t ldx, const float *fisher_k,
                         float threshold, float scale_x, const void *packed_W, int64_t N, float *Y, int64_t ldy,
                         void *workspace, size_t workspace_bytes, hipStream_t st, int score_mode,
                         const PackOut *pack_out)
{
    if (!workspace || !packed_W || (!Y && !pack_out)) return FGMP_ERR_INVALID_ARG;
    if (M <= 0 || N <= 0 || K <= 0) return FGMP_ERR_INVALID_ARG;
    if (K % kBlock != 0 || ldy < N) return FGMP_ERR_BAD_SHAPE;
    if (((uintptr_t)workspace | (uintptr_t)packed_W | (uintptr_t)Y) % 16 != 0) return FGMP_ERR_BAD_ALIGN;
    // (the one-launch kernel addresses X with 32-bit byte offsets)
    const bool x_fits = ldx > 0 && ldx < (int64_t)0xFFFFFF00 / (M * 4);
    // (the decode step quantizes its own results where the caller asks for it)
    const bool stream_pack = pack_out != nullptr && !pack_out->gate && pack_out->one_launch && gemm_stream_packs(M, N, K);
    const bool stream = score_mode == FGMP_SCORE_NVFP4_ERROR && (pack_out == nullptr || stream_pack) && x_fits && gemm_stream_applies(M, N, K);
    if (workspace_bytes < (stream ? (pack_out ? kWsCtrlRegion + gemm_stream_pack_scratch_bytes(M, N, K) : quant_gemm_workspace_need(M, N, K))
                                  : gemm_workspace_bytes(M, N, K)))
        return FGMP_ERR_BUFFER_TOO_SMALL;
    char *ws = static_cast<char *>(workspace) + kWsCtrlRegion;
    if (stream) {
        // decode shapes: one launch quantizes the activation rows and streams the weights (and, with
        // `pack_out`, quantizes and packs the results)
        if (!X || !fisher_k || (!Y && !pack_out)) return FGMP_ERR_INVALID_ARG;
        if (dt != FGMP_F32 && dt != FGMP_BF16) return FGMP_ERR_UNSUPPORTED;
        if (!(scale_x > 0.0f) || !(scale_x < INFINITY) || threshold != threshold) return FGMP_ERR_INVALID_ARG;
        const int64_t esz = dt == FGMP_F32 ? 4 : 2;
        if (ldx < K) return FGMP_ERR_BAD_SHAPE;
        if (((uintptr_t)X | (uintptr_t)fisher_k) % 16 != 0 || (ldx * esz) % 16 != 0) return FGMP_ERR_BAD_ALIGN;
        return gemm_stream(dt == FGMP_F32 ? 1 : 0, X, ldx, fisher_k, threshold, scale_x, nullptr, M, packed_W, N, K, Y, ldy,
                           workspace, ws, st, pack_out);
    }
    const bool in_kernel_prefill = !gemm_skinny_applies(M, N, K) && mixed_kernel_applies(N, K) && kUseHwCvt;
    if (pack_out != nullptr && !in_kernel_prefill) return FGMP_ERR_UNSUPPORTED;   // the caller falls back
    if (gemm_skinny_applies(M, N, K) && kUseHwCvt) {
        // decode shapes: FP16 values of X (rows beyond the last 8-row group stay unwritten: they only
        // feed output rows that are never stored), then the weight-streaming kernel
        const int64_t ld16 = round_up(K, kTileK);
        _Float16 *x16 = reinterpret_cast<_Float16 *>(ws + kHeaderBytes);
        char *sws = ws + kHeaderBytes + skinny_x16_bytes(M, K);
        const SkinnyCounters ctr = gemm_skinny_counters(M, N, K, sws);
        const fgmp_status_t rc = quantize_tensor(X, dt, M, K, ldx, fisher_k, 0, threshold, scale_x, ws,
                                                 sizeof(PackedHeader), nullptr, false, st, x16, ld16, ctr.ptr, ctr.n,
                                                 score_mode);
        if (rc != FGMP_OK) return rc;
        return gemm_skinny(reinterpret_cast<const PackedHeader *>(ws), make_layout(M, K), x16, ld16, packed_W,
                           make_layout(N, K), M, N, K, Y, ldy, sws, st);
    }
    if (in_kernel_prefill) {
        const GemmWorkspace w = gemm_ws_layout(M, N, K);
        const int64_t tiles_m = w.Mp / kBM, tiles_n = w.Np / kBN;
        if (tiles_m * tiles_n > 0x7FFFFFFF) return FGMP_ERR_UNSUPPORTED;
        PackedHeader *hx = reinterpret_cast<PackedHeader *>(ws);
        _Float16 *x16 = reinterpret_cast<_Float16 *>(ws + kHeaderBytes);
        char *split_region = ws + (size_t)make_layout(M, K).total_bytes + w.off_split;
        const SplitTail sp = plan_split_tail(tiles_m * tiles_n, (int)(w.ld / kBK), split_region);
        const fgmp_status_t rc = quantize_tensor(X, dt, M, K, ldx, fisher_k, 0, threshold, scale_x, ws,
                                                 sizeof(PackedHeader), nullptr, false, st, x16, w.ld, sp.counters,
                                                 (int64_t)sp.n_counters, score_mode);
        if (rc != FGMP_OK) return rc;
        const PackedLayout lb = make_layout(N, K);
        const PackedView B = make_view(const_cast<void *>(packed_W), lb);
        launch_gemm_mixed(x16, w.ld, B, lb, Y, ldy, M, N, tiles_m, tiles_n, hx, st, sp, pack_out);
        return hipGetLastError() == hipSuccess ? FGMP_OK : FGMP_ERR_HIP;
    }
    const size_t xbytes = (size_t)make_layout(M, K).total_bytes;
    const fgmp_status_t rc = quantize_tensor(X, dt, M, K, ldx, fisher_k, 0, threshold, scale_x, ws, xbytes,
                                             nullptr, false, st, nullptr, 0, nullptr, 0, score_mode);
    if (rc != FGMP_OK) return rc;
    // (the packed activations sit behind the control region; the product's own workspace starts with one)
    return gemm_packed(ws, M, packed_W, N, K, Y, ldy, workspace, workspace_bytes, st, xbytes);
}

// Fused call whose results are quantized and packed instead of stored as FP32 (Sec. 4.2).  Prefill
// shapes do it in the GEMM's epilogue, decode steps (M <= 32) inside their one launch when asked to
// (FGMP_EPILOGUE_ONE_LAUNCH); otherwise, for other shapes, the gated epilogue at decode sizes and the
// two-pass path, the FP32 results go to the workspace and the standalone quantizer runs over them -- the
// same arithmetic on the same values.
size_t gemm_workspace_bytes_packed_out(int64_t M, int64_t N, int64_t K, int epilogue)
{
    // FP32 staging of the product for the shapes whose epilogue cannot quantize, and of the gated values
    const size_t staged = (size_t)align_up((uint64_t)M * N * 4, 256);
    const size_t gated = epilogue == FGMP_EPILOGUE_SILU_GATE ? (size_t)align_up((uint64_t)M * (N / 2) * 4, 256) : 0;
    return (size_t)align_up(gemm_workspace_bytes(M, N, K), 256) + staged + gated;
}

// h[m][32 q + c] = SiLU(y[m][64 q + c]) * y[m][64 q + 32 + c]: the gated activation over a staged product
// (the shapes whose GEMM epilogue cannot apply it)
__global__ __launch_bounds__(256) void silu_gate_kernel(const float *__restrict__ y, int64_t ldy, int64_t M,
                                                         int64_t n_out, float *__restrict__ h)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= M * n_out) return;
    const int64_t m = i / n_out, c = i % n_out;
    const float *row = y + m * ldy + (c / 32) * kGateGroup + (c % 32);
    h[i] = silu_mul(row[0], row[32]);
}

fgmp_status_t quant_gemm_packed_out(const void *X, fgmp_dtype_t dt, int64_t M, int64_t K, int64_t ldx,
                                    const float *fisher_k, float threshold, float scale_x, const void *packed_W,
                                    int64_t N, const float *fisher_n, float threshold_y, float scale_y,
                                    void *packed_Y, size_t packed_Y_bytes, float *scores_y, void *workspace,
                                    size_t workspace_bytes, hipStream_t st, int epilogue)
{
    if (!fisher_n || !packed_Y || !workspace) return FGMP_ERR_INVALID_ARG;
    if (M <= 0 || N <= 0 || K <= 0) return FGMP_ERR_INVALID_ARG;
    const bool one_launch = (epilogue & FGMP_EPILOGUE_ONE_LAUNCH) != 0;
    epilogue &= ~(int)FGMP_EPILOGUE_ONE_LAUNCH;
    if (epilogue != FGMP_EPILOGUE_NONE && epilogue != FGMP_EPILOGUE_SILU_GATE) return FGMP_ERR_INVALID_ARG;
    if (!(scale_y > 0.0f) || !(scale_y < INFINITY) || threshold_y != threshold_y) return FGMP_ERR_INVALID_ARG;
    const bool gate = epilogue == FGMP_EPILOGUE_SILU_GATE;
    if (N % (gate ? kGateGroup : kBlock) != 0 || K % kBlock != 0) return FGMP_ERR_BAD_SHAPE;
    const int64_t n_out = gate ? N / 2 : N;   // columns of the quantized result
    if (((uintptr_t)fisher_n | (uintptr_t)packed_Y | (uintptr_t)scores_y | (uintptr_t)workspace) % 16 != 0)
        return FGMP_ERR_BAD_ALIGN;
    if (M * (N / kBlock) >= (int64_t)1 << 32) return FGMP_ERR_UNSUPPORTED;
    const PackedLayout ly = make_layout(M, n_out);
    if (packed_Y_bytes < ly.total_bytes) return FGMP_ERR_BUFFER_TOO_SMALL;
    if (workspace_bytes < gemm_workspace_bytes_packed_out(M, N, K, epilogue)) return FGMP_ERR_BUFFER_TOO_SMALL;
    PackOut po;
    po.out = make_view(packed_Y, ly);
    po.layout = ly;
    po.fisher = fisher_n;
    po.T = threshold_y;
    po.S = scale_y;
    po.scores = scores_y;
    po.gate = gate ? 1 : 0;
    po.one_launch = one_launch ? 1 : 0;
    const size_t base_bytes = gemm_workspace_bytes(M, N, K);
    // (the whole workspace: the one-launch decode step keeps its row groups' decisions behind its partial sums)
    fgmp_status_t rc = quant_gemm(X, dt, M, K, ldx, fisher_k, threshold, scale_x, packed_W, N, nullptr, N, workspace,
                                  workspace_bytes, st, FGMP_SCORE_NVFP4_ERROR, &po);
    if (rc != FGMP_ERR_UNSUPPORTED) return rc;
    float *Yf = reinterpret_cast<float *>(static_cast<char *>(workspace) + align_up(base_bytes, 256));
    rc = quant_gemm(X, dt, M, K, ldx, fisher_k, threshold, scale_x, packed_W, N, Yf, N, workspace, base_bytes, st,
                    FGMP_SCORE_NVFP4_ERROR, nullptr);
    if (rc != FGMP_OK) return rc;
    if (gate) {
        float *Hf = Yf + align_up((uint64_t)M * N * 4, 256) / 4;
        const int64_t n = M * n_out;
        hipLaunchKernelGGL(silu_gate_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, Yf, N, M, n_out, Hf);
        if (hipGetLastError() != hipSuccess) return FGMP_ERR_HIP;
        Yf = Hf;
    }
    return quantize_tensor(Yf, FGMP_F32, M, n_out, n_out, fisher_n, 0, threshold_y, scale_y, packed_Y, packed_Y_bytes,
                           scores_y, /*compact=*/false, st);
}

// Measurement reference: independent MFMAs only (8 accumulators per wave, so no instruction waits for
// the previous one's result).
__global__ __launch_bounds__(256) void mfma_rate_kernel(float *sink, int iters)
{
    half8_t a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (_Float16)(0.001f * (float)(threadIdx.x & 63) + (float)i);
        b[i] = (_Float16)(0.5f * (float)i);
    }
    float16_t acc[8];
#pragma unroll
    for (int n = 0; n < 8; ++n)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[n][r] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int n = 0; n < 8; ++n) acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[n], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int n = 0; n < 8; ++n)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[n][r];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

fgmp_status_t selftest_mfma_rate(int64_t workgroups, int32_t iters, float *sink, hipStream_t st)
{
    if (!sink || workgroups <= 0 || workgroups > 0x7FFFFFFF || iters <= 0) return FGMP_ERR_INVALID_ARG;
    hipLaunchKernelGGL(mfma_rate_kernel, dim3((unsigned)workgroups), dim3(256), 0, st, sink, (int)iters);
    return hipGetLastError() == hipSuccess ? FGMP_OK : FGMP_ERR_HIP;
}

}  // namespace fgmp
