// Internal declarations shared by the translation units of libfgmp.
#pragma once
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "../../include/fgmp.h"
#include "fgmp_formats.hpp"
#include "fgmp_layout.hpp"

namespace fgmp {

// Use the gfx950 conversion instructions in the quantizer.  They are only
// enabled because the conversion self-test shows them equal to the integer
// forms for every FP32 input.
#ifndef FGMP_HW_CVT
#define FGMP_HW_CVT 1
#endif
constexpr bool kUseHwCvt = FGMP_HW_CVT != 0;

fgmp_status_t quantize_tensor(const void *X, fgmp_dtype_t dt, int64_t rows, int64_t K, int64_t ldx,
                              const float *fisher, int64_t ld_fisher, float T, float S, void *packed,
                              size_t packed_bytes, float *scores, bool compact, hipStream_t st,
                              _Float16 *x16 = nullptr, int64_t ld16 = 0, uint32_t *zero = nullptr,
                              int64_t zero_n = 0, int score_mode = FGMP_SCORE_NVFP4_ERROR,
                              uint8_t *clip_scales = nullptr);
#ifdef FGMP_MEASUREMENT_HOOKS
fgmp_status_t quantize_traffic_model(const void *X, fgmp_dtype_t dt, int64_t rows, int64_t K, int64_t ldx, const float *fisher,
                                     void *packed, size_t packed_bytes, hipStream_t st);
#endif
fgmp_status_t unpack_tensor(const void *packed, int64_t rows, int64_t K, uint8_t *codes, uint8_t *scales,
                            uint8_t *mask, hipStream_t st);
fgmp_status_t gemm_packed(const void *packed_X, int64_t M, const void *packed_W, int64_t N, int64_t K,
                          float *Y, int64_t ldy, void *workspace, size_t workspace_bytes, hipStream_t st,
                          size_t skip = 0);
size_t gemm_workspace_bytes(int64_t M, int64_t N, int64_t K);
// what fgmp_quant_gemm_fused itself uses of a workspace (control region included)
size_t quant_gemm_workspace_need(int64_t M, int64_t N, int64_t K);
struct PackOut;
// quantize X and multiply in one call; `workspace` holds at least gemm_workspace_bytes(M, N, K)
fgmp_status_t quant_gemm(const void *X, fgmp_dtype_t dt, int64_t M, int64_t K, int64_t ldx, const float *fisher_k,
                         float threshold, float scale_x, const void *packed_W, int64_t N, float *Y, int64_t ldy,
                         void *workspace, size_t workspace_bytes, hipStream_t st,
                         int score_mode = FGMP_SCORE_NVFP4_ERROR, const PackOut *pack_out = nullptr);
size_t gemm_workspace_bytes_packed_out(int64_t M, int64_t N, int64_t K, int epilogue = FGMP_EPILOGUE_NONE);
fgmp_status_t quant_gemm_packed_out(const void *X, fgmp_dtype_t dt, int64_t M, int64_t K, int64_t ldx,
                                    const float *fisher_k, float threshold, float scale_x, const void *packed_W,
                                    int64_t N, const float *fisher_n, float threshold_y, float scale_y,
                                    void *packed_Y, size_t packed_Y_bytes, float *scores_y, void *workspace,
                                    size_t workspace_bytes, hipStream_t st, int epilogue = FGMP_EPILOGUE_NONE);
// Decode shapes (few rows of X): weight-streaming kernel.  X is given as FP16 values (`x16`,
// gemm_skinny_x16_rows(M) rows of ld16 halves; rows from M rounded up to 8 on are never used for a
// stored output) plus the header of its packed form.
constexpr int64_t kSkinnyMaxRows = 256;   // in chunks of 32 rows, one launch each, while that beats the prefill kernel
bool gemm_skinny_applies(int64_t M, int64_t N, int64_t K);
int64_t gemm_skinny_x16_rows(int64_t M);
size_t gemm_skinny_workspace_bytes(int64_t M, int64_t N, int64_t K);
// arrival counters inside a skinny workspace; the kernel that prepares x16 must zero them
struct SkinnyCounters {
    uint32_t *ptr;
    int64_t n;
};
SkinnyCounters gemm_skinny_counters(int64_t M, int64_t N, int64_t K, void *workspace);
fgmp_status_t gemm_skinny(const PackedHeader *xh, const PackedLayout &lx, const _Float16 *x16, int64_t ld16,
                          const void *w, const PackedLayout &lw, int64_t M, int64_t N, int64_t K, float *Y,
                          int64_t ldy, void *workspace, hipStream_t st);
// Every workspace starts with a control region: arrival counters that must be zero when a call starts and
// that every call leaves zero (the caller clears them once, after allocating).  Nothing but the
// single-launch decode kernel touches it; all other scratch starts behind it.
constexpr size_t kWsCtrlRegion = FGMP_WORKSPACE_CONTROL_BYTES;
// Decode shapes (M <= 32) in one launch: the activations are quantized (src 0: bf16 X, 1: fp32 X) or
// decoded (src 2: packed X) inside the kernel that streams the weights.
bool gemm_stream_applies(int64_t M, int64_t N, int64_t K);
size_t gemm_stream_scratch_bytes(int64_t M, int64_t N, int64_t K);
fgmp_status_t gemm_stream(int src, const void *X, int64_t ldx, const float *fisher, float T, float S, const void *packed_X,
                          int64_t M, const void *packed_W, int64_t N, int64_t K, float *Y, int64_t ldy, void *ctrl,
                          void *scratch, hipStream_t st, const PackOut *po = nullptr);
bool gemm_stream_packs(int64_t M, int64_t N, int64_t K);
size_t gemm_stream_pack_scratch_bytes(int64_t M, int64_t N, int64_t K);
// packed -> zero-padded dense FP16 [8 n_rt_pad][ld]; one launch decodes one or two tensors and
// can clear `zero_n` 32-bit counters
struct DecodeJob {
    PackedView v;
    PackedLayout l;
    _Float16 *out;
    int64_t ld, waves;
};
DecodeJob make_decode_job(const PackedView &v, const PackedLayout &l, _Float16 *out, int64_t ld, int64_t n_rt_pad);
fgmp_status_t launch_decode_f16(const DecodeJob &a, const DecodeJob *b, uint32_t *zero, int64_t zero_n,
                                hipStream_t st);
// Output-side quantization of the prefill GEMM: where the packed results go and how they are scored.
struct PackOut {
    PackedView out;        // packed M x N tensor ("strided"), N being the next layer's K
    PackedLayout layout;
    const float *fisher;   // N sensitivities (input channels of the next layer)
    float T, S;            // threshold and tensor scale of the output tensor
    float *scores;         // nullable, M * N / 16
    int gate;              // nonzero: quantize SiLU(gate) * up of the 32 + 32 row groups of W; `out` is M x N / 2
    int one_launch;        // nonzero: a decode step quantizes inside its launch (the default stages FP32 results: measured faster)
};
// The last, partly filled round of tiles of the prefill kernel, split along K (n_split 0: no split).
struct SplitTail {
    int n_whole;              // workgroups [0, n_whole) compute whole tiles
    int n_split;              // tiles n_whole .. n_whole + n_split - 1 are computed by n_parts workgroups each
    int n_parts;              // 2, or 4 when that still fits one round of the chip
    int kt_bound[5];          // part p covers K-steps [kt_bound[p], kt_bound[p + 1]) (all even)
    int n_counters;           // n_split, or 3 n_split with four parts (two pairs, then the pair sums)
    uint32_t partial_bytes;   // n_split * 256 KB * (2, or 6 with four parts: 4 parts + 2 pair sums)
    float *partial;           // accumulators of the parts, 16-byte aligned
    uint32_t *counters;       // arrival counters, zero at launch
};
// Workspace bytes the split of `n_tiles` output tiles needs (0: no split), and the split itself with its
// buffers at `region` (that many bytes, 256-byte aligned); `nk` K-steps of 64.
size_t gemm_mixed_split_bytes(int64_t n_tiles);
SplitTail plan_split_tail(int64_t n_tiles, int nk, void *region);
// `sp.counters` (sp.n_counters words) must be zero when the kernel starts
void launch_gemm_mixed(const _Float16 *a16, int64_t ld, const PackedView &W, const PackedLayout &lw, float *Y,
                       int64_t ldy, int64_t M, int64_t N, int64_t n_tm, int64_t n_tn, const PackedHeader *ha,
                       hipStream_t st, const SplitTail &sp, const PackOut *pack_out = nullptr);
fgmp_status_t selftest_encode_ranges(int format, uint32_t *min_bits, uint32_t *max_bits,
                                     uint32_t *violations, hipStream_t st);
fgmp_status_t selftest_decode_table(int format, float *out, hipStream_t st);
fgmp_status_t selftest_mfma_rate(int64_t workgroups, int32_t iters, float *sink, hipStream_t st);
// element of rank `rank` (0 = smallest) of the union of n_tensors device arrays; result on the host; synchronizes
fgmp_status_t select_rank(const float *const *scores, const int64_t *counts, int32_t n_tensors, int64_t rank, float *result_host,
                          hipStream_t st);
// events recorded around every launch of the prefill GEMM kernel (both null: none); false when the
// library was built without the measurement hooks
bool set_gemm_kernel_events(hipEvent_t start, hipEvent_t stop);

}  // namespace fgmp
