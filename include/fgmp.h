/*
 * libfgmp -- FGMP inference hot path for AMD MI355X (gfx950), C ABI.
 *
 * FGMP (arxiv 2504.14152) keeps every block of 16 consecutive elements along
 * the dot-product dimension either in FP8 E4M3 or in NVFP4 (E2M1 values with
 * one E4M3 scale per block), chosen per block by a Fisher-weighted
 * quantization-error score compared with a calibrated threshold, and
 * multiplies activations and weights stored in that unstructured mix with
 * FP32 accumulation.
 *
 * Conventions for every entry point
 *   - X is M x K (activations), W is N x K (weights), both with K contiguous;
 *     Y = X * W^T is M x N, FP32, row-major with leading dimension ldy.
 *     Blocks run along K for both operands (Sec. 1, Sec. 4).  K % 16 == 0.
 *   - Unless a parameter says "host", every pointer is a DEVICE pointer owned
 *     by the caller.  Input/packed/workspace pointers must be 16-byte aligned.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream).  The hot-path calls (quantize_*, gemm,
 *     quant_gemm_fused, unpack_canonical) never allocate, free or synchronize.
 *   - Return value: FGMP_OK (0) or a negative fgmp_status_t.  After an error
 *     the outputs are unspecified; argument errors are detected on the host
 *     before anything is launched.
 *   - Inputs must be finite; NaN/Inf inputs give unspecified codes.
 *   - A workspace starts with FGMP_WORKSPACE_CONTROL_BYTES of arrival counters.  They must be zero
 *     when the workspace is first used (clear that much once after allocating it; nothing else in a
 *     workspace needs initializing) and every call leaves them zero, so a workspace can be reused
 *     for any sequence of calls and shapes, in or outside a captured graph.  Calls that may overlap
 *     in time need workspaces of their own.
 *   - A packed tensor is an opaque, self-describing device buffer.  Writing one
 *     needs fgmp_packed_bytes(rows, K) bytes (worst case: every block FP8); once
 *     written, its first `bytes_used` bytes (fgmp_packed_info) are all that any
 *     entry point reads.
 */
#ifndef FGMP_H
#define FGMP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FGMP_WORKSPACE_CONTROL_BYTES 65536

typedef int fgmp_status_t;
enum {
    FGMP_OK = 0,
    FGMP_ERR_INVALID_ARG = -1,      /* null pointer, non-positive size, bad enum, S <= 0 */
    FGMP_ERR_BAD_SHAPE = -2,        /* K % 16 != 0, leading dimension < row length */
    FGMP_ERR_BAD_ALIGN = -3,        /* pointer or leading dimension not 16-byte aligned */
    FGMP_ERR_BUFFER_TOO_SMALL = -4, /* packed buffer or workspace smaller than required */
    FGMP_ERR_UNSUPPORTED = -5,      /* dtype or size outside what the kernels handle */
    FGMP_ERR_HIP = -6               /* a HIP runtime call failed */
};

typedef enum { FGMP_F32 = 0, FGMP_BF16 = 1 } fgmp_dtype_t;

/* What a block's score measures (the *_ex entry points; the plain ones use FGMP_SCORE_NVFP4_ERROR).
 *   FGMP_SCORE_NVFP4_ERROR  sum_i F_i (x_i - Q_NVFP4(x_i))^2              (Eq. 6)
 *   FGMP_SCORE_DELTA        sum_i F_i (Q_NVFP4(x_i) - Q_FP8(x_i))^2       (Eq. 7, Eq. 8): the error increase
 *                           from keeping the block in NVFP4 rather than FP8.  With F = 1 this is the
 *                           "quantization error" policy (Eq. 12), with F = the other operand's mean
 *                           squared channel magnitude the "output error" policy (Eq. 13; Sec. 3.4).
 * The stored codes of a block depend only on the decision, not on the mode. */
typedef enum { FGMP_SCORE_NVFP4_ERROR = 0, FGMP_SCORE_DELTA = 1 } fgmp_score_mode_t;

/* Elementwise operator between the product and the output quantizer of
 * fgmp_quant_gemm_fused_packed_out_ex (see there); FGMP_EPILOGUE_ONE_LAUNCH is a flag that may be ORed
 * to an operator. */
typedef enum { FGMP_EPILOGUE_NONE = 0, FGMP_EPILOGUE_SILU_GATE = 1, FGMP_EPILOGUE_ONE_LAUNCH = 0x100 } fgmp_epilogue_t;

/* Host-side summary of a packed tensor (fgmp_packed_info). */
typedef struct {
    int64_t rows, K;
    float tensor_scale;
    int32_t compact;       /* 1: FP8 upper halves stored densely (weights) */
    int64_t n_blocks;      /* rows * K / 16 */
    int64_t n_fp8_blocks;  /* blocks kept in FP8 */
    int64_t bytes_used;    /* no reader touches a byte at or beyond this offset: a packed tensor may be
                              copied into a 16-byte aligned buffer of this many bytes and used there */
} fgmp_packed_info_t;

/* Library version and the name of the target architecture ("gfx950"). */
const char *fgmp_version(void);

/* Bytes of a packed rows x K tensor in the worst case (all blocks FP8),
 * including its header and per-tile tables.  0 on a bad argument. */
size_t fgmp_packed_bytes(int64_t rows, int64_t K);

/* Bytes of workspace fgmp_gemm / fgmp_quant_gemm_fused need for an
 * (M x K) * (N x K)^T product.  0 on a bad argument. */
size_t fgmp_workspace_bytes(int64_t M, int64_t N, int64_t K);

/*
 * Offline weight quantization (Sec. 3.1, Sec. 3.3): score every block of W
 * with sum_i F_i (w_i - Q_NVFP4(w_i))^2 (Eq. 6), keep it in FP8 iff the score
 * exceeds `threshold` (Sec. 4.2), else store NVFP4 with a dynamic-max E4M3
 * block scale, and pack.  The FP8 upper halves are stored compactly, so the
 * tensor occupies about 9 B per FP4 block and 16 B per FP8 block plus one bit
 * per block (Sec. 5.4.1).
 *   W          N x K, dtype dt, leading dimension ldw (elements)
 *   fisher     FP32 sensitivities: ld_fisher == 0 -> K values, one per input
 *              channel, shared by all rows; else N x K with that leading dim
 *   threshold  FP32; +INF keeps every block in FP4, -INF every block in FP8
 *   tensor_scale  S > 0: stored value = w / S; shared by both formats
 *   packed_W   out, packed_bytes >= fgmp_packed_bytes(N, K): the worst case is needed while packing;
 *              afterwards fgmp_packed_info reports bytes_used, and the first bytes_used bytes are a
 *              complete packed tensor wherever they are copied (this is where the memory saving
 *              of Sec. 5.4.1 materializes)
 *   scores_out nullable, N*K/16 FP32 scores, row-major
 */
fgmp_status_t fgmp_quantize_weights(const void *W, fgmp_dtype_t dt, int64_t N, int64_t K, int64_t ldw,
                                    const float *fisher, int64_t ld_fisher, float threshold,
                                    float tensor_scale, void *packed_W, size_t packed_bytes,
                                    float *scores_out, void *stream);

/*
 * On-the-fly activation quantization (Sec. 4.2): the same scoring and
 * decision with one sensitivity per input channel (Sec. 3.1) and a threshold
 * fixed at calibration time; one pass over X, each block written once in the
 * precision chosen for it.
 *   X          M x K, dtype dt, leading dimension ldx (elements)
 *   fisher_k   K FP32 values
 *   packed_X   out, packed_bytes >= fgmp_packed_bytes(M, K)
 *   scores_out nullable, M*K/16 FP32 scores, row-major
 */
fgmp_status_t fgmp_quantize_activations(const void *X, fgmp_dtype_t dt, int64_t M, int64_t K, int64_t ldx,
                                        const float *fisher_k, float threshold, float tensor_scale,
                                        void *packed_X, size_t packed_bytes, float *scores_out,
                                        void *stream);

/*
 * Block-mixed-precision GEMM (Sec. 4.1): Y = S_x * S_w * (X^ * W^^T) where X^,
 * W^ are the stored values (FP8 value, or E2M1 value times its E4M3 block
 * scale); every block pair is multiplied in the precision its two metadata
 * bits select and accumulated in FP32.
 *   packed_X   M x K packed activations; packed_W  N x K packed weights
 *   Y          out, M x N FP32, leading dimension ldy >= N
 *   workspace  >= fgmp_workspace_bytes(M, N, K) bytes of scratch (the decoded
 *              FP16 operands live here during the call, and the partial sums and
 *              arrival counters of output tiles that several workgroups
 *              compute together: calls that may overlap in time need
 *              workspaces of their own)
 * Operands whose headers do not match (M, K) / (N, K) are treated as zeros
 * (the planes of fixed extent -- all but the FP8 upper halves -- are still read
 * at the offsets (M, K) / (N, K) imply, so each buffer must hold a packed tensor
 * of the stated shape or at least fgmp_packed_bytes bytes).
 */
fgmp_status_t fgmp_gemm(const void *packed_X, int64_t M, const void *packed_W, int64_t N, int64_t K,
                        float *Y, int64_t ldy, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Quantize X on the fly and multiply, in one call (Sec. 4.2 followed by
 * Sec. 4.1).  The result equals fgmp_quantize_activations into the workspace
 * followed by fgmp_gemm.
 */
fgmp_status_t fgmp_quant_gemm_fused(const void *X, fgmp_dtype_t dt, int64_t M, int64_t K, int64_t ldx,
                                    const float *fisher_k, float threshold, float scale_x,
                                    const void *packed_W, int64_t N, float *Y, int64_t ldy,
                                    void *workspace, size_t workspace_bytes, void *stream);

/*
 * fgmp_quant_gemm_fused for callers that cannot allocate device memory and have no workspace to
 * hand over -- code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc:
 * the scratch memory (the quantized activations as FP16 values, partial sums and arrival counters
 * of products computed in several parts) lives in a static device array of
 * FGMP_STATIC_SCRATCH_BYTES inside the library, one per GPU, held until the process ends.  The
 * call allocates nothing and frees nothing; same arguments, results (bit for bit) and errors as
 * fgmp_quant_gemm_fused, without the workspace.
 *   limit      the scratch this call uses (never more than fgmp_workspace_bytes(M, N, K); less for the
 *              decode shapes that one kernel handles) <= FGMP_STATIC_SCRATCH_BYTES, else
 *              FGMP_ERR_BUFFER_TOO_SMALL and nothing is launched (all decode shapes, M <= 32, of the
 *              Llama-2-7B linears fit; prefill shapes generally do not)
 *   sharing    every call on a GPU uses that GPU's one array: calls that overlap in time on the
 *              same GPU (different streams or threads) race; calls on one stream are ordered
 *   first call on a device looks up the array's address (hipGetSymbolAddress); make that call
 *              outside a stream capture
 */
#define FGMP_STATIC_SCRATCH_BYTES (16 * 1024 * 1024)
fgmp_status_t fgmp_quant_gemm_fused_static_scratch(const void *X, fgmp_dtype_t dt, int64_t M, int64_t K,
                                                   int64_t ldx, const float *fisher_k, float threshold,
                                                   float scale_x, const void *packed_W, int64_t N, float *Y,
                                                   int64_t ldy, void *stream);

/*
 * The three calls above with the score selected by `score_mode` (Sec. 3.1, Eq. 8; Sec. 3.4);
 * all other arguments, outputs and errors as the plain calls.  FGMP_ERR_INVALID_ARG for an unknown mode.
 */
fgmp_status_t fgmp_quantize_weights_ex(const void *W, fgmp_dtype_t dt, int64_t N, int64_t K, int64_t ldw,
                                       const float *fisher, int64_t ld_fisher, float threshold,
                                       float tensor_scale, fgmp_score_mode_t score_mode, void *packed_W,
                                       size_t packed_bytes, float *scores_out, void *stream);
fgmp_status_t fgmp_quantize_activations_ex(const void *X, fgmp_dtype_t dt, int64_t M, int64_t K, int64_t ldx,
                                           const float *fisher_k, float threshold, float tensor_scale,
                                           fgmp_score_mode_t score_mode, void *packed_X, size_t packed_bytes,
                                           float *scores_out, void *stream);
fgmp_status_t fgmp_quant_gemm_fused_ex(const void *X, fgmp_dtype_t dt, int64_t M, int64_t K, int64_t ldx,
                                       const float *fisher_k, float threshold, float scale_x,
                                       fgmp_score_mode_t score_mode, const void *packed_W, int64_t N, float *Y,
                                       int64_t ldy, void *workspace, size_t workspace_bytes, void *stream);

/*
 * The fused call with output-side quantization (Sec. 4.2: results are quantized before they are
 * written to memory): Y = X^ * W^^T is not stored as FP32; each block of 16 consecutive output
 * columns (= 16 consecutive input channels of the next layer) is scored (Eq. 6) with `fisher_n`,
 * compared with `threshold_y` and stored as FP8 or NVFP4 in `packed_Y`, a packed M x N activation
 * tensor (tensor scale `scale_y`) that the next layer's fgmp_gemm consumes.  The values that are
 * quantized are exactly the FP32 numbers fgmp_quant_gemm_fused would have written.  For shapes that
 * run on the prefill kernel this happens in its epilogue; smaller M stage the FP32 results in the
 * workspace and launch the standalone quantizer.  A decode step (M <= 32) can also do it inside its one
 * launch (FGMP_EPILOGUE_ONE_LAUNCH of the _ex form): the wave that holds the final sums of 16 output
 * columns quantizes them, and the eight such waves behind one 128-column tile of packed_Y settle the
 * tile's mask word and plane-H order through a counter in the workspace's control region.  That chain of
 * memory round trips at the end of the launch measured 1-8 us slower than the second launch, so it is
 * not the default; the packed tensor is the same bit for bit either way.
 *   fisher_n   N FP32 sensitivities; N % 16 == 0
 *   packed_Y   out, packed_Y_bytes >= fgmp_packed_bytes(M, N); scores_y nullable, M*N/16 FP32
 *   workspace  >= fgmp_workspace_bytes_packed_out(M, N, K)
 */
size_t fgmp_workspace_bytes_packed_out(int64_t M, int64_t N, int64_t K);
fgmp_status_t fgmp_quant_gemm_fused_packed_out(const void *X, fgmp_dtype_t dt, int64_t M, int64_t K, int64_t ldx,
                                               const float *fisher_k, float threshold, float scale_x,
                                               const void *packed_W, int64_t N, const float *fisher_n,
                                               float threshold_y, float scale_y, void *packed_Y,
                                               size_t packed_Y_bytes, float *scores_y, void *workspace,
                                               size_t workspace_bytes, void *stream);

/*
 * The same with an elementwise operator in front of the quantizer, so that the gated MLP of the models
 * the paper evaluates (Sec. 5.1: FC1 = gate and up projection, FC2 = down projection) goes from FC1 to
 * FC2 without its intermediate ever being stored unquantized.  FGMP_EPILOGUE_NONE: as above.
 * FGMP_EPILOGUE_SILU_GATE: the N weight rows come in groups of 64 -- rows 64q .. 64q+31 are the gate
 * rows of hidden units 32q .. 32q+31, rows 64q+32 .. 64q+63 their up rows -- and what is scored,
 * quantized and packed is h = SiLU(g) * u per hidden unit, an M x N/2 tensor, with g and u the FP32
 * numbers fgmp_quant_gemm_fused would have written.  The paper does not discuss the operator; since
 * the codes depend on h to the last bit, h is a fixed sequence of FP32 operations, each rounded on its
 * own: E(x) for x clamped to [-87, 88] is p * 2^n with n = rint(x * log2 e), r = (x - n * 0.693359375)
 * - n * (ln 2 - 0.693359375) and p the degree-7 Taylor polynomial of e^r by Horner's rule;
 * h = (g / (1 + E(-g))) * u with a correctly rounded division (within 3 ulp of the exact value).
 * `epilogue | FGMP_EPILOGUE_ONE_LAUNCH` (with FGMP_EPILOGUE_NONE): a decode step quantizes its results
 * inside its launch whenever the one-launch kernel handles the shape (nothing is staged; a single kernel
 * per layer for callers who count launches); shapes that no quantizing epilogue covers are staged as before.
 *   N          N % 64 == 0 with the gate; fisher_n, scores_y and packed_Y then refer to N/2 columns
 *   workspace  >= fgmp_workspace_bytes_packed_out_ex(M, N, K, epilogue)
 * Other arguments and errors as fgmp_quant_gemm_fused_packed_out; an unknown `epilogue` is
 * FGMP_ERR_INVALID_ARG.
 */
size_t fgmp_workspace_bytes_packed_out_ex(int64_t M, int64_t N, int64_t K, fgmp_epilogue_t epilogue);
fgmp_status_t fgmp_quant_gemm_fused_packed_out_ex(const void *X, fgmp_dtype_t dt, int64_t M, int64_t K, int64_t ldx,
                                                  const float *fisher_k, float threshold, float scale_x,
                                                  const void *packed_W, int64_t N, fgmp_epilogue_t epilogue,
                                                  const float *fisher_n, float threshold_y, float scale_y,
                                                  void *packed_Y, size_t packed_Y_bytes, float *scores_y,
                                                  void *workspace, size_t workspace_bytes, void *stream);

/*
 * Offline weight quantization with sensitivity-weighted clipping (Sec. 3.3, Eq. 11): the E4M3
 * scale of every block is the one, among all 127 non-negative E4M3 values, that minimizes
 * sum_i F_i (w_i - Q_s(w_i))^2 (the smallest such code if several tie) instead of the dynamic-max
 * scale; the block's score (Eq. 6) and the FP8/FP4 decision then use that scale.  Everything else as
 * fgmp_quantize_weights.
 *   workspace  device scratch, at least N*K/16 bytes (the chosen scale codes); contents undefined after
 * Errors: as fgmp_quantize_weights; FGMP_ERR_BUFFER_TOO_SMALL for the workspace.
 */
fgmp_status_t fgmp_quantize_weights_clip(const void *W, fgmp_dtype_t dt, int64_t N, int64_t K, int64_t ldw,
                                         const float *fisher, int64_t ld_fisher, float threshold,
                                         float tensor_scale, void *packed_W, size_t packed_bytes,
                                         float *scores_out, void *workspace, size_t workspace_bytes,
                                         void *stream);

/*
 * Expand a packed tensor to layout-independent arrays (for tests and tools):
 *   codes   rows*K bytes: E2M1 code 0..15 (FP4 block) or E4M3 byte (FP8 block)
 *   scales  rows*K/16 bytes: E4M3 block scale, 0 for FP8 blocks
 *   mask    rows*K/16 bytes: 1 = FP8 block
 * Any of the three may be NULL.
 */
fgmp_status_t fgmp_unpack_canonical(const void *packed, int64_t rows, int64_t K, uint8_t *codes,
                                    uint8_t *scales, uint8_t *mask, void *stream);

/*
 * Decode a packed tensor to dense FP16 (IEEE binary16), the operand form the
 * GEMM kernels multiply: FP8 block -> its E4M3 values; FP4 block -> E2M1 value
 * times the E4M3 block scale (exact in FP16); the tensor scale is not applied.
 *   out   rows_out x ld halves, rows_out >= rows a multiple of 8, ld >= K
 *         rounded up to a multiple of 128 exactly; rows and columns beyond the tensor
 *         are written as zeros
 */
fgmp_status_t fgmp_dequantize_f16(const void *packed, int64_t rows, int64_t K, void *out, int64_t rows_out,
                                  int64_t ld, void *stream);

/*
 * Quantize activations (Sec. 3.1-3.3, Eq. 6; same selection as
 * fgmp_quantize_activations) and write, instead of the packed codes, the FP16
 * value of every stored code: the "quantize then dequantize" form of X that the
 * fused prefill path feeds to the GEMM.  Bit-identical to
 * fgmp_quantize_activations followed by fgmp_dequantize_f16; the tensor scale
 * is not applied (x_hat = tensor_scale * out).
 *   X, dt, M, K, ldx, fisher_k, threshold, tensor_scale   as fgmp_quantize_activations
 *   out   device, rows_out x ld halves, 16-byte aligned; rows_out >= M rounded
 *         up to a multiple of 8; ld >= K rounded up to a multiple of 128 and a
 *         multiple of 8; rows M.. of the last 8-row group and columns K.. of the
 *         last 128-column group are written as zeros, nothing beyond them
 * Errors: as fgmp_quantize_activations; FGMP_ERR_BAD_SHAPE for rows_out / ld.
 */
fgmp_status_t fgmp_quantize_dequantize_f16(const void *X, fgmp_dtype_t dt, int64_t M, int64_t K, int64_t ldx,
                                           const float *fisher_k, float threshold, float tensor_scale,
                                           void *out, int64_t rows_out, int64_t ld, void *stream);

/*
 * Offline helpers.  These synchronize `stream` and use host memory.
 */

/* Read a packed tensor's header and count its FP8 blocks. info_host: host. */
fgmp_status_t fgmp_packed_info(const void *packed, fgmp_packed_info_t *info_host, void *stream);

/* Threshold for a target fraction of FP8 blocks (Eq. 9): the score below the
 * round(fraction*J) largest of the J device-resident scores; fraction 0 ->
 * +INF, 1 -> -INF.  threshold_host: host.  Found on the device (an exact radix
 * selection: four passes over the scores, which stay where they are); the call
 * allocates a few KB of device memory for its counters, synchronizes `stream`
 * and frees them. */
fgmp_status_t fgmp_threshold_for_fraction(const float *scores, int64_t J, double fraction,
                                          float *threshold_host, void *stream);

/* One threshold for several tensors (Eq. 10): the same order statistic taken over
 * the union of n_tensors score arrays (e.g. the weights, or the activations, of
 * every layer), so that layers keep different fractions of their blocks in FP8
 * while the total matches `fraction`.
 *   scores  host array of n_tensors device pointers; counts  host array of their lengths
 * The union is never formed: every pass of the selection counts over all the arrays.  Synchronizes
 * `stream`. */
fgmp_status_t fgmp_threshold_for_fraction_multi(const float *const *scores, const int64_t *counts,
                                                int32_t n_tensors, double fraction, float *threshold_host,
                                                void *stream);

/*
 * Conversion self-test hooks: run the library's device-side FP32 -> E2M1
 * (format 0) or FP32 -> E4M3 (format 1) rounding over every non-negative FP32
 * bit pattern 0 .. 0x7F800000 (finite values and +INF) and report, per output
 * code, the smallest and largest input bit pattern that produced it
 * (min_bits/max_bits: 256 uint32 each, device; untouched codes keep
 * 0xFFFFFFFF / 0) plus the number of places where the code decreased as the
 * input grew (violations: 1 uint32, device).
 * fgmp_decode_table writes the device-side decode of all 256 codes of the
 * format as FP32 (out: 256 floats, device; E2M1 uses the low nibble).
 */
fgmp_status_t fgmp_selftest_encode_ranges(int format, uint32_t *min_bits, uint32_t *max_bits,
                                          uint32_t *violations, void *stream);
fgmp_status_t fgmp_selftest_decode_table(int format, float *out, void *stream);

/*
 * Measurement reference: a loop of nothing but independent dense FP16 matrix
 * instructions (32x32x16, FP32 accumulate) -- the rate the prefill GEMM's
 * roofline fraction can also be quoted against.  Launches `workgroups`
 * workgroups of 4 waves, each wave issuing 8 * iters instructions (32768 flops
 * each); the caller times the launch.  sink: device, workgroups * 256 floats,
 * written once at the end (keeps the arithmetic alive).
 */
fgmp_status_t fgmp_selftest_mfma_rate(int64_t workgroups, int32_t iters, float *sink, void *stream);

/*
 * Measurement hook: the duration of the prefill GEMM kernel inside a fused
 * call.  Only libraries built with FGMP_MEASUREMENT_HOOKS have it (the
 * benchmark's libfgmp_hooks.so); in the shipped library setting a pair returns
 * FGMP_ERR_UNSUPPORTED and the launcher records nothing.  While a pair of HIP events (hipEvent_t, created by the caller with
 * timing enabled) is set, every launch of that kernel records `ev_start` on
 * its stream immediately before the launch and `ev_stop` immediately after;
 * the caller synchronizes and reads hipEventElapsedTime.  Two null pointers
 * clear the hook; one null and one non-null pointer is FGMP_ERR_INVALID_ARG.
 * The pair is process-wide state, not synchronized: for single-threaded
 * measurement code only.  The events stay the caller's; clear the hook before
 * destroying them.
 */
fgmp_status_t fgmp_selftest_time_gemm_kernel(void *ev_start, void *ev_stop);

/*
 * Measurement reference for the activation quantizer (Sec. 4.2 as a memory-bound pass): the quantizer's
 * kernel for large tensors with its arithmetic taken out -- the same loads of X, the same stores to the
 * planes of `packed_out` (a fixed tenth of the blocks written as FP8), contents meaningless -- so that
 * the benchmark can put the time the memory system alone takes for this access pattern beside the real
 * kernel's, in the same run.  Arguments as fgmp_quantize_activations (bf16 or fp32 X, per-channel
 * `fisher_k`, which is read but not used).  Only libraries built with FGMP_MEASUREMENT_HOOKS have it;
 * elsewhere, and for tensors too small for that kernel (fewer than 65536 tiles of 8 x 128), it returns
 * FGMP_ERR_UNSUPPORTED.
 */
fgmp_status_t fgmp_selftest_quantizer_traffic(const void *X, fgmp_dtype_t dt, int64_t M, int64_t K, int64_t ldx,
                                              const float *fisher_k, void *packed_out, size_t packed_bytes,
                                              void *stream);

#ifdef __cplusplus
}
#endif
#endif /* FGMP_H */
