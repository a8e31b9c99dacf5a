// C ABI of libfgmp: argument checks and dispatch.  See include/fgmp.h.
#include <algorithm>
#include <atomic>
#include <vector>

#include "fgmp_internal.hpp"

using namespace fgmp;

static inline hipStream_t as_stream(void *s) { return static_cast<hipStream_t>(s); }

// Scratch memory of fgmp_quant_gemm_fused_static_scratch: one array per GPU the library runs on, held
// until the process ends.  The name below is a host-side stand-in, not a device address: host code
// reaches the array only through the address hipGetSymbolAddress returns, looked up once per device.
static __device__ __align__(256) unsigned char scratch[FGMP_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
static std::atomic<void *> g_scratch_ptr[kMaxDevices];

static fgmp_status_t static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return FGMP_ERR_HIP;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        // (two threads may both look it up: they get the same address)
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return FGMP_ERR_HIP;
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return FGMP_OK;
}

extern "C" {

const char *fgmp_version(void) { return "fgmp 0.1 (gfx950)"; }

size_t fgmp_packed_bytes(int64_t rows, int64_t K)
{
    if (rows <= 0 || K <= 0 || K % kBlock != 0) return 0;
    return (size_t)make_layout(rows, K).total_bytes;
}

size_t fgmp_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    if (M <= 0 || N <= 0 || K <= 0 || K % kBlock != 0) return 0;
    return gemm_workspace_bytes(M, N, K);
}

fgmp_status_t fgmp_quantize_weights(const void *W, fgmp_dtype_t dt, int64_t N, int64_t K, int64_t ldw,
                                    const float *fisher, int64_t ld_fisher, float threshold,
                                    float tensor_scale, void *packed_W, size_t packed_bytes,
                                    float *scores_out, void *stream)
{
    return quantize_tensor(W, dt, N, K, ldw, fisher, ld_fisher, threshold, tensor_scale, packed_W,
                           packed_bytes, scores_out, /*compact=*/true, as_stream(stream));
}

fgmp_status_t fgmp_quantize_activations(const void *X, fgmp_dtype_t dt, int64_t M, int64_t K, int64_t ldx,
                                        const float *fisher_k, float threshold, float tensor_scale,
                                        void *packed_X, size_t packed_bytes, float *scores_out,
                                        void *stream)
{
    return quantize_tensor(X, dt, M, K, ldx, fisher_k, /*ld_fisher=*/0, threshold, tensor_scale, packed_X,
                           packed_bytes, scores_out, /*compact=*/false, as_stream(stream));
}

fgmp_status_t fgmp_gemm(const void *packed_X, int64_t M, const void *packed_W, int64_t N, int64_t K,
                        float *Y, int64_t ldy, void *workspace, size_t workspace_bytes, void *stream)
{
    return gemm_packed(packed_X, M, packed_W, N, K, Y, ldy, workspace, workspace_bytes, as_stream(stream));
}

fgmp_status_t fgmp_quant_gemm_fused(const void *X, fgmp_dtype_t dt, int64_t M, int64_t K, int64_t ldx,
                                    const float *fisher_k, float threshold, float scale_x,
                                    const void *packed_W, int64_t N, float *Y, int64_t ldy,
                                    void *workspace, size_t workspace_bytes, void *stream)
{
    return quant_gemm(X, dt, M, K, ldx, fisher_k, threshold, scale_x, packed_W, N, Y, ldy, workspace,
                      workspace_bytes, as_stream(stream));
}

fgmp_status_t fgmp_quant_gemm_fused_static_scratch(const void *X, fgmp_dtype_t dt, int64_t M, int64_t K, int64_t ldx,
                                                   const float *fisher_k, float threshold, float scale_x,
                                                   const void *packed_W, int64_t N, float *Y, int64_t ldy,
                                                   void *stream)
{
    if (M <= 0 || N <= 0 || K <= 0) return FGMP_ERR_INVALID_ARG;
    if (K % kBlock != 0) return FGMP_ERR_BAD_SHAPE;
    // the size check comes first: a product that does not fit must not touch the array
    if (quant_gemm_workspace_need(M, N, K) > (size_t)FGMP_STATIC_SCRATCH_BYTES) return FGMP_ERR_BUFFER_TOO_SMALL;
    void *ws = nullptr;
    const fgmp_status_t rc = static_scratch(&ws);
    if (rc != FGMP_OK) return rc;
    return quant_gemm(X, dt, M, K, ldx, fisher_k, threshold, scale_x, packed_W, N, Y, ldy, ws,
                      (size_t)FGMP_STATIC_SCRATCH_BYTES, as_stream(stream));
}

fgmp_status_t fgmp_quantize_weights_ex(const void *W, fgmp_dtype_t dt, int64_t N, int64_t K, int64_t ldw,
                                       const float *fisher, int64_t ld_fisher, float threshold,
                                       float tensor_scale, fgmp_score_mode_t score_mode, void *packed_W,
                                       size_t packed_bytes, float *scores_out, void *stream)
{
    return quantize_tensor(W, dt, N, K, ldw, fisher, ld_fisher, threshold, tensor_scale, packed_W,
                           packed_bytes, scores_out, /*compact=*/true, as_stream(stream), nullptr, 0, nullptr, 0,
                           (int)score_mode);
}

fgmp_status_t fgmp_quantize_activations_ex(const void *X, fgmp_dtype_t dt, int64_t M, int64_t K, int64_t ldx,
                                           const float *fisher_k, float threshold, float tensor_scale,
                                           fgmp_score_mode_t score_mode, void *packed_X, size_t packed_bytes,
                                           float *scores_out, void *stream)
{
    return quantize_tensor(X, dt, M, K, ldx, fisher_k, /*ld_fisher=*/0, threshold, tensor_scale, packed_X,
                           packed_bytes, scores_out, /*compact=*/false, as_stream(stream), nullptr, 0, nullptr, 0,
                           (int)score_mode);
}

fgmp_status_t fgmp_quant_gemm_fused_ex(const void *X, fgmp_dtype_t dt, int64_t M, int64_t K, int64_t ldx,
                                       const float *fisher_k, float threshold, float scale_x,
                                       fgmp_score_mode_t score_mode, const void *packed_W, int64_t N, float *Y,
                                       int64_t ldy, void *workspace, size_t workspace_bytes, void *stream)
{
    return quant_gemm(X, dt, M, K, ldx, fisher_k, threshold, scale_x, packed_W, N, Y, ldy, workspace,
                      workspace_bytes, as_stream(stream), (int)score_mode);
}

size_t fgmp_workspace_bytes_packed_out(int64_t M, int64_t N, int64_t K)
{
    if (M <= 0 || N <= 0 || K <= 0 || K % kBlock != 0 || N % kBlock != 0) return 0;
    return gemm_workspace_bytes_packed_out(M, N, K);
}

fgmp_status_t fgmp_quant_gemm_fused_packed_out(const void *X, fgmp_dtype_t dt, int64_t M, int64_t K, int64_t ldx,
                                               const float *fisher_k, float threshold, float scale_x,
                                               const void *packed_W, int64_t N, const float *fisher_n,
                                               float threshold_y, float scale_y, void *packed_Y,
                                               size_t packed_Y_bytes, float *scores_y, void *workspace,
                                               size_t workspace_bytes, void *stream)
{
    return quant_gemm_packed_out(X, dt, M, K, ldx, fisher_k, threshold, scale_x, packed_W, N, fisher_n, threshold_y,
                                 scale_y, packed_Y, packed_Y_bytes, scores_y, workspace, workspace_bytes,
                                 as_stream(stream));
}

size_t fgmp_workspace_bytes_packed_out_ex(int64_t M, int64_t N, int64_t K, fgmp_epilogue_t epilogue)
{
    const int op = (int)epilogue & ~(int)FGMP_EPILOGUE_ONE_LAUNCH;
    if (op != FGMP_EPILOGUE_NONE && op != FGMP_EPILOGUE_SILU_GATE) return 0;
    const int64_t n_unit = op == FGMP_EPILOGUE_SILU_GATE ? 64 : kBlock;
    if (M <= 0 || N <= 0 || K <= 0 || K % kBlock != 0 || N % n_unit != 0) return 0;
    return gemm_workspace_bytes_packed_out(M, N, K, op);
}

fgmp_status_t fgmp_quant_gemm_fused_packed_out_ex(const void *X, fgmp_dtype_t dt, int64_t M, int64_t K, int64_t ldx,
                                                  const float *fisher_k, float threshold, float scale_x,
                                                  const void *packed_W, int64_t N, fgmp_epilogue_t epilogue,
                                                  const float *fisher_n, float threshold_y, float scale_y,
                                                  void *packed_Y, size_t packed_Y_bytes, float *scores_y,
                                                  void *workspace, size_t workspace_bytes, void *stream)
{
    return quant_gemm_packed_out(X, dt, M, K, ldx, fisher_k, threshold, scale_x, packed_W, N, fisher_n, threshold_y,
                                 scale_y, packed_Y, packed_Y_bytes, scores_y, workspace, workspace_bytes,
                                 as_stream(stream), (int)epilogue);
}

fgmp_status_t fgmp_quantize_weights_clip(const void *W, fgmp_dtype_t dt, int64_t N, int64_t K, int64_t ldw,
                                         const float *fisher, int64_t ld_fisher, float threshold,
                                         float tensor_scale, void *packed_W, size_t packed_bytes,
                                         float *scores_out, void *workspace, size_t workspace_bytes,
                                         void *stream)
{
    if (!workspace) return FGMP_ERR_INVALID_ARG;
    if (N <= 0 || K <= 0) return FGMP_ERR_INVALID_ARG;
    if (K % kBlock != 0) return FGMP_ERR_BAD_SHAPE;
    if (workspace_bytes < (size_t)(N * (K / kBlock))) return FGMP_ERR_BUFFER_TOO_SMALL;
    return quantize_tensor(W, dt, N, K, ldw, fisher, ld_fisher, threshold, tensor_scale, packed_W,
                           packed_bytes, scores_out, /*compact=*/true, as_stream(stream), nullptr, 0, nullptr, 0,
                           FGMP_SCORE_NVFP4_ERROR, static_cast<uint8_t *>(workspace));
}

fgmp_status_t fgmp_unpack_canonical(const void *packed, int64_t rows, int64_t K, uint8_t *codes,
                                    uint8_t *scales, uint8_t *mask, void *stream)
{
    return unpack_tensor(packed, rows, K, codes, scales, mask, as_stream(stream));
}

fgmp_status_t fgmp_dequantize_f16(const void *packed, int64_t rows, int64_t K, void *out, int64_t rows_out,
                                  int64_t ld, void *stream)
{
    if (!packed || !out || rows <= 0 || K <= 0) return FGMP_ERR_INVALID_ARG;
    if (K % kBlock != 0) return FGMP_ERR_BAD_SHAPE;
    const PackedLayout l = make_layout(rows, K);
    if (rows_out < rows || rows_out % kTileRows != 0 || ld != l.n_kt * kTileK) return FGMP_ERR_BAD_SHAPE;
    if (((uintptr_t)packed | (uintptr_t)out) % 16 != 0) return FGMP_ERR_BAD_ALIGN;
    const DecodeJob job = make_decode_job(make_view(const_cast<void *>(packed), l), l, static_cast<_Float16 *>(out),
                                          ld, rows_out / kTileRows);
    const fgmp_status_t rc = launch_decode_f16(job, nullptr, nullptr, 0, as_stream(stream));
    if (rc != FGMP_OK) return rc;
    return hipGetLastError() == hipSuccess ? FGMP_OK : FGMP_ERR_HIP;
}

fgmp_status_t fgmp_quantize_dequantize_f16(const void *X, fgmp_dtype_t dt, int64_t M, int64_t K, int64_t ldx,
                                           const float *fisher_k, float threshold, float tensor_scale,
                                           void *out, int64_t rows_out, int64_t ld, void *stream)
{
    if (!out || M <= 0 || K <= 0) return FGMP_ERR_INVALID_ARG;
    if (K % kBlock != 0) return FGMP_ERR_BAD_SHAPE;
    if (rows_out < (M + kTileRows - 1) / kTileRows * kTileRows) return FGMP_ERR_BAD_SHAPE;
    return quantize_tensor(X, dt, M, K, ldx, fisher_k, /*ld_fisher=*/0, threshold, tensor_scale, nullptr, 0,
                           nullptr, /*compact=*/false, as_stream(stream), static_cast<_Float16 *>(out), ld);
}

fgmp_status_t fgmp_packed_info(const void *packed, fgmp_packed_info_t *info_host, void *stream)
{
    if (!packed || !info_host) return FGMP_ERR_INVALID_ARG;
    hipStream_t st = as_stream(stream);
    PackedHeader h;
    if (hipMemcpyAsync(&h, packed, sizeof h, hipMemcpyDeviceToHost, st) != hipSuccess) return FGMP_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return FGMP_ERR_HIP;
    if (h.magic != kMagic || h.version != kVersion || h.rows <= 0 || h.K <= 0 || h.K % kBlock != 0)
        return FGMP_ERR_INVALID_ARG;
    const PackedLayout l = make_layout(h.rows, h.K);
    std::vector<uint64_t> mbits((size_t)l.n_tiles);
    if (hipMemcpyAsync(mbits.data(), static_cast<const char *>(packed) + l.off_M, mbits.size() * 8,
                       hipMemcpyDeviceToHost, st) != hipSuccess)
        return FGMP_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return FGMP_ERR_HIP;
    int64_t n_hi = 0;
    for (uint64_t w : mbits) n_hi += __builtin_popcountll(w);
    info_host->rows = h.rows;
    info_host->K = h.K;
    info_host->tensor_scale = h.tensor_scale;
    info_host->compact = (int32_t)h.compact;
    info_host->n_blocks = h.rows * (h.K / kBlock);
    info_host->n_fp8_blocks = n_hi;
    info_host->bytes_used = (int64_t)h.bytes_used;
    return FGMP_OK;
}

fgmp_status_t fgmp_threshold_for_fraction(const float *scores, int64_t J, double fraction,
                                          float *threshold_host, void *stream)
{
    return fgmp_threshold_for_fraction_multi(&scores, &J, 1, fraction, threshold_host, stream);
}

fgmp_status_t fgmp_threshold_for_fraction_multi(const float *const *scores, const int64_t *counts,
                                                int32_t n_tensors, double fraction, float *threshold_host,
                                                void *stream)
{
    if (!scores || !counts || !threshold_host || n_tensors <= 0 || !(fraction >= 0.0) || !(fraction <= 1.0))
        return FGMP_ERR_INVALID_ARG;
    int64_t total = 0;
    for (int32_t i = 0; i < n_tensors; ++i) {
        if (!scores[i] || counts[i] <= 0) return FGMP_ERR_INVALID_ARG;
        total += counts[i];
    }
    // Eq. 9 / Eq. 10 read as: exactly round(fraction * J) of the J scores lie strictly above the threshold
    // (when the boundary score is not tied): the score just below the round(fraction * J) largest ones
    const int64_t n_hi = (int64_t)(fraction * (double)total + 0.5);
    if (n_hi <= 0) { *threshold_host = INFINITY; return FGMP_OK; }
    if (n_hi >= total) { *threshold_host = -INFINITY; return FGMP_OK; }
    return select_rank(scores, counts, n_tensors, total - n_hi - 1, threshold_host, as_stream(stream));
}

fgmp_status_t fgmp_selftest_encode_ranges(int format, uint32_t *min_bits, uint32_t *max_bits,
                                          uint32_t *violations, void *stream)
{
    return selftest_encode_ranges(format, min_bits, max_bits, violations, as_stream(stream));
}

fgmp_status_t fgmp_selftest_decode_table(int format, float *out, void *stream)
{
    return selftest_decode_table(format, out, as_stream(stream));
}

fgmp_status_t fgmp_selftest_mfma_rate(int64_t workgroups, int32_t iters, float *sink, void *stream)
{
    return selftest_mfma_rate(workgroups, iters, sink, as_stream(stream));
}

fgmp_status_t fgmp_selftest_time_gemm_kernel(void *ev_start, void *ev_stop)
{
    if ((ev_start == nullptr) != (ev_stop == nullptr)) return FGMP_ERR_INVALID_ARG;
    return set_gemm_kernel_events(static_cast<hipEvent_t>(ev_start), static_cast<hipEvent_t>(ev_stop))
               ? FGMP_OK
               : (ev_start == nullptr ? FGMP_OK : FGMP_ERR_UNSUPPORTED);   // clearing "nothing" always works
}

fgmp_status_t fgmp_selftest_quantizer_traffic(const void *X, fgmp_dtype_t dt, int64_t M, int64_t K, int64_t ldx,
                                              const float *fisher_k, void *packed_out, size_t packed_bytes, void *stream)
{
#ifdef FGMP_MEASUREMENT_HOOKS
    return quantize_traffic_model(X, dt, M, K, ldx, fisher_k, packed_out, packed_bytes, as_stream(stream));
#else
    (void)X; (void)dt; (void)M; (void)K; (void)ldx; (void)fisher_k; (void)packed_out; (void)packed_bytes; (void)stream;
    return FGMP_ERR_UNSUPPORTED;
#endif
}

}  // extern "C"
