// Threshold for a target fraction of FP8 blocks (Eq. 9; over several tensors, Eq. 10): an exact order
// statistic of the scores, found on the device.  The scores stay where the quantizer wrote them: four
// passes of an 8-bit radix selection over all tensors (most significant digit first) narrow the 32-bit key
// of the wanted element down digit by digit; a pass counts, per value of the current digit, the elements
// whose higher digits equal the prefix found so far (one 256-bin histogram, built per workgroup in LDS and
// merged with 64-bit atomics), and a one-workgroup kernel walks the bins to the one that holds the wanted
// rank.  Keys order like the numbers: the bit pattern of a non-negative float with the sign bit set, that
// of a negative one inverted (-0 sorts just below +0; both compare equal to either as a threshold).  Every
// pass reads every score once -- 16 bytes per lane where the array allows -- so the selection costs four
// reads of the scores, against a copy to the host and a partial sort there.
#include <algorithm>
#include <cstring>

#include "fgmp_internal.hpp"

namespace fgmp {

namespace {

struct SelectState {
    unsigned long long hist[256];   // bins of the pass in progress; zero between passes
    unsigned long long rank;        // wanted element, counted from the smallest among those that match the prefix
    uint32_t prefix, mask;          // digits found so far, and which bits they occupy
    float result;
};

__device__ __forceinline__ uint32_t key_of(float v)
{
    const uint32_t b = __builtin_bit_cast(uint32_t, v);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

__host__ __device__ inline float value_of(uint32_t key)
{
    const uint32_t b = (key & 0x80000000u) ? (key & 0x7FFFFFFFu) : ~key;
#ifdef __HIP_DEVICE_COMPILE__
    return __builtin_bit_cast(float, b);
#else
    float f;
    memcpy(&f, &b, 4);
    return f;
#endif
}

constexpr int kSelThreads = 256;

__global__ __launch_bounds__(kSelThreads) void select_count_kernel(const float *__restrict__ s, int64_t n, int shift, SelectState *st)
{
    __shared__ uint32_t bins[256];
    bins[threadIdx.x] = 0u;
    __syncthreads();
    const uint32_t prefix = st->prefix, mask = st->mask;
    auto take = [&](float v) {
        const uint32_t k = key_of(v);
        if ((k & mask) == prefix) atomicAdd(&bins[(k >> shift) & 0xFFu], 1u);
    };
    // the part of the array that is aligned to 16 bytes in quads, the rest one by one
    const int64_t to_aligned = (int64_t)((16 - ((uintptr_t)s & 15)) & 15) / 4;
    const int64_t head = to_aligned < n ? to_aligned : n;
    const int64_t quads = (n - head) / 4;
    const float4 *q = reinterpret_cast<const float4 *>(s + head);
    const int64_t stride = (int64_t)gridDim.x * kSelThreads;
    for (int64_t i = (int64_t)blockIdx.x * kSelThreads + threadIdx.x; i < quads; i += stride) {
        const float4 v = q[i];
        take(v.x);
        take(v.y);
        take(v.z);
        take(v.w);
    }
    if (blockIdx.x == 0) {
        for (int64_t i = threadIdx.x; i < head; i += kSelThreads) take(s[i]);
        for (int64_t i = head + quads * 4 + threadIdx.x; i < n; i += kSelThreads) take(s[i]);
    }
    __syncthreads();
    const uint32_t c = bins[threadIdx.x];
    if (c != 0u) atomicAdd(&st->hist[threadIdx.x], (unsigned long long)c);
}

__global__ void select_init_kernel(SelectState *st, unsigned long long rank)
{
    st->hist[threadIdx.x] = 0ull;
    if (threadIdx.x == 0) {
        st->rank = rank;
        st->prefix = 0u;
        st->mask = 0u;
        st->result = 0.0f;
    }
}

// the bin that holds the wanted rank becomes the next digit of the prefix; the bins go back to zero
__global__ __launch_bounds__(256) void select_narrow_kernel(int shift, SelectState *st)
{
    __shared__ unsigned long long h[256];
    h[threadIdx.x] = st->hist[threadIdx.x];
    st->hist[threadIdx.x] = 0ull;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long rank = st->rank, below = 0ull;
        uint32_t d = 0;
        for (; d < 255u; ++d) {
            if (rank < below + h[d]) break;
            below += h[d];
        }
        st->rank = rank - below;
        st->prefix |= d << shift;
        st->mask |= 0xFFu << shift;
        if (shift == 0) st->result = value_of(st->prefix);
    }
}

}  // namespace

// The element of rank `rank` (0 = smallest) of the union of the arrays; result on the host.  Synchronizes `st`.
fgmp_status_t select_rank(const float *const *scores, const int64_t *counts, int32_t n_tensors, int64_t rank, float *result_host,
                          hipStream_t st)
{
    SelectState *state = nullptr;
    if (hipMalloc(&state, sizeof(SelectState)) != hipSuccess) return FGMP_ERR_HIP;
    fgmp_status_t rc = FGMP_OK;
    hipLaunchKernelGGL(select_init_kernel, dim3(1), dim3(256), 0, st, state, (unsigned long long)rank);
    for (int shift = 24; shift >= 0 && rc == FGMP_OK; shift -= 8) {
        for (int32_t i = 0; i < n_tensors; ++i) {
            const int64_t quads = counts[i] / 4 + 1;
            const unsigned grid = (unsigned)std::min<int64_t>(2048, (quads + kSelThreads - 1) / kSelThreads);
            hipLaunchKernelGGL(select_count_kernel, dim3(grid), dim3(kSelThreads), 0, st, scores[i], counts[i], shift, state);
        }
        hipLaunchKernelGGL(select_narrow_kernel, dim3(1), dim3(256), 0, st, shift, state);
        if (hipGetLastError() != hipSuccess) rc = FGMP_ERR_HIP;
    }
    if (rc == FGMP_OK && hipMemcpyAsync(result_host, &state->result, sizeof(float), hipMemcpyDeviceToHost, st) != hipSuccess)
        rc = FGMP_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) rc = FGMP_ERR_HIP;
    (void)hipFree(state);
    return rc;
}

}  // namespace fgmp
