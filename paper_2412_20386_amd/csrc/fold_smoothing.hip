// Offline weight preparation for gfx950: fold the smoothing vector into the weight
// (Eq. (smooth), Sec. 2.4) and quantize every output channel symmetrically to int8
// (Sec. 2.3, Delta_W = max|W'| / 127; Sec. 5.1: one Delta_W per output channel).
// Runs once per layer, so it favours exactness (IEEE fp32 division per element) over speed:
// one workgroup per output channel, two passes over the row.
#include <hip/hip_fp16.h>

#include "common.hpp"
#include "quant_device.hpp"

namespace {

using ptq4vm::cvt_i32_f32;

constexpr int kThreads = 256;

// Blocks [0, N) quantize one output channel each; blocks [N, N + ceil(K/256)) write 1/m.
__global__ __launch_bounds__(kThreads) void fold_smoothing_rows(const __half *__restrict__ w,
                                                                const float *__restrict__ m,
                                                                int8_t *__restrict__ wq, float *__restrict__ s_w,
                                                                float *__restrict__ inv_m, int64_t N, int64_t K,
                                                                int64_t ldw, int64_t ldwq) {
    const int64_t o = blockIdx.x;
    if (o >= N) {
        int64_t k = (o - N) * kThreads + threadIdx.x;
        if (k < K) inv_m[k] = 1.0f / m[k];
        return;
    }
    __shared__ float red[kThreads / 64];
    const __half *wrow = w + o * ldw;
    float amax = 0.0f;
    for (int64_t k = threadIdx.x; k < K; k += kThreads) amax = fmaxf(amax, fabsf(__half2float(wrow[k]) * m[k]));
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = amax;
    __syncthreads();
    amax = red[0];
#pragma unroll
    for (int i = 1; i < kThreads / 64; i++) amax = fmaxf(amax, red[i]);

    const float step = (amax == 0.0f) ? 1.0f : amax / 127.0f;
    if (threadIdx.x == 0) s_w[o] = step;
    int8_t *qrow = wq + o * ldwq;
    for (int64_t k = threadIdx.x; k < K; k += kThreads) {
        float wf = __half2float(wrow[k]) * m[k];
        int q = cvt_i32_f32(__builtin_rintf(wf / step));
        qrow[k] = (int8_t)min(max(q, -127), 127);
    }
}

// rowsum[o] = sum_k wq[o,k], one wavefront per output channel: the factor of the per-token zero
// offset in  sum_k (q - z) w = sum_k q w - z rowsum  (offset quantizer of Sec. 2.3 in the linear of Sec. 5.1).
__global__ __launch_bounds__(kThreads) void weight_rowsum_rows(const int8_t *__restrict__ wq,
                                                               int32_t *__restrict__ rowsum, int64_t N, int64_t K,
                                                               int64_t ldwq) {
    const int lane = threadIdx.x & 63;
    const int64_t o = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (o >= N) return;
    int sum = 0;
    for (int64_t k = lane; k < K; k += 64) sum += wq[o * ldwq + k];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
    if (lane == 0) rowsum[o] = sum;
}

}  // namespace

extern "C" int ptq4vm_weight_rowsum(const int8_t *wq, int32_t *rowsum, int64_t N, int64_t K, int64_t ldwq,
                                    void *stream_) {
    if (!wq || !rowsum) return PTQ4VM_ERR_NULL;
    if (N < 0 || K <= 0 || K > PTQ4VM_MAX_K) return PTQ4VM_ERR_SHAPE;
    if (ldwq < K) return PTQ4VM_ERR_STRIDE;
    if (!ptq4vm::aligned_to(rowsum, 4)) return PTQ4VM_ERR_ALIGN;
    if (N == 0) return PTQ4VM_OK;
    const int64_t blocks = ptq4vm::ceil_div(N, kThreads / 64);
    if (blocks > 0x7fffffffLL) return PTQ4VM_ERR_SHAPE;
    weight_rowsum_rows<<<dim3((unsigned)blocks), dim3(kThreads), 0, static_cast<hipStream_t>(stream_)>>>(wq, rowsum, N,
                                                                                                         K, ldwq);
    return ptq4vm::check_launch("weight_rowsum_rows");
}

extern "C" int ptq4vm_fold_smoothing(const void *w_f16, const float *m, int8_t *wq, float *s_w, float *inv_m,
                                     int64_t N, int64_t K, int64_t ldw, int64_t ldwq, void *stream_) {
    if (!w_f16 || !m || !wq || !s_w || !inv_m) return PTQ4VM_ERR_NULL;
    if (N < 0 || K <= 0) return PTQ4VM_ERR_SHAPE;
    if (ldw < K || ldwq < K) return PTQ4VM_ERR_STRIDE;
    if (!ptq4vm::aligned_to(w_f16, 16) || !ptq4vm::aligned_to(wq, 16) || !ptq4vm::aligned_to(m, 4) ||
        !ptq4vm::aligned_to(s_w, 4) || !ptq4vm::aligned_to(inv_m, 4))
        return PTQ4VM_ERR_ALIGN;
    const int64_t blocks = N + ptq4vm::ceil_div(K, kThreads);
    if (blocks > 0x7fffffffLL) return PTQ4VM_ERR_SHAPE;
    fold_smoothing_rows<<<dim3((unsigned)blocks), dim3(kThreads), 0, static_cast<hipStream_t>(stream_)>>>(
        static_cast<const __half *>(w_f16), m, wq, s_w, inv_m, N, K, ldw, ldwq);
    return ptq4vm::check_launch("fold_smoothing_rows");
}
