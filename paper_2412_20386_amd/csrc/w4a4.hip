// 4-bit forms of the offline weight fold and of the PTS activation quantizer for gfx950: the W4A4
// setting of the paper's latency table (Sec. 6.4).  Codes are clipped to +-7 (Sec. 2.3:
// +-(2^(b-1) - 1)) and stored two per byte, the even index in the low nibble, two's complement
// (the packing of App. B.1 "Quantization": the odd index fills the high nibble).
//   ptq4vm_fold_smoothing_w4   W' = W diag(m), s_w = max|W'| / 7, codes packed [N, K / 2]
//   ptq4vm_quantize_pts_a4     clip(rne((f32(x) inv_m[k]) (1 / s_tok[r mod L])), -7, 7), packed [B L, K / 2]
// The quantizer is the same column-stationary stream as the 8-bit one (a thread keeps one group of
// 16 channels for life, smoothing factors in registers, reciprocal steps in LDS); it moves 2.5
// bytes per element instead of 3.
#include <hip/hip_fp16.h>

#include "common.hpp"
#include "quant_device.hpp"

namespace {

using ptq4vm::cvt_i32_f32;

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kMaxLdsTokens = 16384;

__device__ __forceinline__ int code4(float x, float inv_m, float inv_s) {
    float v = x * inv_m;  // two separate fp32 multiplies in this order, as in the 8-bit quantizer
    v = v * inv_s;
    const int q = cvt_i32_f32(__builtin_rintf(v));
    return min(max(q, -7), 7);
}

__device__ __forceinline__ uint32_t pack8_nibbles(const int (&q)[8]) {
    uint32_t r = 0;
#pragma unroll
    for (int i = 0; i < 8; i++) r |= ((uint32_t)q[i] & 15u) << (4 * i);
    return r;
}

__device__ __forceinline__ uint32_t quantize8(u32x4 in, const float *im, float inv_s) {
    int q[8];
#pragma unroll
    for (int e = 0; e < 4; e++) {
        const uint32_t word = in[e];
        const __half2 h = __builtin_bit_cast(__half2, word);
        q[2 * e] = code4(__low2float(h), im[2 * e], inv_s);
        q[2 * e + 1] = code4(__high2float(h), im[2 * e + 1], inv_s);
    }
    return pack8_nibbles(q);
}

// gridDim.x * 256 is a multiple of `chunks` (= K / 16): thread g owns channel group g mod chunks
// and rows g / chunks + i * row_step.
template <bool HAS_M, bool LDS_TABLE>
__global__ __launch_bounds__(kThreads) void quantize_pts_a4_stream(const __half *__restrict__ x,
                                                                   const float *__restrict__ inv_m,
                                                                   const float *__restrict__ s_tok,
                                                                   uint8_t *__restrict__ xq4, int64_t M, int L,
                                                                   int chunks, int64_t ldx, int64_t ldxq,
                                                                   int64_t row_step) {
    extern __shared__ float inv_s_lds[];
    if constexpr (LDS_TABLE) {
        for (int i = threadIdx.x; i < L; i += kThreads) inv_s_lds[i] = 1.0f / s_tok[i];  // IEEE division
        __syncthreads();
    }
    const int64_t gtid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int col = (int)(gtid % chunks);
    int64_t row = gtid / chunks;
    int t = (int)(row % L);
    const int t_step = (int)(row_step % L);
    float im[16];
#pragma unroll
    for (int i = 0; i < 16; i++) im[i] = HAS_M ? inv_m[col * 16 + i] : 1.0f;
    const __half *xp = x + row * ldx + (int64_t)col * 16;
    uint8_t *qp = xq4 + row * ldxq + (int64_t)col * 8;
    const int64_t x_step = row_step * ldx, q_step = row_step * ldxq;
    for (; row < M; row += row_step) {
        const u32x4 lo = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(xp));
        const u32x4 hi = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(xp + 8));
        const float inv_s = LDS_TABLE ? inv_s_lds[t] : 1.0f / s_tok[t];
        t += t_step;
        if (t >= L) t -= L;
        const u32x2 out = {quantize8(lo, im, inv_s), quantize8(hi, im + 8, inv_s)};
        ptq4vm::store_for_next_kernel(reinterpret_cast<u32x2 *>(qp), out);
        xp += x_step;
        qp += q_step;
    }
}

// Any even K and any pitch: one byte (two codes) per thread-iteration.
template <bool HAS_M>
__global__ __launch_bounds__(kThreads) void quantize_pts_a4_generic(const __half *__restrict__ x,
                                                                    const float *__restrict__ inv_m,
                                                                    const float *__restrict__ s_tok,
                                                                    uint8_t *__restrict__ xq4, int64_t M, int64_t L,
                                                                    int64_t K, int64_t ldx, int64_t ldxq) {
    const int64_t half_k = K / 2, total = M * half_k;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = e / half_k, j = e - r * half_k;
        const float inv_s = 1.0f / s_tok[r % L];
        const int lo = code4(__half2float(x[r * ldx + 2 * j]), HAS_M ? inv_m[2 * j] : 1.0f, inv_s);
        const int hi = code4(__half2float(x[r * ldx + 2 * j + 1]), HAS_M ? inv_m[2 * j + 1] : 1.0f, inv_s);
        xq4[r * ldxq + j] = (uint8_t)(((hi & 15) << 4) | (lo & 15));
    }
}

// Blocks [0, N) quantize one output channel each; blocks [N, N + ceil(K/256)) write 1/m.
__global__ __launch_bounds__(kThreads) void fold_smoothing_w4_rows(const __half *__restrict__ w,
                                                                   const float *__restrict__ m,
                                                                   uint8_t *__restrict__ wq4, float *__restrict__ s_w,
                                                                   float *__restrict__ inv_m, int64_t N, int64_t K,
                                                                   int64_t ldw, int64_t ldwq) {
    const int64_t o = blockIdx.x;
    if (o >= N) {
        const int64_t k = (o - N) * kThreads + threadIdx.x;
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
    const float step = (amax == 0.0f) ? 1.0f : amax / 7.0f;
    if (threadIdx.x == 0) s_w[o] = step;
    uint8_t *qrow = wq4 + o * ldwq;
    for (int64_t j = threadIdx.x; j < K / 2; j += kThreads) {
        int q[2];
#pragma unroll
        for (int e = 0; e < 2; e++) {
            const float wf = __half2float(wrow[2 * j + e]) * m[2 * j + e];
            q[e] = min(max(cvt_i32_f32(__builtin_rintf(wf / step)), -7), 7);
        }
        qrow[j] = (uint8_t)(((q[1] & 15) << 4) | (q[0] & 15));
    }
}

int64_t gcd64(int64_t a, int64_t b) {
    while (b) {
        const int64_t t = a % b;
        a = b;
        b = t;
    }
    return a;
}

}  // namespace

extern "C" int ptq4vm_fold_smoothing_w4(const void *w_f16, const float *m, uint8_t *wq4, float *s_w, float *inv_m,
                                        int64_t N, int64_t K, int64_t ldw, int64_t ldwq, void *stream_) {
    if (!w_f16 || !m || !wq4 || !s_w || !inv_m) return PTQ4VM_ERR_NULL;
    if (N < 0 || K <= 0 || K % 2 != 0) return PTQ4VM_ERR_SHAPE;
    if (ldw < K || ldwq < K / 2) return PTQ4VM_ERR_STRIDE;
    if (!ptq4vm::aligned_to(w_f16, 16) || !ptq4vm::aligned_to(wq4, 16) || !ptq4vm::aligned_to(m, 4) ||
        !ptq4vm::aligned_to(s_w, 4) || !ptq4vm::aligned_to(inv_m, 4))
        return PTQ4VM_ERR_ALIGN;
    const int64_t blocks = N + ptq4vm::ceil_div(K, kThreads);
    if (blocks > 0x7fffffffLL) return PTQ4VM_ERR_SHAPE;
    fold_smoothing_w4_rows<<<dim3((unsigned)blocks), dim3(kThreads), 0, static_cast<hipStream_t>(stream_)>>>(
        static_cast<const __half *>(w_f16), m, wq4, s_w, inv_m, N, K, ldw, ldwq);
    return ptq4vm::check_launch("fold_smoothing_w4_rows");
}

extern "C" int ptq4vm_quantize_pts_a4(const void *x_f16, const float *inv_m, const float *s_tok, uint8_t *xq4, int64_t B,
                                      int64_t L, int64_t K, int64_t ldx, int64_t ldxq, void *stream_) {
    if (!x_f16 || !s_tok || !xq4) return PTQ4VM_ERR_NULL;
    if (B < 0 || L <= 0 || K <= 0 || K % 2 != 0) return PTQ4VM_ERR_SHAPE;
    if (L > 0x7fffffffLL || K > 0x7fffffffLL || (B > 0 && L > INT64_MAX / B)) return PTQ4VM_ERR_SHAPE;
    if (ldx < K || ldxq < K / 2) return PTQ4VM_ERR_STRIDE;
    if (!ptq4vm::aligned_to(x_f16, 16) || !ptq4vm::aligned_to(xq4, 16) || !ptq4vm::aligned_to(s_tok, 4) ||
        (inv_m && !ptq4vm::aligned_to(inv_m, 4)))
        return PTQ4VM_ERR_ALIGN;
    const int64_t M = B * L;
    if (M == 0) return PTQ4VM_OK;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const __half *x = static_cast<const __half *>(x_f16);

    if (K % 16 == 0 && ldx % 8 == 0 && ldxq % 8 == 0) {
        const int64_t chunks = K / 16;
        const int64_t unit = chunks / gcd64(chunks, kThreads);
        int64_t want = 768;  // about 3 workgroups per CU striding over the rows together
        const int64_t needed = ptq4vm::ceil_div(M * chunks, kThreads);
        if (want > needed) want = needed;
        const int64_t blocks = ptq4vm::ceil_div(want, unit) * unit;
        if (blocks > 0x7fffffffLL) return PTQ4VM_ERR_SHAPE;
        const int64_t row_step = blocks * kThreads / chunks;
        const bool table = L <= kMaxLdsTokens;
        const size_t lds = table ? (size_t)L * sizeof(float) : 0;
        const dim3 grid((unsigned)blocks), block(kThreads);
#define PTQ4VM_LAUNCH(HAS_M, TABLE)                                                                              \
    quantize_pts_a4_stream<HAS_M, TABLE><<<grid, block, lds, stream>>>(x, inv_m, s_tok, xq4, M, (int)L, (int)chunks, \
                                                                       ldx, ldxq, row_step)
        if (inv_m) {
            if (table) PTQ4VM_LAUNCH(true, true); else PTQ4VM_LAUNCH(true, false);
        } else {
            if (table) PTQ4VM_LAUNCH(false, true); else PTQ4VM_LAUNCH(false, false);
        }
#undef PTQ4VM_LAUNCH
        return ptq4vm::check_launch("quantize_pts_a4_stream");
    }
    int64_t blocks = ptq4vm::ceil_div(M * (K / 2), kThreads);
    if (blocks > 65536) blocks = 65536;
    if (inv_m)
        quantize_pts_a4_generic<true><<<dim3((unsigned)blocks), dim3(kThreads), 0, stream>>>(x, inv_m, s_tok, xq4, M, L, K, ldx, ldxq);
    else
        quantize_pts_a4_generic<false><<<dim3((unsigned)blocks), dim3(kThreads), 0, stream>>>(x, inv_m, s_tok, xq4, M, L, K, ldx, ldxq);
    return ptq4vm::check_launch("quantize_pts_a4_generic");
}
