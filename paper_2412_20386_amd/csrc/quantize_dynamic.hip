// Per-token dynamic activation quantizer for gfx950: the comparison scheme of Sec. 4 and of the
// "Per-token dynamic" rows of the latency table (Sec. 6.4).  The step of a token row is computed
// online from the row itself, after smoothing:
//   v[k] = f32(x[r,k]) * inv_m[k];  s_r = max_k |v[k]| / 127 (1 for an all-zero row);
//   xq[r,k] = clip(rne(v[k] * (1 / s_r)), -127, 127);  s_row[r] = s_r.
// Like the static quantizer it is a pure stream (2 B read + 1 B written per element, + 4 B per
// row), but every row needs a reduction between its read and its write.  A row is held in the
// registers of the 2^n lanes that share it (8 fp16 per 16-byte load, up to 4 loads per lane), the
// maximum travels by lane shuffles inside that group, and the row is quantized from registers:
// the input is read once.  Groups are column-stationary, so the smoothing factors stay in
// registers.  The GEMM takes the result as ptq4vm_w8a8_linear(B = 1, L = M, s_tok = s_row).
#include <hip/hip_fp16.h>

#include "common.hpp"
#include "quant_device.hpp"

namespace {

using ptq4vm::cvt_i32_f32;
using ptq4vm::pack4;

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;

__device__ __forceinline__ int code_of(float v, float inv_s) {
    const int q = cvt_i32_f32(__builtin_rintf(v * inv_s));
    return min(max(q, -127), 127);
}

// lanes_per_row = 2^n <= 64 lanes share a row, lane l of the group holding 16-byte chunks
// l, l + lanes_per_row, ... (CPL of them; chunks beyond K / 8 are empty).  A wavefront handles
// 64 / lanes_per_row rows per pass and strides over the rows with all other wavefronts.
template <int CPL, bool HAS_M>
__global__ __launch_bounds__(kThreads) void quantize_dynamic_rows(const __half *__restrict__ x,
                                                                  const float *__restrict__ inv_m,
                                                                  int8_t *__restrict__ xq, float *__restrict__ s_row,
                                                                  int64_t M, int chunks, int lanes_per_row,
                                                                  int64_t ldx, int64_t ldxq) {
    const int lane = threadIdx.x & 63;
    const int in_row = lane & (lanes_per_row - 1), sub = lane / lanes_per_row;
    const int rows_per_wave = 64 / lanes_per_row;
    const int64_t wave = ((int64_t)blockIdx.x * kThreads + threadIdx.x) >> 6;
    const int64_t waves = ((int64_t)gridDim.x * kThreads) >> 6;

    float im[CPL][8];
    bool have[CPL];
#pragma unroll
    for (int c = 0; c < CPL; c++) {
        const int chunk = in_row + c * lanes_per_row;
        have[c] = chunk < chunks;
#pragma unroll
        for (int e = 0; e < 8; e++) im[c][e] = (HAS_M && have[c]) ? inv_m[chunk * 8 + e] : 1.0f;
    }

    const int64_t row_step = waves * rows_per_wave;
    auto fetch = [&](int64_t row, u32x4 (&raw)[CPL]) {
#pragma unroll
        for (int c = 0; c < CPL; c++) {
            raw[c] = u32x4{0, 0, 0, 0};
            if (row < M && have[c])
                raw[c] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(x + row * ldx + (in_row + c * lanes_per_row) * 8));
        }
    };
    u32x4 raw[CPL], raw_next[CPL];
    int64_t row = wave * rows_per_wave + sub;
    fetch(row, raw);
    for (; row < M + sub; row += row_step) {
        // `row < M + sub` keeps whole wavefronts together for the shuffles; lanes of rows beyond M idle
        const bool live = row < M;
        fetch(row + row_step, raw_next);  // the next row is in flight while this one is reduced and written
        float v[CPL][8];
        float amax = 0.0f;
#pragma unroll
        for (int c = 0; c < CPL; c++) {
#pragma unroll
            for (int e = 0; e < 4; e++) {
                const uint32_t word = raw[c][e];
                const __half2 h = __builtin_bit_cast(__half2, word);
                v[c][2 * e] = __low2float(h) * im[c][2 * e];
                v[c][2 * e + 1] = __high2float(h) * im[c][2 * e + 1];
            }
#pragma unroll
            for (int e = 0; e < 8; e++) amax = fmaxf(amax, fabsf(v[c][e]));  // a NaN never becomes the maximum
        }
        for (int off = lanes_per_row >> 1; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
        const float step = amax == 0.0f ? 1.0f : amax / 127.0f;  // IEEE divisions (compiled without fast-math)
        const float inv_s = 1.0f / step;
        if (live) {
            if (in_row == 0) s_row[row] = step;
#pragma unroll
            for (int c = 0; c < CPL; c++)
                if (have[c]) {
                    int q[8];
#pragma unroll
                    for (int e = 0; e < 8; e++) q[e] = code_of(v[c][e], inv_s);
                    const u32x2 out = {pack4(q[0], q[1], q[2], q[3]), pack4(q[4], q[5], q[6], q[7])};
                    ptq4vm::store_for_next_kernel(reinterpret_cast<u32x2 *>(xq + row * ldxq + (in_row + c * lanes_per_row) * 8), out);
                }
        }
#pragma unroll
        for (int c = 0; c < CPL; c++) raw[c] = raw_next[c];
    }
}

// Any shape and pitch: one wavefront per row, element-wise, two passes over the row.
template <bool HAS_M>
__global__ __launch_bounds__(kThreads) void quantize_dynamic_generic(const __half *__restrict__ x,
                                                                     const float *__restrict__ inv_m,
                                                                     int8_t *__restrict__ xq, float *__restrict__ s_row,
                                                                     int64_t M, int64_t K, int64_t ldx, int64_t ldxq) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = ((int64_t)blockIdx.x * kThreads + threadIdx.x) >> 6;
    const int64_t waves = ((int64_t)gridDim.x * kThreads) >> 6;
    for (int64_t row = wave; row < M; row += waves) {
        float amax = 0.0f;
        for (int64_t k = lane; k < K; k += 64) {
            const float v = __half2float(x[row * ldx + k]) * (HAS_M ? inv_m[k] : 1.0f);
            amax = fmaxf(amax, fabsf(v));
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
        const float step = amax == 0.0f ? 1.0f : amax / 127.0f;
        const float inv_s = 1.0f / step;
        if (lane == 0) s_row[row] = step;
        for (int64_t k = lane; k < K; k += 64) {
            const float v = __half2float(x[row * ldx + k]) * (HAS_M ? inv_m[k] : 1.0f);
            xq[row * ldxq + k] = (int8_t)code_of(v, inv_s);
        }
    }
}

template <int CPL>
int launch_rows(const __half *x, const float *inv_m, int8_t *xq, float *s_row, int64_t M, int chunks, int lanes_per_row,
                int64_t ldx, int64_t ldxq, hipStream_t stream) {
    const int64_t rows_per_wave = 64 / lanes_per_row;
    int64_t blocks = ptq4vm::ceil_div(ptq4vm::ceil_div(M, rows_per_wave), kThreads / 64);
    if (blocks > 2048) blocks = 2048;  // 8 workgroups per CU, each striding over the rows
    dim3 grid((unsigned)blocks), block(kThreads);
    if (inv_m)
        quantize_dynamic_rows<CPL, true><<<grid, block, 0, stream>>>(x, inv_m, xq, s_row, M, chunks, lanes_per_row, ldx, ldxq);
    else
        quantize_dynamic_rows<CPL, false><<<grid, block, 0, stream>>>(x, inv_m, xq, s_row, M, chunks, lanes_per_row, ldx, ldxq);
    return ptq4vm::check_launch("quantize_dynamic_rows");
}

}  // namespace

extern "C" int ptq4vm_quantize_dynamic(const void *x_f16, const float *inv_m, int8_t *xq, float *s_row, int64_t M,
                                       int64_t K, int64_t ldx, int64_t ldxq, void *stream_) {
    if (!x_f16 || !xq || !s_row) return PTQ4VM_ERR_NULL;
    if (M < 0 || K <= 0 || K > 0x7fffffffLL) return PTQ4VM_ERR_SHAPE;
    if (ldx < K || ldxq < K) return PTQ4VM_ERR_STRIDE;
    if (!ptq4vm::aligned_to(x_f16, 16) || !ptq4vm::aligned_to(xq, 16) || !ptq4vm::aligned_to(s_row, 4) ||
        (inv_m && !ptq4vm::aligned_to(inv_m, 4)))
        return PTQ4VM_ERR_ALIGN;
    if (M == 0) return PTQ4VM_OK;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const __half *x = static_cast<const __half *>(x_f16);

    if (K % 8 == 0 && ldx % 8 == 0 && ldxq % 8 == 0 && K <= 2048) {
        const int chunks = (int)(K / 8);
        int lanes_per_row = 1;
        while (lanes_per_row < chunks && lanes_per_row < 64) lanes_per_row <<= 1;
        switch ((chunks + lanes_per_row - 1) / lanes_per_row) {
            case 1: return launch_rows<1>(x, inv_m, xq, s_row, M, chunks, lanes_per_row, ldx, ldxq, stream);
            case 2: return launch_rows<2>(x, inv_m, xq, s_row, M, chunks, lanes_per_row, ldx, ldxq, stream);
            case 3: return launch_rows<3>(x, inv_m, xq, s_row, M, chunks, lanes_per_row, ldx, ldxq, stream);
            default: return launch_rows<4>(x, inv_m, xq, s_row, M, chunks, lanes_per_row, ldx, ldxq, stream);
        }
    }
    int64_t blocks = ptq4vm::ceil_div(M, kThreads / 64);
    if (blocks > 8192) blocks = 8192;
    if (inv_m)
        quantize_dynamic_generic<true><<<dim3((unsigned)blocks), dim3(kThreads), 0, stream>>>(x, inv_m, xq, s_row, M, K, ldx, ldxq);
    else
        quantize_dynamic_generic<false><<<dim3((unsigned)blocks), dim3(kThreads), 0, stream>>>(x, inv_m, xq, s_row, M, K, ldx, ldxq);
    return ptq4vm::check_launch("quantize_dynamic_generic");
}
