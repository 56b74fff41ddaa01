// Per-Token Static activation quantizer for gfx950 (Sec. 5.1; App. B.1 smoothing + quantization
// fused):  xq[r,k] = clip(rne((f32(x[r,k]) * inv_m[k]) * (1 / s_tok[r mod L])), -127, 127).
//
// The kernel is a pure stream (2 B read + 1 B written per element), so everything is arranged
// for HBM: 128-bit loads, consecutive lanes on consecutive addresses, several loads in flight
// per lane, and no per-element index arithmetic.  The grid is a fixed, small number of
// workgroups per CU that stride over the rows together (measured: ~3 workgroups per CU stream
// faster than a grid of many short-lived ones).  The total thread count is a multiple of the
// chunks per row, so a thread keeps ONE column chunk (VEC channels) for its whole life: the
// smoothing factors sit in registers and the row index advances by a constant.  The reciprocal
// steps 1/s_tok[t] of all L token positions are computed once per workgroup into LDS (the only
// place the IEEE division appears); the token position advances incrementally, without a modulo.
#include <hip/hip_fp16.h>

#include "common.hpp"
#include "quant_device.hpp"

namespace {

using ptq4vm::cvt_i32_f32;
using ptq4vm::pack4;

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kMaxThreads = 256;
constexpr int kMaxLdsTokens = 16384;  // reciprocal-step table of up to 64 KiB; longer sequences divide per row

// HAS_Z: per-token zero offset (Sec. 5.1 names it; quantizer form of Sec. 2.3 with the code range shifted
// into int8): the offset is added to the rounded value and the clip range is [-128, 127].
template <bool HAS_Z>
__device__ __forceinline__ int quantize_one(float x, float inv_m, float inv_s, int z) {
    float v = x * inv_m;  // smoothing first (two separate fp32 multiplies, never fused or reordered)
    v = v * inv_s;
    int q = cvt_i32_f32(__builtin_rintf(v));  // round half to even, then NaN -> 0, Inf -> +-INT_MAX
    if constexpr (HAS_Z) {
        q = min(max(q, -(1 << 20)), 1 << 20);  // room for the offset without integer overflow
        return min(max(q + z, -128), 127);
    }
    return min(max(q, -127), 127);
}

template <int VEC>
struct Chunk;
template <>
struct Chunk<8> {
    using In = u32x4;   // 8 x fp16
    using Out = u32x2;  // 8 x int8
};
template <>
struct Chunk<4> {
    using In = u32x2;
    using Out = uint32_t;
};

__device__ __forceinline__ void half2_to_floats(uint32_t packed, float &lo, float &hi) {
    __half2 h = *reinterpret_cast<__half2 *>(&packed);
    lo = __low2float(h);
    hi = __high2float(h);
}

template <bool HAS_Z>
__device__ __forceinline__ u32x2 quantize_chunk(u32x4 in, const float (&im)[8], float inv_s, int z) {
    float f[8];
    half2_to_floats(in.x, f[0], f[1]);
    half2_to_floats(in.y, f[2], f[3]);
    half2_to_floats(in.z, f[4], f[5]);
    half2_to_floats(in.w, f[6], f[7]);
    int q[8];
#pragma unroll
    for (int i = 0; i < 8; i++) q[i] = quantize_one<HAS_Z>(f[i], im[i], inv_s, z);
    u32x2 out = {pack4(q[0], q[1], q[2], q[3]), pack4(q[4], q[5], q[6], q[7])};
    return out;
}

template <bool HAS_Z>
__device__ __forceinline__ uint32_t quantize_chunk(u32x2 in, const float (&im)[4], float inv_s, int z) {
    float f[4];
    half2_to_floats(in.x, f[0], f[1]);
    half2_to_floats(in.y, f[2], f[3]);
    int q[4];
#pragma unroll
    for (int i = 0; i < 4; i++) q[i] = quantize_one<HAS_Z>(f[i], im[i], inv_s, z);
    return pack4(q[0], q[1], q[2], q[3]);
}

// Column-stationary grid-stride stream.  gridDim.x * 256 is a multiple of `chunks` (= K / VEC),
// so thread g owns column chunk g mod chunks and rows g / chunks + i * row_step, i = 0, 1, ...
template <int VEC, bool HAS_M, bool LDS_TABLE, bool HAS_Z, int UNROLL>
__global__ __launch_bounds__(kMaxThreads) void quantize_pts_stream(
    const __half *__restrict__ x, const float *__restrict__ inv_m, const float *__restrict__ s_tok,
    const int32_t *__restrict__ z_tok, int8_t *__restrict__ xq, int64_t M, int L, int chunks, int64_t ldx,
    int64_t ldxq, int64_t row_step) {
    using In = typename Chunk<VEC>::In;
    using Out = typename Chunk<VEC>::Out;
    extern __shared__ float inv_s_lds[];  // [L] reciprocal steps, then (HAS_Z) [L] offsets
    int *const z_lds = reinterpret_cast<int *>(inv_s_lds + L);
    if constexpr (LDS_TABLE) {
        for (int i = threadIdx.x; i < L; i += kMaxThreads) {
            inv_s_lds[i] = 1.0f / s_tok[i];  // IEEE-correct division (compiled without fast-math)
            if constexpr (HAS_Z) z_lds[i] = z_tok[i];
        }
        __syncthreads();
    }
    auto inv_step = [&](int t) { return LDS_TABLE ? inv_s_lds[t] : 1.0f / s_tok[t]; };
    auto offset = [&](int t) { return HAS_Z ? (LDS_TABLE ? z_lds[t] : z_tok[t]) : 0; };

    const int64_t gtid = (int64_t)blockIdx.x * kMaxThreads + threadIdx.x;
    const int col = (int)(gtid % chunks);
    int64_t row = gtid / chunks;
    int t = (int)(row % L);
    const int t_step = (int)(row_step % L);

    float im[VEC];
#pragma unroll
    for (int i = 0; i < VEC; i++) im[i] = HAS_M ? inv_m[col * VEC + i] : 1.0f;

    const __half *xp = x + row * ldx + (int64_t)col * VEC;
    int8_t *qp = xq + row * ldxq + (int64_t)col * VEC;
    const int64_t x_step = row_step * ldx, q_step = row_step * ldxq;

    for (; row + (UNROLL - 1) * row_step < M; row += UNROLL * row_step) {
        In v[UNROLL];
        float is[UNROLL];
        int zs[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; u++) {
            v[u] = __builtin_nontemporal_load(reinterpret_cast<const In *>(xp + u * x_step));
            is[u] = inv_step(t);
            zs[u] = offset(t);
            t += t_step;
            if (t >= L) t -= L;
        }
#pragma unroll
        for (int u = 0; u < UNROLL; u++)
            ptq4vm::store_for_next_kernel(reinterpret_cast<Out *>(qp + u * q_step), quantize_chunk<HAS_Z>(v[u], im, is[u], zs[u]));
        xp += UNROLL * x_step;
        qp += UNROLL * q_step;
    }
    for (; row < M; row += row_step) {
        In v = __builtin_nontemporal_load(reinterpret_cast<const In *>(xp));
        const float is = inv_step(t);
        const int z = offset(t);
        t += t_step;
        if (t >= L) t -= L;
        ptq4vm::store_for_next_kernel(reinterpret_cast<Out *>(qp), quantize_chunk<HAS_Z>(v, im, is, z));
        xp += x_step;
        qp += q_step;
    }
}

// Any shape and pitch: one element per thread-iteration, index arithmetic per element.
template <bool HAS_M, bool HAS_Z>
__global__ __launch_bounds__(kMaxThreads) void quantize_pts_generic(
    const __half *__restrict__ x, const float *__restrict__ inv_m, const float *__restrict__ s_tok,
    const int32_t *__restrict__ z_tok, int8_t *__restrict__ xq, int64_t M, int64_t L, int64_t K, int64_t ldx,
    int64_t ldxq) {
    const int64_t total = M * K;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (int64_t)gridDim.x * blockDim.x) {
        int64_t r = e / K, k = e - r * K;
        float inv_s = 1.0f / s_tok[r % L];
        float m = HAS_M ? inv_m[k] : 1.0f;
        const int z = HAS_Z ? z_tok[r % L] : 0;
        xq[r * ldxq + k] = (int8_t)quantize_one<HAS_Z>(__half2float(x[r * ldx + k]), m, inv_s, z);
    }
}

int64_t gcd64(int64_t a, int64_t b) {
    while (b) {
        int64_t t = a % b;
        a = b;
        b = t;
    }
    return a;
}

template <int VEC>
int launch_stream(const __half *x, const float *inv_m, const float *s_tok, const int32_t *z_tok, int8_t *xq, int64_t M,
                  int64_t L, int64_t K, int64_t ldx, int64_t ldxq, hipStream_t stream) {
    const int64_t chunks = K / VEC;
    // Grid: a multiple of `unit` workgroups (so that threads % chunks == 0), about 3 per CU of
    // the 256-CU part, fewer when the whole problem is smaller than that.
    const int64_t unit = chunks / gcd64(chunks, kMaxThreads);
    const int64_t total_chunks = M * chunks;
    int64_t want = 768;
    const int64_t needed = ptq4vm::ceil_div(total_chunks, kMaxThreads);
    if (want > needed) want = needed;
    int64_t blocks = ptq4vm::ceil_div(want, unit) * unit;
    if (blocks > 0x7fffffffLL) return PTQ4VM_ERR_SHAPE;
    const int64_t row_step = blocks * kMaxThreads / chunks;
    const bool table = L <= (z_tok ? kMaxLdsTokens / 2 : kMaxLdsTokens);
    const size_t lds = table ? (size_t)L * sizeof(float) * (z_tok ? 2 : 1) : 0;
    constexpr int UNROLL = 2;
    dim3 grid((unsigned)blocks), block(kMaxThreads);
#define PTQ4VM_LAUNCH(HAS_M, TABLE, HAS_Z)                                                                       \
    quantize_pts_stream<VEC, HAS_M, TABLE, HAS_Z, UNROLL><<<grid, block, lds, stream>>>(                          \
        x, inv_m, s_tok, z_tok, xq, M, (int)L, (int)chunks, ldx, ldxq, row_step)
    const int variant = (inv_m ? 4 : 0) | (table ? 2 : 0) | (z_tok ? 1 : 0);
    switch (variant) {
        case 0: PTQ4VM_LAUNCH(false, false, false); break;
        case 1: PTQ4VM_LAUNCH(false, false, true); break;
        case 2: PTQ4VM_LAUNCH(false, true, false); break;
        case 3: PTQ4VM_LAUNCH(false, true, true); break;
        case 4: PTQ4VM_LAUNCH(true, false, false); break;
        case 5: PTQ4VM_LAUNCH(true, false, true); break;
        case 6: PTQ4VM_LAUNCH(true, true, false); break;
        default: PTQ4VM_LAUNCH(true, true, true); break;
    }
#undef PTQ4VM_LAUNCH
    return ptq4vm::check_launch("quantize_pts_stream");
}

int quantize_entry(const void *x_f16, const float *inv_m, const float *s_tok, const int32_t *z_tok, int8_t *xq, int64_t B,
                   int64_t L, int64_t K, int64_t ldx, int64_t ldxq, void *stream_) {
    if (B < 0 || L <= 0 || K <= 0) return PTQ4VM_ERR_SHAPE;
    if (L > 0x7fffffffLL || K > 0x7fffffffLL || (B > 0 && L > INT64_MAX / B)) return PTQ4VM_ERR_SHAPE;
    if (ldx < K || ldxq < K) return PTQ4VM_ERR_STRIDE;
    if (!ptq4vm::aligned_to(x_f16, 16) || !ptq4vm::aligned_to(xq, 16) || !ptq4vm::aligned_to(s_tok, 4) ||
        !ptq4vm::aligned_to(z_tok, 4) || (inv_m && !ptq4vm::aligned_to(inv_m, 4)))
        return PTQ4VM_ERR_ALIGN;
    const int64_t M = B * L;
    if (M == 0) return PTQ4VM_OK;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const __half *x = static_cast<const __half *>(x_f16);

    if (K % 8 == 0 && ldx % 8 == 0 && ldxq % 8 == 0)
        return launch_stream<8>(x, inv_m, s_tok, z_tok, xq, M, L, K, ldx, ldxq, stream);
    if (K % 4 == 0 && ldx % 4 == 0 && ldxq % 4 == 0)
        return launch_stream<4>(x, inv_m, s_tok, z_tok, xq, M, L, K, ldx, ldxq, stream);

    int64_t blocks = ptq4vm::ceil_div(M * K, kMaxThreads);
    if (blocks > 65536) blocks = 65536;
    const dim3 grid((unsigned)blocks), block(kMaxThreads);
    if (inv_m && z_tok)
        quantize_pts_generic<true, true><<<grid, block, 0, stream>>>(x, inv_m, s_tok, z_tok, xq, M, L, K, ldx, ldxq);
    else if (inv_m)
        quantize_pts_generic<true, false><<<grid, block, 0, stream>>>(x, inv_m, s_tok, z_tok, xq, M, L, K, ldx, ldxq);
    else if (z_tok)
        quantize_pts_generic<false, true><<<grid, block, 0, stream>>>(x, inv_m, s_tok, z_tok, xq, M, L, K, ldx, ldxq);
    else
        quantize_pts_generic<false, false><<<grid, block, 0, stream>>>(x, inv_m, s_tok, z_tok, xq, M, L, K, ldx, ldxq);
    return ptq4vm::check_launch("quantize_pts_generic");
}

}  // namespace

extern "C" int ptq4vm_quantize_pts(const void *x_f16, const float *inv_m, const float *s_tok, int8_t *xq,
                                   int64_t B, int64_t L, int64_t K, int64_t ldx, int64_t ldxq, void *stream_) {
    if (!x_f16 || !s_tok || !xq) return PTQ4VM_ERR_NULL;
    return quantize_entry(x_f16, inv_m, s_tok, nullptr, xq, B, L, K, ldx, ldxq, stream_);
}

extern "C" int ptq4vm_quantize_pts_offset(const void *x_f16, const float *inv_m, const float *s_tok,
                                          const int32_t *z_tok, int8_t *xq, int64_t B, int64_t L, int64_t K,
                                          int64_t ldx, int64_t ldxq, void *stream_) {
    if (!x_f16 || !s_tok || !z_tok || !xq) return PTQ4VM_ERR_NULL;
    return quantize_entry(x_f16, inv_m, s_tok, z_tok, xq, B, L, K, ldx, ldxq, stream_);
}
