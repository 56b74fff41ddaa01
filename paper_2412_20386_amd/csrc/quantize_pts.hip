// Per-Token Static activation quantizer for gfx950 (Sec. 5.1; App. B.1 smoothing + quantization
// fused):  xq[r,k] = clip(rne((f32(x[r,k]) * inv_m[k]) * (1 / s_tok[r mod L])), -127, 127).
//
// The kernel is a pure stream (2 B read + 1 B written per element), so everything is arranged
// for HBM: 128-bit loads, consecutive lanes on consecutive addresses, several loads in flight
// per lane, and no per-element index arithmetic.  A thread keeps ONE column chunk (VEC
// channels) for its whole life, so the smoothing factors sit in registers; a block owns a
// contiguous band of rows and precomputes their reciprocal steps once into LDS (the only
// place r mod L and the IEEE division appear).
#include <hip/hip_fp16.h>

#include "common.hpp"

namespace {

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kMaxThreads = 256;
constexpr int kMaxBandRows = 1024;  // rows per block; bounds the LDS table of reciprocal steps

// fp32 -> int32 conversion with the hardware's defined behaviour for specials
// (NaN -> 0, out-of-range saturates), which a C++ cast leaves undefined.
__device__ __forceinline__ int cvt_i32_f32(float v) {
    int i;
    asm("v_cvt_i32_f32 %0, %1" : "=v"(i) : "v"(v));
    return i;
}

__device__ __forceinline__ int quantize_one(float x, float inv_m, float inv_s) {
    float v = x * inv_m;  // smoothing first (two separate fp32 multiplies, never fused or reordered)
    v = v * inv_s;
    int q = cvt_i32_f32(__builtin_rintf(v));  // round half to even, then NaN -> 0, Inf -> +-INT_MAX
    return min(max(q, -127), 127);
}

__device__ __forceinline__ uint32_t pack4(int a, int b, int c, int d) {
    uint32_t lo = __builtin_amdgcn_perm((uint32_t)b, (uint32_t)a, 0x0c0c0400u);  // a.b0 | b.b0 << 8
    uint32_t hi = __builtin_amdgcn_perm((uint32_t)d, (uint32_t)c, 0x0c0c0400u);
    return __builtin_amdgcn_perm(hi, lo, 0x05040100u);
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

template <int VEC>
__device__ __forceinline__ typename Chunk<VEC>::Out quantize_chunk(typename Chunk<VEC>::In in,
                                                                   const float (&im)[VEC], float inv_s);

template <>
__device__ __forceinline__ u32x2 quantize_chunk<8>(u32x4 in, const float (&im)[8], float inv_s) {
    float f[8];
    half2_to_floats(in.x, f[0], f[1]);
    half2_to_floats(in.y, f[2], f[3]);
    half2_to_floats(in.z, f[4], f[5]);
    half2_to_floats(in.w, f[6], f[7]);
    int q[8];
#pragma unroll
    for (int i = 0; i < 8; i++) q[i] = quantize_one(f[i], im[i], inv_s);
    u32x2 out = {pack4(q[0], q[1], q[2], q[3]), pack4(q[4], q[5], q[6], q[7])};
    return out;
}

template <>
__device__ __forceinline__ uint32_t quantize_chunk<4>(u32x2 in, const float (&im)[4], float inv_s) {
    float f[4];
    half2_to_floats(in.x, f[0], f[1]);
    half2_to_floats(in.y, f[2], f[3]);
    int q[4];
#pragma unroll
    for (int i = 0; i < 4; i++) q[i] = quantize_one(f[i], im[i], inv_s);
    return pack4(q[0], q[1], q[2], q[3]);
}

// Column-stationary streaming kernel.  blockDim.x = rows_per_pass * cols_per_pass.
//   chunks        K / VEC
//   cols_per_pass min(chunks, 256)           threads side by side along a row
//   rows_per_pass blockDim.x / cols_per_pass rows covered by one pass of the block
//   band          rows owned by one block (multiple of rows_per_pass, <= kMaxBandRows)
template <int VEC, bool HAS_M, int UNROLL>
__global__ __launch_bounds__(kMaxThreads) void quantize_pts_stream(
    const __half *__restrict__ x, const float *__restrict__ inv_m, const float *__restrict__ s_tok,
    int8_t *__restrict__ xq, int64_t M, int L, int K, int64_t ldx, int64_t ldxq, int chunks,
    int cols_per_pass, int rows_per_pass, int band) {
    using In = typename Chunk<VEC>::In;
    using Out = typename Chunk<VEC>::Out;
    __shared__ float inv_s_lds[kMaxBandRows];

    const int64_t row0 = (int64_t)blockIdx.x * band;
    const int rows_here = (int)min((int64_t)band, M - row0);
    {
        int t = (int)((row0 + threadIdx.x) % L);  // the only modulo: once per row, in the prologue
        for (int i = threadIdx.x; i < rows_here; i += blockDim.x) {
            inv_s_lds[i] = 1.0f / s_tok[t];  // IEEE-correct division (compiled without fast-math)
            t = (int)((t + (int64_t)blockDim.x) % L);
        }
    }
    __syncthreads();

    const int col = threadIdx.x % cols_per_pass;
    const int row_in_pass = threadIdx.x / cols_per_pass;

    for (int c = col; c < chunks; c += cols_per_pass) {
        float im[VEC];
#pragma unroll
        for (int i = 0; i < VEC; i++) im[i] = HAS_M ? inv_m[c * VEC + i] : 1.0f;

        const __half *xcol = x + row0 * ldx + (int64_t)c * VEC;
        int8_t *qcol = xq + row0 * ldxq + (int64_t)c * VEC;
        for (int rb = row_in_pass; rb < rows_here; rb += rows_per_pass * UNROLL) {
            In v[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; u++) {
                int r = rb + u * rows_per_pass;
                if (r < rows_here) v[u] = __builtin_nontemporal_load(reinterpret_cast<const In *>(xcol + (int64_t)r * ldx));
            }
#pragma unroll
            for (int u = 0; u < UNROLL; u++) {
                int r = rb + u * rows_per_pass;
                if (r < rows_here) {
                    Out o = quantize_chunk<VEC>(v[u], im, inv_s_lds[r]);
                    __builtin_nontemporal_store(o, reinterpret_cast<Out *>(qcol + (int64_t)r * ldxq));
                }
            }
        }
    }
}

// Any shape and pitch: one element per thread-iteration, index arithmetic per element.
template <bool HAS_M>
__global__ __launch_bounds__(kMaxThreads) void quantize_pts_generic(
    const __half *__restrict__ x, const float *__restrict__ inv_m, const float *__restrict__ s_tok,
    int8_t *__restrict__ xq, int64_t M, int64_t L, int64_t K, int64_t ldx, int64_t ldxq) {
    const int64_t total = M * K;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (int64_t)gridDim.x * blockDim.x) {
        int64_t r = e / K, k = e - r * K;
        float inv_s = 1.0f / s_tok[r % L];
        float m = HAS_M ? inv_m[k] : 1.0f;
        xq[r * ldxq + k] = (int8_t)quantize_one(__half2float(x[r * ldx + k]), m, inv_s);
    }
}

template <int VEC>
int launch_stream(const __half *x, const float *inv_m, const float *s_tok, int8_t *xq, int64_t M, int64_t L,
                  int64_t K, int64_t ldx, int64_t ldxq, hipStream_t stream) {
    const int chunks = (int)(K / VEC);
    const int cols_per_pass = chunks < kMaxThreads ? chunks : kMaxThreads;
    const int rows_per_pass = kMaxThreads / cols_per_pass;
    const int threads = rows_per_pass * cols_per_pass;
    constexpr int UNROLL = 4;
    // A block streams about 64 KiB of input, but no fewer rows than one unrolled pass.
    int64_t want_rows = (64 * 1024) / (K * 2);
    int64_t pass_rows = (int64_t)rows_per_pass * UNROLL;
    int64_t band = ptq4vm::ceil_div(want_rows > 1 ? want_rows : 1, pass_rows) * pass_rows;
    if (band > kMaxBandRows) band = (kMaxBandRows / rows_per_pass) * rows_per_pass;
    if (band < rows_per_pass) band = rows_per_pass;  // rows_per_pass <= 256 <= kMaxBandRows
    const int64_t blocks = ptq4vm::ceil_div(M, band);
    if (blocks > 0x7fffffffLL) return PTQ4VM_ERR_SHAPE;
    dim3 grid((unsigned)blocks), block((unsigned)threads);
    if (inv_m)
        quantize_pts_stream<VEC, true, UNROLL><<<grid, block, 0, stream>>>(
            x, inv_m, s_tok, xq, M, (int)L, (int)K, ldx, ldxq, chunks, cols_per_pass, rows_per_pass, (int)band);
    else
        quantize_pts_stream<VEC, false, UNROLL><<<grid, block, 0, stream>>>(
            x, inv_m, s_tok, xq, M, (int)L, (int)K, ldx, ldxq, chunks, cols_per_pass, rows_per_pass, (int)band);
    return ptq4vm::check_launch("quantize_pts_stream");
}

}  // namespace

extern "C" int ptq4vm_quantize_pts(const void *x_f16, const float *inv_m, const float *s_tok, int8_t *xq,
                                   int64_t B, int64_t L, int64_t K, int64_t ldx, int64_t ldxq, void *stream_) {
    if (!x_f16 || !s_tok || !xq) return PTQ4VM_ERR_NULL;
    if (B < 0 || L <= 0 || K <= 0) return PTQ4VM_ERR_SHAPE;
    if (L > 0x7fffffffLL || K > 0x7fffffffLL || (B > 0 && L > INT64_MAX / B)) return PTQ4VM_ERR_SHAPE;
    if (ldx < K || ldxq < K) return PTQ4VM_ERR_STRIDE;
    if (!ptq4vm::aligned_to(x_f16, 16) || !ptq4vm::aligned_to(xq, 16) || !ptq4vm::aligned_to(s_tok, 4) ||
        (inv_m && !ptq4vm::aligned_to(inv_m, 4)))
        return PTQ4VM_ERR_ALIGN;
    const int64_t M = B * L;
    if (M == 0) return PTQ4VM_OK;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const __half *x = static_cast<const __half *>(x_f16);

    if (K % 8 == 0 && ldx % 8 == 0 && ldxq % 8 == 0)
        return launch_stream<8>(x, inv_m, s_tok, xq, M, L, K, ldx, ldxq, stream);
    if (K % 4 == 0 && ldx % 4 == 0 && ldxq % 4 == 0)
        return launch_stream<4>(x, inv_m, s_tok, xq, M, L, K, ldx, ldxq, stream);

    int64_t blocks = ptq4vm::ceil_div(M * K, kMaxThreads);
    if (blocks > 65536) blocks = 65536;
    if (inv_m)
        quantize_pts_generic<true><<<dim3((unsigned)blocks), dim3(kMaxThreads), 0, stream>>>(x, inv_m, s_tok, xq, M,
                                                                                           L, K, ldx, ldxq);
    else
        quantize_pts_generic<false><<<dim3((unsigned)blocks), dim3(kMaxThreads), 0, stream>>>(x, inv_m, s_tok, xq,
                                                                                            M, L, K, ldx, ldxq);
    return ptq4vm::check_launch("quantize_pts_generic");
}
