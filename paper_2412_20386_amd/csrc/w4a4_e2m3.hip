// The 4-bit weight fold and PTS activation quantizer of w4a4.hip writing their codes as FP6 (E2M3) numbers:
// the operand format of gfx950's v_mfma_f32_16x16x128_f8f6f4, which runs at twice the int8 MFMA rate.  Every
// code -7..7 (Sec. 2.3: +-(2^(b-1) - 1) with b = 4, the W4A4 setting of the latency table of Sec. 6.4) is
// exactly an E2M3 number (1 sign, 2 exponent, 3 mantissa bits, bias 1), so the matrix product on these
// containers is the integer product of App. B.1 "INT GEMM", exactly.
//   ptq4vm_fold_smoothing_w4_e2m3   W' = W diag(m), s_w = max|W'| / 7, codes as E2M3 [N, 96 ceil(K / 128)]
//   ptq4vm_quantize_pts_a4_e2m3     clip(rne((f32(x) inv_m[k]) (1 / s_tok[r mod L])), -7, 7), same container
// Container: a row is zero padded to a multiple of 128 codes and written as 96-byte blocks of 128 codes; in a
// block, group g = 0..3 holds codes 32 g .. 32 g + 31 as a 192-bit little-endian string (code j at bits
// [6 j, 6 j + 6)), the string's first 16 bytes at block offset 16 g, its last 8 bytes at offset 64 + 8 g: a
// lane of the MFMA reads its 32 codes with one 16-byte and one 8-byte access.  Storage is block-major: block b
// of row r starts at byte b * pitch + 96 r (plane pitch >= 96 rows), so the blocks that 16 consecutive rows have
// in one block column are one contiguous 1536-byte span.
// The integer decision is the one of the nibble quantizer (same fp32 products, rint, hardware float -> int
// conversion, clamp); the integer is then converted back to fp32 (exact) and 32 of them are packed by one
// v_cvt_scalef32_2xpk16_fp6_f32 (scale 1: exact for these values; -0 cannot occur because the value comes
// from an integer).
#include <hip/hip_fp16.h>

#include "common.hpp"
#include "quant_device.hpp"

namespace {

using ptq4vm::cvt_i32_f32;

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x6 __attribute__((ext_vector_type(6)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kMaxLdsTokens = 16384;
constexpr int kBlockBytes = 96;   // 128 codes
constexpr int kGroupCodes = 32;   // codes of one lane of the MFMA

__device__ __forceinline__ float code4_as_float(float x, float inv_m, float inv_s) {
    float v = x * inv_m;  // two separate fp32 multiplies in this order, as in the 8-bit quantizer
    v = v * inv_s;
    const int q = cvt_i32_f32(__builtin_rintf(v));  // NaN -> 0
    return (float)min(max(q, -7), 7);
}

// 32 integer-valued floats in [-7, 7] -> their E2M3 patterns, value j at bits [6 j, 6 j + 6).
// The instruction interleaves its two sources: field 2 i comes from the first, field 2 i + 1 from the second.
__device__ __forceinline__ u32x6 pack32_e2m3(const float (&v)[32]) {
    v16f even, odd;
#pragma unroll
    for (int i = 0; i < 16; i++) even[i] = v[2 * i], odd[i] = v[2 * i + 1];
    return __builtin_amdgcn_cvt_scalef32_2xpk16_fp6_f32(even, odd, 1.0f);
}

// `base`: the container; group: 4 * block + g; pitch: plane pitch in bytes
__device__ __forceinline__ void store_group(uint8_t *base, int64_t row, int group, int64_t pitch, const u32x6 &s) {
    uint8_t *block = base + (group >> 2) * pitch + row * kBlockBytes;
    const int g = group & 3;
    const u32x4 lo = {s[0], s[1], s[2], s[3]};
    const u32x2 hi = {s[4], s[5]};
    ptq4vm::store_for_next_kernel(reinterpret_cast<u32x4 *>(block + 16 * g), lo);
    ptq4vm::store_for_next_kernel(reinterpret_cast<u32x2 *>(block + 64 + 8 * g), hi);
}

// Column-stationary stream (K % 32 == 0, 16-byte aligned rows): gridDim.x * 256 is a multiple of `groups_padded`
// (4 per block of 128 codes); thread g owns group g mod groups_padded (32 channels, smoothing factors in
// registers) and rows g / groups_padded + i * row_step.  Groups at or beyond K / 32 are padding: zeros.
template <bool HAS_M, bool LDS_TABLE>
__global__ __launch_bounds__(kThreads) void quantize_pts_a4_e2m3_stream(const __half *__restrict__ x,
                                                                        const float *__restrict__ inv_m,
                                                                        const float *__restrict__ s_tok,
                                                                        uint8_t *__restrict__ xq6, int64_t M, int L,
                                                                        int groups, int groups_padded, int64_t ldx,
                                                                        int64_t ldxq, int64_t row_step) {
    extern __shared__ float inv_s_lds[];
    if constexpr (LDS_TABLE) {
        for (int i = threadIdx.x; i < L; i += kThreads) inv_s_lds[i] = 1.0f / s_tok[i];  // IEEE division
        __syncthreads();
    }
    const int64_t gtid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int group = (int)(gtid % groups_padded);
    int64_t row = gtid / groups_padded;
    if (group >= groups) {
        const u32x6 zero = {0, 0, 0, 0, 0, 0};
        for (; row < M; row += row_step) store_group(xq6, row, group, ldxq, zero);
        return;
    }
    int t = (int)(row % L);
    const int t_step = (int)(row_step % L);
    float im[kGroupCodes];
#pragma unroll
    for (int i = 0; i < kGroupCodes; i++) im[i] = HAS_M ? inv_m[group * kGroupCodes + i] : 1.0f;
    const __half *xp = x + row * ldx + (int64_t)group * kGroupCodes;
    const int64_t x_step = row_step * ldx;
    for (; row < M; row += row_step) {
        u32x4 in[4];
#pragma unroll
        for (int c = 0; c < 4; c++) in[c] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(xp) + c);
        const float inv_s = LDS_TABLE ? inv_s_lds[t] : 1.0f / s_tok[t];
        t += t_step;
        if (t >= L) t -= L;
        float v[kGroupCodes];
#pragma unroll
        for (int c = 0; c < 4; c++)
#pragma unroll
            for (int e = 0; e < 4; e++) {
                const uint32_t word = in[c][e];  // a scalar first: a bit cast applied to a vector element misreads it
                const __half2 h = __builtin_bit_cast(__half2, word);
                const int k = 8 * c + 2 * e;
                v[k] = code4_as_float(__low2float(h), im[k], inv_s);
                v[k + 1] = code4_as_float(__high2float(h), im[k + 1], inv_s);
            }
        store_group(xq6, row, group, ldxq, pack32_e2m3(v));
        xp += x_step;
    }
}

// Block-column stream (K % 128 == 0, 16-byte aligned rows).  A wavefront owns one block column (128 channels) and
// walks down the rows 16 at a time.  Loads are whole 256-byte row segments: lane l of load c reads the 8 values
// of chunk (l mod 16) of row 4 c + l / 16, so a lane keeps the smoothing factors of 8 channels for life.  The 32
// values of a group are spread over 4 lanes, and the packing instruction wants them in one: the integer-valued
// floats cross through a wavefront-private LDS patch (group pitch 144 bytes: the 16 lanes of an access phase
// start 4 banks apart), after which lane G holds group G mod 4 of row G / 4; its 24 bytes go to a second patch laid
// out like the unit's 1536 contiguous bytes of the container, which leave as 16-byte stores of consecutive lines.
constexpr int kPatchPitch = 144;
constexpr int kOutBytes = 16 * kBlockBytes;                // the unit's 16 blocks as they lie in memory
constexpr int kPatchBytes = 64 * kPatchPitch + kOutBytes;  // per wavefront
constexpr int kMaxBlockTokens = 4096;        // reciprocal steps of all token positions sit next to the patches (52 KiB in all)

template <bool HAS_M>
__global__ __launch_bounds__(kThreads) void quantize_pts_a4_e2m3_blocks(const __half *__restrict__ x,
                                                                        const float *__restrict__ inv_m,
                                                                        const float *__restrict__ s_tok,
                                                                        uint8_t *__restrict__ xq6, int64_t M, int L,
                                                                        int n_blocks, int64_t ldx, int64_t ldxq,
                                                                        int64_t unit_step) {
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    float *const inv_s_lds = reinterpret_cast<float *>(lds_raw + (kThreads / 64) * kPatchBytes);
    for (int i = threadIdx.x; i < L; i += kThreads) inv_s_lds[i] = 1.0f / s_tok[i];  // IEEE division
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    char *const patch = lds_raw + wave * kPatchBytes;
    const int64_t gwave = (int64_t)blockIdx.x * (kThreads / 64) + wave;
    const int block = (int)(gwave % n_blocks);
    const int chunk = lane & 15, sub = lane >> 4;
    float im[8];
#pragma unroll
    for (int i = 0; i < 8; i++) im[i] = HAS_M ? inv_m[block * 128 + chunk * 8 + i] : 1.0f;
    // write side: row 4 c + sub, group chunk / 4, floats 8 (chunk mod 4) ..; read side: group `lane`
    const int wr_off = (sub * 4 + (chunk >> 2)) * kPatchPitch + (chunk & 3) * 32;
    const int rd_off = lane * kPatchPitch;
    for (int64_t unit = gwave / n_blocks; unit * 16 < M; unit += unit_step) {
        const int64_t r0 = unit * 16;
        u32x4 in[4];
#pragma unroll
        for (int c = 0; c < 4; c++) {
            const int64_t r = r0 + 4 * c + sub;
            in[c] = u32x4{0, 0, 0, 0};
            if (r < M) in[c] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(x + r * ldx + block * 128 + chunk * 8));
        }
        const int t0 = (int)(r0 % L);
#pragma unroll
        for (int c = 0; c < 4; c++) {
            int t = t0 + 4 * c + sub;
            t = t >= L ? t % L : t;
            const float inv_s = inv_s_lds[t];
            float q[8];
#pragma unroll
            for (int e = 0; e < 4; e++) {
                const uint32_t word = in[c][e];  // a scalar first: a bit cast applied to a vector element misreads it
                const __half2 h = __builtin_bit_cast(__half2, word);
                q[2 * e] = code4_as_float(__low2float(h), im[2 * e], inv_s);
                q[2 * e + 1] = code4_as_float(__high2float(h), im[2 * e + 1], inv_s);
            }
            float *dst = reinterpret_cast<float *>(patch + c * 16 * kPatchPitch + wr_off);
            *reinterpret_cast<float4 *>(dst) = float4{q[0], q[1], q[2], q[3]};
            *reinterpret_cast<float4 *>(dst + 4) = float4{q[4], q[5], q[6], q[7]};
        }
        asm volatile("" ::: "memory");  // wavefront-private patch: LDS runs a wavefront's accesses in order
        float v[kGroupCodes];
#pragma unroll
        for (int i = 0; i < 8; i++) {
            const float4 f = *reinterpret_cast<const float4 *>(patch + rd_off + 16 * i);
            v[4 * i] = f.x, v[4 * i + 1] = f.y, v[4 * i + 2] = f.z, v[4 * i + 3] = f.w;
        }
        asm volatile("" ::: "memory");
        const u32x6 packed = pack32_e2m3(v);
        char *out = patch + 64 * kPatchPitch;
        *reinterpret_cast<u32x4 *>(out + (lane >> 2) * kBlockBytes + 16 * (lane & 3)) = u32x4{packed[0], packed[1], packed[2], packed[3]};
        *reinterpret_cast<u32x2 *>(out + (lane >> 2) * kBlockBytes + 64 + 8 * (lane & 3)) = u32x2{packed[4], packed[5]};
        asm volatile("" ::: "memory");
        const int valid = (int)min((int64_t)16, M - r0) * kBlockBytes;  // bytes of the unit inside the matrix
        uint8_t *dst = xq6 + block * ldxq + r0 * kBlockBytes;
#pragma unroll
        for (int h = 0; h < 2; h++) {
            const int off = (h * 64 + lane) * 16;
            if (off < valid && (h == 0 || lane < 32)) {
                const u32x4 data = *reinterpret_cast<const u32x4 *>(out + off);
                ptq4vm::store_for_next_kernel(reinterpret_cast<u32x4 *>(dst + off), data);
            }
        }
        asm volatile("" ::: "memory");
    }
}

// Any K and any fp16 pitch: one group (32 codes, element-wise guarded loads) per thread-iteration.
template <bool HAS_M>
__global__ __launch_bounds__(kThreads) void quantize_pts_a4_e2m3_generic(const __half *__restrict__ x,
                                                                         const float *__restrict__ inv_m,
                                                                         const float *__restrict__ s_tok,
                                                                         uint8_t *__restrict__ xq6, int64_t M, int64_t L,
                                                                         int64_t K, int groups_padded, int64_t ldx,
                                                                         int64_t ldxq) {
    const int64_t total = M * groups_padded;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = e / groups_padded;
        const int group = (int)(e - r * groups_padded);
        const float inv_s = 1.0f / s_tok[r % L];
        float v[kGroupCodes];
#pragma unroll
        for (int j = 0; j < kGroupCodes; j++) {
            const int64_t k = (int64_t)group * kGroupCodes + j;
            v[j] = k < K ? code4_as_float(__half2float(x[r * ldx + k]), HAS_M ? inv_m[k] : 1.0f, inv_s) : 0.0f;
        }
        store_group(xq6, r, group, ldxq, pack32_e2m3(v));
    }
}

// Blocks [0, N) quantize one output channel each; blocks [N, N + ceil(K/256)) write 1/m.
__global__ __launch_bounds__(kThreads) void fold_smoothing_w4_e2m3_rows(const __half *__restrict__ w,
                                                                        const float *__restrict__ m,
                                                                        uint8_t *__restrict__ wq6,
                                                                        float *__restrict__ s_w,
                                                                        float *__restrict__ inv_m, int64_t N, int64_t K,
                                                                        int groups_padded, int64_t ldw, int64_t ldwq) {
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
    for (int group = threadIdx.x; group < groups_padded; group += kThreads) {
        float v[kGroupCodes];
#pragma unroll
        for (int j = 0; j < kGroupCodes; j++) {
            const int64_t k = (int64_t)group * kGroupCodes + j;
            float q = 0.0f;
            if (k < K) {
                const float wf = __half2float(wrow[k]) * m[k];
                q = (float)min(max(cvt_i32_f32(__builtin_rintf(wf / step)), -7), 7);
            }
            v[j] = q;
        }
        store_group(wq6, o, group, ldwq, pack32_e2m3(v));
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

extern "C" int ptq4vm_fold_smoothing_w4_e2m3(const void *w_f16, const float *m, uint8_t *wq6, float *s_w, float *inv_m,
                                             int64_t N, int64_t K, int64_t ldw, int64_t ldwq, void *stream_) {
    if (!w_f16 || !m || !wq6 || !s_w || !inv_m) return PTQ4VM_ERR_NULL;
    if (N < 0 || K <= 0 || K > PTQ4VM_MAX_K_E2M3) return PTQ4VM_ERR_SHAPE;
    if (ldw < K || ldwq / 96 < N || ldwq % 16 != 0) return PTQ4VM_ERR_STRIDE;
    if (!ptq4vm::aligned_to(w_f16, 2) || !ptq4vm::aligned_to(wq6, 16) || !ptq4vm::aligned_to(m, 4) ||
        !ptq4vm::aligned_to(s_w, 4) || !ptq4vm::aligned_to(inv_m, 4))
        return PTQ4VM_ERR_ALIGN;
    const int64_t blocks = N + ptq4vm::ceil_div(K, kThreads);
    if (blocks > 0x7fffffffLL) return PTQ4VM_ERR_SHAPE;
    const int groups_padded = (int)(ptq4vm::ceil_div(K, 128) * 4);
    fold_smoothing_w4_e2m3_rows<<<dim3((unsigned)blocks), dim3(kThreads), 0, static_cast<hipStream_t>(stream_)>>>(
        static_cast<const __half *>(w_f16), m, wq6, s_w, inv_m, N, K, groups_padded, ldw, ldwq);
    return ptq4vm::check_launch("fold_smoothing_w4_e2m3_rows");
}

extern "C" int ptq4vm_quantize_pts_a4_e2m3(const void *x_f16, const float *inv_m, const float *s_tok, uint8_t *xq6,
                                           int64_t B, int64_t L, int64_t K, int64_t ldx, int64_t ldxq, void *stream_) {
    if (!x_f16 || !s_tok || !xq6) return PTQ4VM_ERR_NULL;
    if (B < 0 || L <= 0 || K <= 0 || K > PTQ4VM_MAX_K_E2M3) return PTQ4VM_ERR_SHAPE;
    if (L > 0x7fffffffLL || (B > 0 && L > INT64_MAX / B)) return PTQ4VM_ERR_SHAPE;
    if (ldx < K || (B > 0 && ldxq / 96 < B * L) || ldxq % 16 != 0) return PTQ4VM_ERR_STRIDE;
    if (!ptq4vm::aligned_to(x_f16, 2) || !ptq4vm::aligned_to(xq6, 16) || !ptq4vm::aligned_to(s_tok, 4) ||
        (inv_m && !ptq4vm::aligned_to(inv_m, 4)))
        return PTQ4VM_ERR_ALIGN;
    const int64_t M = B * L;
    if (M == 0) return PTQ4VM_OK;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const __half *x = static_cast<const __half *>(x_f16);
    const int64_t groups_padded = ptq4vm::ceil_div(K, 128) * 4;

    if (K % 128 == 0 && ldx % 8 == 0 && ptq4vm::aligned_to(x_f16, 16) && L <= kMaxBlockTokens) {
        const int64_t n_blocks = K / 128, units = ptq4vm::ceil_div(M, 16);
        constexpr int kWavesPerWg = kThreads / 64;
        // about 3 workgroups per CU; the wavefront count is a multiple of the block columns so that every
        // wavefront keeps its column
        int64_t waves = 768 * kWavesPerWg;
        if (waves > units * n_blocks) waves = units * n_blocks;
        const int64_t lcm = n_blocks * kWavesPerWg / gcd64(n_blocks, kWavesPerWg);
        waves = ptq4vm::ceil_div(waves, lcm) * lcm;
        const int64_t blocks = waves / kWavesPerWg;
        if (blocks > 0x7fffffffLL) return PTQ4VM_ERR_SHAPE;
        const size_t lds = (size_t)kWavesPerWg * kPatchBytes + (size_t)L * sizeof(float);
        const dim3 grid((unsigned)blocks), block(kThreads);
        if (inv_m)
            quantize_pts_a4_e2m3_blocks<true><<<grid, block, lds, stream>>>(x, inv_m, s_tok, xq6, M, (int)L, (int)n_blocks, ldx, ldxq, waves / n_blocks);
        else
            quantize_pts_a4_e2m3_blocks<false><<<grid, block, lds, stream>>>(x, inv_m, s_tok, xq6, M, (int)L, (int)n_blocks, ldx, ldxq, waves / n_blocks);
        return ptq4vm::check_launch("quantize_pts_a4_e2m3_blocks");
    }
    if (K % kGroupCodes == 0 && ldx % 8 == 0 && ptq4vm::aligned_to(x_f16, 16)) {
        const int64_t unit = groups_padded / gcd64(groups_padded, kThreads);
        int64_t want = 768;  // about 3 workgroups per CU striding over the rows together
        const int64_t needed = ptq4vm::ceil_div(M * groups_padded, kThreads);
        if (want > needed) want = needed;
        const int64_t blocks = ptq4vm::ceil_div(want, unit) * unit;
        if (blocks > 0x7fffffffLL) return PTQ4VM_ERR_SHAPE;
        const int64_t row_step = blocks * kThreads / groups_padded;
        const bool table = L <= kMaxLdsTokens;
        const size_t lds = table ? (size_t)L * sizeof(float) : 0;
        const dim3 grid((unsigned)blocks), block(kThreads);
#define PTQ4VM_LAUNCH(HAS_M, TABLE)                                                                             \
    quantize_pts_a4_e2m3_stream<HAS_M, TABLE><<<grid, block, lds, stream>>>(x, inv_m, s_tok, xq6, M, (int)L,    \
                                                                            (int)(K / kGroupCodes),             \
                                                                            (int)groups_padded, ldx, ldxq, row_step)
        if (inv_m) {
            if (table) PTQ4VM_LAUNCH(true, true); else PTQ4VM_LAUNCH(true, false);
        } else {
            if (table) PTQ4VM_LAUNCH(false, true); else PTQ4VM_LAUNCH(false, false);
        }
#undef PTQ4VM_LAUNCH
        return ptq4vm::check_launch("quantize_pts_a4_e2m3_stream");
    }
    int64_t blocks = ptq4vm::ceil_div(M * groups_padded, kThreads);
    if (blocks > 65536) blocks = 65536;
    if (inv_m)
        quantize_pts_a4_e2m3_generic<true><<<dim3((unsigned)blocks), dim3(kThreads), 0, stream>>>(x, inv_m, s_tok, xq6, M, L, K, (int)groups_padded, ldx, ldxq);
    else
        quantize_pts_a4_e2m3_generic<false><<<dim3((unsigned)blocks), dim3(kThreads), 0, stream>>>(x, inv_m, s_tok, xq6, M, L, K, (int)groups_padded, ldx, ldxq);
    return ptq4vm::check_launch("quantize_pts_a4_e2m3_generic");
}
