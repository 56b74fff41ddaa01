// Shared pieces of the MFMA linear kernels for gfx950: operand/accumulator types of the int8 and
// fp16 paths, the kernel argument block, the LDS swizzle, the XCD-aware tile order, the MFMA loop over
// one 64-byte slab, the fused dequantization epilogue and the zero-filling chunk loader.
#pragma once
#include <hip/hip_fp16.h>
#include <math.h>

#include "common.hpp"

namespace ptq4vm {
namespace mfma {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kSlabBytes = 64;  // K bytes per LDS stage per row: two MFMA k-steps of 32 bytes
constexpr int kXcds = 8;
#ifndef PTQ4VM_PERSISTENT_SLAB
#define PTQ4VM_PERSISTENT_SLAB 128   // K bytes per LDS row that the 256 x 256 persistent kernel needs K to divide by
#endif

struct Int8Path {
    static constexpr int kElemBytes = 1;
    static constexpr bool kOffset = false;
    static constexpr bool kPacked4 = false;
    using Acc = v16i;
    static __device__ __forceinline__ Acc mfma(v4i a, v4i b, Acc c) {
        return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
    }
    // 16 x 16 output block, 64 bytes of K per instruction: lane feeds row (lane mod 16), bytes 16 (lane / 16) ..
    using Acc16 = v4i;
    static __device__ __forceinline__ Acc16 mfma16(v4i a, v4i b, Acc16 c) {
        return __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, 0, 0, 0);
    }
};

// int8 codes carrying a per-token zero offset: the epilogue subtracts z_tok[r mod L] * rowsum[o]
// from the accumulator (sum_k (q - z) w = sum_k q w - z sum_k w) before the rescale.
struct Int8OffsetPath : Int8Path {
    static constexpr bool kOffset = true;
};

// Two 4-bit codes per byte, the even index in the low nibble (App. B.1 "Quantization").  gfx950
// has no int4 MFMA, so packed operands travel through memory, L2 and LDS at half the bytes and are
// expanded in registers right before the int8 MFMA: `p & 0xF0F0F0F0` is the odd codes times 16 as
// int8 bytes and `(p << 4) & 0xF0F0F0F0` the even codes times 16 (the nibble's two's complement sits
// in the byte's top bits, so no sign extension is needed).  One packed 16-byte operand becomes two
// MFMA operands (even and odd reduction indices; both matrices split the same way, so the sum is
// unchanged); the accumulator is 256 times the true one and is shifted back, exactly, in the epilogue.
struct Int4Path : Int8Path {
    static constexpr bool kPacked4 = true;
    static __device__ __forceinline__ v4i even_codes(v4i p) { return (p << 4) & (int)0xF0F0F0F0; }
    static __device__ __forceinline__ v4i odd_codes(v4i p) { return p & (int)0xF0F0F0F0; }
};

struct Half16Path {
    static constexpr int kElemBytes = 2;
    static constexpr bool kOffset = false;
    static constexpr bool kPacked4 = false;
    using Acc = v16f;
    static __device__ __forceinline__ Acc mfma(v4i a, v4i b, Acc c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), c, 0,
                                                      0, 0);
    }
    using Acc16 = v4f;
    static __device__ __forceinline__ Acc16 mfma16(v4i a, v4i b, Acc16 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), c, 0,
                                                      0, 0);
    }
};

struct LinearArgs {
    const char *x;       // [M, ldx] activations (B operand), K-contiguous
    const char *w;       // [N, ldw] weights (A operand), K-contiguous
    const float *s_tok;  // [L] or nullptr (fp16 path)
    const float *s_w;    // [N] or nullptr (fp16 path)
    const __half *bias;  // [N] or nullptr
    __half *y;           // [M, ldy]
    int32_t *acc_out;    // [M, N] dense or nullptr (int8 path only)
    int64_t M, N;
    int64_t k_bytes;     // K * element size
    int64_t ldx_bytes, ldw_bytes;
    int64_t ldy;         // elements
    int64_t L;
    int tiles_o, tiles_r;
    int y_vec;           // widest store the pitch and base of y allow, in fp16 elements: 8, 4 or 1
    // Fused activation quantizer only: x then holds fp16 activations (ldx_bytes = 2 * pitch) and k_bytes
    // is still K, the reduction length in int8 codes.
    // Per-token zero offset only (Int8OffsetPath):
    const int32_t *z_tok;   // [L] offsets in the int8 range
    const int32_t *rowsum;  // [N] sum_k wq[o,k]
    const float *inv_m;  // [K] reciprocal smoothing factors or nullptr (no smoothing)
    int8_t *xq_out;      // [M, ldxq_out] optional copy of the int8 codes, or nullptr
    int64_t ldxq_out;
};

extern __shared__ __attribute__((aligned(16))) char lds_dyn[];

__device__ __forceinline__ int swizzle(int row) { return ((row >> 1) ^ (row >> 2)) & 3; }

// XCD-aware tile order: workgroup ids go round-robin over the 8 XCDs, so give each XCD a
// contiguous range of tiles, output-channel tiles fastest (they share the activation strip).
__device__ __forceinline__ bool tile_of_block(const LinearArgs &p, int &tile_r, int &tile_o) {
    const int total_tiles = p.tiles_o * p.tiles_r;
    const int per_xcd = (total_tiles + kXcds - 1) / kXcds;
    const int tile = (int)(blockIdx.x % kXcds) * per_xcd + (int)(blockIdx.x / kXcds);
    if (tile >= total_tiles) return false;
    tile_o = tile % p.tiles_o;
    tile_r = tile / p.tiles_o;
    return true;
}

// MFMA work on one 64-byte slab held in LDS: x_rows/w_rows point at the wave's first row.
template <class Path, int FO, int FR>
__device__ __forceinline__ void mfma_slab(typename Path::Acc (&acc)[FO][FR], const char *x_rows, const char *w_rows,
                                          int l32, int lhalf) {
#pragma unroll
    for (int s = 0; s < 2; s++) {
        const int kc = 2 * s + lhalf;
        v4i fw[FO], fx[FR];
#pragma unroll
        for (int i = 0; i < FO; i++) {
            const int row = i * 32 + l32;  // wave row offsets are multiples of 32: swizzle(row) is unchanged
            fw[i] = *reinterpret_cast<const v4i *>(w_rows + row * kSlabBytes + ((kc ^ swizzle(row)) << 4));
        }
#pragma unroll
        for (int j = 0; j < FR; j++) {
            const int row = j * 32 + l32;
            fx[j] = *reinterpret_cast<const v4i *>(x_rows + row * kSlabBytes + ((kc ^ swizzle(row)) << 4));
        }
        if constexpr (Path::kPacked4) {
#pragma unroll
            for (int half = 0; half < 2; half++) {
                v4i ew[FO], ex[FR];
#pragma unroll
                for (int i = 0; i < FO; i++) ew[i] = half ? Path::odd_codes(fw[i]) : Path::even_codes(fw[i]);
#pragma unroll
                for (int j = 0; j < FR; j++) ex[j] = half ? Path::odd_codes(fx[j]) : Path::even_codes(fx[j]);
#pragma unroll
                for (int i = 0; i < FO; i++)
#pragma unroll
                    for (int j = 0; j < FR; j++) acc[i][j] = Path::mfma(ew[i], ex[j], acc[i][j]);
            }
        } else {
#pragma unroll
            for (int i = 0; i < FO; i++)
#pragma unroll
                for (int j = 0; j < FR; j++) acc[i][j] = Path::mfma(fw[i], fx[j], acc[i][j]);
        }
    }
}

// Epilogue of one wavefront.  Accumulator register v of a lane in block (i, j):
//   token row       r = r_base + 32 j + (lane mod 32)
//   output channel  o = o_base + 32 i + 8 (v / 4) + 4 (lane / 32) + (v mod 4)
// A lane therefore owns 8-byte runs scattered over 32 rows.  The wavefront transposes its
// results through a private LDS patch (JB*32 rows x WAVE_O fp16 at a time, 16-byte chunks
// XOR-swizzled by the row) so that the global stores are 16 bytes per lane with the lanes of a
// row side by side: every store instruction writes whole, contiguous row segments.  Only this
// wavefront touches `patch`, and the LDS executes a wavefront's instructions in order, so no
// barrier is needed; the empty asm statements only stop the compiler from reordering LDS
// accesses.  Column scales and biases are fetched per group of four channels (outer loops) so
// that they do not have to live in registers next to the accumulators.
template <class Path, int FO, int FR, int JB>
__device__ __forceinline__ void epilogue(const typename Path::Acc (&acc)[FO][FR], const LinearArgs &p, char *patch,
                                         int64_t r_base, int64_t o_base, int lane) {
    constexpr int WAVE_O = FO * 32;
    constexpr int CPR = WAVE_O / 8;           // 16-byte chunks per staged row
    constexpr int ROWS_PER_STORE = 64 / CPR;  // rows covered by one store instruction
    static_assert(CPR <= 64 && (CPR & (CPR - 1)) == 0, "wave tile width must be 32, 64 or 128 channels");
    static_assert(FR % JB == 0, "row blocks are staged in equal groups");
    const int l32 = lane & 31, lhalf = lane >> 5;
    auto patch_chunk = [&](int row, int chunk) {  // byte offset of a 16-byte chunk
        const int sw = CPR >= 8 ? (row & 7) : ((row / (8 / CPR)) & (CPR - 1));
        return row * (WAVE_O * 2) + ((chunk ^ sw) << 4);
    };

#pragma unroll
    for (int jb = 0; jb < FR; jb += JB) {
        float row_scale[JB];
        int row_z[JB];
#pragma unroll
        for (int jj = 0; jj < JB; jj++) {
            const int64_t r = r_base + (jb + jj) * 32 + l32;
            row_scale[jj] = 1.0f;
            row_z[jj] = 0;
            if constexpr (Path::kElemBytes == 1) row_scale[jj] = p.s_tok[(r < p.M ? r : 0) % p.L];
            if constexpr (Path::kOffset) row_z[jj] = p.z_tok[(r < p.M ? r : 0) % p.L];
        }
#pragma unroll
        for (int i = 0; i < FO; i++) {
#pragma unroll
            for (int g = 0; g < 4; g++) {
                float col_scale[4], col_bias[4];
                int col_sum[4];
#pragma unroll
                for (int c = 0; c < 4; c++) {
                    const int64_t o = o_base + i * 32 + g * 8 + lhalf * 4 + c;
                    const bool ok = o < p.N;
                    col_bias[c] = (ok && p.bias) ? __half2float(p.bias[o]) : 0.0f;
                    col_scale[c] = 1.0f;
                    col_sum[c] = 0;
                    if constexpr (Path::kElemBytes == 1) col_scale[c] = ok ? p.s_w[o] : 0.0f;
                    if constexpr (Path::kOffset) col_sum[c] = ok ? p.rowsum[o] : 0;
                }
#pragma unroll
                for (int jj = 0; jj < JB; jj++) {
                    const int j = jb + jj;
                    float out[4];
#pragma unroll
                    for (int c = 0; c < 4; c++) {
                        if constexpr (Path::kElemBytes == 1) {
                            int a = acc[i][j][g * 4 + c];
                            if constexpr (Path::kPacked4) a >>= 8;  // operands were codes times 16: exact
                            if (p.acc_out) {
                                const int64_t r = r_base + j * 32 + l32;
                                const int64_t o = o_base + i * 32 + g * 8 + lhalf * 4 + c;
                                if (r < p.M && o < p.N) p.acc_out[r * p.N + o] = a;
                            }
                            int corrected = a;
                            // 24-bit multiply (full rate): |z| < 2^8 and |rowsum| <= 127 K < 2^23 for every accepted K
                            if constexpr (Path::kOffset) corrected = a - __mul24(row_z[jj], col_sum[c]);
                            out[c] = (float)corrected * (row_scale[jj] * col_scale[c]) + col_bias[c];
                        } else {
                            out[c] = acc[i][j][g * 4 + c] + col_bias[c];
                        }
                    }
                    __half2 lo = __floats2half2_rn(out[0], out[1]);
                    __half2 hi = __floats2half2_rn(out[2], out[3]);
                    u32x2 packed = {*reinterpret_cast<uint32_t *>(&lo), *reinterpret_cast<uint32_t *>(&hi)};
                    *reinterpret_cast<u32x2 *>(patch + patch_chunk(jj * 32 + l32, i * 4 + g) + lhalf * 8) = packed;
                }
            }
        }
        asm volatile("" ::: "memory");
#pragma unroll
        for (int s = 0; s < JB * 32 / ROWS_PER_STORE; s++) {
            const int row = s * ROWS_PER_STORE + lane / CPR, chunk = lane % CPR;
            const v4i data = *reinterpret_cast<const v4i *>(patch + patch_chunk(row, chunk));
            const int64_t rr = r_base + jb * 32 + row;
            const int64_t oc = o_base + chunk * 8;
            if (rr < p.M && oc < p.N) {
                __half *dst = p.y + rr * p.ldy + oc;
                if (p.y_vec == 8 && oc + 8 <= p.N) {
                    *reinterpret_cast<v4i *>(dst) = data;
                } else if (p.y_vec >= 4 && oc + 8 <= p.N) {
                    u32x2 a = {(uint32_t)data[0], (uint32_t)data[1]}, b = {(uint32_t)data[2], (uint32_t)data[3]};
                    *reinterpret_cast<u32x2 *>(dst) = a;
                    *reinterpret_cast<u32x2 *>(dst + 4) = b;
                } else {
#pragma unroll
                    for (int e = 0; e < 8; e++)
                        if (oc + e < p.N)
                            reinterpret_cast<uint16_t *>(dst)[e] = (uint16_t)((uint32_t)data[e >> 1] >> (16 * (e & 1)));
                }
            }
        }
        asm volatile("" ::: "memory");
    }
}

// The dequantization of two neighbouring outputs, y = fp16(a * scale + bias) each, as ONE instruction per
// output: v_fma_mix computes the multiply-add in fp32 from fp32 a and scale and the fp16 bias and rounds
// the result to fp16.  Left to itself the compiler picks this form or fma + conversion (two roundings)
// from one inlined copy of the same source line to the next, and the two differ in the last bit of a few
// outputs per million; writing the instruction out keeps every kernel that uses this helper on the same
// bits.  `bias_pair` holds the two fp16 biases (low half: first output) as a raw word; the result is the
// two fp16 outputs as a raw word.
__device__ __forceinline__ float dequantize_pair_f16(float a0, float scale0, float a1, float scale1, float bias_pair) {
    float packed;
    asm("v_fma_mixlo_f16 %0, %1, %2, %3 op_sel_hi:[0,0,1]" : "=v"(packed) : "v"(a0), "v"(scale0), "v"(bias_pair));
    asm("v_fma_mixhi_f16 %0, %1, %2, %3 op_sel:[0,0,1] op_sel_hi:[0,0,1]"
        : "+v"(packed)
        : "v"(a1), "v"(scale1), "v"(bias_pair));
    return packed;
}

__device__ __forceinline__ uint32_t keep_low_bytes(uint32_t v, int nbytes) {
    return nbytes >= 4 ? v : (nbytes <= 0 ? 0u : (v & ((1u << (8 * nbytes)) - 1u)));
}

// One 16-byte chunk of row `row_ptr` at byte offset `kb`; bytes at or beyond k_bytes read as 0.
// LOAD_ALIGN 16: pitch and base are multiples of 16, so the full chunk is inside the row's pitch.
// LOAD_ALIGN 4:  same with 4.  LOAD_ALIGN 0: element-wise (ELEM bytes each), any pitch.
template <int LOAD_ALIGN, int ELEM>
__device__ __forceinline__ v4i load_chunk(const char *row_ptr, int64_t kb, int64_t k_bytes, bool row_ok) {
    v4i out = {0, 0, 0, 0};
    if (!row_ok || kb >= k_bytes) return out;
    const int valid = (int)min((int64_t)16, k_bytes - kb);
    if constexpr (LOAD_ALIGN == 16) {
        out = *reinterpret_cast<const v4i *>(row_ptr + kb);
        if (valid < 16) {
#pragma unroll
            for (int j = 0; j < 4; j++) out[j] = (int)keep_low_bytes((uint32_t)out[j], valid - 4 * j);
        }
    } else if constexpr (LOAD_ALIGN == 4) {
#pragma unroll
        for (int j = 0; j < 4; j++) {
            if (4 * j < valid) {
                uint32_t v = *reinterpret_cast<const uint32_t *>(row_ptr + kb + 4 * j);
                out[j] = (int)keep_low_bytes(v, valid - 4 * j);
            }
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; j++) {
            uint32_t v = 0;
#pragma unroll
            for (int b = 0; b < 4; b += ELEM) {
                if (4 * j + b < valid) {
                    if constexpr (ELEM == 1)
                        v |= (uint32_t) * reinterpret_cast<const uint8_t *>(row_ptr + kb + 4 * j + b) << (8 * b);
                    else
                        v |= (uint32_t) * reinterpret_cast<const uint16_t *>(row_ptr + kb + 4 * j + b) << (8 * b);
                }
            }
            out[j] = (int)v;
        }
    }
    return out;
}

template <int BR, int BO>
inline bool set_grid(LinearArgs &a, dim3 &grid) {
    const int64_t tiles_r = ptq4vm::ceil_div(a.M, BR), tiles_o = ptq4vm::ceil_div(a.N, BO);
    if (tiles_r * tiles_o > 0x3fffffffLL) return false;
    a.tiles_r = (int)tiles_r;
    a.tiles_o = (int)tiles_o;
    grid = dim3((unsigned)(ptq4vm::ceil_div(tiles_r * tiles_o, kXcds) * kXcds));
    return true;
}


// LDS accesses of the epilogue are written as inline asm: the compiler does not see them, so it
// cannot tie them to the outstanding global -> LDS copies (for which it would insert a full
// vmcnt(0) drain).  Every read block ends with its own s_waitcnt inside the same asm statement,
// so the outputs are valid as soon as the compiler may touch them.  Outputs are float vectors:
// this compiler reads every element of an integer-vector asm output from its first register.
__device__ __forceinline__ uint32_t lds_addr(const void *p) { return (uint32_t)(uintptr_t)p; }

// eight 16-byte reads at base + STEP n (n = 0..3) and base + JUMP + STEP n
template <int STEP, int JUMP>
__device__ __forceinline__ void lds_read_8x_b128(uint32_t base, v4f (&v)[8]) {
    asm volatile(
        "ds_read_b128 %0, %8 offset:%9\n ds_read_b128 %1, %8 offset:%10\n ds_read_b128 %2, %8 offset:%11\n"
        "ds_read_b128 %3, %8 offset:%12\n ds_read_b128 %4, %8 offset:%13\n ds_read_b128 %5, %8 offset:%14\n"
        "ds_read_b128 %6, %8 offset:%15\n ds_read_b128 %7, %8 offset:%16\n s_waitcnt lgkmcnt(0)"
        : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3]), "=&v"(v[4]), "=&v"(v[5]), "=&v"(v[6]), "=&v"(v[7])
        : "v"(base), "n"(0), "n"(STEP), "n"(2 * STEP), "n"(3 * STEP), "n"(JUMP), "n"(JUMP + STEP), "n"(JUMP + 2 * STEP),
          "n"(JUMP + 3 * STEP)
        : "memory");
}
// four 16-byte reads at base + STEP n
template <int STEP>
__device__ __forceinline__ void lds_read_4x_b128(uint32_t base, v4f (&v)[4]) {
    asm volatile(
        "ds_read_b128 %0, %4 offset:%5\n ds_read_b128 %1, %4 offset:%6\n ds_read_b128 %2, %4 offset:%7\n"
        "ds_read_b128 %3, %4 offset:%8\n s_waitcnt lgkmcnt(0)"
        : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3])
        : "v"(base), "n"(0), "n"(STEP), "n"(2 * STEP), "n"(3 * STEP)
        : "memory");
}
// eight 4-byte reads at base + STEP n
template <int STEP>
__device__ __forceinline__ void lds_read_8x_b32(uint32_t base, float (&v)[8]) {
    asm volatile(
        "ds_read_b32 %0, %8 offset:%9\n ds_read_b32 %1, %8 offset:%10\n ds_read_b32 %2, %8 offset:%11\n"
        "ds_read_b32 %3, %8 offset:%12\n ds_read_b32 %4, %8 offset:%13\n ds_read_b32 %5, %8 offset:%14\n"
        "ds_read_b32 %6, %8 offset:%15\n ds_read_b32 %7, %8 offset:%16\n s_waitcnt lgkmcnt(0)"
        : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3]), "=&v"(v[4]), "=&v"(v[5]), "=&v"(v[6]), "=&v"(v[7])
        : "v"(base), "n"(0), "n"(STEP), "n"(2 * STEP), "n"(3 * STEP), "n"(4 * STEP), "n"(5 * STEP), "n"(6 * STEP),
          "n"(7 * STEP)
        : "memory");
}
// four 4-byte reads at base + STEP n
template <int STEP>
__device__ __forceinline__ void lds_read_4x_b32(uint32_t base, float (&v)[4]) {
    asm volatile(
        "ds_read_b32 %0, %4 offset:%5\n ds_read_b32 %1, %4 offset:%6\n ds_read_b32 %2, %4 offset:%7\n"
        "ds_read_b32 %3, %4 offset:%8\n s_waitcnt lgkmcnt(0)"
        : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3])
        : "v"(base), "n"(0), "n"(STEP), "n"(2 * STEP), "n"(3 * STEP)
        : "memory");
}
// four 16-byte reads at arbitrary addresses
__device__ __forceinline__ void lds_read_4_b128(const uint32_t (&addr)[4], v4f (&v)[4]) {
    asm volatile(
        "ds_read_b128 %0, %4\n ds_read_b128 %1, %5\n ds_read_b128 %2, %6\n ds_read_b128 %3, %7\n"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3])
        : "v"(addr[0]), "v"(addr[1]), "v"(addr[2]), "v"(addr[3])
        : "memory");
}
__device__ __forceinline__ void lds_write_b64(uint32_t addr, u32x2 v) {
    asm volatile("ds_write_b64 %0, %1" ::"v"(addr), "v"(v) : "memory");
}

template <int KEEP>
__device__ __forceinline__ void wait_vmcnt_at_most() {
    // s_waitcnt immediate on gfx9: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] << 14
    static_assert(KEEP >= 0 && KEEP <= 63, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (KEEP & 15) | ((KEEP >> 4) << 14));
}

__device__ __forceinline__ void lds_read_1x_b128(uint32_t addr, v4f &v) {
    asm volatile("ds_read_b128 %0, %1\n s_waitcnt lgkmcnt(0)" : "=&v"(v) : "v"(addr) : "memory");
}
// two 16-byte reads at base and base + STEP
template <int STEP>
__device__ __forceinline__ void lds_read_2x_b128(uint32_t base, v4f (&v)[2]) {
    asm volatile("ds_read_b128 %0, %2 offset:%3\n ds_read_b128 %1, %2 offset:%4\n s_waitcnt lgkmcnt(0)"
                 : "=&v"(v[0]), "=&v"(v[1])
                 : "v"(base), "n"(0), "n"(STEP)
                 : "memory");
}
// Reads that are only ISSUED here (eight 4-byte reads at base + STEP n; three 16-byte reads at base +
// STEP n): the caller must pass every destination through lds_wait_all before using it.
template <int STEP>
__device__ __forceinline__ void lds_issue_8x_b32(uint32_t base, float (&v)[8]) {
    asm volatile(
        "ds_read_b32 %0, %8 offset:%9\n ds_read_b32 %1, %8 offset:%10\n ds_read_b32 %2, %8 offset:%11\n"
        "ds_read_b32 %3, %8 offset:%12\n ds_read_b32 %4, %8 offset:%13\n ds_read_b32 %5, %8 offset:%14\n"
        "ds_read_b32 %6, %8 offset:%15\n ds_read_b32 %7, %8 offset:%16"
        : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3]), "=&v"(v[4]), "=&v"(v[5]), "=&v"(v[6]), "=&v"(v[7])
        : "v"(base), "n"(0), "n"(STEP), "n"(2 * STEP), "n"(3 * STEP), "n"(4 * STEP), "n"(5 * STEP), "n"(6 * STEP),
          "n"(7 * STEP)
        : "memory");
}
template <int STEP>
__device__ __forceinline__ void lds_issue_3x_b128(uint32_t base, v4f (&v)[3]) {
    asm volatile("ds_read_b128 %0, %3 offset:%4\n ds_read_b128 %1, %3 offset:%5\n ds_read_b128 %2, %3 offset:%6"
                 : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2])
                 : "v"(base), "n"(0), "n"(STEP), "n"(2 * STEP)
                 : "memory");
}
// s_waitcnt lgkmcnt(0) that the given registers depend on: no use of them can be scheduled ahead of it.
__device__ __forceinline__ void lds_wait_all(float (&a)[8], v4f (&b)[3]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(a[5]), "+v"(a[6]), "+v"(a[7]),
                   "+v"(b[0]), "+v"(b[1]), "+v"(b[2])
                 :
                 : "memory");
}
__device__ __forceinline__ void lds_write_b128(uint32_t addr, v4f v) {
    asm volatile("ds_write_b128 %0, %1" ::"v"(addr), "v"(v) : "memory");
}

// Row-streaming kernel for short reductions (K <= 128), defined next to the fused kernels.
// quantize: x holds fp16 activations and inv_m / xq_out are honoured; otherwise x holds int8 codes.
// Returns PTQ4VM_OK after a launch, a negative status on error, or 1 if the shape does not fit
// this kernel (nothing was launched; the caller picks another one).
// packed4: x and w hold two 4-bit codes per byte (k_bytes = K / 2), expanded on chip; with `quantize` (the fused
// 4-bit form) x holds fp16 activations, only w is packed and k_bytes = K.
// offset: z_tok / rowsum are honoured (per-token zero offset; with `quantize` the codes carry the offset); not with `packed4`.
int launch_stream_smallk(const LinearArgs &a, bool quantize, hipStream_t stream, bool packed4 = false, bool offset = false);

// Weights-in-registers kernel for wide int8 linears with a short reduction (K = 384 or 768, e.g. the
// in_proj of the Vim-S / Vim-B stacks), defined in gemm_wreg.hip.  Same return convention.
int launch_wreg(const LinearArgs &a, hipStream_t stream);

}  // namespace mfma
}  // namespace ptq4vm
