// MFMA linear layers for gfx950.
//
//   ptq4vm_w8a8_linear  int8 x int8 -> int32 GEMM with the PTS dequantization fused into the
//                       epilogue (PTS equation of Sec. 5.1: diag(Delta_W)(W-bar X-bar)diag(Delta_X);
//                       App. B.1 "INT GEMM" + "Dequantization" without the materialised
//                       step-size outer product).
//   ptq4vm_f16_linear   the unquantized FP16 linear the paper's latency table compares with,
//                       on the same tiling skeleton.
//
// Both operands are K-contiguous (X[M,K], W[N,K]), which is exactly what the CDNA4 MFMA wants:
// a lane feeds 16 consecutive bytes of K per instruction (16 int8 for v_mfma_i32_32x32x32_i8,
// 8 fp16 for v_mfma_f32_32x32x16_f16), so one 128-bit load from either matrix is one operand.
// The weight is the MFMA "A" operand and the activation the "B" operand: the accumulator of a
// lane then holds one token row r and runs of four consecutive output channels, which become
// 8-byte fp16 stores, and the per-token step s_tok[r mod L] is one scalar per lane.
//
// Tiling: a workgroup of 4 wavefronts owns BR token rows x BO output channels; K is walked in
// slabs of 64 bytes, double buffered in LDS (register-staged global loads, one barrier per
// slab).  LDS rows are 64 bytes with the 16-byte chunk index XOR-swizzled by the row so that
// both the 128-bit writes and the MFMA-fragment reads spread over all banks.  Workgroup ids
// are remapped so that the tiles sharing one activation strip run on the same XCD (shared L2).
#include <hip/hip_fp16.h>

#include "common.hpp"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kSlabBytes = 64;  // K bytes per LDS stage per row: two MFMA k-steps of 32 bytes
constexpr int kXcds = 8;

struct Int8Path {
    static constexpr int kElemBytes = 1;
    using Acc = v16i;
    static __device__ __forceinline__ Acc mfma(v4i a, v4i b, Acc c) {
        return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
    }
};

struct Half16Path {
    static constexpr int kElemBytes = 2;
    using Acc = v16f;
    static __device__ __forceinline__ Acc mfma(v4i a, v4i b, Acc c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), c, 0,
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
    int y_vec4_ok;       // rows of y are 8-byte aligned: runs of 4 outputs may use one 64-bit store
};

__device__ __forceinline__ int swizzle(int row) { return ((row >> 1) ^ (row >> 2)) & 3; }

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

template <class Path, int BR, int BO, int WR, int WO, int LOAD_ALIGN>
__global__ __launch_bounds__(kThreads, 2) void linear_mfma(const LinearArgs p) {
    static_assert(WR * WO == kWaves, "four wavefronts per workgroup");
    constexpr int WAVE_R = BR / WR, WAVE_O = BO / WO;  // wave tile
    constexpr int FR = WAVE_R / 32, FO = WAVE_O / 32;  // 32x32 MFMA blocks per wave tile
    static_assert(WAVE_R % 32 == 0 && WAVE_O % 32 == 0, "wave tile must be whole MFMA blocks");
    constexpr int X_CHUNKS = (BR * 4 + kThreads - 1) / kThreads;  // 16-byte chunks per thread per slab
    constexpr int W_CHUNKS = (BO * 4 + kThreads - 1) / kThreads;
    using Acc = typename Path::Acc;

    __shared__ __attribute__((aligned(16))) char lds_x[2][BR * kSlabBytes];
    __shared__ __attribute__((aligned(16))) char lds_w[2][BO * kSlabBytes];

    // XCD-aware tile order: workgroup ids go round-robin over the 8 XCDs, so give each XCD a
    // contiguous range of tiles, output-channel tiles fastest (they share the activation strip).
    const int total_tiles = p.tiles_o * p.tiles_r;
    const int per_xcd = (total_tiles + kXcds - 1) / kXcds;
    const int tile = (int)(blockIdx.x % kXcds) * per_xcd + (int)(blockIdx.x / kXcds);
    if (tile >= total_tiles) return;
    const int tile_o = tile % p.tiles_o, tile_r = tile / p.tiles_o;
    const int64_t r0 = (int64_t)tile_r * BR;
    const int64_t o0 = (int64_t)tile_o * BO;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_r = (wave / WO) * WAVE_R, wave_o = (wave % WO) * WAVE_O;
    const int l32 = lane & 31, lhalf = lane >> 5;

    Acc acc[FO][FR];
#pragma unroll
    for (int i = 0; i < FO; i++)
#pragma unroll
        for (int j = 0; j < FR; j++)
#pragma unroll
            for (int v = 0; v < 16; v++) acc[i][j][v] = 0;

    v4i stage_x[X_CHUNKS], stage_w[W_CHUNKS];

    auto fetch = [&](int64_t kb0) {
#pragma unroll
        for (int i = 0; i < X_CHUNKS; i++) {
            const int cid = tid + kThreads * i, row = cid >> 2, kc = cid & 3;
            const bool ok = (cid < BR * 4) && (r0 + row < p.M);
            stage_x[i] = load_chunk<LOAD_ALIGN, Path::kElemBytes>(p.x + (r0 + row) * p.ldx_bytes, kb0 + kc * 16,
                                                                  p.k_bytes, ok);
        }
#pragma unroll
        for (int i = 0; i < W_CHUNKS; i++) {
            const int cid = tid + kThreads * i, row = cid >> 2, kc = cid & 3;
            const bool ok = (cid < BO * 4) && (o0 + row < p.N);
            stage_w[i] = load_chunk<LOAD_ALIGN, Path::kElemBytes>(p.w + (o0 + row) * p.ldw_bytes, kb0 + kc * 16,
                                                                  p.k_bytes, ok);
        }
    };
    auto commit = [&](int buf) {
#pragma unroll
        for (int i = 0; i < X_CHUNKS; i++) {
            const int cid = tid + kThreads * i, row = cid >> 2, kc = cid & 3;
            if (cid < BR * 4)
                *reinterpret_cast<v4i *>(&lds_x[buf][row * kSlabBytes + ((kc ^ swizzle(row)) << 4)]) = stage_x[i];
        }
#pragma unroll
        for (int i = 0; i < W_CHUNKS; i++) {
            const int cid = tid + kThreads * i, row = cid >> 2, kc = cid & 3;
            if (cid < BO * 4)
                *reinterpret_cast<v4i *>(&lds_w[buf][row * kSlabBytes + ((kc ^ swizzle(row)) << 4)]) = stage_w[i];
        }
    };

    const int n_slabs = (int)((p.k_bytes + kSlabBytes - 1) / kSlabBytes);
    fetch(0);
    commit(0);
    __syncthreads();

    for (int it = 0; it < n_slabs; it++) {
        const int buf = it & 1;
        const bool more = it + 1 < n_slabs;
        if (more) fetch((int64_t)(it + 1) * kSlabBytes);
#pragma unroll
        for (int s = 0; s < 2; s++) {
            const int kc = 2 * s + lhalf;
            v4i fw[FO], fx[FR];
#pragma unroll
            for (int i = 0; i < FO; i++) {
                const int row = wave_o + i * 32 + l32;
                fw[i] = *reinterpret_cast<const v4i *>(&lds_w[buf][row * kSlabBytes + ((kc ^ swizzle(row)) << 4)]);
            }
#pragma unroll
            for (int j = 0; j < FR; j++) {
                const int row = wave_r + j * 32 + l32;
                fx[j] = *reinterpret_cast<const v4i *>(&lds_x[buf][row * kSlabBytes + ((kc ^ swizzle(row)) << 4)]);
            }
#pragma unroll
            for (int i = 0; i < FO; i++)
#pragma unroll
                for (int j = 0; j < FR; j++) acc[i][j] = Path::mfma(fw[i], fx[j], acc[i][j]);
        }
        if (more) commit(buf ^ 1);
        __syncthreads();
    }

    // Epilogue.  Accumulator register v of a lane in block (i, j):
    //   token row       r = r0 + wave_r + 32 j + (lane mod 32)
    //   output channel  o = o0 + wave_o + 32 i + 8 (v / 4) + 4 (lane / 32) + (v mod 4)
#pragma unroll
    for (int j = 0; j < FR; j++) {
        const int64_t r = r0 + wave_r + j * 32 + l32;
        if (r >= p.M) continue;
        float row_scale = 1.0f;
        if constexpr (Path::kElemBytes == 1) row_scale = p.s_tok[r % p.L];
        __half *yrow = p.y + r * p.ldy;
#pragma unroll
        for (int i = 0; i < FO; i++) {
#pragma unroll
            for (int g = 0; g < 4; g++) {
                const int64_t ob = o0 + wave_o + i * 32 + g * 8 + lhalf * 4;
                if (ob >= p.N) continue;
                float out[4];
#pragma unroll
                for (int c = 0; c < 4; c++) {
                    const int64_t o = ob + c;
                    float val = 0.0f;
                    if (o < p.N) {
                        const float b = p.bias ? __half2float(p.bias[o]) : 0.0f;
                        if constexpr (Path::kElemBytes == 1) {
                            const int a = acc[i][j][g * 4 + c];
                            if (p.acc_out) p.acc_out[r * p.N + o] = a;
                            val = (float)a * (row_scale * p.s_w[o]) + b;
                        } else {
                            val = acc[i][j][g * 4 + c] + b;
                        }
                    }
                    out[c] = val;
                }
                if (p.y_vec4_ok && ob + 3 < p.N) {
                    __half2 lo = __floats2half2_rn(out[0], out[1]);
                    __half2 hi = __floats2half2_rn(out[2], out[3]);
                    u32x2 packed = {*reinterpret_cast<uint32_t *>(&lo), *reinterpret_cast<uint32_t *>(&hi)};
                    __builtin_nontemporal_store(packed, reinterpret_cast<u32x2 *>(yrow + ob));
                } else {
#pragma unroll
                    for (int c = 0; c < 4; c++)
                        if (ob + c < p.N) yrow[ob + c] = __float2half_rn(out[c]);
                }
            }
        }
    }
}

template <class Path, int BR, int BO, int WR, int WO>
int launch_tiles(LinearArgs a, int load_align, hipStream_t stream) {
    const int64_t tiles_r = ptq4vm::ceil_div(a.M, BR), tiles_o = ptq4vm::ceil_div(a.N, BO);
    if (tiles_r * tiles_o > 0x3fffffffLL) return PTQ4VM_ERR_SHAPE;
    a.tiles_r = (int)tiles_r;
    a.tiles_o = (int)tiles_o;
    const int64_t total = tiles_r * tiles_o;
    dim3 grid((unsigned)(ptq4vm::ceil_div(total, kXcds) * kXcds)), block(kThreads);
    if (load_align == 16)
        linear_mfma<Path, BR, BO, WR, WO, 16><<<grid, block, 0, stream>>>(a);
    else if (load_align == 4)
        linear_mfma<Path, BR, BO, WR, WO, 4><<<grid, block, 0, stream>>>(a);
    else
        linear_mfma<Path, BR, BO, WR, WO, 0><<<grid, block, 0, stream>>>(a);
    return ptq4vm::check_launch("linear_mfma");
}

// Widest load granularity that base pointers and pitches allow for both operands.
int pick_load_align(const LinearArgs &a) {
    auto ok = [&](uintptr_t g) {
        return ptq4vm::aligned_to(a.x, g) && ptq4vm::aligned_to(a.w, g) && a.ldx_bytes % g == 0 &&
               a.ldw_bytes % g == 0;
    };
    return ok(16) ? 16 : (ok(4) ? 4 : 0);
}

template <class Path>
int dispatch(LinearArgs a, hipStream_t stream) {
    const int la = pick_load_align(a);
    a.y_vec4_ok = (a.ldy % 4 == 0 && ptq4vm::aligned_to(a.y, 8)) ? 1 : 0;
    if (a.N > 64) return launch_tiles<Path, 256, 128, 2, 2>(a, la, stream);
    return launch_tiles<Path, 256, 64, 4, 1>(a, la, stream);
}

}  // namespace

extern "C" int ptq4vm_w8a8_linear(const int8_t *xq, const int8_t *wq, const float *s_tok, const float *s_w,
                                  const void *bias_f16, void *y_f16, int32_t *acc_out, int64_t B, int64_t L,
                                  int64_t K, int64_t N, int64_t ldxq, int64_t ldwq, int64_t ldy, void *stream_) {
    if (!xq || !wq || !s_tok || !s_w || !y_f16) return PTQ4VM_ERR_NULL;
    if (B < 0 || N < 0 || L <= 0 || K <= 0 || K > PTQ4VM_MAX_K) return PTQ4VM_ERR_SHAPE;
    if (B > 0 && L > INT64_MAX / B) return PTQ4VM_ERR_SHAPE;
    if (ldxq < K || ldwq < K || ldy < N) return PTQ4VM_ERR_STRIDE;
    if (!ptq4vm::aligned_to(xq, 16) || !ptq4vm::aligned_to(wq, 16) || !ptq4vm::aligned_to(y_f16, 2) ||
        !ptq4vm::aligned_to(s_tok, 4) || !ptq4vm::aligned_to(s_w, 4) || !ptq4vm::aligned_to(bias_f16, 2) ||
        !ptq4vm::aligned_to(acc_out, 4))
        return PTQ4VM_ERR_ALIGN;
    const int64_t M = B * L;
    if (M == 0 || N == 0) return PTQ4VM_OK;
    LinearArgs a{};
    a.x = reinterpret_cast<const char *>(xq);
    a.w = reinterpret_cast<const char *>(wq);
    a.s_tok = s_tok;
    a.s_w = s_w;
    a.bias = static_cast<const __half *>(bias_f16);
    a.y = static_cast<__half *>(y_f16);
    a.acc_out = acc_out;
    a.M = M;
    a.N = N;
    a.k_bytes = K;
    a.ldx_bytes = ldxq;
    a.ldw_bytes = ldwq;
    a.ldy = ldy;
    a.L = L;
    return dispatch<Int8Path>(a, static_cast<hipStream_t>(stream_));
}

extern "C" int ptq4vm_f16_linear(const void *x_f16, const void *w_f16, const void *bias_f16, void *y_f16,
                                 int64_t M, int64_t K, int64_t N, int64_t ldx, int64_t ldw, int64_t ldy,
                                 void *stream_) {
    if (!x_f16 || !w_f16 || !y_f16) return PTQ4VM_ERR_NULL;
    if (M < 0 || N < 0 || K <= 0 || K > (int64_t)1 << 40) return PTQ4VM_ERR_SHAPE;
    if (ldx < K || ldw < K || ldy < N) return PTQ4VM_ERR_STRIDE;
    if (!ptq4vm::aligned_to(x_f16, 16) || !ptq4vm::aligned_to(w_f16, 16) || !ptq4vm::aligned_to(y_f16, 2) ||
        !ptq4vm::aligned_to(bias_f16, 2))
        return PTQ4VM_ERR_ALIGN;
    if (M == 0 || N == 0) return PTQ4VM_OK;
    LinearArgs a{};
    a.x = static_cast<const char *>(x_f16);
    a.w = static_cast<const char *>(w_f16);
    a.bias = static_cast<const __half *>(bias_f16);
    a.y = static_cast<__half *>(y_f16);
    a.M = M;
    a.N = N;
    a.k_bytes = K * 2;
    a.ldx_bytes = ldx * 2;
    a.ldw_bytes = ldw * 2;
    a.ldy = ldy;
    a.L = 1;
    return dispatch<Half16Path>(a, static_cast<hipStream_t>(stream_));
}
