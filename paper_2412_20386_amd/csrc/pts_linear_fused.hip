// ptq4vm_w8a8_linear_fused: Per-Token-Static activation quantizer and W8A8 linear in ONE launch
// (App. B.1 lists "Activation smoothing", "Quantization", "INT GEMM" and "Dequantization" as four
// kernels; PTS equation of Sec. 5.1).  The int8 activation codes exist only in registers / LDS:
//   q[r,k]   = clip(rne((f32(x[r,k]) * inv_m[k]) * (1 / s_tok[r mod L])), -127, 127)
//   y[r,o]   = fp16(f32(sum_k q[r,k] wq[o,k]) * (s_tok[r mod L] * s_w[o]) + bias[o])
// i.e. bit for bit what ptq4vm_quantize_pts followed by ptq4vm_w8a8_linear produce, without the
// 1 byte written + 1 byte read per activation element in between.
//
// Fusing pays when an activation element is quantized once or a few times: a tiled GEMM quantizes
// every element once per tile column (N / tile width times), so for wide outputs the separate
// quantizer is cheaper.  Kernels:
//   pts_linear_wres     N <= 128 over many rows (x_proj): weight resident in LDS, every fp16
//                       activation read once from HBM in whole 128-byte lines, quantized once.
//   pts_linear_generic  every other shape: the register-staged tiled kernel with the quantizer in
//                       its loader (correct everywhere, re-quantizes per tile column).
#include <type_traits>

#include "mfma_linear.hpp"
#include "quant_device.hpp"

namespace {

using ptq4vm::cvt_i32_f32;
using ptq4vm::pack4;

using namespace ptq4vm::mfma;

// One PTS code (Sec. 5.1): smoothing multiply, step multiply, round half to even, clip.  Two
// separate fp32 multiplies in this order: the codes must equal the stand-alone quantizer's.
// BITS4: clip to +-7 (Sec. 2.3 with b = 4) instead of +-127.
// OFFSET: per-token zero offset z (Sec. 5.1; the quantizer of Sec. 2.3 with its code range shifted into int8):
// clip(q + z, -128, 127), formed as clip(q, -128 - z, 127 - z) + z so that a saturated q cannot overflow.
template <bool BITS4, bool OFFSET>
__device__ __forceinline__ int clip_code(int q, int z) {
    if constexpr (OFFSET) return min(max(q, -128 - z), 127 - z) + z;
    return BITS4 ? min(max(q, -7), 7) : min(max(q, -127), 127);
}

template <bool BITS4 = false, bool OFFSET = false>
__device__ __forceinline__ int quantize_one(float x, float inv_m, float inv_s, int z = 0) {
    float v = x * inv_m;
    v = v * inv_s;
    return clip_code<BITS4, OFFSET>(cvt_i32_f32(__builtin_rintf(v)), z);
}

// Four int8 bytes holding 4-bit codes -> the same codes times 16 (what the int8 MFMA is fed on the 4-bit path:
// the accumulator is then 256 times the sum, undone exactly in the channel steps).
__device__ __forceinline__ uint32_t times16(uint32_t packed_codes) { return (packed_codes << 4) & 0xF0F0F0F0u; }

// 32 packed 4-bit codes (16 bytes, even index in the low nibble) -> 32 int8 bytes, codes times 16, in index order.
__device__ __forceinline__ void expand_nibbles_in_order(const v4i &packed, v4i &first16, v4i &last16) {
    uint32_t out[8];
#pragma unroll
    for (int e = 0; e < 4; e++) {
        const uint32_t p = (uint32_t)packed[e];
        const uint32_t even = (p << 4) & 0xF0F0F0F0u, odd = p & 0xF0F0F0F0u;  // codes 0, 2, 4, 6 / 1, 3, 5, 7 of this dword, times 16
        out[2 * e] = __builtin_amdgcn_perm(odd, even, 0x05010400u);      // even.b0, odd.b0, even.b1, odd.b1
        out[2 * e + 1] = __builtin_amdgcn_perm(odd, even, 0x07030602u);  // even.b2, odd.b2, even.b3, odd.b3
    }
    first16 = v4i{(int)out[0], (int)out[1], (int)out[2], (int)out[3]};
    last16 = v4i{(int)out[4], (int)out[5], (int)out[6], (int)out[7]};
}

// f32(fp16 half of `pair`) * m in one instruction: v_fma_mix_f32 converts the selected half exactly,
// multiplies and rounds once to fp32 - the same value as a conversion followed by v_mul_f32.
template <bool HIGH>
__device__ __forceinline__ float half_times(int pair, float m) {
    float d;
    if constexpr (HIGH)
        asm("v_fma_mix_f32 %0, %1, %2, 0 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(pair), "v"(m));
    else
        asm("v_fma_mix_f32 %0, %1, %2, 0 op_sel_hi:[1,0,0]" : "=v"(d) : "v"(pair), "v"(m));
    return d;
}

template <bool BITS4, bool OFFSET>
__device__ __forceinline__ int code_of_smoothed(float v, float inv_s, int z) {
    return clip_code<BITS4, OFFSET>(cvt_i32_f32(__builtin_rintf(v * inv_s)), z);
}

// Eight fp16 values (one 16-byte load) -> eight int8 codes (BITS4: 4-bit codes times 16).
template <bool BITS4, bool OFFSET>
__device__ __forceinline__ u32x2 quantize_8(v4i raw, const float (&im)[8], float inv_s, int z) {
    int q[8];
#pragma unroll
    for (int e = 0; e < 4; e++) {
        const int word = raw[e];  // (a bit_cast applied directly to a vector element reads element 0 with this compiler)
        q[2 * e] = code_of_smoothed<BITS4, OFFSET>(half_times<false>(word, im[2 * e]), inv_s, z);
        q[2 * e + 1] = code_of_smoothed<BITS4, OFFSET>(half_times<true>(word, im[2 * e + 1]), inv_s, z);
    }
    u32x2 out = {pack4(q[0], q[1], q[2], q[3]), pack4(q[4], q[5], q[6], q[7])};
    if constexpr (BITS4) out = u32x2{times16(out[0]), times16(out[1])};
    return out;
}

// ------------------------------------------------------------------------------------------
// Skinny-N fused kernel.  One workgroup of 16 wavefronts per CU (PTQ4VM_FUSED_RB = 1; 8 with 32-row units); LDS
// holds, for the whole kernel,
//   the int8 weight (row pitch K + 32 bytes, see fused_layout),
//   inv_m[K], 1 / s_tok[L] (the only place the IEEE division appears), s_w[N] and the bias as fp32.
// A wavefront owns units of 16 RB token rows.  Per k-step (64 codes = one 128-byte line of fp16 per
// row) it fetches the unit's lines with 2 RB loads (lane s: row 8 i + s / 8, 16-byte piece s mod 8,
// so every request is a whole cache line), D k-steps ahead (D = 4, 2 or 1); at consumption the eight fp16 of a
// lane become eight codes, go through a wavefront-private (16 RB) x 64-byte LDS tile (chunks XOR-swizzled
// by the row) and come back as RB MFMA operands (lane t: row t mod 16, 16 codes t / 16), which
// meet the weight fragments of all ceil(N / 16) channel blocks in v_mfma_i32_16x16x64_i8.
// There is no barrier after the set-up.  The epilogue is the dequantization of the PTS equation,
// staged through the same private LDS region and written as whole contiguous row segments.
// Requirements (host-checked): K % 64 == 0, 16-byte aligned fp16 rows and weight rows, N <= 128,
// M, L < 2^31, all tables fit the LDS.
// ------------------------------------------------------------------------------------------
#ifndef PTQ4VM_FUSED_RB
#define PTQ4VM_FUSED_RB 1
#endif
constexpr int kFusedRB = PTQ4VM_FUSED_RB;       // 16-row MFMA blocks per unit (2: 32-row units on 8 wavefronts, 1: 16-row units on 16)
constexpr int kFusedWaves = 16 / kFusedRB;
constexpr int kFusedPatchRows = 8 * kFusedRB;   // result rows staged per pass of the epilogue
constexpr int kFusedMaxBlocks = 8;   // 16-channel blocks: N <= 128
constexpr int kLdsBytes = 160 * 1024;
constexpr int64_t kFusedMinRows = 2048;   // below this the one-off table copies per workgroup do not pay (4 k rows: 11 us against 48 us for the tiled fused kernel at 384 -> 44)

struct FusedLayout {
    int nb, n4, pw, w_bytes, inv_m_off, inv_s_off, z_off, scale_off, tile_off, tile_bytes, total;
};
// offset: room for the per-token zero offsets [L] and the weight row sums (zero-offset form)
__host__ __device__ __forceinline__ FusedLayout fused_layout(int N, int K, int L, bool offset = false) {
    FusedLayout l;
    l.nb = (N + 15) >> 4;
    l.n4 = (N + 3) & ~3;
    l.pw = K + 32;  // in 16-byte chunks 2 mod 4: operand reads of 16 rows run at 235-240 bytes per clock and CU (K + 16: 120)
    l.w_bytes = (l.nb * 16 * l.pw + 1023) & ~1023;  // whole 1 KiB wavefront copies
    l.inv_m_off = l.w_bytes;
    l.inv_s_off = l.inv_m_off + K * 4;
    l.z_off = l.inv_s_off + ((L * 4 + 15) & ~15);
    l.scale_off = l.z_off + (offset ? ((L * 4 + 15) & ~15) : 0);
    l.tile_off = l.scale_off + l.nb * 16 * 4 * (offset ? 3 : 2);
    const int patch = kFusedPatchRows * l.n4 * 2;    // one pass of fp16 results
    const int codes = 1024 * kFusedRB;               // or the (16 RB) x 64-byte tile of codes
    l.tile_bytes = patch > codes ? patch : codes;
    l.total = l.tile_off + kFusedWaves * l.tile_bytes;
    return l;
}

// DUMP: also write the int8 codes (xq_out) and the int32 accumulators (acc_out), the parity aids; without it
// their address arithmetic (a third of the VALU instructions of the k loop) is not even compiled in.
// BITS4: the weight arrives as packed 4-bit codes ([N, K / 2] bytes) and is expanded once into LDS (codes times 16, in
// index order); activations are clipped to +-7 and also fed times 16; the factor 256 is undone in the channel steps.
// OFFSET: the zero-offset form (8 bits): codes carry z_tok[t], the epilogue takes z_tok[t] * rowsum[o] off the accumulator.
template <int NB, int D, bool DUMP, bool BITS4 = false, bool OFFSET = false>
__global__ __launch_bounds__(kFusedWaves * 64) void pts_linear_wres(const LinearArgs p) {
    static_assert(!(BITS4 && OFFSET), "the zero-offset form is 8-bit");
    using Acc = v4i;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: unit numbers and row bounds stay in SGPRs
    const int l16 = lane & 15, lq = lane >> 4;  // MFMA operand position: row, 16-code chunk
    const int rr = lane >> 3, pc = lane & 7;    // load position: row within a group of 8, 16-byte piece
    const int N = (int)p.N, K = (int)p.k_bytes, L = (int)p.L, n_ksteps = K >> 6;
    const FusedLayout lay = fused_layout(N, K, L, OFFSET);
    const int n4 = lay.n4, pw = lay.pw;
    char *const w_lds = lds_dyn;
    float *const inv_m_lds = reinterpret_cast<float *>(lds_dyn + lay.inv_m_off);
    float *const inv_s_lds = reinterpret_cast<float *>(lds_dyn + lay.inv_s_off);
    float *const cs_lds = reinterpret_cast<float *>(lds_dyn + lay.scale_off);
    float *const cb_lds = cs_lds + NB * 16;
    int *const z_lds = reinterpret_cast<int *>(lds_dyn + lay.z_off);   // zero-offset form only
    int *const cz_lds = reinterpret_cast<int *>(cb_lds + NB * 16);     // weight row sums (zero-offset form only)
    char *const tile = lds_dyn + lay.tile_off + wave * lay.tile_bytes;  // codes in the K loop, results after it

    // Work items.  A wavefront handles units of up to UNIT rows, one per pass over the matrix; in a pass the
    // units are dealt wavefront-major, so that a launch with fewer units than wavefronts still spreads them
    // over all workgroups.  The kernel is bound by the VALU work of the quantizer, which is proportional to the
    // rows a SIMD's wavefronts load, and with about one unit per wavefront (M = 50 432: 3152 units of 16 rows on
    // 4096 wavefronts) whole units cannot be dealt evenly: some SIMDs would get four and most three.  So the
    // last, partial pass is dealt in groups of 8 rows (the rows of one load instruction): every workgroup gets
    // a contiguous share of the groups and hands them to its wavefronts two at a time (16 rows) until the rest
    // is one group per wavefront; wavefront w sits on SIMD w mod 4, so the SIMDs' row counts differ by at most 8.
    constexpr int RB = kFusedRB, UNIT = 16 * RB, NL = 2 * RB, PR = kFusedPatchRows;  // NL loads of 8 rows per k-step
    const int64_t wavefronts = (int64_t)gridDim.x * kFusedWaves;
    const int64_t full_passes = p.M / (wavefronts * UNIT);
    const int64_t tail_row0 = full_passes * wavefronts * UNIT;
    const int64_t tail_groups = (p.M - tail_row0 + 7) / 8;  // fewer than NL groups per wavefront on average
    auto item = [&](int64_t k, int64_t &r0, int &nrows) -> bool {  // k-th item of this wavefront: rows r0 .. r0 + nrows - 1
#ifdef PTQ4VM_FUSED_NO_BALANCE  // timing experiment: whole units only, dealt wavefront-major
        const int64_t first_row = ((k * wavefronts) + (int64_t)wave * gridDim.x + blockIdx.x) * UNIT;
        if (first_row >= p.M) return false;
        r0 = first_row;
        nrows = UNIT;
        return true;
#endif
        if (k < full_passes) {
            r0 = ((k * wavefronts) + (int64_t)wave * gridDim.x + blockIdx.x) * UNIT;
            nrows = UNIT;
            return true;
        }
        if (k > full_passes || tail_groups == 0) return false;
        const int64_t per_wg = tail_groups / gridDim.x, extra = tail_groups % gridDim.x;
        const int64_t g0 = blockIdx.x * per_wg + min((int64_t)blockIdx.x, extra);
        const int n = (int)(per_wg + (blockIdx.x < extra ? 1 : 0));  // this workgroup's groups: at most NL per wavefront
        // the first `big` wavefronts take NL groups, the others NL / 2 (or what is left), so that every group is taken once
        constexpr int small_size = NL / 2, big_size = NL;
        const int big = max(0, min(kFusedWaves, (n - small_size * kFusedWaves + (big_size - small_size) - 1) / (big_size - small_size)));
        int first, count;
        if (wave < big) {
            first = wave * big_size, count = big_size;
        } else {
            first = big * big_size + (wave - big) * small_size, count = small_size;
        }
        count = min(count, n - first);
        if (count <= 0) return false;
        r0 = tail_row0 + (g0 + first) * 8;
        nrows = count * 8;
        return true;
    };
    int64_t item_k = 0, unit_r0 = 0, next_r0 = 0;
    int unit_rows = 0, next_rows = 0;
    bool have = item(0, unit_r0, unit_rows);

    v4i raw[D][NL];
    const char *xrow[NL];
    uint32_t tok[NL];
    // 8-row groups (load instructions per k-step) of the unit being loaded: all NL, or half of them for a short
    // unit, whose further groups are neither loaded nor quantized.  The k loop is compiled once for either count
    // (branches inside it would cost the counted waits on the loads).
    int groups = 0;
    auto load_x = [&](int d, int ks) {  // outside the k loop only
#pragma unroll
        for (int i = 0; i < NL; i++)
            if (i < groups) raw[d][i] = __builtin_nontemporal_load(reinterpret_cast<const v4i *>(xrow[i] + ks * 128));
    };
    auto start_unit = [&](int64_t r0, int nrows) {  // first D k-steps of the unit's rows
        groups = nrows > 8 * (NL / 2) ? NL : NL / 2;
#pragma unroll
        for (int i = 0; i < NL; i++) {
            const int64_t r = min(r0 + i * 8 + rr, p.M - 1);  // clamped rows are never stored
            xrow[i] = p.x + r * p.ldx_bytes + pc * 16;
            tok[i] = (uint32_t)r % (uint32_t)L;
        }
#pragma unroll
        for (int d = 0; d < D; d++) load_x(d, d);
    };
    if (have) start_unit(unit_r0, unit_rows);

    // Tables, once per workgroup.  The weight goes global -> LDS in 1 KiB copies, linear on the LDS
    // side; the lane picks the global chunk that belongs at its LDS position (pad chunks and pad
    // rows re-read a valid neighbour).
    {
        if constexpr (BITS4) {
            const int packed_chunks = K >> 5;  // 16-byte chunks of 32 packed codes per weight row (K is a multiple of 64)
            for (int idx = tid; idx < NB * 16 * packed_chunks; idx += kFusedWaves * 64) {
                const int row = idx / packed_chunks, c = idx - row * packed_chunks;
                const v4i packed = *reinterpret_cast<const v4i *>(p.w + (int64_t)min(row, N - 1) * p.ldw_bytes + c * 16);  // pad rows re-read a valid one
                v4i first16, last16;
                expand_nibbles_in_order(packed, first16, last16);
                *reinterpret_cast<v4i *>(w_lds + row * pw + c * 32) = first16;
                *reinterpret_cast<v4i *>(w_lds + row * pw + c * 32 + 16) = last16;
            }
        } else {
        const int chunks_per_row = pw >> 4;
        for (int c = wave; c < (lay.w_bytes >> 10); c += kFusedWaves) {
            const int chunk = c * 64 + lane;
            const int row = chunk / chunks_per_row, cc = chunk - row * chunks_per_row;
            const char *src = p.w + (int64_t)min(row, N - 1) * p.ldw_bytes + min(cc, chunks_per_row - 3) * 16;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                             (__attribute__((address_space(3))) void *)(w_lds + c * 1024), 16, 0, 0);
        }
        }
        for (int k = tid; k < K; k += kFusedWaves * 64) inv_m_lds[k] = p.inv_m ? p.inv_m[k] : 1.0f;
        for (int t = tid; t < L; t += kFusedWaves * 64) inv_s_lds[t] = 1.0f / p.s_tok[t];  // IEEE division
        for (int o = tid; o < NB * 16; o += kFusedWaves * 64) {
            // 4-bit path: operands are codes times 16, the accumulator 256 times the sum; undone here (a power of two: exact)
            cs_lds[o] = o < N ? (BITS4 ? p.s_w[o] * (1.0f / 256.0f) : p.s_w[o]) : 0.0f;
            cb_lds[o] = (o < N && p.bias) ? __half2float(p.bias[o]) : 0.0f;
            if constexpr (OFFSET) cz_lds[o] = o < N ? p.rowsum[o] : 0;
        }
        if constexpr (OFFSET) {
            for (int t = tid; t < L; t += kFusedWaves * 64) z_lds[t] = p.z_tok[t];
        }
    }
    __builtin_amdgcn_s_waitcnt(0);  // vmcnt(0) expcnt(0) lgkmcnt(0): this wavefront's copies have landed
    __syncthreads();

    const bool dense_y = n4 == N && p.ldy == p.N && (reinterpret_cast<uintptr_t>(p.y) & 15) == 0;
    const int chunks8_per_row = n4 >> 2;  // 8-byte groups of four channels per result row
    const char *const w_lane = w_lds + l16 * pw + lq * 16;
    // Code tile: row pitch 64 bytes, 16-byte chunk c of row r stored at chunk position c ^ (((r >> 1) ^ (r >> 2)) & 3)
    // (operand reads at 236 bytes per clock and CU in a read loop; with (r >> 2) & 3: 120).
    uint32_t tile_wr[NL];
#pragma unroll
    for (int i = 0; i < NL; i++) {
        const int row = i * 8 + rr;
        tile_wr[i] = row * 64 + (((pc >> 1) ^ (((row >> 1) ^ (row >> 2)) & 3)) << 4) + (pc & 1) * 8;
    }
    const uint32_t tile_rd = l16 * 64 + ((lq ^ (((l16 >> 1) ^ (l16 >> 2)) & 3)) << 4);  // + 1024 for rows 16..31

    bool next_have = false;
    for (; have; have = next_have, unit_r0 = next_r0, unit_rows = next_rows) {
        Acc acc[RB][NB];
#pragma unroll
        for (int j = 0; j < RB; j++)
#pragma unroll
            for (int i = 0; i < NB; i++)
#pragma unroll
                for (int v = 0; v < 4; v++) acc[j][i][v] = 0;
        float inv_s[NL];
#pragma unroll
        for (int i = 0; i < NL; i++) inv_s[i] = inv_s_lds[tok[i]];
        int zq[NL];  // zero offsets of the rows this lane quantizes
#pragma unroll
        for (int i = 0; i < NL; i++) zq[i] = OFFSET ? z_lds[tok[i]] : 0;
        const int64_t r_unit = unit_r0;
        const int64_t r_end = min(p.M, unit_r0 + unit_rows);  // rows at or beyond it are not this unit's
        const int unit_groups = groups;                        // (`groups` moves on to the next unit before the epilogue)

        auto k_loop = [&](auto g_tag) {
            constexpr int G = decltype(g_tag)::value;
            auto load_g = [&](int d, int ks) {
#pragma unroll
                for (int i = 0; i < G; i++)
                    raw[d][i] = __builtin_nontemporal_load(reinterpret_cast<const v4i *>(xrow[i] + ks * 128));
            };
            auto compute = [&](int d, int ks) {
                float im[8];
                const v4f im_lo = *reinterpret_cast<const v4f *>(inv_m_lds + ks * 64 + pc * 8);
                const v4f im_hi = *reinterpret_cast<const v4f *>(inv_m_lds + ks * 64 + pc * 8 + 4);
#pragma unroll
                for (int e = 0; e < 4; e++) im[e] = im_lo[e], im[4 + e] = im_hi[e];
#pragma unroll
                for (int i = 0; i < G; i++) {  // tile rows of further groups keep stale codes: results of rows nobody stores
                    const u32x2 codes = quantize_8<BITS4, OFFSET>(raw[d][i], im, inv_s[i], zq[i]);
                    *reinterpret_cast<u32x2 *>(tile + tile_wr[i]) = codes;
                    if (DUMP && p.xq_out) {  // parity aid: the codes that the MFMA will see (4-bit path: divided by 16 again)
                        const int64_t r = r_unit + i * 8 + rr;
                        u32x2 plain = codes;
                        if constexpr (BITS4) {
#pragma unroll
                            for (int h = 0; h < 2; h++) {
                                uint32_t w = 0;
#pragma unroll
                                for (int b = 0; b < 4; b++) w |= (uint32_t)(uint8_t)((int8_t)(codes[h] >> (8 * b)) >> 4) << (8 * b);
                                plain[h] = w;
                            }
                        }
                        if (r < p.M) *reinterpret_cast<u32x2 *>(p.xq_out + r * p.ldxq_out + ks * 64 + pc * 8) = plain;
                    }
                    __builtin_amdgcn_sched_barrier(0);  // one load's eight codes at a time: bounds the live registers
                }
                v4i fw[NB], fb[RB];
#pragma unroll
                for (int j = 0; j < RB; j++) fb[j] = *reinterpret_cast<const v4i *>(tile + tile_rd + j * 1024);
#pragma unroll
                for (int i = 0; i < NB; i++) fw[i] = *reinterpret_cast<const v4i *>(w_lane + i * 16 * pw + ks * 64);
                __builtin_amdgcn_sched_barrier(0);  // all LDS traffic of the k-step in flight before its first MFMA
#pragma unroll
                for (int i = 0; i < NB; i++) {
#pragma unroll
                    for (int j = 0; j < RB; j++) acc[j][i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fw[i], fb[j], acc[j][i], 0, 0, 0);
                }
            };
            // The scheduling barriers keep each refill right behind the work that frees its registers;
            // left alone the scheduler sinks all loads of a group to its end and the wavefront then
            // waits for the whole group before every pass.
            int ks0 = 0;
            for (; ks0 + D < n_ksteps; ks0 += D) {  // every register slot is refilled (K is a multiple of 64 D)
#pragma unroll
                for (int d = 0; d < D; d++) {
                    compute(d, ks0 + d);
                    load_g(d, ks0 + d + D);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
#pragma unroll
            for (int d = 0; d < D; d++) {  // last group: drain
                compute(d, ks0 + d);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        if (unit_groups == NL)
            k_loop(std::integral_constant<int, NL>{});
        else
            k_loop(std::integral_constant<int, NL / 2>{});

        // Accumulator register v of block (j, i): token row 16 j + (lane mod 16), channel 16 i + 4 (lane / 16) + v.
        float rs[RB];
#pragma unroll
        for (int j = 0; j < RB; j++) rs[j] = p.s_tok[(uint32_t)min(r_unit + j * 16 + l16, p.M - 1) % (uint32_t)L];
        int rz[RB];  // zero offset of the lane's result row
#pragma unroll
        for (int j = 0; j < RB; j++) rz[j] = OFFSET ? z_lds[(uint32_t)min(r_unit + j * 16 + l16, p.M - 1) % (uint32_t)L] : 0;
        item_k++;
        next_have = item(item_k, next_r0, next_rows);
        if (next_have) start_unit(next_r0, next_rows);  // in flight while this unit's results are written

#pragma unroll
        for (int pass = 0; pass < UNIT / PR; pass++) {  // PR result rows at a time through the private region
            const int j = pass * PR / 16, row_in_block = (pass * PR) % 16;  // rows row_in_block .. + PR - 1 of block j
            const int64_t r0 = r_unit + pass * PR;
            const int rows_valid = (int)min((int64_t)PR, r_end - r0);
            if (rows_valid <= 0) break;
            const int prow = l16 - row_in_block;         // this lane's row inside the pass
            const bool mine = prow >= 0 && prow < PR;
#pragma unroll
            for (int i = 0; i < NB; i++) {
                const int col = i * 16 + lq * 4;
                if (col < n4 && mine) {
                    const v4f cs = *reinterpret_cast<const v4f *>(cs_lds + col);
                    const v4f cb = *reinterpret_cast<const v4f *>(cb_lds + col);
                    v4i cz = {0, 0, 0, 0};
                    if constexpr (OFFSET) cz = *reinterpret_cast<const v4i *>(cz_lds + col);
                    float out[4];
#pragma unroll
                    for (int c = 0; c < 4; c++) {
                        int a = acc[j][i][c];
                        if (DUMP && p.acc_out && prow < rows_valid && col + c < N) p.acc_out[(r0 + prow) * p.N + col + c] = BITS4 ? a >> 8 : a;
                        if constexpr (OFFSET) a -= __mul24(rz[j], cz[c]);  // |z| < 2^8, |rowsum| < 2^23
                        out[c] = (float)a * (rs[j] * cs[c]) + cb[c];
                    }
                    __half2 lo = __floats2half2_rn(out[0], out[1]);
                    __half2 hi = __floats2half2_rn(out[2], out[3]);
                    u32x2 packed = {__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi)};
                    *reinterpret_cast<u32x2 *>(tile + prow * (n4 * 2) + col * 2) = packed;
                }
            }
            asm volatile("" ::: "memory");  // wavefront-private region: LDS runs a wavefront's accesses in order
            if (dense_y) {
                const int valid_bytes = rows_valid * N * 2, block_bytes = PR * 2 * N;
                char *dst = reinterpret_cast<char *>(p.y + r0 * p.N);
                for (int off = lane * 16; off < block_bytes; off += 64 * 16) {
                    const v4i data = *reinterpret_cast<const v4i *>(tile + off);
                    if (off + 16 <= valid_bytes) {
                        __builtin_nontemporal_store(data, reinterpret_cast<v4i *>(dst + off));
                    } else {
#pragma unroll
                        for (int e = 0; e < 8; e++)
                            if (off + 2 * e < valid_bytes)
                                reinterpret_cast<uint16_t *>(dst + off)[e] = (uint16_t)((uint32_t)data[e >> 1] >> (16 * (e & 1)));
                    }
                }
            } else {
                for (int idx = lane; idx < PR * chunks8_per_row; idx += 64) {
                    const int row = idx / chunks8_per_row, cc = idx - row * chunks8_per_row;
                    if (row >= rows_valid) continue;
                    const u32x2 data = *reinterpret_cast<const u32x2 *>(tile + row * (n4 * 2) + cc * 8);
                    __half *dst = p.y + (r0 + row) * p.ldy + cc * 4;
                    if (p.y_vec >= 4 && cc * 4 + 4 <= N) {
                        *reinterpret_cast<u32x2 *>(dst) = data;
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; e++)
                            if (cc * 4 + e < N)
                                reinterpret_cast<uint16_t *>(dst)[e] = (uint16_t)(data[e >> 1] >> (16 * (e & 1)));
                    }
                }
            }
            asm volatile("" ::: "memory");
        }
        // Stores and loads share the vmcnt counter and complete out of order with each other, so with
        // stores possibly outstanding every wait on a fetched line would have to be a full drain.
        // Drain once here instead: the next unit's first lines were fetched during the epilogue.
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    }
}

// Sixteen codes of row `row_ptr` (fp16) starting at code index k0; codes at or beyond K are 0.
// im[j] is the smoothing factor of code k0 + j (any value for codes at or beyond K).
template <int X_ALIGN, bool BITS4 = false, bool OFFSET = false>
__device__ __forceinline__ v4i load_quantized_chunk(const char *row_ptr, int64_t k0, int64_t K, bool row_ok,
                                                    const float (&im)[16], float inv_s, int z = 0) {
    v4i out = {0, 0, 0, 0};
    if (!row_ok || k0 >= K) return out;
    const int valid = (int)min((int64_t)16, K - k0);
    uint32_t h2[8];  // 16 fp16 values, two per word
#pragma unroll
    for (int j = 0; j < 8; j++) h2[j] = 0;
    const char *src = row_ptr + k0 * 2;
    if constexpr (X_ALIGN == 16) {
#pragma unroll
        for (int j = 0; j < 2; j++)
            if (8 * j < valid) {
                const v4i v = *reinterpret_cast<const v4i *>(src + 16 * j);
#pragma unroll
                for (int e = 0; e < 4; e++) h2[4 * j + e] = (uint32_t)v[e];
            }
    } else if constexpr (X_ALIGN == 4) {
#pragma unroll
        for (int j = 0; j < 8; j++)
            if (2 * j < valid) h2[j] = *reinterpret_cast<const uint32_t *>(src + 4 * j);
    } else {
#pragma unroll
        for (int j = 0; j < 16; j++)
            if (j < valid) h2[j >> 1] |= (uint32_t) * reinterpret_cast<const uint16_t *>(src + 2 * j) << (16 * (j & 1));
    }
    int q[16];
#pragma unroll
    for (int j = 0; j < 16; j++) {
        const __half h = __builtin_bit_cast(__half, (uint16_t)(h2[j >> 1] >> (16 * (j & 1))));
        q[j] = j < valid ? quantize_one<BITS4, OFFSET>(__half2float(h), im[j], inv_s, z) : 0;
    }
#pragma unroll
    for (int j = 0; j < 4; j++) {
        const uint32_t packed = pack4(q[4 * j], q[4 * j + 1], q[4 * j + 2], q[4 * j + 3]);
        out[j] = (int)(BITS4 ? times16(packed) : packed);  // 4-bit path: codes times 16
    }
    return out;
}

// ------------------------------------------------------------------------------------------
// Short-reduction kernel (K <= 128, e.g. dt_proj 48 -> 1536): almost all traffic is the fp16
// output, so the kernel is arranged around the stores.  One workgroup of 16 wavefronts per CU; LDS
// holds the whole int8 weight (64 or 128 bytes per channel, 16-byte chunks XOR-swizzled by the row),
// s_w and the bias as fp32.  A wavefront owns units of 16 token rows and ALL output channels of
// them: it reads (and, fused, quantizes) the unit's activations once into two MFMA operands, then
// walks over the channels 64 at a time - weight fragments and scales from LDS, v_mfma_i32_16x16x64_i8,
// dequantization, transposition through a private 4 KiB LDS patch, 16-byte non-temporal stores of
// whole 128-byte lines.  A unit's output is one contiguous 16-row span of y written by at most four
// wavefronts (the channel groups of a unit are dealt in up to four parts) within a few microseconds.  No barrier
// after the set-up.
// QUANT: activations are fp16 and pass through the PTS quantizer; otherwise they are int8 codes.
// Any pitch and alignment (X_ALIGN / W_ALIGN: 16, 4 or 0 = element-wise loads).
// ------------------------------------------------------------------------------------------
#ifndef PTQ4VM_STREAM_RB
#define PTQ4VM_STREAM_RB 1
#endif
#ifndef PTQ4VM_STREAM_SKIP
#define PTQ4VM_STREAM_SKIP 0
#endif
constexpr int kStreamRB = PTQ4VM_STREAM_RB;       // 16-row MFMA blocks per unit
constexpr int kStreamWaves = 16 / kStreamRB;      // wavefronts per workgroup
constexpr int kStreamPatch = 2048 * kStreamRB;    // bytes of the per-wavefront transposition patch
// A unit (16 rows x all channels) is one serial chain per wavefront and costs ~1 us per 64 channels however
// few rows there are; the channel-strip kernel is faster below ~20 k rows (N = 384 ... 1536).  The fused form
// has only the tiled fused kernel as an alternative and takes over much earlier.
constexpr int64_t kStreamMinRows = 20480, kStreamMinRowsFused = 1024;

struct StreamLayout {
    int groups, rows, pitch, w_bytes, scale_off, inv_m_off, patch_off, total;
};
__host__ __device__ __forceinline__ StreamLayout stream_layout(int N, int ksteps) {
    StreamLayout l;
    l.groups = (N + 63) >> 6;      // 64-channel groups
    l.rows = l.groups * 64;        // weight rows in LDS, zero beyond N
    l.pitch = 64 * ksteps;
    l.w_bytes = l.rows * l.pitch;
    l.scale_off = l.w_bytes;
    l.inv_m_off = l.scale_off + l.rows * 12;         // steps, biases, weight row sums; then 64 ksteps smoothing factors (fused form)
    l.patch_off = l.inv_m_off + 64 * ksteps * 4;
    l.total = l.patch_off + kStreamWaves * kStreamPatch;
    return l;
}

template <int KSTEPS, bool QUANT, int X_ALIGN, int W_ALIGN, bool PACKED4 = false, bool OFFSET = false>
__global__ __launch_bounds__(kStreamWaves * 64) void linear_stream_smallk(const LinearArgs p) {
    // QUANT && PACKED4: the fused 4-bit form - fp16 activations clipped to +-7, packed 4-bit weight; both fed times 16
    static_assert(!(OFFSET && PACKED4), "the zero-offset form is 8-bit");
    constexpr bool BITS4 = QUANT && PACKED4;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: unit numbers and row bounds stay in SGPRs
    const int l16 = lane & 15, lq = lane >> 4;
    const int N = (int)p.N, K = (int)p.k_bytes;
    const StreamLayout lay = stream_layout(N, KSTEPS);
    char *const w_lds = lds_dyn;
    float *const cs_lds = reinterpret_cast<float *>(lds_dyn + lay.scale_off);
    float *const cb_lds = cs_lds + lay.rows;
    int *const cz_lds = reinterpret_cast<int *>(cb_lds + lay.rows);  // weight row sums (zero-offset form)
    float *const inv_m_lds = reinterpret_cast<float *>(lds_dyn + lay.inv_m_off);
    char *const patch = lds_dyn + lay.patch_off + wave * kStreamPatch;
    constexpr int RB = kStreamRB, UNIT = 16 * RB;
    // 64-byte rows: measured in a read loop, ((row >> 1) ^ (row >> 2)) & 3 reads 16-byte operands at 236 bytes per clock
    // and CU, (row >> 2) & 3 at 120
    auto swz = [](int row) { return KSTEPS == 1 ? (((row >> 1) ^ (row >> 2)) & 3) : ((row >> 1) & 3); };

    // Set-up: weight (zero beyond N and K), scales, bias.
    {
        constexpr int CPR = 4 * KSTEPS;  // 16-byte chunks per weight row in LDS
        if constexpr (PACKED4) {
            // a packed chunk (32 codes) becomes two int8 chunks, codes times 16: even reduction indices, then odd ones
            // (two-launch form: the activations are split the same way) or in index order (fused form)
            const int packed_bytes = BITS4 ? K / 2 : K;
            for (int idx = tid; idx < lay.rows * (CPR / 2); idx += kStreamWaves * 64) {
                const int row = idx / (CPR / 2), c = idx - row * (CPR / 2);
                const v4i v = load_chunk<W_ALIGN, 1>(p.w + (int64_t)min(row, N - 1) * p.ldw_bytes, c * 16, packed_bytes, row < N);
                v4i first, second;
                if constexpr (BITS4) expand_nibbles_in_order(v, first, second);
                else first = Int4Path::even_codes(v), second = Int4Path::odd_codes(v);
                *reinterpret_cast<v4i *>(w_lds + row * lay.pitch + (((2 * c) ^ swz(row)) << 4)) = first;
                *reinterpret_cast<v4i *>(w_lds + row * lay.pitch + (((2 * c + 1) ^ swz(row)) << 4)) = second;
            }
        } else
        for (int idx = tid; idx < lay.rows * CPR; idx += kStreamWaves * 64) {
            const int row = idx / CPR, c = idx - row * CPR;
            const v4i v = load_chunk<W_ALIGN, 1>(p.w + (int64_t)min(row, N - 1) * p.ldw_bytes, c * 16, K, row < N);
            *reinterpret_cast<v4i *>(w_lds + row * lay.pitch + ((c ^ swz(row)) << 4)) = v;
        }
        for (int o = tid; o < lay.rows; o += kStreamWaves * 64) {
            // packed operands are codes times 16: the accumulator is 256 times the sum, undone here (a power of two: exact)
            cs_lds[o] = o < N ? (PACKED4 ? p.s_w[o] * (1.0f / 256.0f) : p.s_w[o]) : 0.0f;
            cb_lds[o] = (o < N && p.bias) ? __half2float(p.bias[o]) : 0.0f;
            if constexpr (OFFSET) cz_lds[o] = o < N ? p.rowsum[o] : 0;
        }
        if constexpr (QUANT) {
            for (int k = tid; k < 64 * KSTEPS; k += kStreamWaves * 64) inv_m_lds[k] = (p.inv_m && k < K) ? p.inv_m[k] : 1.0f;
        }
    }
    __syncthreads();

    // Work items: a unit (UNIT rows) times a part of the channel groups.  The time of a SIMD is the sum of its
    // wavefronts' items (dequantization VALU work and store issue), and whole units do not divide evenly: at
    // M = 50 432 there are 3152 of them for 4096 wavefronts, so some SIMDs would carry four units and most three.
    // In quarters a SIMD carries 12 or 13 items.  The parts of a unit go to neighbouring workgroups at the same
    // time (they read the same rows).
    const int64_t units = (p.M + UNIT - 1) / UNIT;
    const int parts = min(4, lay.groups), groups_per_part = (lay.groups + parts - 1) / parts;
    const int64_t items = units * parts;
    const int64_t item_step = (int64_t)gridDim.x * kStreamWaves;
    const bool y_wide = p.y_vec == 8;
    auto patch_chunk = [&](int row, int chunk) { return row * 128 + ((chunk ^ (row & 7)) << 4); };

    for (int64_t it = (int64_t)wave * gridDim.x + blockIdx.x; it < items; it += item_step) {
        const int64_t unit = it / parts;
        const int part = (int)(it - unit * parts);
        const int g_begin = part * groups_per_part, g_end = min(lay.groups, g_begin + groups_per_part);
        const int64_t r_unit = unit * UNIT;
        // ---- the unit's two activation operands (lane: row 16 jb + lane mod 16, codes 64 ks + 16 (lane / 16) ..)
        v4i fx[RB][KSTEPS];
        float rs[RB];
        int rz[RB];  // per-token zero offset of the lane's row (zero-offset form)
#pragma unroll
        for (int jb = 0; jb < RB; jb++) {
            const int64_t r = min(r_unit + jb * 16 + l16, p.M - 1);  // clamped rows are never stored
            const float step = p.s_tok[(uint32_t)r % (uint32_t)p.L];
            rs[jb] = step;
            rz[jb] = 0;
            if constexpr (OFFSET) rz[jb] = p.z_tok[(uint32_t)r % (uint32_t)p.L];
            const char *xrow = p.x + r * p.ldx_bytes;
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ks++) {
                const int k0 = 64 * ks + 16 * lq;
                if constexpr (QUANT) {
                    const float inv_s = 1.0f / step;  // IEEE division
                    float im[16];
#pragma unroll
                    for (int e = 0; e < 4; e++) {
                        const v4f f = *reinterpret_cast<const v4f *>(inv_m_lds + k0 + 4 * e);
                        im[4 * e] = f.x, im[4 * e + 1] = f.y, im[4 * e + 2] = f.z, im[4 * e + 3] = f.w;
                    }
                    const v4i codes = load_quantized_chunk<X_ALIGN, BITS4, OFFSET>(xrow, k0, K, true, im, inv_s, rz[jb]);
                    if (p.xq_out && part == 0 && r_unit + jb * 16 + l16 < p.M) {  // parity aid (4-bit form: the codes, not times 16)
#pragma unroll
                        for (int b = 0; b < 16; b++)
                            if (k0 + b < K) {
                                const int8_t fed = (int8_t)((uint32_t)codes[b >> 2] >> (8 * (b & 3)));
                                p.xq_out[r * p.ldxq_out + k0 + b] = BITS4 ? (int8_t)(fed >> 4) : fed;
                            }
                    }
                    fx[jb][ks] = codes;
                } else if constexpr (PACKED4) {
                    // int8 chunk 4 ks + lq comes from packed chunk (4 ks + lq) / 2: its even codes, or its odd ones
                    const v4i packed = load_chunk<X_ALIGN, 1>(xrow, ((4 * ks + lq) >> 1) * 16, K, true);
                    fx[jb][ks] = (lq & 1) ? Int4Path::odd_codes(packed) : Int4Path::even_codes(packed);
                } else {
                    fx[jb][ks] = load_chunk<X_ALIGN, 1>(xrow, k0, K, true);
                }
            }
        }

        // ---- the part's output channels, 64 at a time
        for (int g = g_begin; g < g_end; g++) {
            v4i acc[RB][4];
            v4f cs[4], cb[4];
            v4i cz[4];
#pragma unroll
            for (int i = 0; i < 4; i++) {
                if constexpr (OFFSET) cz[i] = *reinterpret_cast<const v4i *>(cz_lds + g * 64 + i * 16 + lq * 4);
                const int row = g * 64 + i * 16 + l16;
                v4i fw[KSTEPS];
#pragma unroll
                for (int ks = 0; ks < KSTEPS; ks++)
                    fw[ks] = *reinterpret_cast<const v4i *>(w_lds + row * lay.pitch + (((4 * ks + lq) ^ swz(row)) << 4));
                cs[i] = *reinterpret_cast<const v4f *>(cs_lds + g * 64 + i * 16 + lq * 4);
                cb[i] = *reinterpret_cast<const v4f *>(cb_lds + g * 64 + i * 16 + lq * 4);
#pragma unroll
                for (int jb = 0; jb < RB; jb++) {
                    v4i a = {0, 0, 0, 0};
#pragma unroll
                    for (int ks = 0; ks < KSTEPS; ks++) a = __builtin_amdgcn_mfma_i32_16x16x64_i8(fw[ks], fx[jb][ks], a, 0, 0, 0);
#if PTQ4VM_STREAM_SKIP & 4
                    a = fx[jb][0] + i;
#endif
                    acc[jb][i] = a;
                }
            }
            const int cols_valid = min(64, N - g * 64);
            // Accumulator register v of block (jb, i): token row 16 jb + (lane mod 16), channel 64 g + 16 i + 4 (lane / 16) + v.
            if (p.acc_out) {  // parity aid, off the timed path
#pragma unroll
                for (int jb = 0; jb < RB; jb++)
#pragma unroll
                    for (int i = 0; i < 4; i++)
#pragma unroll
                        for (int c = 0; c < 4; c++) {
                            const int64_t r = r_unit + jb * 16 + l16;
                            const int col = i * 16 + lq * 4 + c;
                            if (r < p.M && col < cols_valid) p.acc_out[r * p.N + g * 64 + col] = PACKED4 ? acc[jb][i][c] >> 8 : acc[jb][i][c];  // 4-bit forms: 256 times the sum
                        }
            }
#pragma unroll
            for (int jb = 0; jb < RB; jb++)
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    float out[4];
#pragma unroll
                    for (int c = 0; c < 4; c++) {
                        int a = acc[jb][i][c];
                        if constexpr (OFFSET) a -= __mul24(rz[jb], cz[i][c]);  // |z| < 2^8, |rowsum| < 2^23
                        out[c] = (float)a * (rs[jb] * cs[i][c]) + cb[i][c];
                    }
                    __half2 lo = __floats2half2_rn(out[0], out[1]);
                    __half2 hi = __floats2half2_rn(out[2], out[3]);
                    u32x2 packed = {__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi)};
#if PTQ4VM_STREAM_SKIP & 2
                    packed = u32x2{(uint32_t)acc[jb][i][0] ^ (uint32_t)acc[jb][i][1], (uint32_t)acc[jb][i][2] ^ (uint32_t)acc[jb][i][3]};
#endif
                    *reinterpret_cast<u32x2 *>(patch + patch_chunk(jb * 16 + l16, 2 * i + (lq >> 1)) + (lq & 1) * 8) = packed;
                }
            asm volatile("" ::: "memory");  // wavefront-private patch: LDS runs a wavefront's accesses in order
#if PTQ4VM_STREAM_SKIP & 1
            if (p.M < 0)
#endif
            if (y_wide && cols_valid == 64 && r_unit + UNIT <= p.M) {  // uniform: whole lines, no per-lane tests
                __half *dst = p.y + (r_unit + (lane >> 3)) * p.ldy + g * 64 + (lane & 7) * 8;
#pragma unroll
                for (int s = 0; s < 2 * RB; s++) {  // 8 rows x 128 bytes per store instruction
                    const v4i data = *reinterpret_cast<const v4i *>(patch + patch_chunk(s * 8 + (lane >> 3), lane & 7));
                    __builtin_nontemporal_store(data, reinterpret_cast<v4i *>(dst + s * 8 * p.ldy));
                }
            } else
#pragma unroll
            for (int s = 0; s < 2 * RB; s++) {
                const int row = s * 8 + (lane >> 3), chunk = lane & 7;
                const v4i data = *reinterpret_cast<const v4i *>(patch + patch_chunk(row, chunk));
                const int64_t rr = r_unit + row;
                if (rr < p.M) {
                    __half *dst = p.y + rr * p.ldy + g * 64 + chunk * 8;
                    if (y_wide && chunk * 8 + 8 <= cols_valid) {
                        __builtin_nontemporal_store(data, reinterpret_cast<v4i *>(dst));
                    } else if (p.y_vec >= 4 && chunk * 8 + 8 <= cols_valid) {
                        u32x2 a = {(uint32_t)data[0], (uint32_t)data[1]}, b = {(uint32_t)data[2], (uint32_t)data[3]};
                        *reinterpret_cast<u32x2 *>(dst) = a;
                        *reinterpret_cast<u32x2 *>(dst + 4) = b;
                    } else {
#pragma unroll
                        for (int e = 0; e < 8; e++)
                            if (chunk * 8 + e < cols_valid)
                                reinterpret_cast<uint16_t *>(dst)[e] = (uint16_t)((uint32_t)data[e >> 1] >> (16 * (e & 1)));
                    }
                }
            }
            asm volatile("" ::: "memory");
        }
    }
}

// ------------------------------------------------------------------------------------------
// Generic fused kernel: the register-staged tiled kernel (4 wavefronts, BR x BO tile, 64-code
// slabs, double-buffered LDS) whose activation loader reads fp16 and quantizes on the way to LDS.
// Any shape, pitch and alignment (X_ALIGN / W_ALIGN: 16, 4 or 0 = element-wise).
// ------------------------------------------------------------------------------------------
template <int BR, int BO, int WR, int WO, int X_ALIGN, int W_ALIGN>
__global__ __launch_bounds__(kThreads, 2) void pts_linear_generic(const LinearArgs p) {
    using Path = Int8Path;
    static_assert(WR * WO == kWaves, "four wavefronts per workgroup");
    constexpr int WAVE_R = BR / WR, WAVE_O = BO / WO;
    constexpr int FR = WAVE_R / 32, FO = WAVE_O / 32;
    static_assert(WAVE_R % 32 == 0 && WAVE_O % 32 == 0, "wave tile must be whole MFMA blocks");
    static_assert(BR * 4 % kThreads == 0, "every thread stages the same rows in every slab");
    constexpr int X_CHUNKS = BR * 4 / kThreads;  // 16-code chunks per thread per slab
    constexpr int W_CHUNKS = (BO * 4 + kThreads - 1) / kThreads;
    using Acc = typename Path::Acc;

    __shared__ __attribute__((aligned(16))) char lds_x[2][BR * kSlabBytes];
    __shared__ __attribute__((aligned(16))) char lds_w[2][BO * kSlabBytes];
    constexpr int JB = (FR % 2 == 0 && kWaves * 64 * WAVE_O * 2 <= 2 * BR * kSlabBytes) ? 2 : 1;
    static_assert(kWaves * JB * 32 * WAVE_O * 2 <= 2 * BR * kSlabBytes, "epilogue patches must fit the activation buffers");

    int tile_r, tile_o;
    if (!tile_of_block(p, tile_r, tile_o)) return;
    const int64_t r0 = (int64_t)tile_r * BR, o0 = (int64_t)tile_o * BO;
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

    // A thread stages the same X_CHUNKS rows in every slab: their reciprocal steps are computed once.
    float inv_s[X_CHUNKS];
#pragma unroll
    for (int i = 0; i < X_CHUNKS; i++) {
        const int64_t r = r0 + ((tid + kThreads * i) >> 2);
        inv_s[i] = 1.0f / p.s_tok[(r < p.M ? r : 0) % p.L];  // IEEE division
    }

    v4i stage_x[X_CHUNKS], stage_w[W_CHUNKS];
    auto fetch = [&](int64_t kb0) {
#pragma unroll
        for (int i = 0; i < X_CHUNKS; i++) {
            const int cid = tid + kThreads * i, row = cid >> 2, kc = cid & 3;
            const bool ok = r0 + row < p.M;
            float im[16];
#pragma unroll
            for (int e = 0; e < 16; e++) im[e] = (p.inv_m && kb0 + kc * 16 + e < p.k_bytes) ? p.inv_m[kb0 + kc * 16 + e] : 1.0f;
            stage_x[i] = load_quantized_chunk<X_ALIGN>(p.x + (r0 + row) * p.ldx_bytes, kb0 + kc * 16, p.k_bytes, ok,
                                                       im, inv_s[i]);
            if (p.xq_out && tile_o == 0 && ok) {  // parity aid: the codes exactly as the MFMA will see them
#pragma unroll
                for (int b = 0; b < 16; b++)
                    if (kb0 + kc * 16 + b < p.k_bytes)
                        p.xq_out[(r0 + row) * p.ldxq_out + kb0 + kc * 16 + b] = (int8_t)((uint32_t)stage_x[i][b >> 2] >> (8 * (b & 3)));
            }
        }
#pragma unroll
        for (int i = 0; i < W_CHUNKS; i++) {
            const int cid = tid + kThreads * i, row = cid >> 2, kc = cid & 3;
            const bool ok = (cid < BO * 4) && (o0 + row < p.N);
            stage_w[i] = load_chunk<W_ALIGN, 1>(p.w + (o0 + row) * p.ldw_bytes, kb0 + kc * 16, p.k_bytes, ok);
        }
    };
    auto commit = [&](int buf) {
#pragma unroll
        for (int i = 0; i < X_CHUNKS; i++) {
            const int cid = tid + kThreads * i, row = cid >> 2, kc = cid & 3;
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
        mfma_slab<Path, FO, FR>(acc, &lds_x[buf][wave_r * kSlabBytes], &lds_w[buf][wave_o * kSlabBytes], l32, lhalf);
        if (more) commit(buf ^ 1);
        __syncthreads();
    }
    epilogue<Path, FO, FR, JB>(acc, p, &lds_x[0][0] + wave * (JB * 32 * WAVE_O * 2), r0 + wave_r, o0 + wave_o, lane);
}

// ------------------------------------------------------------------------------------------
// Host side
// ------------------------------------------------------------------------------------------
template <int KSTEPS, bool QUANT, bool PACKED4 = false, bool OFFSET = false>
int launch_stream_aligned(const LinearArgs &a, int xa, int wa, const StreamLayout &lay, unsigned wgs, hipStream_t stream) {
    using Kernel = void (*)(const LinearArgs);
    // [activation alignment 16 / 4 / 0][weight alignment 16 / 4 / 0]
    static const Kernel kernels[3][3] = {
        {linear_stream_smallk<KSTEPS, QUANT, 16, 16, PACKED4, OFFSET>, linear_stream_smallk<KSTEPS, QUANT, 16, 4, PACKED4, OFFSET>,
         linear_stream_smallk<KSTEPS, QUANT, 16, 0, PACKED4, OFFSET>},
        {linear_stream_smallk<KSTEPS, QUANT, 4, 16, PACKED4, OFFSET>, linear_stream_smallk<KSTEPS, QUANT, 4, 4, PACKED4, OFFSET>,
         linear_stream_smallk<KSTEPS, QUANT, 4, 0, PACKED4, OFFSET>},
        {linear_stream_smallk<KSTEPS, QUANT, 0, 16, PACKED4, OFFSET>, linear_stream_smallk<KSTEPS, QUANT, 0, 4, PACKED4, OFFSET>,
         linear_stream_smallk<KSTEPS, QUANT, 0, 0, PACKED4, OFFSET>}};
    auto idx = [](int al) { return al == 16 ? 0 : (al == 4 ? 1 : 2); };
    const Kernel kernel = kernels[idx(xa)][idx(wa)];
    if (int rc = ptq4vm::set_lds_limit(reinterpret_cast<const void *>(kernel), kLdsBytes, "hipFuncSetAttribute(linear_stream_smallk)")) return rc;
    kernel<<<dim3(wgs), dim3(kStreamWaves * 64), lay.total, stream>>>(a);
    return ptq4vm::check_launch("linear_stream_smallk");
}

// Form of a fused launch: 8-bit codes, 4-bit codes (packed weight), or 8-bit codes with a per-token zero offset.
enum class Form { kInt8 = 0, kBits4 = 1, kOffset = 2 };

int launch_wres(const LinearArgs &a, hipStream_t stream, Form form) {
    const FusedLayout lay = fused_layout((int)a.N, (int)a.k_bytes, (int)a.L, form == Form::kOffset);
    int device = 0, cus = 0;
    hipError_t err = hipGetDevice(&device);
    if (err == hipSuccess) err = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device);
    if (err != hipSuccess) return ptq4vm::record_hip_error(err, "hipDeviceGetAttribute(multiprocessor count)");
    if (cus < 1) cus = 1;
    const int64_t units = ptq4vm::ceil_div(a.M, 16 * kFusedRB);
    int64_t wgs = ptq4vm::ceil_div(units, kFusedWaves);
    if (wgs > cus) wgs = cus;  // one workgroup per CU: the resident tables take most of its LDS
    using Kernel = void (*)(const LinearArgs);
    // four k-steps in flight need too many registers next to the accumulators of 7 or 8 channel blocks
#ifndef PTQ4VM_FUSED_MAXD
#define PTQ4VM_FUSED_MAXD (PTQ4VM_FUSED_RB == 1 ? 2 : 4)  // 16 wavefronts of 128 registers: two k-steps in flight (measured best)
#endif
    constexpr int kDeepest = PTQ4VM_FUSED_MAXD >= 4 ? 4 : 2;  // (the depth-4 kernels are not even compiled when they cannot be chosen)
#define PTQ4VM_WRES_ROW(D, DUMP, B4, OFS) \
    {pts_linear_wres<1, D, DUMP, B4, OFS>, pts_linear_wres<2, D, DUMP, B4, OFS>, pts_linear_wres<3, D, DUMP, B4, OFS>, \
     pts_linear_wres<4, D, DUMP, B4, OFS>, pts_linear_wres<5, D, DUMP, B4, OFS>, pts_linear_wres<6, D, DUMP, B4, OFS>, \
     pts_linear_wres<7, D, DUMP, B4, OFS>, pts_linear_wres<8, D, DUMP, B4, OFS>}
#define PTQ4VM_WRES_FORM(B4, OFS) \
    {{PTQ4VM_WRES_ROW(kDeepest, false, B4, OFS), PTQ4VM_WRES_ROW(2, false, B4, OFS), PTQ4VM_WRES_ROW(1, false, B4, OFS)}, \
     {PTQ4VM_WRES_ROW(kDeepest, true, B4, OFS), PTQ4VM_WRES_ROW(2, true, B4, OFS), PTQ4VM_WRES_ROW(1, true, B4, OFS)}}
    // [form][parity aids][k-steps in flight: 4, 2, 1][number of 16-channel blocks - 1]
    static const Kernel kernels[3][2][3][kFusedMaxBlocks] = {PTQ4VM_WRES_FORM(false, false), PTQ4VM_WRES_FORM(true, false),
                                                             PTQ4VM_WRES_FORM(false, true)};
#undef PTQ4VM_WRES_FORM
#undef PTQ4VM_WRES_ROW
    const int n_ksteps = (int)(a.k_bytes / 64);
    const int depth_row = (PTQ4VM_FUSED_MAXD >= 4 && n_ksteps % 4 == 0 && lay.nb <= 6) ? 0 : (n_ksteps % 2 == 0 ? 1 : 2);
    const Kernel kernel = kernels[(int)form][(a.xq_out || a.acc_out) ? 1 : 0][depth_row][lay.nb - 1];
    if (int rc = ptq4vm::set_lds_limit(reinterpret_cast<const void *>(kernel), kLdsBytes, "hipFuncSetAttribute(pts_linear_wres)")) return rc;
    kernel<<<dim3((unsigned)wgs), dim3(kFusedWaves * 64), lay.total, stream>>>(a);
    return ptq4vm::check_launch("pts_linear_wres");
}

template <int BR, int BO, int WR, int WO>
int launch_generic(LinearArgs a, int x_align, int w_align, hipStream_t stream) {
    dim3 grid;
    if (!set_grid<BR, BO>(a, grid)) return PTQ4VM_ERR_SHAPE;
    const dim3 block(kThreads);
#define PTQ4VM_LAUNCH(XA, WA) pts_linear_generic<BR, BO, WR, WO, XA, WA><<<grid, block, 0, stream>>>(a)
    if (x_align == 16 && w_align == 16) PTQ4VM_LAUNCH(16, 16);
    else if (x_align == 16 && w_align == 4) PTQ4VM_LAUNCH(16, 4);
    else if (x_align == 16) PTQ4VM_LAUNCH(16, 0);
    else if (x_align == 4 && w_align == 16) PTQ4VM_LAUNCH(4, 16);
    else if (x_align == 4 && w_align == 4) PTQ4VM_LAUNCH(4, 4);
    else if (x_align == 4) PTQ4VM_LAUNCH(4, 0);
    else if (w_align == 16) PTQ4VM_LAUNCH(0, 16);
    else if (w_align == 4) PTQ4VM_LAUNCH(0, 4);
    else PTQ4VM_LAUNCH(0, 0);
#undef PTQ4VM_LAUNCH
    return ptq4vm::check_launch("pts_linear_generic");
}

// The 4-bit form (weight packed two codes per byte, activations clipped to +-7) and the zero-offset form run on the
// weight-resident and the row-streaming kernel only; other shapes return PTQ4VM_ERR_SHAPE (the two-call forms cover them).
int dispatch(LinearArgs a, hipStream_t stream, Form form = Form::kInt8) {
    auto align_of = [](const void *base, int64_t pitch_bytes) {
        if (ptq4vm::aligned_to(base, 16) && pitch_bytes % 16 == 0) return 16;
        if (ptq4vm::aligned_to(base, 4) && pitch_bytes % 4 == 0) return 4;
        return 0;
    };
    const int xa = align_of(a.x, a.ldx_bytes), wa = align_of(a.w, a.ldw_bytes);
    a.y_vec = (a.ldy % 8 == 0 && ptq4vm::aligned_to(a.y, 16)) ? 8
              : ((a.ldy % 4 == 0 && ptq4vm::aligned_to(a.y, 8)) ? 4 : 1);
    const bool small = a.M < (1LL << 31) && a.L < (1LL << 31) && a.k_bytes < (1LL << 20);
    const bool wres_ok = small && xa == 16 && wa == 16 && a.k_bytes % 64 == 0 && a.N <= 16 * kFusedMaxBlocks &&
                         a.M >= kFusedMinRows && a.L <= 65536 &&
                         (!a.xq_out || (ptq4vm::aligned_to(a.xq_out, 8) && a.ldxq_out % 8 == 0)) &&
                         fused_layout((int)a.N, (int)a.k_bytes, (int)a.L, form == Form::kOffset).total <= kLdsBytes;
    if (wres_ok) return launch_wres(a, stream, form);
    if (a.k_bytes <= 128) {
        const int rc = launch_stream_smallk(a, true, stream, form == Form::kBits4, form == Form::kOffset);
        if (rc <= 0) return rc;
    }
    if (form != Form::kInt8) return PTQ4VM_ERR_SHAPE;
    if (a.N > 64) return launch_generic<256, 128, 2, 2>(a, xa, wa, stream);
    return launch_generic<256, 64, 4, 1>(a, xa, wa, stream);
}

}  // namespace

int ptq4vm::mfma::launch_stream_smallk(const LinearArgs &a, bool quantize, hipStream_t stream, bool packed4, bool offset) {
    auto align_of = [](const void *base, int64_t pitch_bytes) {
        if (ptq4vm::aligned_to(base, 16) && pitch_bytes % 16 == 0) return 16;
        if (ptq4vm::aligned_to(base, 4) && pitch_bytes % 4 == 0) return 4;
        return 0;
    };
    const int xa = align_of(a.x, a.ldx_bytes), wa = align_of(a.w, a.ldw_bytes);
    // bytes of K per row once the operands are int8 (two-launch 4-bit form: k_bytes counts packed bytes; fused 4-bit form: codes)
    const int64_t k_codes = (packed4 && !quantize) ? 2 * a.k_bytes : a.k_bytes;
    if (k_codes > 128 || (offset && packed4) || a.M < (quantize ? kStreamMinRowsFused : kStreamMinRows) || a.M >= (1LL << 31) || a.L >= (1LL << 31) || a.N > 8192) return 1;
    const int ksteps = k_codes <= 64 ? 1 : 2;
    const StreamLayout lay = stream_layout((int)a.N, ksteps);
    if (lay.total > kLdsBytes) return 1;
    int device = 0, cus = 0;
    hipError_t err = hipGetDevice(&device);
    if (err == hipSuccess) err = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device);
    if (err != hipSuccess) return ptq4vm::record_hip_error(err, "hipDeviceGetAttribute(multiprocessor count)");
    if (cus < 1) cus = 1;
    const int64_t items = ptq4vm::ceil_div(a.M, 16 * kStreamRB) * (lay.groups < 4 ? lay.groups : 4);  // as the kernel counts them
    int64_t wgs = ptq4vm::ceil_div(items, kStreamWaves);
    if (wgs > cus) wgs = cus;  // one workgroup per CU: the resident weight takes most of its LDS
    if (offset && quantize)
        return ksteps == 1 ? launch_stream_aligned<1, true, false, true>(a, xa, wa, lay, (unsigned)wgs, stream)
                           : launch_stream_aligned<2, true, false, true>(a, xa, wa, lay, (unsigned)wgs, stream);
    if (offset)
        return ksteps == 1 ? launch_stream_aligned<1, false, false, true>(a, xa, wa, lay, (unsigned)wgs, stream)
                           : launch_stream_aligned<2, false, false, true>(a, xa, wa, lay, (unsigned)wgs, stream);
    if (packed4 && quantize)
        return ksteps == 1 ? launch_stream_aligned<1, true, true>(a, xa, wa, lay, (unsigned)wgs, stream)
                           : launch_stream_aligned<2, true, true>(a, xa, wa, lay, (unsigned)wgs, stream);
    if (packed4)
        return ksteps == 1 ? launch_stream_aligned<1, false, true>(a, xa, wa, lay, (unsigned)wgs, stream)
                           : launch_stream_aligned<2, false, true>(a, xa, wa, lay, (unsigned)wgs, stream);
    if (quantize)
        return ksteps == 1 ? launch_stream_aligned<1, true>(a, xa, wa, lay, (unsigned)wgs, stream)
                           : launch_stream_aligned<2, true>(a, xa, wa, lay, (unsigned)wgs, stream);
    return ksteps == 1 ? launch_stream_aligned<1, false>(a, xa, wa, lay, (unsigned)wgs, stream)
                       : launch_stream_aligned<2, false>(a, xa, wa, lay, (unsigned)wgs, stream);
}

extern "C" int ptq4vm_w4a4_linear_fused(const void *x_f16, const float *inv_m, const float *s_tok, const uint8_t *wq4,
                                        const float *s_w, const void *bias_f16, void *y_f16, int32_t *acc_out,
                                        int8_t *xq_out, int64_t B, int64_t L, int64_t K, int64_t N, int64_t ldx,
                                        int64_t ldwq, int64_t ldy, int64_t ldxq, void *stream_) {
    if (!x_f16 || !s_tok || !wq4 || !s_w || !y_f16) return PTQ4VM_ERR_NULL;
    if (B < 0 || N < 0 || L <= 0 || K <= 0 || K > PTQ4VM_MAX_K_W4 || K % 2 != 0) return PTQ4VM_ERR_SHAPE;
    if (B > 0 && L > INT64_MAX / B) return PTQ4VM_ERR_SHAPE;
    if (ldx < K || ldwq < K / 2 || ldy < N || (xq_out && ldxq < K)) return PTQ4VM_ERR_STRIDE;
    if (!ptq4vm::aligned_to(x_f16, 16) || !ptq4vm::aligned_to(wq4, 16) || !ptq4vm::aligned_to(y_f16, 2) ||
        !ptq4vm::aligned_to(inv_m, 4) || !ptq4vm::aligned_to(s_tok, 4) || !ptq4vm::aligned_to(s_w, 4) ||
        !ptq4vm::aligned_to(bias_f16, 2) || !ptq4vm::aligned_to(acc_out, 4))
        return PTQ4VM_ERR_ALIGN;
    const int64_t M = B * L;
    if (M == 0 || N == 0) return PTQ4VM_OK;
    LinearArgs a{};
    a.x = static_cast<const char *>(x_f16);
    a.w = reinterpret_cast<const char *>(wq4);
    a.s_tok = s_tok;
    a.s_w = s_w;
    a.bias = static_cast<const __half *>(bias_f16);
    a.y = static_cast<__half *>(y_f16);
    a.acc_out = acc_out;
    a.M = M;
    a.N = N;
    a.k_bytes = K;  // codes per row
    a.ldx_bytes = ldx * 2;
    a.ldw_bytes = ldwq;  // packed bytes
    a.ldy = ldy;
    a.L = L;
    a.inv_m = inv_m;
    a.xq_out = xq_out;
    a.ldxq_out = ldxq;
    return dispatch(a, static_cast<hipStream_t>(stream_), Form::kBits4);
}

extern "C" int ptq4vm_w8a8_linear_offset_fused(const void *x_f16, const float *inv_m, const float *s_tok, const int32_t *z_tok,
                                               const int8_t *wq, const int32_t *rowsum, const float *s_w,
                                               const void *bias_f16, void *y_f16, int32_t *acc_out, int8_t *xq_out,
                                               int64_t B, int64_t L, int64_t K, int64_t N, int64_t ldx, int64_t ldwq,
                                               int64_t ldy, int64_t ldxq, void *stream_) {
    if (!x_f16 || !s_tok || !z_tok || !wq || !rowsum || !s_w || !y_f16) return PTQ4VM_ERR_NULL;
    if (B < 0 || N < 0 || L <= 0 || K <= 0 || K > PTQ4VM_MAX_K_OFFSET) return PTQ4VM_ERR_SHAPE;
    if (B > 0 && L > INT64_MAX / B) return PTQ4VM_ERR_SHAPE;
    if (ldx < K || ldwq < K || ldy < N || (xq_out && ldxq < K)) return PTQ4VM_ERR_STRIDE;
    if (!ptq4vm::aligned_to(x_f16, 16) || !ptq4vm::aligned_to(wq, 16) || !ptq4vm::aligned_to(y_f16, 2) ||
        !ptq4vm::aligned_to(inv_m, 4) || !ptq4vm::aligned_to(s_tok, 4) || !ptq4vm::aligned_to(z_tok, 4) ||
        !ptq4vm::aligned_to(rowsum, 4) || !ptq4vm::aligned_to(s_w, 4) || !ptq4vm::aligned_to(bias_f16, 2) ||
        !ptq4vm::aligned_to(acc_out, 4))
        return PTQ4VM_ERR_ALIGN;
    const int64_t M = B * L;
    if (M == 0 || N == 0) return PTQ4VM_OK;
    LinearArgs a{};
    a.x = static_cast<const char *>(x_f16);
    a.w = reinterpret_cast<const char *>(wq);
    a.s_tok = s_tok;
    a.s_w = s_w;
    a.bias = static_cast<const __half *>(bias_f16);
    a.y = static_cast<__half *>(y_f16);
    a.acc_out = acc_out;
    a.M = M;
    a.N = N;
    a.k_bytes = K;
    a.ldx_bytes = ldx * 2;
    a.ldw_bytes = ldwq;
    a.ldy = ldy;
    a.L = L;
    a.inv_m = inv_m;
    a.xq_out = xq_out;
    a.ldxq_out = ldxq;
    a.z_tok = z_tok;
    a.rowsum = rowsum;
    return dispatch(a, static_cast<hipStream_t>(stream_), Form::kOffset);
}

extern "C" int ptq4vm_w8a8_linear_fused(const void *x_f16, const float *inv_m, const float *s_tok, const int8_t *wq,
                                        const float *s_w, const void *bias_f16, void *y_f16, int32_t *acc_out,
                                        int8_t *xq_out, int64_t B, int64_t L, int64_t K, int64_t N, int64_t ldx,
                                        int64_t ldwq, int64_t ldy, int64_t ldxq, void *stream_) {
    if (!x_f16 || !s_tok || !wq || !s_w || !y_f16) return PTQ4VM_ERR_NULL;
    if (B < 0 || N < 0 || L <= 0 || K <= 0 || K > PTQ4VM_MAX_K) return PTQ4VM_ERR_SHAPE;
    if (B > 0 && L > INT64_MAX / B) return PTQ4VM_ERR_SHAPE;
    if (ldx < K || ldwq < K || ldy < N || (xq_out && ldxq < K)) return PTQ4VM_ERR_STRIDE;
    if (!ptq4vm::aligned_to(x_f16, 16) || !ptq4vm::aligned_to(wq, 16) || !ptq4vm::aligned_to(y_f16, 2) ||
        !ptq4vm::aligned_to(inv_m, 4) || !ptq4vm::aligned_to(s_tok, 4) || !ptq4vm::aligned_to(s_w, 4) ||
        !ptq4vm::aligned_to(bias_f16, 2) || !ptq4vm::aligned_to(acc_out, 4))
        return PTQ4VM_ERR_ALIGN;
    const int64_t M = B * L;
    if (M == 0 || N == 0) return PTQ4VM_OK;
    LinearArgs a{};
    a.x = static_cast<const char *>(x_f16);
    a.w = reinterpret_cast<const char *>(wq);
    a.s_tok = s_tok;
    a.s_w = s_w;
    a.bias = static_cast<const __half *>(bias_f16);
    a.y = static_cast<__half *>(y_f16);
    a.acc_out = acc_out;
    a.M = M;
    a.N = N;
    a.k_bytes = K;
    a.ldx_bytes = ldx * 2;
    a.ldw_bytes = ldwq;
    a.ldy = ldy;
    a.L = L;
    a.inv_m = inv_m;
    a.xq_out = xq_out;
    a.ldxq_out = ldxq;
    return dispatch(a, static_cast<hipStream_t>(stream_));
}
