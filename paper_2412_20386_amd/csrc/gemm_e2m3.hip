// W4A4 linear for gfx950 on FP6 (E2M3) containers: the integer product of App. B.1 "INT GEMM" carried by
// v_mfma_f32_16x16x128_f8f6f4 (128 codes per instruction, twice the rate of the int8 MFMA), with the PTS
// dequantization fused behind it (PTS equation of Sec. 5.1; App. B.1 "Dequantization").  The 4-bit codes
// -7..7 (Sec. 2.3; the W4A4 setting of the latency table, Sec. 6.4) are exactly representable in E2M3, their
// products and partial sums are integers below 2^24, so the fp32 accumulators hold sum_k xq wq exactly.
//
// Operand layout of the instruction (checked against integer dot products on the device): lane l feeds row
// (l mod 16) of its matrix with the 32 codes of group (l / 16) of the current 128-code block, as 6 dwords;
// accumulator register v of lane l is (first-operand row 4 (l / 16) + v) x (second-operand row l mod 16).
// The weight is the first operand: a lane's four results are four consecutive channels of one token row.
//
// Two kernels:
//   linear_e2m3_persistent  one workgroup of 8 wavefronts per CU walks 256 x 256 tiles (wave tile 128 token rows x
//                           64 channels); a ring of 3 stages, each one 128-code block of the tile's 256 + 256
//                           rows, is filled by direct global -> LDS copies that run two stages ahead.
//   linear_e2m3_generic     64 x 64 tiles staged through registers, any shape and alignment of y.
#include "mfma_linear.hpp"

// Timing experiments only (results are wrong when any bit is set): 1 no output stores, 2 no epilogue at all,
// 4 no global -> LDS copies of the operands, 8 no MFMAs.
#ifndef PTQ4VM_E2M3_SKIP
#define PTQ4VM_E2M3_SKIP 0
#endif

namespace ptq4vm {
namespace mfma {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v2i __attribute__((ext_vector_type(2)));

constexpr int kBlockBytes = 96;  // one row's 128 codes: 4 x 16 bytes (groups' low parts), 4 x 8 bytes (high parts)

__device__ __forceinline__ v4f mfma_e2m3(const v8i &w, const v8i &x, const v4f &c) {
    // cbsz = blgp = 2: both operands are FP6 E2M3; no block scales
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(w, x, c, 2, 2, 0, 0, 0, 0);
}
__device__ __forceinline__ v8i make_fragment(const v4i &lo, const v2i &hi) {
    return v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], 0, 0};
}

// ------------------------------------------------------------------------------------------
// Small tiled kernel: 4 wavefronts, 64 token rows x 64 channels per workgroup, wavefront w owns rows
// 16 w .. 16 w + 15 against the 64 channels.  One 128-code block per trip, staged through registers.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void linear_e2m3_generic(const LinearArgs p) {
    __shared__ __attribute__((aligned(16))) char xs[64 * kBlockBytes];
    __shared__ __attribute__((aligned(16))) char ws[64 * kBlockBytes];
    int tile_r, tile_o;
    if (!tile_of_block(p, tile_r, tile_o)) return;
    const int64_t r0 = (int64_t)tile_r * 64, o0 = (int64_t)tile_o * 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, lq = lane >> 4;

    v4f acc[4];
#pragma unroll
    for (int i = 0; i < 4; i++) acc[i] = v4f{0.0f, 0.0f, 0.0f, 0.0f};

    const int n_blocks = (int)(p.k_bytes / kBlockBytes);
    for (int kb = 0; kb < n_blocks; kb++) {
        for (int q = tid; q < 64 * 6; q += kThreads) {  // 16-byte chunks of the two 64-row tiles
            const int row = q / 6, c = q - row * 6;
            v4i vx = {0, 0, 0, 0}, vw = {0, 0, 0, 0};
            if (r0 + row < p.M) vx = *reinterpret_cast<const v4i *>(p.x + kb * p.ldx_bytes + (r0 + row) * kBlockBytes + c * 16);
            if (o0 + row < p.N) vw = *reinterpret_cast<const v4i *>(p.w + kb * p.ldw_bytes + (o0 + row) * kBlockBytes + c * 16);
            *reinterpret_cast<v4i *>(xs + q * 16) = vx;
            *reinterpret_cast<v4i *>(ws + q * 16) = vw;
        }
        __syncthreads();
        const char *xrow = xs + (wave * 16 + l16) * kBlockBytes;
        const v8i fx = make_fragment(*reinterpret_cast<const v4i *>(xrow + lq * 16), *reinterpret_cast<const v2i *>(xrow + 64 + lq * 8));
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const char *wrow = ws + (i * 16 + l16) * kBlockBytes;
            const v8i fw = make_fragment(*reinterpret_cast<const v4i *>(wrow + lq * 16), *reinterpret_cast<const v2i *>(wrow + 64 + lq * 8));
            acc[i] = mfma_e2m3(fw, fx, acc[i]);
        }
        __syncthreads();
    }

    const int64_t r = r0 + wave * 16 + l16;
    if (r >= p.M) return;
    const float rs = p.s_tok[r % p.L];
    uint16_t *yrow = reinterpret_cast<uint16_t *>(p.y) + r * p.ldy;
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
        for (int h = 0; h < 2; h++) {
            const int64_t o = o0 + i * 16 + lq * 4 + 2 * h;
            const bool ok0 = o < p.N, ok1 = o + 1 < p.N;
            const float a0 = acc[i][2 * h], a1 = acc[i][2 * h + 1];
            if (p.acc_out) {
                if (ok0) p.acc_out[r * p.N + o] = (int)a0;
                if (ok1) p.acc_out[r * p.N + o + 1] = (int)a1;
            }
            const float cs0 = ok0 ? p.s_w[o] : 0.0f, cs1 = ok1 ? p.s_w[o + 1] : 0.0f;
            uint32_t bias_word = 0;
            if (p.bias) {
                const uint16_t *b = reinterpret_cast<const uint16_t *>(p.bias);
                bias_word = (ok0 ? (uint32_t)b[o] : 0u) | (ok1 ? (uint32_t)b[o + 1] << 16 : 0u);
            }
            const uint32_t out = __builtin_bit_cast(
                uint32_t, dequantize_pair_f16(a0, rs * cs0, a1, rs * cs1, __builtin_bit_cast(float, bias_word)));
            if (ok0) yrow[o] = (uint16_t)out;
            if (ok1) yrow[o + 1] = (uint16_t)(out >> 16);
        }
}

// ------------------------------------------------------------------------------------------
// Persistent kernel.  LDS: ring of kStages stages, each (256 token rows + 256 channels) x 96 bytes, then two
// buffers of per-tile scale vectors.  The containers are block-major, so what a stage receives is two contiguous
// 24 KiB spans of memory.  A stage row is the 96-byte block as in memory, except that rows with bit 3 set keep
// their last two 16-byte chunks (the groups' 8-byte high parts) swapped.  Measured with a stand-alone read loop
// (bytes per clock and CU, 16-byte low-part reads / 8-byte high-part reads / both): rows as in memory 228 / 118 /
// 168, high chunks swapped by row bit 3: 245 / 174 / 203, all chunk pairs swapped by row bit 3: 127 / 170 / 141.
// Ring discipline: barrier B(g) sits before the MFMAs of block g - 1, after its fragments have arrived in
// registers.  Passing it means every wavefront's copies of block g have landed and nobody reads block g - 1's
// stage again, so that stage is refilled at once with block g + 2 (after a tile's last block the refill waits
// until the epilogue, which borrows the stage, has finished).
// Requirements (host-checked): K a multiple of 128 and at least 256 codes, 16-byte aligned operand rows,
// N a multiple of 8, y rows 16-byte aligned, 4-byte aligned bias, 256 row pitches below 2^31, L < 2^31.
// ------------------------------------------------------------------------------------------
// Tile geometry: BR token rows x 256 channels; 4 wavefronts side by side along the channels per 128 rows.
#ifndef PTQ4VM_E2M3_BR
#define PTQ4VM_E2M3_BR 256
#endif
#ifndef PTQ4VM_E2M3_STAGES
#define PTQ4VM_E2M3_STAGES 3
#endif
// Which 16-byte chunk of a row's block goes to chunk position c of its stage row.
__device__ __forceinline__ int stage_chunk_source(int row, int c) { return c < 4 ? c : 4 + ((c - 4) ^ ((row >> 3) & 1)); }

constexpr int kTile = 256;                 // channels per tile
constexpr int kTileRows = PTQ4VM_E2M3_BR;  // token rows per tile: 256 (one workgroup of 8 wavefronts per CU) or 128 (two of 4)
constexpr int kStages = PTQ4VM_E2M3_STAGES;
constexpr int kWavesPerWg = 4 * kTileRows / 128;
constexpr int kStageBytes = (kTileRows + kTile) * kBlockBytes;
constexpr int kScaleBytes = kTile * 4 + kTileRows * 4 + kTile * 2;
constexpr int kPersistentLds = kStages * kStageBytes + 2 * kScaleBytes;
static_assert(kTileRows == 256 || kTileRows == 128, "tile height");

template <bool HAS_BIAS, bool DUMP_ACC>
__global__ __launch_bounds__(kWavesPerWg * 64, 2) void linear_e2m3_persistent(const LinearArgs p) {
    constexpr int NW = kWavesPerWg, FR = 8, FO = 4, WAVE_R = 128, WAVE_O = 64;
    constexpr int X_COPIES = kTileRows * 6 / 64 / NW;  // 1 KiB copies per wavefront and stage: 3 of token rows,
    constexpr int W_COPIES = kTile * 6 / 64 / NW;      // 3 or 6 of weight rows
    constexpr int LOADS_PER_BLOCK = X_COPIES + W_COPIES;
    constexpr int KEEP = (kStages - 2) * LOADS_PER_BLOCK;  // copies allowed in flight when a block is needed

    char *const ring = lds_dyn;
    char *const scales = lds_dyn + kStages * kStageBytes;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_r = (wave >> 2) * WAVE_R, wave_o = (wave & 3) * WAVE_O;
    const int l16 = lane & 15, lq = lane >> 4;
    const int swap = (l16 >> 3) & 1;
    // byte offsets of this lane's fragment parts inside a stage row block of 16 rows
    const int frag_lo = l16 * kBlockBytes + (lq << 4);
    const int frag_hi = l16 * kBlockBytes + ((4 + ((lq >> 1) ^ swap)) << 4) + (lq & 1) * 8;

    // work split: XCD x owns a contiguous range of tiles (channel tiles fastest), its workgroups interleave in it
    const int total_tiles = p.tiles_o * p.tiles_r;
    const int per_xcd = (total_tiles + kXcds - 1) / kXcds;
    const int wpx = (int)gridDim.x / kXcds, xcd = (int)(blockIdx.x % kXcds), wj = (int)(blockIdx.x / kXcds);
    const int lo_tile = xcd * per_xcd, hi_tile = min(lo_tile + per_xcd, total_tiles);
    const int n_range = max(hi_tile - lo_tile, 0);
    const int n_my = n_range / wpx + (wj < n_range % wpx ? 1 : 0);
    const int first = lo_tile + wj, last = first + n_my * wpx;

    const int n_blocks = (int)(p.k_bytes / kBlockBytes);
    const int total_blocks = n_my * n_blocks;
    if (total_blocks == 0) return;  // the whole workgroup: no barrier has been executed yet

    // ---- producer: the next block to copy, possibly of a later tile than the one being computed
    int pf_tile = first, pf_block = 0, pf_stage = 0, issued = 0;
    const char *pf_x = nullptr, *pf_w = nullptr;
    uint32_t x_off[X_COPIES], w_off[W_COPIES];
    auto pf_setup = [&]() {
        const int to = pf_tile % p.tiles_o, tr = pf_tile / p.tiles_o;
        const int64_t r0 = (int64_t)tr * kTileRows, o0 = (int64_t)to * kTile;
        pf_x = p.x + r0 * kBlockBytes;  // in plane 0; block b is b plane pitches further
        pf_w = p.w + o0 * kBlockBytes;
        const int rows_x = (int)min((int64_t)kTileRows, p.M - r0), rows_w = (int)min((int64_t)kTile, p.N - o0);
        // 16-byte chunk q of a stage half: row q / 6, chunk q mod 6; rows with bit 3 set keep chunks 4 and 5 swapped.
        // Rows beyond the matrix are clamped: their results are never stored.
#pragma unroll
        for (int i = 0; i < X_COPIES; i++) {
            const int q = (wave + NW * i) * 64 + lane;
            const int row = q / 6, c = q - row * 6;
            x_off[i] = (uint32_t)min(row, rows_x - 1) * kBlockBytes + stage_chunk_source(row, c) * 16;
        }
#pragma unroll
        for (int i = 0; i < W_COPIES; i++) {
            const int q = (wave + NW * i) * 64 + lane;
            const int row = q / 6, c = q - row * 6;
            w_off[i] = (uint32_t)min(row, rows_w - 1) * kBlockBytes + stage_chunk_source(row, c) * 16;
        }
    };
    auto issue = [&]() {  // copy the producer's block into ring stage pf_stage, then advance
        char *sx = ring + pf_stage * kStageBytes;
        char *sw = sx + kTileRows * kBlockBytes;
        const char *gx = pf_x + (int64_t)pf_block * p.ldx_bytes;
        const char *gw = pf_w + (int64_t)pf_block * p.ldw_bytes;
#pragma unroll
        for (int i = 0; i < ((PTQ4VM_E2M3_SKIP & 4) ? 0 : X_COPIES); i++)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(gx + x_off[i]),
                                             (__attribute__((address_space(3))) void *)(sx + (wave + NW * i) * 1024),
                                             16, 0, 0);
#pragma unroll
        for (int i = 0; i < ((PTQ4VM_E2M3_SKIP & 4) ? 0 : W_COPIES); i++)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(gw + w_off[i]),
                                             (__attribute__((address_space(3))) void *)(sw + (wave + NW * i) * 1024),
                                             16, 0, 0);
        issued++;
        if (++pf_stage == kStages) pf_stage = 0;
        if (++pf_block == n_blocks) {
            pf_block = 0;
            pf_tile += wpx;
            if (pf_tile < last) pf_setup();
        }
    };
    auto wait_block = [&](int g) {  // block g has landed for this wavefront
        if (g + kStages - 2 < total_blocks)
            wait_vmcnt_at_most<KEEP>();
        else
            wait_vmcnt_at_most<0>();
    };

    pf_setup();
    while (issued < kStages - 1 && issued < total_blocks) issue();
    wait_block(0);
    __builtin_amdgcn_s_barrier();  // B(0)
    if (issued < total_blocks) issue();

    int stage = 0, g = 0, parity = 0;  // consumer: ring stage, running block number, scale buffer
    for (int tile = first; tile < last; tile += wpx, parity ^= 1) {
        const int tile_o = tile % p.tiles_o, tile_r = tile / p.tiles_o;
        const int64_t r0 = (int64_t)tile_r * kTileRows, o0 = (int64_t)tile_o * kTile;
        const int rows_valid = (int)min((int64_t)kTileRows, p.M - r0), cols_valid = (int)min((int64_t)kTile, p.N - o0);
        float *const cs_lds = reinterpret_cast<float *>(scales + parity * kScaleBytes);  // s_w of the tile's channels
        float *const rs_lds = cs_lds + kTile;                                           // s_tok of the tile's rows
        uint32_t *const cb_lds = reinterpret_cast<uint32_t *>(rs_lds + kTileRows);      // bias, two fp16 per word

        // Scale vectors of this tile, one 4-byte element per lane, straight into LDS (indices beyond the
        // matrix are clamped; those rows / channels are never stored).  Tasks 0-3: s_w, then s_tok (64 rows each), then 2 of bias.
        constexpr int kRowTasks = kTileRows / 64;
#pragma unroll
        for (int task = 0; task < 4 + kRowTasks + 2; task++) {
            if (task % NW != wave) continue;
            if (task < 4) {
                const int c = min(task * 64 + lane, cols_valid - 1);
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(p.s_w + o0 + c),
                                                 (__attribute__((address_space(3))) void *)(cs_lds + task * 64), 4, 0, 0);
            } else if (task < 4 + kRowTasks) {
                const int blk = task - 4;
                const int r = min(blk * 64 + lane, rows_valid - 1);
                const uint32_t t = ((uint32_t)(r0 % p.L) + (uint32_t)r) % (uint32_t)p.L;
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(p.s_tok + t),
                                                 (__attribute__((address_space(3))) void *)(rs_lds + blk * 64), 4, 0, 0);
            } else if constexpr (HAS_BIAS) {
                const int blk = task - 4 - kRowTasks;
                const int c2 = min(blk * 64 + lane, cols_valid / 2 - 1);
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void *)(reinterpret_cast<const uint32_t *>(p.bias + o0) + c2),
                    (__attribute__((address_space(3))) void *)(cb_lds + blk * 64), 4, 0, 0);
            }
        }
        int loads_after_scales = 0;

        v4f acc[FO][FR];
#pragma unroll
        for (int i = 0; i < FO; i++)
#pragma unroll
            for (int j = 0; j < FR; j++) acc[i][j] = v4f{0.0f, 0.0f, 0.0f, 0.0f};

        // An operand is dead after its last MFMA of a block and is fetched again at once for the next block.
        v8i fw[FO], fx[FR];
        auto load_fw = [&](int i, int stg) {
            const char *sw = ring + stg * kStageBytes + (kTileRows + wave_o + i * 16) * kBlockBytes;
            fw[i] = make_fragment(*reinterpret_cast<const v4i *>(sw + frag_lo), *reinterpret_cast<const v2i *>(sw + frag_hi));
        };
        auto load_fx = [&](int j, int stg) {
            const char *sx = ring + stg * kStageBytes + (wave_r + j * 16) * kBlockBytes;
            fx[j] = make_fragment(*reinterpret_cast<const v4i *>(sx + frag_lo), *reinterpret_cast<const v2i *>(sx + frag_hi));
        };

        // B(g) for the tile's first block was passed during the previous tile (or before the loop)
#pragma unroll
        for (int i = 0; i < FO; i++) load_fw(i, stage);
#pragma unroll
        for (int j = 0; j < FR; j++) load_fx(j, stage);

        for (int s = 0; s < n_blocks; s++, g++) {
            int next_stage = stage + 1;
            if (next_stage == kStages) next_stage = 0;
            bool has_next = false;
            if (g + 1 < total_blocks) {
                // B(g+1): this wavefront holds the fragments of block g in registers and its copies of block g+1 have landed
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                wait_block(g + 1);
                __builtin_amdgcn_s_barrier();
                if (s + 1 < n_blocks) {
                    if (issued < total_blocks) {
                        issue();  // refills the stage of block g
                        loads_after_scales += LOADS_PER_BLOCK;
                    }
                    has_next = true;
                }  // after the tile's last block that stage first serves the epilogue
            }
#pragma unroll
            for (int j = 0; j < FR; j++) {
#pragma unroll
                for (int i = 0; i < FO; i++) {
                    if constexpr (!(PTQ4VM_E2M3_SKIP & 8)) acc[i][j] = mfma_e2m3(fw[i], fx[j], acc[i][j]);
                    else acc[i][j][0] += __builtin_bit_cast(float, fw[i][0] ^ fx[j][5]);
                    if (j == FR - 1 && has_next) load_fw(i, next_stage);
                }
                if (has_next) load_fx(j, next_stage);
            }
            stage = next_stage;
        }

        // ---- epilogue of this tile.  The ring stage of the tile's last block is free: B(g) was passed with that
        // block's fragments in registers and its refill has been held back; it holds the wavefronts' fp16
        // patches until the barrier that ends the epilogue.
        if (loads_after_scales >= KEEP && KEEP > 0)
            wait_vmcnt_at_most<KEEP>();
        else
            wait_vmcnt_at_most<0>();
        __builtin_amdgcn_s_barrier();  // scale vectors are visible to every wavefront
        const int free_stage = stage == 0 ? kStages - 1 : stage - 1;  // stage of the tile's last block
        char *patch = ring + free_stage * kStageBytes + wave * (32 * WAVE_O * 2);
        char *y_tile = reinterpret_cast<char *>(p.y + r0 * p.ldy + o0);
        const uint32_t ldy_bytes = (uint32_t)p.ldy * 2;
        auto patch_chunk = [&](int row, int chunk) { return row * (WAVE_O * 2) + ((chunk ^ (row & 7)) << 4); };
        const bool full_tile = rows_valid == kTileRows && cols_valid == kTile;

        // Accumulator register v of block (i, j): token row 16 j + (lane mod 16), channel 16 i + 4 (lane / 16) + v.
        // cs_raw[i]: steps of this lane's four channels of block i; cb_raw[i]: the eight fp16 biases around them.
        v4f cs_raw[4], cb_raw[4];
        float rs_raw[8];
        lds_read_4x_b128<64>(lds_addr(cs_lds + wave_o + lq * 4), cs_raw);
        if constexpr (HAS_BIAS) lds_read_4x_b128<32>(lds_addr(cb_lds + (wave_o + (lq >> 1) * 8) / 2), cb_raw);
        lds_read_8x_b32<64>(lds_addr(rs_lds + wave_r + l16), rs_raw);

        if constexpr (PTQ4VM_E2M3_SKIP & 2) {
            float sum = 0.0f;
#pragma unroll
            for (int i = 0; i < FO; i++)
#pragma unroll
                for (int j = 0; j < FR; j++) sum += acc[i][j][0] + acc[i][j][1] + acc[i][j][2] + acc[i][j][3];
            if (sum == 1.2345e-30f) p.y[0] = __float2half(sum);
        } else
#pragma unroll
        for (int jp = 0; jp < FR / 2; jp++) {  // 32 rows per round through the patch
#pragma unroll
            for (int jj = 0; jj < 2; jj++) {
                const int j = 2 * jp + jj;
#pragma unroll
                for (int i = 0; i < FO; i++) {
                    float b01 = 0.0f, b23 = 0.0f;  // two fp16 biases each, raw
                    if constexpr (HAS_BIAS) {
                        b01 = (lq & 1) ? cb_raw[i].z : cb_raw[i].x;
                        b23 = (lq & 1) ? cb_raw[i].w : cb_raw[i].y;
                    }
                    if constexpr (DUMP_ACC) {
                        const int64_t r = r0 + wave_r + j * 16 + l16;
#pragma unroll
                        for (int c = 0; c < 4; c++) {
                            const int64_t o = o0 + wave_o + i * 16 + lq * 4 + c;
                            if (r < p.M && o < p.N) p.acc_out[r * p.N + o] = (int)acc[i][j][c];
                        }
                    }
                    const float lo = dequantize_pair_f16(acc[i][j][0], rs_raw[j] * cs_raw[i][0], acc[i][j][1],
                                                         rs_raw[j] * cs_raw[i][1], b01);
                    const float hi = dequantize_pair_f16(acc[i][j][2], rs_raw[j] * cs_raw[i][2], acc[i][j][3],
                                                         rs_raw[j] * cs_raw[i][3], b23);
                    const u32x2 packed = {__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi)};
                    lds_write_b64(lds_addr(patch + patch_chunk(jj * 16 + l16, 2 * i + (lq >> 1)) + (lq & 1) * 8), packed);
                }
            }
            v4f data[4];
            uint32_t src[4];
#pragma unroll
            for (int q = 0; q < 4; q++)  // 8 rows x 128 bytes per store instruction
                src[q] = lds_addr(patch + patch_chunk(q * 8 + (lane >> 3), lane & 7));
            lds_read_4_b128(src, data);
            const uint32_t base = (uint32_t)(wave_r + jp * 32 + (lane >> 3)) * ldy_bytes + (uint32_t)(wave_o + (lane & 7) * 8) * 2;
            if constexpr (PTQ4VM_E2M3_SKIP & 1) {
                if (data[0][0] == 1.2345e-30f) p.y[0] = __float2half(data[1][1]);
            } else if (full_tile) {
#pragma unroll
                for (int q = 0; q < 4; q++)
                    __builtin_nontemporal_store(data[q], reinterpret_cast<v4f *>(y_tile + base + (uint32_t)(q * 8) * ldy_bytes));
            } else {
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const int rr = wave_r + jp * 32 + q * 8 + (lane >> 3), cc = wave_o + (lane & 7) * 8;
                    if (rr < rows_valid && cc < cols_valid)
                        *reinterpret_cast<v4f *>(y_tile + base + (uint32_t)(q * 8) * ldy_bytes) = data[q];
                }
            }
        }
        __builtin_amdgcn_s_barrier();  // every wavefront has read its patch back: the stage can be refilled
        if (issued < total_blocks) issue();
    }
}

int launch_persistent(LinearArgs a, hipStream_t stream) {
    int device = 0, cus = 0;
    hipError_t err = hipGetDevice(&device);
    if (err == hipSuccess) err = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device);
    if (err != hipSuccess) return ptq4vm::record_hip_error(err, "hipDeviceGetAttribute(multiprocessor count)");
    const int64_t tiles_r = ptq4vm::ceil_div(a.M, kTileRows), tiles_o = ptq4vm::ceil_div(a.N, kTile);
    a.tiles_r = (int)tiles_r;
    a.tiles_o = (int)tiles_o;
    // 8 wavefronts per CU (one workgroup, or two of 4), a multiple of the XCD count
    const unsigned wgs = (unsigned)max(1, cus / kXcds) * kXcds * (8 / kWavesPerWg);
    using Kernel = void (*)(const LinearArgs);
    static const Kernel kernels[2][2] = {{linear_e2m3_persistent<false, false>, linear_e2m3_persistent<false, true>},
                                         {linear_e2m3_persistent<true, false>, linear_e2m3_persistent<true, true>}};
    const Kernel kernel = kernels[a.bias ? 1 : 0][a.acc_out ? 1 : 0];
    if (int rc = ptq4vm::set_lds_limit(reinterpret_cast<const void *>(kernel), kPersistentLds, "hipFuncSetAttribute(linear_e2m3_persistent)")) return rc;
    kernel<<<dim3(wgs), dim3(kWavesPerWg * 64), kPersistentLds, stream>>>(a);
    return ptq4vm::check_launch("linear_e2m3_persistent");
}

int launch_generic(LinearArgs a, hipStream_t stream) {
    dim3 grid;
    if (!set_grid<64, 64>(a, grid)) return PTQ4VM_ERR_SHAPE;
    linear_e2m3_generic<<<grid, dim3(kThreads), 0, stream>>>(a);
    return ptq4vm::check_launch("linear_e2m3_generic");
}

}  // namespace
}  // namespace mfma
}  // namespace ptq4vm

extern "C" int ptq4vm_w4a4_linear_e2m3(const uint8_t *xq6, const uint8_t *wq6, const float *s_tok, const float *s_w,
                                       const void *bias_f16, void *y_f16, int32_t *acc_out, int64_t B, int64_t L,
                                       int64_t K, int64_t N, int64_t ldxq, int64_t ldwq, int64_t ldy, void *stream_) {
    using namespace ptq4vm::mfma;
    if (!xq6 || !wq6 || !s_tok || !s_w || !y_f16) return PTQ4VM_ERR_NULL;
    if (B < 0 || N < 0 || L <= 0 || K <= 0 || K > PTQ4VM_MAX_K_E2M3) return PTQ4VM_ERR_SHAPE;
    if (B > 0 && L > INT64_MAX / B) return PTQ4VM_ERR_SHAPE;
    const int64_t row_bytes = PTQ4VM_E2M3_BLOCKS(K) * kBlockBytes;
    // ldxq / ldwq: plane pitches of the block-major containers
    if ((B > 0 && ldxq / kBlockBytes < B * L) || ldwq / kBlockBytes < N || ldxq % 16 != 0 || ldwq % 16 != 0 || ldy < N)
        return PTQ4VM_ERR_STRIDE;
    if (!ptq4vm::aligned_to(xq6, 16) || !ptq4vm::aligned_to(wq6, 16) || !ptq4vm::aligned_to(y_f16, 2) ||
        !ptq4vm::aligned_to(s_tok, 4) || !ptq4vm::aligned_to(s_w, 4) || !ptq4vm::aligned_to(bias_f16, 2) ||
        !ptq4vm::aligned_to(acc_out, 4))
        return PTQ4VM_ERR_ALIGN;
    const int64_t M = B * L;
    if (M == 0 || N == 0) return PTQ4VM_OK;
    LinearArgs a{};
    a.x = reinterpret_cast<const char *>(xq6);
    a.w = reinterpret_cast<const char *>(wq6);
    a.s_tok = s_tok;
    a.s_w = s_w;
    a.bias = static_cast<const __half *>(bias_f16);
    a.y = static_cast<__half *>(y_f16);
    a.acc_out = acc_out;
    a.M = M;
    a.N = N;
    a.k_bytes = row_bytes;
    a.ldx_bytes = ldxq;
    a.ldw_bytes = ldwq;
    a.ldy = ldy;
    a.L = L;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const int64_t tiles = ptq4vm::ceil_div(M, 256) * ptq4vm::ceil_div(N, kTile);
    const bool persistent_ok = K % 128 == 0 && K >= 256 && N % 8 == 0 && ptq4vm::aligned_to(y_f16, 16) && ldy % 8 == 0 &&
                               ptq4vm::aligned_to(bias_f16, 4) &&
                               ldy * 2 * kTile < (1LL << 31) && L < (1LL << 31) && tiles >= 128 && tiles <= 0x3fffffffLL;
    if (persistent_ok) return launch_persistent(a, stream);
    return launch_generic(a, stream);
}
