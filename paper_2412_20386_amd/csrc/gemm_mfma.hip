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
// lane then holds one token row r and runs of four consecutive output channels, and the
// per-token step s_tok[r mod L] is one scalar per lane.
//
// Tiling: a workgroup of 4 wavefronts owns BR token rows x BO output channels; K is walked in
// slabs of 64 bytes.  LDS rows are 64 bytes with the 16-byte chunk index XOR-swizzled by the
// row.  Workgroup ids are remapped so that the tiles sharing one activation strip run on the
// same XCD (shared L2).  Two kernels share fragments, MFMA loop and epilogue:
//   linear_mfma_dma      fast path (16-byte aligned pitches, K bytes a multiple of 64): slabs are
//                        copied global -> LDS directly (global_load_lds_dwordx4), several slabs
//                        in flight in a ring of LDS stages, one s_barrier per slab and explicit
//                        s_waitcnt vmcnt so that younger slabs stay in flight across the barrier.
//   linear_mfma_generic  any pitch, alignment and K: register-staged loads with zero fill.
// The epilogue transposes each wavefront's results through a private LDS patch so that global
// stores are 16 bytes per lane and cover whole contiguous row segments.
#include "mfma_linear.hpp"

#ifndef PTQ4VM_PERSISTENT_BO
#define PTQ4VM_PERSISTENT_BO 256
#endif
#ifndef PTQ4VM_PERSISTENT_PHYS_SLAB
#define PTQ4VM_PERSISTENT_PHYS_SLAB 128  // K bytes per LDS row of a ring stage (64: twice the stages in the same LDS)
#define PTQ4VM_PERSISTENT_STAGES 2
#endif
#ifndef PTQ4VM_STREAM_SMALLK
#define PTQ4VM_STREAM_SMALLK 1
#endif

namespace {

using namespace ptq4vm::mfma;

// ------------------------------------------------------------------------------------------
// Fast path: direct global -> LDS copies, STAGES-deep ring.
// Requirements (checked on the host): k_bytes % 64 == 0, pitches and bases 16-byte aligned,
// 256 * pitch below 2^31.
// A wavefront copies 1 KiB blocks (16 rows x 64 bytes): the LDS side of the copy is linear in the
// lane index, so the swizzle is applied by choosing which global chunk each lane fetches.  Rows
// beyond M or N are clamped to the last valid row; their results are never stored.
// ------------------------------------------------------------------------------------------
template <class Path, int BR, int BO, int WR, int WO, int STAGES>
__global__ __launch_bounds__(kThreads, 2) void linear_mfma_dma(const LinearArgs p) {
    static_assert(WR * WO == kWaves, "four wavefronts per workgroup");
    constexpr int WAVE_R = BR / WR, WAVE_O = BO / WO;
    constexpr int FR = WAVE_R / 32, FO = WAVE_O / 32;
    static_assert(WAVE_R % 32 == 0 && WAVE_O % 32 == 0, "wave tile must be whole MFMA blocks");
    static_assert(BR % 64 == 0 && BO % 64 == 0, "each wavefront copies whole 16-row blocks");
    constexpr int X_BLOCKS = BR / 16 / kWaves, W_BLOCKS = BO / 16 / kWaves;  // 1 KiB copies per wave per slab
    constexpr int LOADS_PER_SLAB = X_BLOCKS + W_BLOCKS;
    constexpr int STAGE_BYTES = (BR + BO) * kSlabBytes;
    static_assert((STAGES - 2) * LOADS_PER_SLAB <= 63, "vmcnt is a 6-bit counter");
    static_assert(BR * BO * 2 <= STAGES * STAGE_BYTES, "the output tile must fit the LDS ring for the epilogue");
    using Acc = typename Path::Acc;

    int tile_r, tile_o;
    if (!tile_of_block(p, tile_r, tile_o)) return;
    const int64_t r0 = (int64_t)tile_r * BR, o0 = (int64_t)tile_o * BO;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_r = (wave / WO) * WAVE_R, wave_o = (wave % WO) * WAVE_O;
    const int l32 = lane & 31, lhalf = lane >> 5;

    // Per-lane source offsets (bytes from the tile's first row, slab 0) of the copies.
    const char *x_tile = p.x + r0 * p.ldx_bytes;
    const char *w_tile = p.w + o0 * p.ldw_bytes;
    const int rows_x = (int)min((int64_t)BR, p.M - r0), rows_w = (int)min((int64_t)BO, p.N - o0);
    uint32_t x_off[X_BLOCKS], w_off[W_BLOCKS];
#pragma unroll
    for (int i = 0; i < X_BLOCKS; i++) {
        const int row = (wave + kWaves * i) * 16 + (lane >> 2);
        const int kc = (lane & 3) ^ swizzle(row);
        x_off[i] = (uint32_t)min(row, rows_x - 1) * (uint32_t)p.ldx_bytes + kc * 16;
    }
#pragma unroll
    for (int i = 0; i < W_BLOCKS; i++) {
        const int row = (wave + kWaves * i) * 16 + (lane >> 2);
        const int kc = (lane & 3) ^ swizzle(row);
        w_off[i] = (uint32_t)min(row, rows_w - 1) * (uint32_t)p.ldw_bytes + kc * 16;
    }
    auto issue = [&](int slab, int stage) {
        char *sx = lds_dyn + stage * STAGE_BYTES;
        char *sw = sx + BR * kSlabBytes;
        const char *gx = x_tile + (int64_t)slab * kSlabBytes;
        const char *gw = w_tile + (int64_t)slab * kSlabBytes;
#pragma unroll
        for (int i = 0; i < X_BLOCKS; i++)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(gx + x_off[i]),
                                             (__attribute__((address_space(3))) void *)(sx + (wave + kWaves * i) * 1024),
                                             16, 0, 0);
#pragma unroll
        for (int i = 0; i < W_BLOCKS; i++)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(gw + w_off[i]),
                                             (__attribute__((address_space(3))) void *)(sw + (wave + kWaves * i) * 1024),
                                             16, 0, 0);
    };

    Acc acc[FO][FR];
#pragma unroll
    for (int i = 0; i < FO; i++)
#pragma unroll
        for (int j = 0; j < FR; j++)
#pragma unroll
            for (int v = 0; v < 16; v++) acc[i][j][v] = 0;

    const int n_slabs = (int)(p.k_bytes / kSlabBytes);
#pragma unroll
    for (int s = 0; s < STAGES - 1; s++)
        if (s < n_slabs) issue(s, s);

    int stage = 0;
    for (int it = 0; it < n_slabs; it++) {
        // Slab `it` must have landed; up to STAGES-2 younger slabs may stay in flight.
        // s_waitcnt immediate on gfx9: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] << 14.
        constexpr int KEEP = (STAGES - 2) * LOADS_PER_SLAB;
        if (it + STAGES - 2 < n_slabs)
            __builtin_amdgcn_s_waitcnt(0x0F70 | (KEEP & 15) | ((KEEP >> 4) << 14));
        else
            __builtin_amdgcn_s_waitcnt(0x0F70);
        __builtin_amdgcn_s_barrier();  // everyone's copies of slab `it` are visible; slab it-1 is fully consumed
        int refill = stage + STAGES - 1;
        if (refill >= STAGES) refill -= STAGES;
        if (it + STAGES - 1 < n_slabs) issue(it + STAGES - 1, refill);
        const char *sx = lds_dyn + stage * STAGE_BYTES;
        mfma_slab<Path, FO, FR>(acc, sx + wave_r * kSlabBytes, sx + (BR + wave_o) * kSlabBytes, l32, lhalf);
        if (++stage == STAGES) stage = 0;
    }
    __syncthreads();  // all MFMA reads of LDS are done: the ring becomes the epilogue patches
    epilogue<Path, FO, FR, FR>(acc, p, lds_dyn + wave * (WAVE_R * WAVE_O * 2), r0 + wave_r, o0 + wave_o, lane);
}

// ------------------------------------------------------------------------------------------
// Large-problem path: persistent workgroups, one per CU, 8 wavefronts on a 256 x 256 tile
// (wave tile 128 token rows x 64 channels), LDS ring fed by direct global -> LDS copies.
// Compared with linear_mfma_dma:
//   * the 256 x 256 tile halves the L2 -> LDS traffic per MAC (the 256 x 128 tile needs more
//     L2 bandwidth than the chip has once the MFMA pipes are kept busy); with SLAB = 128 every
//     copied row segment is a whole 128-byte cache line (measured: 64-byte segments cap the
//     L2 -> LDS path at ~16 TB/s, 128-byte ones reach 22 TB/s and more);
//   * the slab pipeline never drains: a workgroup walks its tiles in a loop and the copies for
//     the next tile's first slabs are issued during the current tile's last slabs and epilogue;
//   * the MFMA is v_mfma_i32_16x16x64_i8 (v_mfma_f32_16x16x32_f16 on the fp16 path): with random
//     operand bytes it sustains ~18 % more than the 32x32x32 form on this part (3.5 vs 3.0 POP/s in
//     an isolated LDS-fed loop; the matrix pipes are clock/power limited once operands toggle),
//     for the same LDS traffic per MAC;
//   * MFMA fragments are double buffered in registers: the LDS reads of k-step n+1 are issued
//     before the MFMAs of k-step n, so LDS latency hides behind the matrix pipe even though all
//     wavefronts of the workgroup run in lock step;
//   * per-tile scale vectors (s_w, bias, s_tok[r mod L]) are copied into LDS by the same
//     asynchronous path at the start of a tile (double buffered), so the epilogue issues no
//     register loads and never forces the in-flight slabs to land early;
//   * the epilogue stages fp16 results in the ring stage that was consumed last (free until
//     the next refill), index arithmetic is 32-bit and tile-relative, full tiles take a
//     branch-free path.
// Ring discipline: barrier B(g) sits before the MFMAs of the LAST k-step of slab g-1, after the
// fragments of that k-step have arrived in registers.  Passing it means (a) every wavefront's
// copies of slab g have landed (each waited on its own vmcnt first) and (b) nobody will read slab
// g-1's stage again, so that stage is refilled at once with slab g-1+STAGES (after a tile's last
// slab the refill waits until the epilogue, which borrows the stage, has finished).
// Requirements (host-checked): as linear_mfma_dma, plus k_bytes % SLAB == 0, k_bytes >= 2 SLAB,
// N % 8 == 0, 16-byte aligned y pitch, 4-byte aligned bias, 256 * ldy * 2 < 2^31, L < 2^31.
// ------------------------------------------------------------------------------------------
// The tiles `first`, `first + stride`, ... (n_my of them) of the grid of (32 FR)-row x BO-channel
// tiles, channel tiles fastest, processed by the whole workgroup.  FR = 8: 256-row tiles; FR = 4:
// 128-row half tiles (used to spread a last, partial round of tiles over idle workgroups).
template <class Path, int BO, int SLAB, int STAGES, bool HAS_BIAS, bool DUMP_ACC, int FR>
__device__ __forceinline__ void persistent_tiles(const LinearArgs &p, const int first, const int stride,
                                                 const int n_my) {
    // (32 FR) x 256 tile on 8 wavefronts (one workgroup per CU) or (32 FR) x 128 on 4 (two per CU)
    constexpr int BR = 32 * FR, WO = BO / 64, NW = 2 * WO;
    constexpr int WAVE_R = 16 * FR, WAVE_O = 64;
    constexpr int FO = WAVE_O / 16;  // 16 x 16 MFMA blocks of the wave tile: FO x FR
    static_assert(FR == 8 || FR == 4, "wave tile height");
    static_assert(BO == 256 || BO == 128, "tile width");
    constexpr int KS = SLAB / 64;             // MFMA k-steps (64 bytes of K each) per slab
    constexpr int CHUNKS = SLAB / 16;         // 16-byte chunks per LDS row
    constexpr int ROWS_PER_COPY = 64 / CHUNKS;  // rows in one wavefront-wide 1 KiB copy
    constexpr int X_COPIES = BR / ROWS_PER_COPY / NW, W_COPIES = BO / ROWS_PER_COPY / NW;
    constexpr int LOADS_PER_SLAB = X_COPIES + W_COPIES;
    constexpr int STAGE_BYTES = (BR + BO) * SLAB;
    constexpr int KEEP = (STAGES - 2) * LOADS_PER_SLAB;  // copies allowed in flight when a slab is needed
    static_assert(SLAB == 64 || SLAB == 128, "LDS rows hold 64 or 128 bytes of K");
    static_assert(NW * 32 * WAVE_O * 2 <= STAGE_BYTES, "epilogue patches must fit one stage");
    constexpr bool kInt8 = Path::kElemBytes == 1;
    using Acc = typename Path::Acc16;

    char *const ring = lds_dyn;
    // per-tile scale vectors, double buffered by tile parity
    constexpr int SCALE_BYTES = BO * 4 + BR * 4 + BO * 2 + (Path::kOffset ? BO * 4 + BR * 4 : 0);
    char *const scales = lds_dyn + STAGES * STAGE_BYTES;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_r = (wave / WO) * WAVE_R, wave_o = (wave % WO) * WAVE_O;
    const int l16 = lane & 15, lq = lane >> 4;
    auto lds_chunk = [&](int row, int chunk) {  // byte offset of a 16-byte chunk inside a stage half
        return row * SLAB + ((chunk ^ (SLAB == 64 ? swizzle(row) : (row & 7))) << 4);
    };

    const int wgs_per_xcd = stride, last = first + n_my * stride;
    const int n_slabs = (int)(p.k_bytes / SLAB);
    const int total_slabs = n_my * n_slabs;
    if (total_slabs == 0) return;

    // ---- producer: the next slab to copy, possibly of a later tile than the one being computed
    int pf_tile = first, pf_slab = 0, pf_stage = 0, issued = 0;
    const char *pf_x = nullptr, *pf_w = nullptr;
    uint32_t x_off[X_COPIES], w_off[W_COPIES];
    auto pf_setup = [&]() {
        const int to = pf_tile % p.tiles_o, tr = pf_tile / p.tiles_o;
        const int64_t r0 = (int64_t)tr * BR, o0 = (int64_t)to * BO;
        pf_x = p.x + r0 * p.ldx_bytes;
        pf_w = p.w + o0 * p.ldw_bytes;
        const int rows_x = (int)min((int64_t)BR, p.M - r0), rows_w = (int)min((int64_t)BO, p.N - o0);
#pragma unroll
        for (int i = 0; i < X_COPIES; i++) {
            const int row = (wave + NW * i) * ROWS_PER_COPY + lane / CHUNKS;
            const int chunk = (lane % CHUNKS) ^ (SLAB == 64 ? swizzle(row) : (row & 7));
            x_off[i] = (uint32_t)min(row, rows_x - 1) * (uint32_t)p.ldx_bytes + chunk * 16;
        }
#pragma unroll
        for (int i = 0; i < W_COPIES; i++) {
            const int row = (wave + NW * i) * ROWS_PER_COPY + lane / CHUNKS;
            const int chunk = (lane % CHUNKS) ^ (SLAB == 64 ? swizzle(row) : (row & 7));
            w_off[i] = (uint32_t)min(row, rows_w - 1) * (uint32_t)p.ldw_bytes + chunk * 16;
        }
    };
    auto issue = [&]() {  // copy the producer's slab into ring stage pf_stage, then advance
        char *sx = ring + pf_stage * STAGE_BYTES;
        char *sw = sx + BR * SLAB;
        const char *gx = pf_x + (int64_t)pf_slab * SLAB;
        const char *gw = pf_w + (int64_t)pf_slab * SLAB;
#pragma unroll
        for (int i = 0; i < X_COPIES; i++)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(gx + x_off[i]),
                                             (__attribute__((address_space(3))) void *)(sx + (wave + NW * i) * 1024),
                                             16, 0, 0);
#pragma unroll
        for (int i = 0; i < W_COPIES; i++)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(gw + w_off[i]),
                                             (__attribute__((address_space(3))) void *)(sw + (wave + NW * i) * 1024),
                                             16, 0, 0);
        issued++;
        if (++pf_stage == STAGES) pf_stage = 0;
        if (++pf_slab == n_slabs) {
            pf_slab = 0;
            pf_tile += wgs_per_xcd;
            if (pf_tile < last) pf_setup();
        }
    };
    // Slab g has landed for this wavefront once at most `younger` of its copies are outstanding.
    auto wait_slab = [&](int g) {
        if (g + STAGES - 2 < total_slabs)
            wait_vmcnt_at_most<KEEP>();
        else
            wait_vmcnt_at_most<0>();
    };

    pf_setup();
    while (issued < STAGES - 1 && issued < total_slabs) issue();
    wait_slab(0);
    __builtin_amdgcn_s_barrier();  // B(0)
    if (issued < total_slabs) issue();

    int stage = 0, g = 0, parity = 0;  // consumer: ring stage, running slab number, scale buffer
    for (int tile = first; tile < last; tile += wgs_per_xcd, parity ^= 1) {
        const int tile_o = tile % p.tiles_o, tile_r = tile / p.tiles_o;
        const int64_t r0 = (int64_t)tile_r * BR, o0 = (int64_t)tile_o * BO;
        const int rows_valid = (int)min((int64_t)BR, p.M - r0), cols_valid = (int)min((int64_t)BO, p.N - o0);
        float *const cs_lds = reinterpret_cast<float *>(scales + parity * SCALE_BYTES);  // s_w of the tile's channels
        float *const rs_lds = cs_lds + BO;                                              // s_tok of the tile's rows
        uint32_t *const cb_lds = reinterpret_cast<uint32_t *>(rs_lds + BR);             // bias, two fp16 per word
        int *const cz_lds = reinterpret_cast<int *>(cb_lds + BO / 2);                   // rowsum of the tile's channels
        int *const rz_lds = cz_lds + BO;                                                // z_tok of the tile's rows

        // Scale vectors of this tile, one 4-byte element per lane, straight into LDS.  Indices
        // beyond the matrix are clamped; those rows / channels are never stored.
        constexpr int kScaleTasks = BO / 64 + BR / 64 + BO / 128;
        constexpr int kOffsetTasks = Path::kOffset ? BO / 64 + BR / 64 : 0;
#pragma unroll
        for (int task = kScaleTasks; task < kScaleTasks + kOffsetTasks; task++) {
            if (task % NW != wave) continue;
            if constexpr (Path::kOffset) {
                const int blk = task - kScaleTasks;
                if (blk < BO / 64) {  // rowsum of 64 channels
                    const int c = min(blk * 64 + lane, cols_valid - 1);
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(p.rowsum + o0 + c),
                                                     (__attribute__((address_space(3))) void *)(cz_lds + blk * 64), 4, 0, 0);
                } else {  // z_tok of 64 rows
                    const int rblk = blk - BO / 64;
                    const int r = min(rblk * 64 + lane, rows_valid - 1);
                    const uint32_t t = ((uint32_t)(r0 % p.L) + (uint32_t)r) % (uint32_t)p.L;
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(p.z_tok + t),
                                                     (__attribute__((address_space(3))) void *)(rz_lds + rblk * 64), 4, 0, 0);
                }
            }
        }
#pragma unroll
        for (int task = 0; task < kScaleTasks; task++) {
            if (task % NW != wave) continue;  // the copies are dealt round-robin to the wavefronts
            if (task < BO / 64) {             // s_w of 64 channels
                if constexpr (kInt8) {
                    const int c = min(task * 64 + lane, cols_valid - 1);
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(p.s_w + o0 + c),
                                                     (__attribute__((address_space(3))) void *)(cs_lds + task * 64), 4, 0, 0);
                }
            } else if (task < BO / 64 + BR / 64) {  // s_tok of 64 rows
                if constexpr (kInt8) {
                    const int blk = task - BO / 64;
                    const int r = min(blk * 64 + lane, rows_valid - 1);
                    const uint32_t t = ((uint32_t)(r0 % p.L) + (uint32_t)r) % (uint32_t)p.L;
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(p.s_tok + t),
                                                     (__attribute__((address_space(3))) void *)(rs_lds + blk * 64), 4, 0, 0);
                }
            } else {  // bias of 128 channels, two fp16 per lane
                if constexpr (HAS_BIAS) {
                    const int blk = task - BO / 64 - BR / 64;
                    const int c2 = min(blk * 64 + lane, cols_valid / 2 - 1);
                    __builtin_amdgcn_global_load_lds(
                        (const __attribute__((address_space(1))) void *)(reinterpret_cast<const uint32_t *>(p.bias + o0) + c2),
                        (__attribute__((address_space(3))) void *)(cb_lds + blk * 64), 4, 0, 0);
                }
            }
        }
        int loads_after_scales = 0;

        Acc acc[FO][FR];
#pragma unroll
        for (int i = 0; i < FO; i++)
#pragma unroll
            for (int j = 0; j < FR; j++)
#pragma unroll
                for (int v = 0; v < 4; v++) acc[i][j][v] = 0;

        // Weight fragments are double buffered; an activation fragment is dead after its FO MFMAs
        // of a k-step, so the next k-step's fragment is fetched into the same registers right then.
        v4i fw[2][FO], fx[FR];
        auto load_fw = [&](int buf, int stg, int ks) {
            const char *sw = ring + stg * STAGE_BYTES + (BR + wave_o) * SLAB;
#pragma unroll
            for (int i = 0; i < FO; i++) fw[buf][i] = *reinterpret_cast<const v4i *>(sw + lds_chunk(i * 16 + l16, 4 * ks + lq));
        };
        auto load_fx = [&](int j, int stg, int ks) {
            const char *sx = ring + stg * STAGE_BYTES + wave_r * SLAB;
            fx[j] = *reinterpret_cast<const v4i *>(sx + lds_chunk(j * 16 + l16, 4 * ks + lq));
        };

        load_fw(0, stage, 0);  // B(g) for the tile's first slab was passed during the previous tile
#pragma unroll
        for (int j = 0; j < FR; j++) load_fx(j, stage, 0);
        // U slabs per trip of the loop, so that the register buffer of the weight fragments, which
        // alternates per k-step, starts every trip (and every tile) at buffer 0.
        constexpr int U = (KS % 2 == 0) ? 1 : 2;
        for (int s0 = 0; s0 < n_slabs; s0 += U)
#pragma unroll
        for (int h = 0; h < U; h++, g++) {
            const int s = s0 + h;
            int next_stage = stage + 1;
            if (next_stage == STAGES) next_stage = 0;
#pragma unroll
            for (int ks = 0; ks < KS; ks++) {
                const int cur = (h * KS + ks) & 1;
                bool has_next = false;
                int nstg = stage, nks = ks + 1;
                if (ks + 1 < KS) {
                    has_next = true;
                } else if (g + 1 < total_slabs) {
                    // B(g+1): this wavefront holds the last fragments of slab g in registers and its
                    // copies of slab g+1 have landed.
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                    wait_slab(g + 1);
                    __builtin_amdgcn_s_barrier();
                    if (s + 1 < n_slabs) {
                        if (issued < total_slabs) {
                            issue();  // refills the stage of slab g
                            loads_after_scales += LOADS_PER_SLAB;
                        }
                        has_next = true, nstg = next_stage, nks = 0;
                    }  // after the tile's last slab that stage first serves the epilogue
                }
                if constexpr (Path::kPacked4) {
                    // a packed 16-byte fragment is two MFMA operands: even and odd reduction indices
                    v4i we[FO], wo[FO];
#pragma unroll
                    for (int i = 0; i < FO; i++) we[i] = Path::even_codes(fw[cur][i]), wo[i] = Path::odd_codes(fw[cur][i]);
                    if (has_next) load_fw(cur ^ 1, nstg, nks);
#pragma unroll
                    for (int j = 0; j < FR; j++) {
                        const v4i xe = Path::even_codes(fx[j]), xo = Path::odd_codes(fx[j]);
                        if (has_next) load_fx(j, nstg, nks);
#pragma unroll
                        for (int i = 0; i < FO; i++) acc[i][j] = Path::mfma16(we[i], xe, acc[i][j]);
#pragma unroll
                        for (int i = 0; i < FO; i++) acc[i][j] = Path::mfma16(wo[i], xo, acc[i][j]);
                    }
                } else {
                    if (has_next) load_fw(cur ^ 1, nstg, nks);
#pragma unroll
                    for (int j = 0; j < FR; j++) {
#pragma unroll
                        for (int i = 0; i < FO; i++) acc[i][j] = Path::mfma16(fw[cur][i], fx[j], acc[i][j]);
                        if (has_next) load_fx(j, nstg, nks);
                    }
                }
            }
            stage = next_stage;
        }

        // ---- epilogue of this tile.  The ring stage of the tile's last slab is free: B(g) was passed
        // with that slab's fragments in registers and its refill has been held back; it holds the
        // wavefronts' fp16 patches until the barrier that ends the epilogue.
        if (loads_after_scales >= KEEP && KEEP > 0)
            wait_vmcnt_at_most<KEEP>();
        else
            wait_vmcnt_at_most<0>();
        __builtin_amdgcn_s_barrier();  // scale vectors are visible to every wavefront
        const int free_stage = stage == 0 ? STAGES - 1 : stage - 1;  // stage of the tile's last slab
        char *patch = ring + free_stage * STAGE_BYTES + wave * (32 * WAVE_O * 2);
        char *y_tile = reinterpret_cast<char *>(p.y + r0 * p.ldy + o0);
        const uint32_t ldy_bytes = (uint32_t)p.ldy * 2;
        auto patch_chunk = [&](int row, int chunk) { return row * (WAVE_O * 2) + ((chunk ^ (row & 7)) << 4); };
        const bool full_tile = rows_valid == BR && cols_valid == BO;

        // Accumulator register v of block (i, j):  token row 16 j + (lane mod 16),
        // channel 16 i + 4 (lane / 16) + v.  Column scales / biases of this lane's 16 channels
        // (cb_raw[i] holds the eight fp16 biases around them), row scales of its 8 rows.
        v4f cs_raw[4], cb_raw[4];
        float rs_raw[8];
        if constexpr (kInt8) lds_read_4x_b128<64>(lds_addr(cs_lds + wave_o + lq * 4), cs_raw);
        if constexpr (HAS_BIAS) lds_read_4x_b128<32>(lds_addr(cb_lds + (wave_o + (lq >> 1) * 8) / 2), cb_raw);
        if constexpr (kInt8) {
            if constexpr (FR == 8) {
                lds_read_8x_b32<64>(lds_addr(rs_lds + wave_r + l16), rs_raw);
            } else {
                float half_rs[4];
                lds_read_4x_b32<64>(lds_addr(rs_lds + wave_r + l16), half_rs);
#pragma unroll
                for (int j = 0; j < 4; j++) rs_raw[j] = half_rs[j];
            }
        }
        v4f cz_raw[4];   // rowsum of the lane's channels and z_tok of its rows (zero-offset path), as raw bits
        float rz_raw[8];
        if constexpr (Path::kOffset) {
            lds_read_4x_b128<64>(lds_addr(cz_lds + wave_o + lq * 4), cz_raw);
            if constexpr (FR == 8) {
                lds_read_8x_b32<64>(lds_addr(rz_lds + wave_r + l16), rz_raw);
            } else {
                float half_rz[4];
                lds_read_4x_b32<64>(lds_addr(rz_lds + wave_r + l16), half_rz);
#pragma unroll
                for (int j = 0; j < 4; j++) rz_raw[j] = half_rz[j];
            }
        }
        float bias4[FO][4];
#pragma unroll
        for (int i = 0; i < FO; i++) {
#pragma unroll
            for (int c = 0; c < 4; c++) bias4[i][c] = 0.0f;
            if constexpr (HAS_BIAS) {
                const float w01 = (lq & 1) ? cb_raw[i].z : cb_raw[i].x, w23 = (lq & 1) ? cb_raw[i].w : cb_raw[i].y;
                const __half2 b01 = __builtin_bit_cast(__half2, w01), b23 = __builtin_bit_cast(__half2, w23);
                bias4[i][0] = __low2float(b01), bias4[i][1] = __high2float(b01);
                bias4[i][2] = __low2float(b23), bias4[i][3] = __high2float(b23);
            }
        }

#pragma unroll
        for (int jp = 0; jp < FR / 2; jp++) {  // 32 rows per round through the patch
#pragma unroll
            for (int jj = 0; jj < 2; jj++) {
                const int j = 2 * jp + jj;
#pragma unroll
                for (int i = 0; i < FO; i++) {
                    float out[4];
#pragma unroll
                    for (int c = 0; c < 4; c++) {
                        if constexpr (kInt8) {
                            int a = acc[i][j][c];
                            if constexpr (Path::kPacked4) a >>= 8;  // operands were codes times 16: exact
                            if constexpr (DUMP_ACC) {
                                const int64_t r = r0 + wave_r + j * 16 + l16;
                                const int64_t o = o0 + wave_o + i * 16 + lq * 4 + c;
                                if (r < p.M && o < p.N) p.acc_out[r * p.N + o] = a;
                            }
                            if constexpr (Path::kOffset) {
                                const float zf = rz_raw[j], sf = cz_raw[i][c];  // scalars first: bit casts of vector elements misread
                                a -= __mul24(__builtin_bit_cast(int, zf), __builtin_bit_cast(int, sf));  // |z| < 2^8, |rowsum| < 2^23
                            }
                            out[c] = (float)a * (rs_raw[j] * cs_raw[i][c]) + bias4[i][c];
                        } else {
                            out[c] = acc[i][j][c] + bias4[i][c];
                        }
                    }
                    __half2 lo = __floats2half2_rn(out[0], out[1]);
                    __half2 hi = __floats2half2_rn(out[2], out[3]);
                    u32x2 packed = {__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi)};
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
            if (full_tile) {
#pragma unroll
                for (int q = 0; q < 4; q++)
                    // non-temporal: measured 4-8 % faster than write-back stores here
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
        if (issued < total_slabs) issue();
    }
}

// Work split.  Workgroup ids go round-robin over the XCDs; XCD x owns a contiguous range of tiles
// (channel tiles fastest, so tiles sharing an activation strip share one L2) and its workgroups
// interleave in it.  FRM = 8: 256-row tiles.  A range is whole rounds of tiles plus a partial last
// round; when that round has at most half as many tiles as the XCD has workgroups, its tiles are cut
// into two 128-row halves, which twice as many workgroups take BEFORE their whole tiles (Vim-B
// out_proj: 2.31 rounds -> 1/2 + 2 instead of 3, measured 81 -> 70 us).  A half-tile pass costs ~0.7
// of a tile (its own slab pipeline, more LDS traffic per MAC); doing it first also moves those
// workgroups' epilogues out of step with the others' (in_proj, 9.23 rounds: 149.4 -> 146.9 us; with
// the halves last it gained nothing there).  FRM = 4: every tile has 128 rows (packed 4-bit operands,
// whose expanded fragments would not fit the register file next to a 256-row tile's accumulators).
template <class Path, int BO, int SLAB, int STAGES, bool HAS_BIAS, bool DUMP_ACC, int FRM>
__global__ __launch_bounds__(BO * 2, 2) void linear_mfma_persistent(const LinearArgs p) {
    const int total_tiles = p.tiles_o * p.tiles_r;
    const int per_xcd = (total_tiles + kXcds - 1) / kXcds;
    const int wpx = (int)gridDim.x / kXcds, xcd = (int)(blockIdx.x % kXcds), j = (int)(blockIdx.x / kXcds);
    const int lo = xcd * per_xcd, hi = min(lo + per_xcd, total_tiles);
    const int n = max(hi - lo, 0);
    const int rounds = n / wpx, tail = n - rounds * wpx;
    if constexpr (FRM == 8) {
        const bool halves = tail > 0 && 2 * tail <= wpx;
        const int n_full = rounds + ((!halves && j < tail) ? 1 : 0);
        if (halves && j < 2 * tail) {
            const int tile = lo + rounds * wpx + (j >> 1);
            const int half_tile = ((tile / p.tiles_o) * 2 + (j & 1)) * p.tiles_o + tile % p.tiles_o;  // in the 128-row grid
            if ((int64_t)(half_tile / p.tiles_o) * 128 < p.M) {
                persistent_tiles<Path, BO, SLAB, STAGES, HAS_BIAS, DUMP_ACC, 4>(p, half_tile, 1, 1);
                __syncthreads();  // the ring and the scale buffers change layout
            }
        }
        persistent_tiles<Path, BO, SLAB, STAGES, HAS_BIAS, DUMP_ACC, 8>(p, lo + j, wpx, n_full);
    } else {
        persistent_tiles<Path, BO, SLAB, STAGES, HAS_BIAS, DUMP_ACC, 4>(p, lo + j, wpx, rounds + (j < tail ? 1 : 0));
    }
}

// ------------------------------------------------------------------------------------------
// Small-K path (K bytes <= 128, e.g. dt_proj with K = dt_rank): the whole reduction is 1-4 MFMA
// k-steps, so the kernel is a stream of output rows bound by the fp16 stores.  A wavefront owns
// 64 output channels for its whole life and keeps their weight fragments, scales and biases in
// registers; it walks over 32-row blocks, fetching the activation fragments straight from
// global memory (no LDS staging of operands), and transposes results through a private LDS
// patch so that every store instruction writes eight whole 128-byte row segments.
// LOAD_ALIGN 16: pitches and bases are multiples of 16 bytes; 4: multiples of 4 bytes.
// ------------------------------------------------------------------------------------------
template <int LOAD_ALIGN>
__device__ __forceinline__ v4i load_fragment_chunk(const char *row_ptr, int kb, int k_bytes) {
    v4i out = {0, 0, 0, 0};
    if (kb >= k_bytes) return out;
    const int valid = min(16, k_bytes - kb);
    if constexpr (LOAD_ALIGN == 16) {
        out = *reinterpret_cast<const v4i *>(row_ptr + kb);
    } else {
#pragma unroll
        for (int j = 0; j < 4; j++)
            if (4 * j < valid) out[j] = *reinterpret_cast<const int *>(row_ptr + kb + 4 * j);
    }
    if (valid < 16) {
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const int nb = valid - 4 * j;
            out[j] = nb >= 4 ? out[j] : (nb <= 0 ? 0 : (out[j] & ((1 << (8 * nb)) - 1)));
        }
    }
    return out;
}

template <class Path, int KSTEPS, int LOAD_ALIGN, bool HAS_BIAS, bool DUMP_ACC>
__global__ __launch_bounds__(kThreads) void linear_mfma_smallk(const LinearArgs p) {
    constexpr bool kInt8 = Path::kElemBytes == 1;
    using Acc = typename Path::Acc;
    __shared__ __attribute__((aligned(16))) char patches[kWaves][32 * 64 * 2];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, lhalf = lane >> 5;
    const int k_bytes = (int)p.k_bytes;
    const int64_t o_base = ((int64_t)blockIdx.y * kWaves + wave) * 64;
    if (o_base >= p.N) return;  // whole wavefront out of range; no barriers are used below
    const int cols_valid = (int)min((int64_t)64, p.N - o_base);

    // weight fragments of the strip's 64 channels: block i covers channels 32 i .. 32 i + 31
    v4i fw[2][KSTEPS];
#pragma unroll
    for (int i = 0; i < 2; i++) {
        const int row = min(i * 32 + l32, cols_valid - 1);  // clamped rows are never stored
        const char *wrow = p.w + (o_base + row) * p.ldw_bytes;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ks++) fw[i][ks] = load_fragment_chunk<LOAD_ALIGN>(wrow, (2 * ks + lhalf) * 16, k_bytes);
    }
    // packed 4-bit codes: the resident weight fragments are split once into their even / odd operands
    v4i fw_odd[2][Path::kPacked4 ? KSTEPS : 1];
    if constexpr (Path::kPacked4) {
#pragma unroll
        for (int i = 0; i < 2; i++)
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ks++) {
                fw_odd[i][ks] = Path::odd_codes(fw[i][ks]);
                fw[i][ks] = Path::even_codes(fw[i][ks]);
            }
    }
    // scales and biases of this lane's channels: o_base + 32 i + 8 g + 4 lhalf + c
    float cs[2][4][4], cb[2][4][4];
    int cz[2][4][Path::kOffset ? 4 : 1];  // their weight row sums (zero-offset path)
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
        for (int g = 0; g < 4; g++)
#pragma unroll
            for (int c = 0; c < 4; c++) {
                const int col = min(i * 32 + g * 8 + lhalf * 4 + c, cols_valid - 1);
                cs[i][g][c] = 1.0f;
                if constexpr (kInt8) cs[i][g][c] = p.s_w[o_base + col];
                cb[i][g][c] = 0.0f;
                if constexpr (HAS_BIAS) cb[i][g][c] = __half2float(p.bias[o_base + col]);
                if constexpr (Path::kOffset) cz[i][g][c] = p.rowsum[o_base + col];
            }

    const int64_t n_blocks = (p.M + 31) / 32;
    int64_t rb = blockIdx.x;
    uint32_t t = 0, t_step = 0;
    if constexpr (kInt8) {
        t = (uint32_t)((rb * 32 + l32) % p.L);
        t_step = (uint32_t)(((int64_t)gridDim.x * 32) % p.L);
    }
    auto load_x = [&](int64_t block, v4i (&fx)[KSTEPS]) {
        const int64_t row = min(block * 32 + l32, p.M - 1);
        const char *xrow = p.x + row * p.ldx_bytes;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ks++) fx[ks] = load_fragment_chunk<LOAD_ALIGN>(xrow, (2 * ks + lhalf) * 16, k_bytes);
    };
    char *patch = patches[wave];
    auto patch_chunk = [&](int row, int chunk) { return row * 128 + ((chunk ^ (row & 7)) << 4); };
    const bool y_fast = p.y_vec == 8 && cols_valid == 64;

    v4i fx[KSTEPS], fx_next[KSTEPS];
    if (rb < n_blocks) load_x(rb, fx);
    for (; rb < n_blocks; rb += gridDim.x) {
        const int64_t nb = rb + gridDim.x;
        if (nb < n_blocks) load_x(nb, fx_next);  // in flight while this block is computed and stored
        Acc acc[2];
#pragma unroll
        for (int i = 0; i < 2; i++) {
#pragma unroll
            for (int v = 0; v < 16; v++) acc[i][v] = 0;
        }
        if constexpr (Path::kPacked4) {
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ks++) {
                const v4i xe = Path::even_codes(fx[ks]), xo = Path::odd_codes(fx[ks]);
#pragma unroll
                for (int i = 0; i < 2; i++) acc[i] = Path::mfma(fw[i][ks], xe, acc[i]);
#pragma unroll
                for (int i = 0; i < 2; i++) acc[i] = Path::mfma(fw_odd[i][ks], xo, acc[i]);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 2; i++)
#pragma unroll
                for (int ks = 0; ks < KSTEPS; ks++) acc[i] = Path::mfma(fw[i][ks], fx[ks], acc[i]);
        }
        float rs = 1.0f;
        int rz = 0;
        if constexpr (kInt8) {
            rs = p.s_tok[t];
            if constexpr (Path::kOffset) rz = p.z_tok[t];
            t += t_step;
            if (t >= (uint32_t)p.L) t -= (uint32_t)p.L;
        }
        const int64_t r = rb * 32 + l32;
#pragma unroll
        for (int i = 0; i < 2; i++)
#pragma unroll
            for (int g = 0; g < 4; g++) {
                float out[4];
#pragma unroll
                for (int c = 0; c < 4; c++) {
                    if constexpr (kInt8) {
                        int a = acc[i][g * 4 + c];
                        if constexpr (Path::kPacked4) a >>= 8;  // operands were codes times 16: exact
                        if constexpr (DUMP_ACC) {
                            const int col = i * 32 + g * 8 + lhalf * 4 + c;
                            if (r < p.M && col < cols_valid) p.acc_out[r * p.N + o_base + col] = a;
                        }
                        if constexpr (Path::kOffset) a -= __mul24(rz, cz[i][g][c]);  // |z| < 2^8, |rowsum| < 2^23
                        out[c] = (float)a * (rs * cs[i][g][c]) + cb[i][g][c];
                    } else {
                        out[c] = acc[i][g * 4 + c] + cb[i][g][c];
                    }
                }
                __half2 lo = __floats2half2_rn(out[0], out[1]);
                __half2 hi = __floats2half2_rn(out[2], out[3]);
                u32x2 packed = {__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi)};
                *reinterpret_cast<u32x2 *>(patch + patch_chunk(l32, i * 4 + g) + lhalf * 8) = packed;
            }
        asm volatile("" ::: "memory");  // wavefront-private patch: LDS runs a wavefront's accesses in order
#pragma unroll
        for (int q = 0; q < 4; q++) {
            const int row = q * 8 + (lane >> 3), chunk = lane & 7;
            const v4i data = *reinterpret_cast<const v4i *>(patch + patch_chunk(row, chunk));
            const int64_t rr = rb * 32 + row;
            if (rr < p.M) {
                __half *dst = p.y + rr * p.ldy + o_base + chunk * 8;
                if (y_fast) {
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
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ks++) fx[ks] = fx_next[ks];
    }
}

// ------------------------------------------------------------------------------------------
// Skinny-N path (N <= 128 over very many rows, e.g. x_proj 1536 -> 80): the activation is read
// exactly once from HBM and is almost all of the traffic, the weight is small.  One workgroup of 8
// wavefronts per CU keeps the WHOLE weight in LDS (row pitch K bytes + 32: measured in a read loop, operand
// reads of 16 rows run at 235-240 bytes per clock and CU, at pitch K + 16 at half of that) together with s_w and the bias as
// fp32.  A wavefront owns units of 32 token rows (two 16 x 16 MFMA row blocks against all
// ceil(N / 16) channel blocks): its activation fragments go from global memory straight into
// registers in MFMA operand layout (16 rows x 64 contiguous bytes per load instruction),
// kWresDepth k-steps ahead, and there is no barrier after the weight has landed.  Results leave
// through a wavefront-private LDS patch laid out like the output rows; when the output is dense
// (ldy == N, N a multiple of 4, 16-byte aligned base) a 16-row block is one contiguous span and is
// written with 16-byte stores.
// Requirements (host-checked): pitches and bases 16-byte aligned, k_bytes % 64 == 0, N <= 128,
// M, L < 2^31, everything fits the 160 KiB of LDS.
// ------------------------------------------------------------------------------------------
constexpr int kWresWaves = 8;
constexpr int kWresDepth = 8;      // k-steps of activation fragments in flight per row block
constexpr int kWresMaxBlocks = 8;  // 16-channel blocks: N <= 128
constexpr int kLdsBytes = 160 * 1024;
constexpr int64_t kWresMinRows = 2048;   // and at least a quarter as many rows as the weight has bytes: below that the one-off weight copy per workgroup does not pay

struct WresLayout {
    int nb, n4, pw, w_bytes, scale_bytes, patch_bytes, total;
};
__host__ __device__ __forceinline__ WresLayout wres_layout(int N, int k_bytes) {
    WresLayout l;
    l.nb = (N + 15) >> 4;
    l.n4 = (N + 3) & ~3;
    l.pw = k_bytes + 32;  // in 16-byte chunks 2 mod 4: operand reads of 16 rows run at 235-240 bytes per clock and CU (k_bytes + 16: 120)
    l.w_bytes = (l.nb * 16 * l.pw + 1023) & ~1023;  // whole 1 KiB wavefront copies
    l.scale_bytes = l.nb * 16 * 4 * 3;  // step, bias and (zero-offset path) weight row sum per channel
    l.patch_bytes = 16 * l.n4 * 2;                   // one 16-row block of fp16 results
    l.total = l.w_bytes + l.scale_bytes + kWresWaves * l.patch_bytes;
    return l;
}

template <class Path, int NB>
__global__ __launch_bounds__(kWresWaves * 64) void linear_mfma_wres(const LinearArgs p) {
    constexpr bool kInt8 = Path::kElemBytes == 1;
    constexpr int D = kWresDepth;
    using Acc = typename Path::Acc16;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, lq = lane >> 4;
    const int N = (int)p.N, k_bytes = (int)p.k_bytes, n_ksteps = k_bytes >> 6;
    const WresLayout lay = wres_layout(N, k_bytes);
    const int n4 = lay.n4, pw = lay.pw;
    char *const w_lds = lds_dyn;
    float *const cs_lds = reinterpret_cast<float *>(lds_dyn + lay.w_bytes);
    float *const cb_lds = cs_lds + NB * 16;
    int *const cz_lds = reinterpret_cast<int *>(cb_lds + NB * 16);  // weight row sums (zero-offset path)
    char *const patch = lds_dyn + lay.w_bytes + lay.scale_bytes + wave * lay.patch_bytes;

    // Units are dealt wavefront-major, so that a launch with fewer units than wavefronts still
    // spreads them over all workgroups.
    const int64_t units = (p.M + 31) >> 5;
    const int64_t unit_step = (int64_t)gridDim.x * kWresWaves;
    int64_t unit = (int64_t)wave * gridDim.x + blockIdx.x;

    v4i fx[2][D];
    const char *xrow[2];
    auto load_x = [&](int d, int ks) {
#pragma unroll
        for (int j = 0; j < 2; j++)
            fx[j][d] = __builtin_nontemporal_load(reinterpret_cast<const v4i *>(xrow[j] + ks * 64));
    };
    auto start_unit = [&](int64_t u) {  // first D k-steps of the unit's two row blocks
#pragma unroll
        for (int j = 0; j < 2; j++)
            xrow[j] = p.x + min(u * 32 + j * 16 + l16, p.M - 1) * p.ldx_bytes + lq * 16;  // clamped rows are never stored
#pragma unroll
        for (int d = 0; d < D; d++)
            if (d < n_ksteps) load_x(d, d);
    };
    if (unit < units) start_unit(unit);

    // The weight, once: 1 KiB copies, linear on the LDS side; the lane picks the global chunk that
    // belongs at its LDS position (pad chunks and pad rows re-read a valid neighbour).
    {
        const int chunks_per_row = pw >> 4;
        for (int c = wave; c < (lay.w_bytes >> 10); c += kWresWaves) {
            const int chunk = c * 64 + lane;
            const int row = chunk / chunks_per_row, cc = chunk - row * chunks_per_row;
            const char *src = p.w + (int64_t)min(row, N - 1) * p.ldw_bytes + min(cc, chunks_per_row - 3) * 16;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                             (__attribute__((address_space(3))) void *)(w_lds + c * 1024), 16, 0, 0);
        }
        for (int o = tid; o < NB * 16; o += kWresWaves * 64) {
            float s = 0.0f, b = 0.0f;
            if (o < N) {
                s = 1.0f;
                if constexpr (kInt8) s = p.s_w[o];
                if (p.bias) b = __half2float(p.bias[o]);
            }
            cs_lds[o] = s;
            cb_lds[o] = b;
            if constexpr (Path::kOffset) cz_lds[o] = o < N ? p.rowsum[o] : 0;
        }
    }
    __builtin_amdgcn_s_waitcnt(0);  // vmcnt(0) expcnt(0) lgkmcnt(0): this wavefront's copies have landed
    __syncthreads();

    const bool dense_y = n4 == N && p.ldy == p.N && (reinterpret_cast<uintptr_t>(p.y) & 15) == 0;
    const int chunks8_per_row = n4 >> 2;  // 8-byte groups of four channels per patch row
    const char *const w_lane = w_lds + l16 * pw + lq * 16;

    for (; unit < units; unit += unit_step) {
        Acc acc[2][NB];
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
            for (int i = 0; i < NB; i++)
#pragma unroll
                for (int v = 0; v < 4; v++) acc[j][i][v] = 0;
        auto compute = [&](int d, int ks) {
            v4i fw[NB];
#pragma unroll
            for (int i = 0; i < NB; i++) fw[i] = *reinterpret_cast<const v4i *>(w_lane + i * 16 * pw + ks * 64);
            __builtin_amdgcn_sched_barrier(0);  // all LDS reads of the k-step in flight before its first MFMA
#pragma unroll
            for (int i = 0; i < NB; i++) {
                acc[0][i] = Path::mfma16(fw[i], fx[0][d], acc[0][i]);
                acc[1][i] = Path::mfma16(fw[i], fx[1][d], acc[1][i]);
            }
        };
        // The scheduling barriers keep each refill right behind the MFMAs that free its registers;
        // left alone the scheduler sinks all loads of a group to its end and the wavefront then
        // waits for the whole group before every pass.

        int ks0 = 0;
        for (; ks0 + 2 * D <= n_ksteps; ks0 += D) {  // steady state: every register slot is refilled
#pragma unroll
            for (int d = 0; d < D; d++) {
                compute(d, ks0 + d);
                load_x(d, ks0 + d + D);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#pragma unroll
        for (int d = 0; d < D; d++) {  // last refills
            if (ks0 + d < n_ksteps) {
                compute(d, ks0 + d);
                if (ks0 + d + D < n_ksteps) load_x(d, ks0 + d + D);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        ks0 += D;
#pragma unroll
        for (int d = 0; d < D; d++) {  // drain
            if (ks0 + d < n_ksteps) compute(d, ks0 + d);
            __builtin_amdgcn_sched_barrier(0);
        }

        // Accumulator register v of block (j, i): token row 16 j + (lane mod 16), channel 16 i + 4 (lane / 16) + v.
        const int64_t r_unit = unit * 32;
        float rs[2] = {1.0f, 1.0f};
        int rz[2] = {0, 0};  // per-token zero offsets of the lane's two rows (zero-offset path)
        if constexpr (kInt8) {
#pragma unroll
            for (int j = 0; j < 2; j++) {
                const uint32_t t = (uint32_t)min(r_unit + j * 16 + l16, p.M - 1) % (uint32_t)p.L;
                rs[j] = p.s_tok[t];
                if constexpr (Path::kOffset) rz[j] = p.z_tok[t];
            }
        }
        const int64_t next = unit + unit_step;
        if (next < units) start_unit(next);  // in flight while this unit's results are written

#pragma unroll
        for (int j = 0; j < 2; j++) {
            const int64_t r0 = r_unit + j * 16;
            const int rows_valid = (int)min((int64_t)16, p.M - r0);
            if (rows_valid <= 0) break;
#pragma unroll
            for (int i = 0; i < NB; i++) {
                const int col = i * 16 + lq * 4;
                if (col < n4) {
                    const v4f cs = *reinterpret_cast<const v4f *>(cs_lds + col);
                    const v4f cb = *reinterpret_cast<const v4f *>(cb_lds + col);
                    v4i cz = {0, 0, 0, 0};
                    if constexpr (Path::kOffset) cz = *reinterpret_cast<const v4i *>(cz_lds + col);
                    float out[4];
#pragma unroll
                    for (int c = 0; c < 4; c++) {
                        if constexpr (kInt8) {
                            int a = acc[j][i][c];
                            if (p.acc_out && l16 < rows_valid && col + c < N) p.acc_out[(r0 + l16) * p.N + col + c] = a;
                            if constexpr (Path::kOffset) a -= __mul24(rz[j], cz[c]);  // |z| < 2^8, |rowsum| < 2^23
                            out[c] = (float)a * (rs[j] * cs[c]) + cb[c];
                        } else {
                            out[c] = acc[j][i][c] + cb[c];
                        }
                    }
                    __half2 lo = __floats2half2_rn(out[0], out[1]);
                    __half2 hi = __floats2half2_rn(out[2], out[3]);
                    u32x2 packed = {__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi)};
                    *reinterpret_cast<u32x2 *>(patch + l16 * (n4 * 2) + col * 2) = packed;
                }
            }
            asm volatile("" ::: "memory");  // wavefront-private patch: LDS runs a wavefront's accesses in order
            if (dense_y) {
                const int valid_bytes = rows_valid * N * 2, block_bytes = 32 * N;
                char *dst = reinterpret_cast<char *>(p.y + r0 * p.N);
                for (int off = lane * 16; off < block_bytes; off += 64 * 16) {
                    const v4i data = *reinterpret_cast<const v4i *>(patch + off);
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
                for (int idx = lane; idx < 16 * chunks8_per_row; idx += 64) {
                    const int row = idx / chunks8_per_row, cc = idx - row * chunks8_per_row;
                    if (row >= rows_valid) continue;
                    const u32x2 data = *reinterpret_cast<const u32x2 *>(patch + row * (n4 * 2) + cc * 8);
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
        // stores possibly outstanding every wait on a fragment would have to be a full drain.  Drain
        // once here instead: the next unit's first fragments were fetched during the epilogue.
        wait_vmcnt_at_most<0>();
    }
}

// ------------------------------------------------------------------------------------------
// Generic path: register-staged loads, zero fill beyond M, N and K, any pitch.
// ------------------------------------------------------------------------------------------
template <class Path, int BR, int BO, int WR, int WO, int LOAD_ALIGN>
__global__ __launch_bounds__(kThreads, 2) void linear_mfma_generic(const LinearArgs p) {
    static_assert(WR * WO == kWaves, "four wavefronts per workgroup");
    constexpr int WAVE_R = BR / WR, WAVE_O = BO / WO;
    constexpr int FR = WAVE_R / 32, FO = WAVE_O / 32;
    static_assert(WAVE_R % 32 == 0 && WAVE_O % 32 == 0, "wave tile must be whole MFMA blocks");
    constexpr int X_CHUNKS = (BR * 4 + kThreads - 1) / kThreads;  // 16-byte chunks per thread per slab
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
        mfma_slab<Path, FO, FR>(acc, &lds_x[buf][wave_r * kSlabBytes], &lds_w[buf][wave_o * kSlabBytes], l32, lhalf);
        if (more) commit(buf ^ 1);
        __syncthreads();
    }
    epilogue<Path, FO, FR, JB>(acc, p, &lds_x[0][0] + wave * (JB * 32 * WAVE_O * 2), r0 + wave_r, o0 + wave_o, lane);
}

// ------------------------------------------------------------------------------------------
// Host side
// ------------------------------------------------------------------------------------------
template <class Path, int BR, int BO, int WR, int WO, int STAGES>
int launch_dma(LinearArgs a, hipStream_t stream) {
    dim3 grid;
    if (!set_grid<BR, BO>(a, grid)) return PTQ4VM_ERR_SHAPE;
    constexpr int lds_bytes = STAGES * (BR + BO) * kSlabBytes;
    auto kernel = linear_mfma_dma<Path, BR, BO, WR, WO, STAGES>;
    if (int rc = ptq4vm::set_lds_limit(reinterpret_cast<const void *>(kernel), lds_bytes, "hipFuncSetAttribute(linear_mfma_dma)")) return rc;
    kernel<<<grid, dim3(kThreads), lds_bytes, stream>>>(a);
    return ptq4vm::check_launch("linear_mfma_dma");
}

template <class Path, int BO, int SLAB, int STAGES>
int launch_persistent(LinearArgs a, hipStream_t stream) {
    constexpr int FRM = Path::kPacked4 ? 4 : 8;  // tile rows / 32
    dim3 grid;
    if (!set_grid<32 * FRM, BO>(a, grid)) return PTQ4VM_ERR_SHAPE;
    // One 8-wavefront or two 4-wavefront workgroups per CU (all that LDS allows), a multiple of the XCD count.
    int device = 0, cus = 0;
    hipError_t err = hipGetDevice(&device);
    if (err == hipSuccess) err = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device);
    if (err != hipSuccess) return ptq4vm::record_hip_error(err, "hipDeviceGetAttribute(multiprocessor count)");
    unsigned wgs = (unsigned)(cus / kXcds * kXcds) * (BO == 256 ? 1 : 2);
    if (wgs == 0) wgs = kXcds;
    if (wgs > grid.x) wgs = grid.x;  // grid.x is the tile count rounded up to a multiple of kXcds
    constexpr int lds_bytes = STAGES * (256 + BO) * SLAB + 2 * (BO * 4 + 256 * 4 + BO * 2 + (Path::kOffset ? BO * 4 + 256 * 4 : 0));
    using Kernel = void (*)(const LinearArgs);
    // [has bias][also write the int32 accumulators]
    static const Kernel kernels[2][2] = {{linear_mfma_persistent<Path, BO, SLAB, STAGES, false, false, FRM>,
                                          linear_mfma_persistent<Path, BO, SLAB, STAGES, false, true, FRM>},
                                         {linear_mfma_persistent<Path, BO, SLAB, STAGES, true, false, FRM>,
                                          linear_mfma_persistent<Path, BO, SLAB, STAGES, true, true, FRM>}};
    const Kernel kernel = kernels[a.bias ? 1 : 0][a.acc_out ? 1 : 0];
    if (int rc = ptq4vm::set_lds_limit(reinterpret_cast<const void *>(kernel), lds_bytes, "hipFuncSetAttribute(linear_mfma_persistent)")) return rc;
    kernel<<<dim3(wgs), dim3(BO * 2), lds_bytes, stream>>>(a);
    return ptq4vm::check_launch("linear_mfma_persistent");
}

template <class Path, int KSTEPS, int LOAD_ALIGN>
int launch_smallk(const LinearArgs &a, hipStream_t stream) {
    const int64_t strips = ptq4vm::ceil_div(a.N, 64 * kWaves), blocks = ptq4vm::ceil_div(a.M, 32);
    if (strips > 65535) return PTQ4VM_ERR_SHAPE;
    // about 8 workgroups per CU in total, each walking over row blocks
    int64_t gx = ptq4vm::ceil_div(2048, strips);
    if (gx > blocks) gx = blocks;
    dim3 grid((unsigned)gx, (unsigned)strips), block(kThreads);
    const bool bias = a.bias != nullptr, dump = a.acc_out != nullptr;
    if (bias && dump)
        linear_mfma_smallk<Path, KSTEPS, LOAD_ALIGN, true, true><<<grid, block, 0, stream>>>(a);
    else if (bias)
        linear_mfma_smallk<Path, KSTEPS, LOAD_ALIGN, true, false><<<grid, block, 0, stream>>>(a);
    else if (dump)
        linear_mfma_smallk<Path, KSTEPS, LOAD_ALIGN, false, true><<<grid, block, 0, stream>>>(a);
    else
        linear_mfma_smallk<Path, KSTEPS, LOAD_ALIGN, false, false><<<grid, block, 0, stream>>>(a);
    return ptq4vm::check_launch("linear_mfma_smallk");
}

template <class Path, int LOAD_ALIGN>
int launch_smallk_ksteps(const LinearArgs &a, hipStream_t stream) {
    switch ((int)ptq4vm::ceil_div(a.k_bytes, 32)) {
        case 1: return launch_smallk<Path, 1, LOAD_ALIGN>(a, stream);
        case 2: return launch_smallk<Path, 2, LOAD_ALIGN>(a, stream);
        case 3: return launch_smallk<Path, 3, LOAD_ALIGN>(a, stream);
        default: return launch_smallk<Path, 4, LOAD_ALIGN>(a, stream);
    }
}

template <class Path>
int launch_wres(const LinearArgs &a, hipStream_t stream) {
    const WresLayout lay = wres_layout((int)a.N, (int)a.k_bytes);
    int device = 0, cus = 0;
    hipError_t err = hipGetDevice(&device);
    if (err == hipSuccess) err = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device);
    if (err != hipSuccess) return ptq4vm::record_hip_error(err, "hipDeviceGetAttribute(multiprocessor count)");
    if (cus < 1) cus = 1;
    const int64_t units = ptq4vm::ceil_div(a.M, 32);
    int64_t wgs = ptq4vm::ceil_div(units, kWresWaves);
    if (wgs > cus) wgs = cus;  // one workgroup per CU: the resident weight takes most of its LDS
    using Kernel = void (*)(const LinearArgs);
    static const Kernel kernels[kWresMaxBlocks] = {  // by the number of 16-channel blocks
        linear_mfma_wres<Path, 1>, linear_mfma_wres<Path, 2>, linear_mfma_wres<Path, 3>, linear_mfma_wres<Path, 4>,
        linear_mfma_wres<Path, 5>, linear_mfma_wres<Path, 6>, linear_mfma_wres<Path, 7>, linear_mfma_wres<Path, 8>};
    if (int rc = ptq4vm::set_lds_limit(reinterpret_cast<const void *>(kernels[lay.nb - 1]), kLdsBytes, "hipFuncSetAttribute(linear_mfma_wres)")) return rc;
    kernels[lay.nb - 1]<<<dim3((unsigned)wgs), dim3(kWresWaves * 64), lay.total, stream>>>(a);
    return ptq4vm::check_launch("linear_mfma_wres");
}

template <class Path, int BR, int BO, int WR, int WO>
int launch_generic(LinearArgs a, int load_align, hipStream_t stream) {
    dim3 grid;
    if (!set_grid<BR, BO>(a, grid)) return PTQ4VM_ERR_SHAPE;
    if (load_align == 16)
        linear_mfma_generic<Path, BR, BO, WR, WO, 16><<<grid, dim3(kThreads), 0, stream>>>(a);
    else if (load_align == 4)
        linear_mfma_generic<Path, BR, BO, WR, WO, 4><<<grid, dim3(kThreads), 0, stream>>>(a);
    else
        linear_mfma_generic<Path, BR, BO, WR, WO, 0><<<grid, dim3(kThreads), 0, stream>>>(a);
    return ptq4vm::check_launch("linear_mfma_generic");
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
    a.y_vec = (a.ldy % 8 == 0 && ptq4vm::aligned_to(a.y, 16)) ? 8
              : ((a.ldy % 4 == 0 && ptq4vm::aligned_to(a.y, 8)) ? 4 : 1);
    const bool dma_ok = la == 16 && a.k_bytes % kSlabBytes == 0 && a.ldx_bytes * 256 < (1LL << 31) &&
                        a.ldw_bytes * 256 < (1LL << 31);
#if PTQ4VM_STREAM_SMALLK
    if constexpr (Path::kElemBytes == 1) {
        if (a.k_bytes <= (Path::kPacked4 ? 64 : 128)) {  // many rows: whole rows of y streamed out by one wavefront each
            const int rc = launch_stream_smallk(a, false, stream, Path::kPacked4, Path::kOffset);
            if (rc <= 0) return rc;
        }
    }
#endif
    if (a.k_bytes <= 128 && la >= 4 && a.L < (1LL << 31))
        return la == 16 ? launch_smallk_ksteps<Path, 16>(a, stream) : launch_smallk_ksteps<Path, 4>(a, stream);
    if constexpr (Path::kElemBytes == 1 && !Path::kOffset && !Path::kPacked4) {
        // wide output, short reduction (in_proj of the Vim-S / Vim-B stacks): weight rows held in registers
        const int rc = launch_wreg(a, stream);
        if (rc <= 0) return rc;
    }
    const bool persistent_ok = dma_ok && a.N % 8 == 0 && a.y_vec == 8 && ptq4vm::aligned_to(a.bias, 4) &&
                               a.ldy * 512 < (1LL << 31) && a.L < (1LL << 31) && a.N >= 256 &&
                               a.k_bytes % PTQ4VM_PERSISTENT_SLAB == 0 && a.k_bytes >= 2 * PTQ4VM_PERSISTENT_SLAB &&
                               ptq4vm::ceil_div(a.M, 256) * ptq4vm::ceil_div(a.N, 256) >= 256;
    // 256 x 256 tiles on one 8-wavefront workgroup per CU.  (The 256 x 128 / two 4-wavefront workgroups
    // per CU instantiation balances few-tile problems better but moves 1.5x the bytes through L2; it
    // measured 3 % slower on out_proj and 10 % slower on in_proj of the Vim-B stack.)
    if (persistent_ok) return launch_persistent<Path, PTQ4VM_PERSISTENT_BO, PTQ4VM_PERSISTENT_PHYS_SLAB, PTQ4VM_PERSISTENT_STAGES>(a, stream);
    if constexpr (Path::kElemBytes == 1 && !Path::kOffset && !Path::kPacked4 && PTQ4VM_PERSISTENT_BO == 256) {
        // Too few 256 x 256 tiles for the kernel above, and the second of two column tiles at most half full (N = 384 at
        // 25 216 rows: the out_proj of the Vim-S stack, batch 128): 256 x 128 tiles of the same kernel.  Measured there
        // 26.2 us against 29.3 us on the tiled kernel below.  (With enough 256 x 256 tiles - 50 240 rows - the wide tiles
        // are faster in spite of the half-empty column: 33.3 against 36.9 us.)
        const bool narrow_ok = dma_ok && a.N % 8 == 0 && a.y_vec == 8 && ptq4vm::aligned_to(a.bias, 4) &&
                               a.ldy * 512 < (1LL << 31) && a.L < (1LL << 31) && a.N > 256 && a.N <= 384 &&
                               a.k_bytes % PTQ4VM_PERSISTENT_SLAB == 0 && a.k_bytes >= 2 * PTQ4VM_PERSISTENT_SLAB &&
                               ptq4vm::ceil_div(a.M, 256) * ptq4vm::ceil_div(a.N, 128) >= 256;
        if (narrow_ok) return launch_persistent<Path, 128, PTQ4VM_PERSISTENT_PHYS_SLAB, PTQ4VM_PERSISTENT_STAGES>(a, stream);
    }
    // Few output channels over many rows: weight resident in LDS, activations streamed once.
    const bool wres_ok = dma_ok && a.N <= 16 * kWresMaxBlocks && a.M >= kWresMinRows &&
                         4 * a.M >= ptq4vm::ceil_div(a.N, 16) * 16 * a.k_bytes && a.M < (1LL << 31) &&
                         a.L < (1LL << 31) && a.k_bytes < (1LL << 20) &&
                         wres_layout((int)a.N, (int)a.k_bytes).total <= kLdsBytes;
    if constexpr (!Path::kPacked4) {
        if (wres_ok) return launch_wres<Path>(a, stream);
    }
    if (a.N > 64) {
        if (dma_ok && a.N <= 128) return launch_dma<Path, 128, 128, 2, 2, 4>(a, stream);  // skinny N: many small tiles
        if (dma_ok) return launch_dma<Path, 256, 128, 2, 2, 3>(a, stream);
        return launch_generic<Path, 256, 128, 2, 2>(a, la, stream);
    }
    if (dma_ok) return launch_dma<Path, 256, 64, 4, 1, 3>(a, stream);
    return launch_generic<Path, 256, 64, 4, 1>(a, la, stream);
}

}  // namespace

extern "C" int ptq4vm_w8a8_linear_offset(const int8_t *xq, const int8_t *wq, const float *s_tok, const int32_t *z_tok,
                                         const int32_t *rowsum, const float *s_w, const void *bias_f16, void *y_f16,
                                         int32_t *acc_out, int64_t B, int64_t L, int64_t K, int64_t N, int64_t ldxq,
                                         int64_t ldwq, int64_t ldy, void *stream_) {
    if (!xq || !wq || !s_tok || !z_tok || !rowsum || !s_w || !y_f16) return PTQ4VM_ERR_NULL;
    if (B < 0 || N < 0 || L <= 0 || K <= 0 || K > PTQ4VM_MAX_K_OFFSET) return PTQ4VM_ERR_SHAPE;  // |acc| + |z rowsum| < 2^31
    if (B > 0 && L > INT64_MAX / B) return PTQ4VM_ERR_SHAPE;
    if (ldxq < K || ldwq < K || ldy < N) return PTQ4VM_ERR_STRIDE;
    if (!ptq4vm::aligned_to(xq, 16) || !ptq4vm::aligned_to(wq, 16) || !ptq4vm::aligned_to(y_f16, 2) ||
        !ptq4vm::aligned_to(s_tok, 4) || !ptq4vm::aligned_to(z_tok, 4) || !ptq4vm::aligned_to(rowsum, 4) ||
        !ptq4vm::aligned_to(s_w, 4) || !ptq4vm::aligned_to(bias_f16, 2) || !ptq4vm::aligned_to(acc_out, 4))
        return PTQ4VM_ERR_ALIGN;
    const int64_t M = B * L;
    if (M == 0 || N == 0) return PTQ4VM_OK;
    LinearArgs a{};
    a.x = reinterpret_cast<const char *>(xq);
    a.w = reinterpret_cast<const char *>(wq);
    a.s_tok = s_tok;
    a.s_w = s_w;
    a.z_tok = z_tok;
    a.rowsum = rowsum;
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
    return dispatch<Int8OffsetPath>(a, static_cast<hipStream_t>(stream_));
}

extern "C" int ptq4vm_w4a4_linear(const uint8_t *xq4, const uint8_t *wq4, const float *s_tok, const float *s_w,
                                  const void *bias_f16, void *y_f16, int32_t *acc_out, int64_t B, int64_t L,
                                  int64_t K, int64_t N, int64_t ldxq, int64_t ldwq, int64_t ldy, void *stream_) {
    if (!xq4 || !wq4 || !s_tok || !s_w || !y_f16) return PTQ4VM_ERR_NULL;
    // operands are codes times 16: the accumulator holds 256 acc, at most 2^14 K with the nibble -8
    if (B < 0 || N < 0 || L <= 0 || K <= 0 || K > PTQ4VM_MAX_K_W4 || K % 2 != 0) return PTQ4VM_ERR_SHAPE;
    if (B > 0 && L > INT64_MAX / B) return PTQ4VM_ERR_SHAPE;
    if (ldxq < K / 2 || ldwq < K / 2 || ldy < N) return PTQ4VM_ERR_STRIDE;
    if (!ptq4vm::aligned_to(xq4, 16) || !ptq4vm::aligned_to(wq4, 16) || !ptq4vm::aligned_to(y_f16, 2) ||
        !ptq4vm::aligned_to(s_tok, 4) || !ptq4vm::aligned_to(s_w, 4) || !ptq4vm::aligned_to(bias_f16, 2) ||
        !ptq4vm::aligned_to(acc_out, 4))
        return PTQ4VM_ERR_ALIGN;
    const int64_t M = B * L;
    if (M == 0 || N == 0) return PTQ4VM_OK;
    LinearArgs a{};
    a.x = reinterpret_cast<const char *>(xq4);
    a.w = reinterpret_cast<const char *>(wq4);
    a.s_tok = s_tok;
    a.s_w = s_w;
    a.bias = static_cast<const __half *>(bias_f16);
    a.y = static_cast<__half *>(y_f16);
    a.acc_out = acc_out;
    a.M = M;
    a.N = N;
    a.k_bytes = K / 2;  // packed bytes
    a.ldx_bytes = ldxq;
    a.ldw_bytes = ldwq;
    a.ldy = ldy;
    a.L = L;
    return dispatch<Int4Path>(a, static_cast<hipStream_t>(stream_));
}

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
