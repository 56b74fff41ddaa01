// W8A8 linear for gfx950 with the WEIGHT HELD IN REGISTERS: int8 x int8 -> int32 MFMA GEMM with the
// PTS dequantization fused behind it (PTS equation of Sec. 5.1; App. B.1 "INT GEMM" +
// "Dequantization").  For wide linears with a short reduction (K = 384 or 768 codes: the in_proj of
// the Vim-S / Vim-B stacks), where the output stream is as long as the matrix work.
//
// One workgroup of 8 wavefronts per CU owns a strip of 256 output channels for (almost) its whole
// life.  A wavefront keeps the weight rows of 32 channels, all K of them, as MFMA "A" operands in
// registers (96 VGPRs at K = 768) and never reads the weight again.  Token rows arrive in units of
// 128 rows: their int8 codes are copied global -> LDS (direct copies, no VGPR staging) into a ring
// of 5 slots, each slot one sixth of K for the 128 rows, and every wavefront reads all of them as
// "B" operands.  Per 128 x 256 unit that is 96 KiB through L2 -> LDS, half of what a 256 x 256
// tile with both operands in LDS needs per output, and the ring runs 3 slots ahead.
//
// Step g of a workgroup consumes ring slot g: MFMAs of all but the last k-step of the slot; wait;
// s_barrier; MFMAs of the last k-step while the operands of the next slot's first k-step are fetched.
// At the barrier of step g every copy of slot g + 1 has landed and slot g - 1 has been read into
// registers by everyone, so its place is refilled with slot g + 4.
// A unit's last step is different: after its barrier the MFMAs run row block by row block (all
// k-steps of the slot for 16 rows), and each block's results are converted to fp16 and written to an
// LDS staging tile right behind its MFMAs.  The conversion is three VALU instructions per output and
// a lone wavefront issues at most one VALU instruction in ~8 cycles: done as a phase of its own it
// would leave the matrix pipes idle for a third of the time; woven between the MFMAs of both
// wavefronts of a SIMD it runs at the SIMD's full VALU rate with the MFMAs underneath.
// The staged 128 x 256 fp16 tile leaves for memory during the first four steps of the next unit, in
// whole 512-byte row segments, so the store stream is spread over the unit instead of bursting.
// Roles: wavefronts 0-3 issue every global -> LDS copy and never store; wavefronts 4-7 issue every
// output store and never wait for a copy.  Loads and stores share one counter (vmcnt) and complete
// out of order with each other, so a wavefront that did both could only wait for a copy by draining
// its stores.
//
// Output channel order inside a wavefront: MFMA block i (0, 1), A-operand row a (0..15) carries
// strip channel 32 w + 8 (a / 4) + 4 i + (a mod 4).  A lane's eight results of a token row are then
// eight consecutive channels, 16 bytes of fp16.
//
// Requirements (host-checked): int8 path without zero offset, K = 384 or 768, pitches and bases
// 16-byte aligned, N a multiple of 256, y 16-byte aligned with 16-byte pitch, M, L < 2^31.
#include <type_traits>

#include "mfma_linear.hpp"
#include "unit_order.hpp"

// Timing experiments only (results are wrong when any bit is set): 1 no output stores, 2 no conversion,
// 4 no global -> LDS copies, 8 no operand refetch from LDS, 16 no step barriers, 32 no MFMAs.
#ifndef PTQ4VM_WREG_SKIP
#define PTQ4VM_WREG_SKIP 0
#endif

#ifndef PTQ4VM_WREG_TRACE
#define PTQ4VM_WREG_TRACE 0
#endif
#if PTQ4VM_WREG_TRACE
// Debug build only: wall-clock ticks (100 MHz) of workgroups 0 and 77, per wavefront.
__device__ unsigned long long ptq4vm_wreg_trace[2][8][256];
extern "C" int ptq4vm_debug_wreg_trace(void *host_dst) {
    return (int)hipMemcpyFromSymbol(host_dst, HIP_SYMBOL(ptq4vm_wreg_trace), sizeof(ptq4vm_wreg_trace));
}
#define WREG_TRACE()                                                                                     \
    do {                                                                                                 \
        if (tr_wg >= 0 && tr_n < 256) {                                                                  \
            const unsigned long long now = __builtin_amdgcn_s_memrealtime();                             \
            if (lane == 0) ptq4vm_wreg_trace[tr_wg][wave][tr_n] = now;                                   \
            tr_n++;                                                                                      \
        }                                                                                                \
    } while (0)
#else
#define WREG_TRACE() do {} while (0)
#endif

namespace ptq4vm {
namespace mfma {
namespace {

constexpr int kUnitRows = 128;    // token rows per unit
constexpr int kStripCols = 256;   // output channels per workgroup
constexpr int kSteps = 6;         // ring slots per unit
constexpr int kSlots = 5;         // ring depth
constexpr int kAhead = kSlots - 1;  // slots copied ahead of the one being consumed
constexpr int kStagePitch = 528;  // bytes per staged row: 256 channels of fp16 + 16 (bank spread)
constexpr int kStageBytes = kUnitRows * kStagePitch;
constexpr int kRowScaleBufs = 4;  // per-row step vectors of the units in flight
#ifndef PTQ4VM_WREG_PREFETCH
#define PTQ4VM_WREG_PREFETCH 3
#endif
constexpr int kPrefetchAhead = PTQ4VM_WREG_PREFETCH;  // units between a row tile's L2 prefetch and its first copy (0: none)
constexpr int kPrefetchSinkBytes = 4 * 256;           // where the prefetch loads land: 256 bytes per storing wavefront

template <int KSTEPS, bool HAS_BIAS, bool DUMP_ACC>
__global__ __launch_bounds__(512, 1) void linear_mfma_wreg(const LinearArgs p) {
    constexpr int KPS = KSTEPS / kSteps;  // k-steps (64 bytes of K) per ring slot: 1 or 2
    static_assert(KPS * kSteps == KSTEPS && (KPS == 1 || KPS == 2), "K is 384 or 768");
    constexpr int SLAB = 64 * KPS;               // bytes of K per row in a slot
    constexpr int SLOT_BYTES = kUnitRows * SLAB;
    constexpr int CHUNKS = SLAB / 16;            // 16-byte chunks per slot row
    constexpr int ROWS_PER_COPY = 64 / CHUNKS;   // rows in one wavefront-wide 1 KiB copy
    constexpr int COPIES = kUnitRows / ROWS_PER_COPY / 4;  // copies per copying wavefront and slot
    using Acc = Int8Path::Acc16;

    char *const ring = lds_dyn;
    char *const stage = lds_dyn + kSlots * SLOT_BYTES;
    float *const rs_lds = reinterpret_cast<float *>(stage + kStageBytes);  // [kRowScaleBufs][kUnitRows]
    // steps and biases of the strip's channels, 48 bytes per group of 8 channels: 8 fp32 steps, 8 fp16 biases
    char *const cs_lds = reinterpret_cast<char *>(rs_lds + kRowScaleBufs * kUnitRows);
    char *const pf_sink = cs_lds + 32 * 48 + 16;  // never read

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int gw = wave & 3;  // wavefront inside its group of four
    const int l16 = lane & 15, lq = lane >> 4;

#if PTQ4VM_WREG_TRACE
    const int tr_wg = blockIdx.x == 0 ? 0 : (blockIdx.x == 77 ? 1 : -1);
    int tr_n = 0;
#endif
    WREG_TRACE();
    const WorkRange wr = work_range(p);
    if (wr.count == 0) return;  // the whole workgroup: no barrier has been executed yet
    const int total_steps = wr.count * kSteps;

    auto unit_row0 = [&](const UnitCursor &c) { return (int64_t)(wr.t_lo + c.band * wr.band_h + c.row) * kUnitRows; };
    auto slot_chunk = [&](int row, int chunk) {  // byte offset of a 16-byte chunk inside a slot
        return row * SLAB + ((chunk ^ (SLAB == 64 ? swizzle(row) : (row & 7))) << 4);
    };

    // ---- the wavefront's weight rows (registers) and the steps and biases of its channels (a
    // wavefront-private LDS table, read back at conversion time), reloaded when the strip changes.
    v4i fw[2][KSTEPS];
    auto load_strip = [&](int strip) {
        const int64_t o0 = (int64_t)strip * kStripCols;
        const char *w_strip = p.w + o0 * p.ldw_bytes;
#pragma unroll
        for (int i = 0; i < 2; i++) {
            const int ch = wave * 32 + 8 * (l16 >> 2) + 4 * i + (l16 & 3);
            const uint32_t off = (uint32_t)ch * (uint32_t)p.ldw_bytes + lq * 16;
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ks++) fw[i][ks] = *reinterpret_cast<const v4i *>(w_strip + off + ks * 64);
        }
        if (lane < 32) {  // channel wave * 32 + lane: lanes 0..31 write the wavefront's own 4 x 48 bytes
            const int ch = wave * 32 + lane;
            char *slot8 = cs_lds + (wave * 4 + (lane >> 3)) * 48;
            reinterpret_cast<float *>(slot8)[lane & 7] = p.s_w[o0 + ch];
            __half bias = __float2half(0.0f);
            if constexpr (HAS_BIAS) bias = p.bias[o0 + ch];
            reinterpret_cast<__half *>(slot8 + 32)[lane & 7] = bias;
        }
    };

    // ---- operand fetch from the ring
    v4i fx[8];
    uint32_t frag_off[KPS];
#pragma unroll
    for (int k2 = 0; k2 < KPS; k2++) frag_off[k2] = (uint32_t)slot_chunk(l16, 4 * k2 + lq);  // row 16 j + l16: same swizzle
    auto operand = [&](int j, int slot, int k2) {
        return *reinterpret_cast<const v4i *>(ring + slot * SLOT_BYTES + frag_off[k2] + j * 16 * SLAB);
    };

    Acc acc[2][8];
    // One MFMA k-step over the 8 row blocks.  REFETCH: operand j is dead after its two MFMAs and is
    // fetched again at once for the k-step named by (slot, k2).
    auto k_step = [&](const v4i &w0, const v4i &w1, bool fresh, bool refetch, int slot, int k2) {
#pragma unroll
        for (int j = 0; j < 8; j++) {
            const Acc zero = {0, 0, 0, 0};
            if constexpr (!(PTQ4VM_WREG_SKIP & 32)) {
                acc[0][j] = Int8Path::mfma16(w0, fx[j], fresh ? zero : acc[0][j]);
                acc[1][j] = Int8Path::mfma16(w1, fx[j], fresh ? zero : acc[1][j]);
            } else if (fresh) {
                acc[0][j] = fx[j], acc[1][j] = fx[j] + w0 + w1;
            }
            if (refetch && !(PTQ4VM_WREG_SKIP & 8)) fx[j] = operand(j, slot, k2);
            __builtin_amdgcn_sched_barrier(0);  // keep the refetch behind its MFMAs: hoisted, it would need a second register set
        }
    };

    // A zero the compiler cannot see through: lane-derived addresses built on it are computed where they
    // are used instead of being hoisted out of the unit loop into (spilled) registers.
    auto opaque_zero = [&]() {
        uint32_t z;
        asm volatile("v_mov_b32 %0, 0" : "=v"(z));
        return z;
    };

    // ---- the unit's last step.  Operands come through a four-deep rotation (fx[0..3]); the per-row
    // steps and the channels' steps / biases are fetched before the step's barrier (`prefetch`) and are
    // waited for together with everything else there.
    struct LastStep {
        float rs[8];   // s_tok of rows 16 j + l16
        v4f csb[3];    // 8 channel steps, 8 fp16 biases
        uint32_t dst;  // staging address of row l16, this lane's 16 bytes
    };
    constexpr int LOOKAHEAD = 4 / KPS;  // row blocks whose operands are in flight
    auto last_step_prefetch = [&](LastStep &ls, int slot, int rs_buf) {
        const uint32_t ln = threadIdx.x + opaque_zero();
        const uint32_t l16_now = ln & 15, lq_now = (ln >> 4) & 3;
        lds_issue_8x_b32<64>(lds_addr(rs_lds + rs_buf * kUnitRows) + l16_now * 4, ls.rs);
        lds_issue_3x_b128<16>(lds_addr(cs_lds) + (wave * 4 + lq_now) * 48, ls.csb);
        ls.dst = lds_addr(stage) + l16_now * kStagePitch + wave * 64 + lq_now * 16;
#pragma unroll
        for (int j = 0; j < LOOKAHEAD; j++)
#pragma unroll
            for (int k2 = 0; k2 < KPS; k2++) fx[j * KPS + k2] = operand(j, slot, k2);
    };
    auto convert_block = [&](const LastStep &ls, int j, int64_t r0, int64_t o0) {
        if constexpr (PTQ4VM_WREG_SKIP & 2) {
            if (acc[0][j][0] == 0x12345678 && acc[1][j][3] == 0x7654321) p.y[0] = __float2half(1.0f);
            return;
        }
        v4f packed;
#pragma unroll
        for (int i = 0; i < 2; i++) {  // four results at a time: keeps the temporaries few
#pragma unroll
            for (int h = 0; h < 2; h++) {
                const int e = 4 * i + 2 * h;
                const int a0 = acc[i][j][2 * h], a1 = acc[i][j][2 * h + 1];
                if constexpr (DUMP_ACC) {
                    const int64_t r = r0 + j * 16 + l16, o = o0 + wave * 32 + lq * 8 + e;
                    if (r < p.M) p.acc_out[r * p.N + o] = a0, p.acc_out[r * p.N + o + 1] = a1;
                }
                const float bias_word = HAS_BIAS ? ls.csb[2][e >> 1] : 0.0f;  // two fp16 biases
                packed[2 * i + h] = dequantize_pair_f16((float)a0, ls.rs[j] * ls.csb[i][2 * h], (float)a1,
                                                        ls.rs[j] * ls.csb[i][2 * h + 1], bias_word);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        lds_write_b128(ls.dst + j * 16 * kStagePitch, packed);
    };
    // fx[(j % LOOKAHEAD) * KPS + k2] holds the operand of row block j, k-step k2 of the slot.  Block j - 1
    // is converted behind the MFMAs of block j: its own MFMAs have left the pipe by then.
    auto last_step_run = [&](const LastStep &ls, int slot, int64_t r0, int64_t o0) {
#pragma unroll
        for (int j = 0; j < 8; j++) {
#pragma unroll
            for (int k2 = 0; k2 < KPS; k2++) {
                const int f = (j % LOOKAHEAD) * KPS + k2, ks = (kSteps - 1) * KPS + k2;
                if constexpr (!(PTQ4VM_WREG_SKIP & 32)) {
                    acc[0][j] = Int8Path::mfma16(fw[0][ks], fx[f], acc[0][j]);
                    acc[1][j] = Int8Path::mfma16(fw[1][ks], fx[f], acc[1][j]);
                }
                if (j + LOOKAHEAD < 8 && !(PTQ4VM_WREG_SKIP & 8)) fx[f] = operand(j + LOOKAHEAD, slot, k2);
            }
            if (j > 0) convert_block(ls, j - 1, r0, o0);
            __builtin_amdgcn_sched_barrier(0);
        }
        convert_block(ls, 7, r0, o0);
    };

    const uint32_t ldy_bytes = (uint32_t)p.ldy * 2;

    // ---- copies (wavefronts 0-3): slot `pf_step` of the unit list goes to ring place pf_step mod 5
    UnitCursor pc = wr.start;
    int pf_step = 0, pf_in_unit = 0, pf_slot = 0, pf_unit = 0;
    const char *pf_x = nullptr;
    int64_t pf_r0 = 0;
    int pf_rows_valid = 0;
    auto pf_setup = [&]() {
        pf_r0 = unit_row0(pc);
        pf_x = p.x + pf_r0 * p.ldx_bytes;
        pf_rows_valid = (int)min((int64_t)kUnitRows, p.M - pf_r0);
    };
    auto issue = [&]() {
        const uint32_t ln = (threadIdx.x + opaque_zero()) & 63;
        if (pf_in_unit == 0 && gw < 2) {  // the unit's per-row steps s_tok[r mod L], 64 rows per wavefront
            const int r = min((int)(gw * 64 + ln), pf_rows_valid - 1);
            const uint32_t t = ((uint32_t)(pf_r0 % p.L) + (uint32_t)r) % (uint32_t)p.L;
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void *)(p.s_tok + t),
                (__attribute__((address_space(3))) void *)(rs_lds + (pf_unit & (kRowScaleBufs - 1)) * kUnitRows + gw * 64), 4, 0, 0);
        }
        const char *gx = pf_x + (int64_t)pf_in_unit * SLAB;
        char *dst = ring + pf_slot * SLOT_BYTES;
#pragma unroll
        for (int c = 0; c < ((PTQ4VM_WREG_SKIP & 4) ? 0 : COPIES); c++) {
            const int row = (gw + 4 * c) * ROWS_PER_COPY + (int)(ln / CHUNKS);
            const int chunk = (int)(ln % CHUNKS) ^ (SLAB == 64 ? swizzle(row) : (row & 7));
            // rows beyond M are clamped to row M - 1: their results are copies of that row's (see `drain`)
            const uint32_t off = (uint32_t)min(row, pf_rows_valid - 1) * (uint32_t)p.ldx_bytes + chunk * 16;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(gx + off),
                                             (__attribute__((address_space(3))) void *)(dst + (gw + 4 * c) * 1024), 16, 0, 0);
        }
        pf_step++;
        if (++pf_slot == kSlots) pf_slot = 0;
        if (++pf_in_unit == kSteps) {
            pf_in_unit = 0;
            pf_unit++;
            advance(pc, wr);
            if (pf_step < total_steps) pf_setup();
        }
    };

    // ---- output stores (wavefronts 4-7): a quarter of this wavefront's 32 staged rows, two stores of
    // 2 rows x 512 bytes.  No masks and no branches: any control flow inside the unrolled steps, even
    // uniform, costs this kernel registers it does not have.  N is a multiple of 256, so a unit has all
    // of its channels.  Rows beyond M hold copies of row M - 1's results (their codes and steps were
    // clamped to that row when they were copied), so they are written onto row M - 1 again: same bytes,
    // same address.
    auto drain = [&](int part, int64_t r0, int64_t o0) {
        const uint32_t ln = (threadIdx.x + opaque_zero()) & 63;
        const int row0 = gw * 32 + part * 8 + (int)(ln >> 5), chunk = (int)(ln & 31);
        const int rows_valid = (int)min((int64_t)kUnitRows, p.M - r0);
        char *dst = reinterpret_cast<char *>(p.y + r0 * p.ldy + o0) + chunk * 16;
        const uint32_t src = lds_addr(stage) + row0 * kStagePitch + chunk * 16;
#pragma unroll
        for (int q = 0; q < 4; q++) {
            v4f data;
            lds_read_1x_b128(src + q * 2 * kStagePitch, data);
            const int row = min(row0 + q * 2, rows_valid - 1);
            if (!(PTQ4VM_WREG_SKIP & 1))
                __builtin_nontemporal_store(data, reinterpret_cast<v4f *>(dst + (uint32_t)row * ldy_bytes));
        }
    };

    // ---- L2 prefetch (wavefronts 4-7): one 4-byte load per 128-byte line of a unit's codes, kPrefetchAhead units
    // before the unit is worked on.  At K = 384 a step is 16 MFMAs per wavefront and the ring's three slots of
    // lookahead are shorter than the latency of a row tile that comes from memory: measured 63 -> 59 us at
    // M = 50 240 and 32.8 -> 31.5 us at M = 25 216 (at K = 768 the steps are twice as long and nothing changes).
    // The ring cannot grow: LDS is full.  The loads land in an LDS sink that nobody reads (no destination register
    // to keep alive), and they are issued by the wavefronts that never wait for a load: loads return in order, so in
    // a copying wavefront every later copy would wait for them.
    auto prefetch_unit = [&](const UnitCursor &c) {
        const uint32_t ln = (threadIdx.x + opaque_zero()) & 63;
        const int64_t r0 = unit_row0(c);
        const int rows_valid = (int)min((int64_t)kUnitRows, p.M - r0);
        constexpr int LINES_PER_ROW = KSTEPS / 2, LINES = kUnitRows * LINES_PER_ROW, PER_WAVE = LINES / 4;
        const char *base = p.x + r0 * p.ldx_bytes;
#pragma unroll
        for (int c2 = 0; c2 < (PER_WAVE + 63) / 64; c2++) {
            const int idx = min(gw * PER_WAVE + c2 * 64 + (int)ln, LINES - 1);
            const int row = idx / LINES_PER_ROW, line = idx - row * LINES_PER_ROW;
            const uint32_t off = (uint32_t)min(row, rows_valid - 1) * (uint32_t)p.ldx_bytes + line * 128;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(base + off),
                                             (__attribute__((address_space(3))) void *)(pf_sink + gw * 256), 4, 0, 0);
        }
    };

    // One source for both roles; COPIER is a compile-time flag so that neither role's code has branches
    // on the other's duties.
    auto run = [&](auto copier_tag) {
        constexpr bool COPIER = decltype(copier_tag)::value;
        UnitCursor cc = wr.start;
        if constexpr (COPIER) {
            pf_setup();
#pragma unroll
            for (int t = 0; t < kAhead; t++) issue();  // slots 0..3 (every unit list has at least 6)
        }
        int g = 0, slot = 0, u = 0;
        int64_t prev_r0 = 0, prev_o0 = 0;
        bool first_run = true;
        UnitCursor qc = wr.start;  // the unit kPrefetchAhead after the current one
        if constexpr (!COPIER && kPrefetchAhead > 0) {
#pragma unroll 1
            for (int a = 0; a < kPrefetchAhead; a++) {
                advance(qc, wr);
                if (a + 1 < kPrefetchAhead && a + 1 < wr.count) prefetch_unit(qc);  // units 1 .. kPrefetchAhead - 1
            }
        }
#pragma unroll 1
        while (u < wr.count) {
            // A run of units of one strip: the weight rows stay in registers for all of it.
            const int strip = cc.strip;
            load_strip(strip);
            wait_vmcnt_at_most<0>();  // also lands every copy in flight; happens once or twice per launch
            if (first_run) __builtin_amdgcn_s_barrier();  // slot 0 is visible to everyone
            first_run = false;
            WREG_TRACE();
            const int64_t o0 = (int64_t)strip * kStripCols;
#pragma unroll 1
            do {
                const int64_t r0 = unit_row0(cc);
                if constexpr (!COPIER && kPrefetchAhead > 0) {
                    if (u + kPrefetchAhead < wr.count) prefetch_unit(qc);
                    advance(qc, wr);
                }
#pragma unroll
                for (int j = 0; j < 8; j++) fx[j] = operand(j, slot, 0);  // the unit's first operands (its slot has landed)
#pragma unroll
                for (int s = 0; s < kSteps; s++, g++) {
                    int next_slot = slot + 1;
                    if (next_slot == kSlots) next_slot = 0;
                    LastStep ls;
                    if (s < kSteps - 1) {
                        if constexpr (KPS == 2) k_step(fw[0][2 * s], fw[1][2 * s], s == 0, true, slot, 1);
                        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // this slot's operands are all in registers
                    } else {
                        last_step_prefetch(ls, slot, u & (kRowScaleBufs - 1));
                        lds_wait_all(ls.rs, ls.csb);
                    }
                    if constexpr (COPIER) {
                        if (g + 1 < total_steps) {  // slot g + 1 has landed for this wavefront
                            if (g + kAhead - 1 < total_steps && !DUMP_ACC)
                                wait_vmcnt_at_most<(kAhead - 2) * COPIES>();  // slots g + 2, g + 3 may still be in flight
                            else
                                wait_vmcnt_at_most<0>();
                        }
                    }
                    if constexpr (!(PTQ4VM_WREG_SKIP & 16)) __builtin_amdgcn_s_barrier();
                    WREG_TRACE();
                    if constexpr (COPIER) {
                        if (pf_step < total_steps) issue();  // slot g + 4 into the ring place of slot g - 1
                    }
                    if (s < kSteps - 1)
                        k_step(fw[0][KPS * s + KPS - 1], fw[1][KPS * s + KPS - 1], KPS == 1 && s == 0, s + 2 < kSteps, next_slot, 0);
                    else
                        last_step_run(ls, slot, r0, o0);
                    if constexpr (!COPIER) {  // the previous unit's staged tile, a quarter per step
                        if (s < 4 && u > 0) drain(s, prev_r0, prev_o0);
                    }
                    slot = next_slot;
                }
                WREG_TRACE();
                prev_r0 = r0, prev_o0 = o0;
                advance(cc, wr);
                u++;
            } while (u < wr.count && cc.strip == strip);
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the last unit's staged results are in LDS before the barrier
        __builtin_amdgcn_s_barrier();
        if constexpr (!COPIER) {
#pragma unroll 1
            for (int part = 0; part < 4; part++) drain(part, prev_r0, prev_o0);
        }
    };
    if (wave < 4)
        run(std::true_type{});
    else
        run(std::false_type{});
}

}  // namespace

int launch_wreg(const LinearArgs &a_in, hipStream_t stream) {
    LinearArgs a = a_in;
    const bool shape_ok = (a.k_bytes == 384 || a.k_bytes == 768) && a.N % kStripCols == 0 && a.N > 0 &&
                          a.M >= 64 * kUnitRows && a.M < (1LL << 31) && a.L < (1LL << 31) && a.y_vec == 8 &&
                          ptq4vm::aligned_to(a.x, 16) && ptq4vm::aligned_to(a.w, 16) && a.ldx_bytes % 16 == 0 &&
                          a.ldw_bytes % 16 == 0 && a.ldx_bytes * kUnitRows < (1LL << 31) &&
                          a.ldy * 2 * kUnitRows < (1LL << 31) && ptq4vm::aligned_to(a.bias, 4) && a.ldw_bytes * kStripCols < (1LL << 31);
    if (!shape_ok) return 1;
    const int64_t tiles_r = ptq4vm::ceil_div(a.M, kUnitRows), tiles_o = ptq4vm::ceil_div(a.N, kStripCols);
    if (tiles_r * tiles_o > 0x3fffffffLL) return 1;
    a.tiles_r = (int)tiles_r;
    a.tiles_o = (int)tiles_o;
    int device = 0, cus = 0;
    hipError_t err = hipGetDevice(&device);
    if (err == hipSuccess) err = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device);
    if (err != hipSuccess) return ptq4vm::record_hip_error(err, "hipDeviceGetAttribute(multiprocessor count)");
    const unsigned wgs = (unsigned)max(1, cus / kXcds) * kXcds;  // one workgroup per CU, a multiple of the XCD count
    using Kernel = void (*)(const LinearArgs);
    // [K = 768][has bias][also write the int32 accumulators]
    static const Kernel kernels[2][2][2] = {
        {{linear_mfma_wreg<6, false, false>, linear_mfma_wreg<6, false, true>},
         {linear_mfma_wreg<6, true, false>, linear_mfma_wreg<6, true, true>}},
        {{linear_mfma_wreg<12, false, false>, linear_mfma_wreg<12, false, true>},
         {linear_mfma_wreg<12, true, false>, linear_mfma_wreg<12, true, true>}}};
    const Kernel kernel = kernels[a.k_bytes == 768 ? 1 : 0][a.bias ? 1 : 0][a.acc_out ? 1 : 0];
    const int slab = a.k_bytes == 768 ? 128 : 64;
    const int lds_bytes = kSlots * kUnitRows * slab + kStageBytes + kRowScaleBufs * kUnitRows * 4 + 32 * 48 + 16 + kPrefetchSinkBytes;
    if (int rc = ptq4vm::set_lds_limit(reinterpret_cast<const void *>(kernel), lds_bytes, "hipFuncSetAttribute(linear_mfma_wreg)")) return rc;
    kernel<<<dim3(wgs), dim3(512), lds_bytes, stream>>>(a);
    return ptq4vm::check_launch("linear_mfma_wreg");
}

}  // namespace mfma
}  // namespace ptq4vm
