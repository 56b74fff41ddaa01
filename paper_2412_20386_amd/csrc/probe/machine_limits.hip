// Standalone probe of the MI355X (gfx950) limits that the kernel designs in this package lean on.
// Not part of libptq4vm.so.  Build: hipcc --offload-arch=gfx950 -O3 machine_limits.hip -o machine_limits
// Every kernel here is bounded (fixed trip counts, in-bounds addresses) and writes nothing but
// one guarded word.
//
//   hbm     streaming read / write / copy / 2:1 (read 16 B, write 8 B) over 1 GiB buffers
//   l2lds   direct global -> LDS copies of an L2-resident region, 64- vs 128-byte row segments
//   lds     ds_read_b128 rate
//   mfma    v_mfma_i32_32x32x32_i8 and v_mfma_i32_16x16x64_i8 with all-zero and random operand
//           bytes, operands in registers or re-read from LDS every k-step (the GEMM's inner loop)
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
#define CK(x)                                                                     \
    do {                                                                          \
        hipError_t e = (x);                                                       \
        if (e != hipSuccess) {                                                    \
            printf("HIP error %s at line %d\n", hipGetErrorString(e), __LINE__);  \
            exit(1);                                                              \
        }                                                                         \
    } while (0)

extern __shared__ __attribute__((aligned(16))) char lds[];

template <class F>
static float best_ms(F f, int reps = 5) {
    hipEvent_t a, b;
    CK(hipEventCreate(&a));
    CK(hipEventCreate(&b));
    f();
    CK(hipDeviceSynchronize());
    float best = 1e30f;
    for (int r = 0; r < reps; r++) {
        CK(hipEventRecord(a));
        f();
        CK(hipEventRecord(b));
        CK(hipEventSynchronize(b));
        float ms;
        CK(hipEventElapsedTime(&ms, a, b));
        if (ms < best) best = ms;
    }
    CK(hipEventDestroy(a));
    CK(hipEventDestroy(b));
    return best;
}

// ------------------------------------------------------------------ HBM streams
__global__ __launch_bounds__(256) void k_read(const u32x4 *__restrict__ in, int *out, size_t n) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x, stride = (size_t)gridDim.x * 256;
    u32x4 acc = {0, 0, 0, 0};
    for (; i < n; i += stride) acc ^= __builtin_nontemporal_load(in + i);
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678u) out[0] = 1;
}
__global__ __launch_bounds__(256) void k_fill(u32x4 *__restrict__ out, size_t n) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x, stride = (size_t)gridDim.x * 256;
    u32x4 v = {1, 2, 3, (unsigned)i};
    for (; i < n; i += stride) __builtin_nontemporal_store(v, out + i);
}
__global__ __launch_bounds__(256) void k_copy(const u32x4 *__restrict__ in, u32x4 *__restrict__ out, size_t n) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x, stride = (size_t)gridDim.x * 256;
    for (; i < n; i += stride) __builtin_nontemporal_store(__builtin_nontemporal_load(in + i), out + i);
}
__global__ __launch_bounds__(256) void k_halve(const u32x4 *__restrict__ in, u32x2 *__restrict__ out, size_t n) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x, stride = (size_t)gridDim.x * 256;
    for (; i < n; i += stride) {
        u32x4 v = __builtin_nontemporal_load(in + i);
        u32x2 o = {v.x ^ v.y, v.z ^ v.w};
        __builtin_nontemporal_store(o, out + i);
    }
}

static void probe_hbm(int cus, int *dout) {
    const size_t bytes = (size_t)1 << 30, n = bytes / 16;
    void *a, *b;
    CK(hipMalloc(&a, bytes));
    CK(hipMalloc(&b, bytes));
    CK(hipMemset(a, 1, bytes));
    CK(hipMemset(b, 2, bytes));
    for (int per_cu : {3, 4, 8}) {
        const int blocks = cus * per_cu;
        float ms = best_ms([&] { k_read<<<blocks, 256>>>((const u32x4 *)a, dout, n); });
        printf("hbm read   %d wg/CU: %6.2f TB/s\n", per_cu, bytes / ms / 1e9);
        ms = best_ms([&] { k_fill<<<blocks, 256>>>((u32x4 *)b, n); });
        printf("hbm write  %d wg/CU: %6.2f TB/s\n", per_cu, bytes / ms / 1e9);
        ms = best_ms([&] { k_copy<<<blocks, 256>>>((const u32x4 *)a, (u32x4 *)b, n); });
        printf("hbm copy   %d wg/CU: %6.2f TB/s (read + write)\n", per_cu, 2.0 * bytes / ms / 1e9);
        ms = best_ms([&] { k_halve<<<blocks, 256>>>((const u32x4 *)a, (u32x2 *)b, n); });
        printf("hbm 2:1    %d wg/CU: %6.2f TB/s (16 B read + 8 B written per lane)\n", per_cu, 1.5 * bytes / ms / 1e9);
    }
    CK(hipFree(a));
    CK(hipFree(b));
}

// ------------------------------------------------------------------ L2 -> LDS direct copies
// A workgroup copies [256 rows x SEG bytes] blocks of a row-major region with `pitch` bytes per row.
template <int SEG>
__global__ __launch_bounds__(256) void k_dma(const char *base, long pitch, int rows_total, int kbytes, int iters,
                                             int depth, int *out) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int LPR = SEG / 16, RPB = 64 / LPR, BLOCKS = 256 / RPB / 4;
    int r0 = (blockIdx.x * 256) % rows_total, k0 = 0;
    for (int it = 0; it < iters; it++) {
        char *dst = lds + (it % depth) * (256 * SEG);
#pragma unroll
        for (int b = 0; b < BLOCKS; b++) {
            const int row = (wave * BLOCKS + b) * RPB + lane / LPR;
            const char *src = base + (long)(r0 + row) * pitch + k0 + (lane % LPR) * 16;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                             (__attribute__((address_space(3))) void *)(dst + (wave * BLOCKS + b) * 1024),
                                             16, 0, 0);
        }
        if (it + 1 >= depth) {  // keep depth-1 groups of BLOCKS copies in flight
            constexpr int KEEP3 = BLOCKS * 3;
            if (depth == 4)
                __builtin_amdgcn_s_waitcnt(0x0F70 | (KEEP3 & 15) | ((KEEP3 >> 4) << 14));
            else
                __builtin_amdgcn_s_waitcnt(0x0F70);
        }
        k0 += SEG;
        if (k0 >= kbytes) {
            k0 = 0;
            r0 += 256;
            if (r0 + 256 > rows_total) r0 = 0;
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    if (((int *)lds)[tid] == 0x12345678) out[0] = 1;
}

static void probe_l2lds(int cus, int *dout) {
    char *buf;
    const size_t bytes = (size_t)64 << 20;
    CK(hipMalloc(&buf, bytes));
    CK(hipMemset(buf, 1, bytes));
    CK(hipFuncSetAttribute((const void *)k_dma<64>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
    CK(hipFuncSetAttribute((const void *)k_dma<128>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
    const int K = 768, iters = 2000;
    for (int rows_total : {4096, 65536}) {  // 3 MB (L2-resident per XCD) and 50 MB (last-level cache)
        for (int depth : {2, 4}) {
            const int blocks = cus;
            float ms = best_ms([&] { k_dma<64><<<blocks, 256, depth * 256 * 64>>>(buf, K, rows_total, K, iters, depth, dout); });
            printf("l2->lds region %5.1f MB, %d copies deep,  64-B row segments: %6.2f TB/s\n", rows_total * 768.0 / 1e6,
                   depth, (double)blocks * iters * 256 * 64 / ms / 1e9);
            ms = best_ms([&] { k_dma<128><<<blocks, 256, depth * 256 * 128>>>(buf, K, rows_total, K, iters, depth, dout); });
            printf("l2->lds region %5.1f MB, %d copies deep, 128-B row segments: %6.2f TB/s\n", rows_total * 768.0 / 1e6,
                   depth, (double)blocks * iters * 256 * 128 / ms / 1e9);
        }
    }
    CK(hipFree(buf));
}

// ------------------------------------------------------------------ LDS read rate
__global__ __launch_bounds__(256) void k_ldsread(int iters, int *out) {
    for (int i = threadIdx.x; i < 32768 / 4; i += 256) ((int *)lds)[i] = i;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned addr = (unsigned)((lane * 16 + wave * 4096) & 16383);
    v4i a0, a1, a2, a3, a4, a5, a6, a7;
    for (int i = 0; i < iters; i++) {
        asm volatile(
            "ds_read_b128 %0, %8\n ds_read_b128 %1, %8 offset:2048\n ds_read_b128 %2, %8 offset:4096\n"
            "ds_read_b128 %3, %8 offset:6144\n ds_read_b128 %4, %8 offset:8192\n ds_read_b128 %5, %8 offset:10240\n"
            "ds_read_b128 %6, %8 offset:12288\n ds_read_b128 %7, %8 offset:14336\n s_waitcnt lgkmcnt(0)"
            : "=&v"(a0), "=&v"(a1), "=&v"(a2), "=&v"(a3), "=&v"(a4), "=&v"(a5), "=&v"(a6), "=&v"(a7)
            : "v"(addr)
            : "memory");
    }
    if (a0[0] + a1[0] + a2[0] + a3[0] + a4[0] + a5[0] + a6[0] + a7[0] == 123456789) out[0] = 1;
}

// ------------------------------------------------------------------ MFMA loops
__device__ unsigned hash32(unsigned i) {
    unsigned h = i * 2654435761u;
    h ^= h >> 15;
    h *= 2246822519u;
    h ^= h >> 13;
    return h;
}
// One workgroup of 8 wavefronts per CU, wave tile 128 x 64, 128 bytes of K per "slab" as in
// linear_mfma_persistent.  SHAPE 0: 32x32x32 (8 accumulators of 16 registers), 1: 16x16x64 (32 of 4).
// FROM_LDS: fragments are re-read from LDS every k-step (double buffered), else they stay in registers.
template <int SHAPE, bool FROM_LDS>
__global__ __launch_bounds__(512, 1) void k_mfma(int iters, int *out, int random_data) {
    constexpr int SLAB = 128;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < 131072 / 4; i += 512) ((int *)lds)[i] = random_data ? (int)hash32(i + blockIdx.x * 7919) : 0;
    __syncthreads();
    const int wave_r = (wave / 4) * 128, wave_o = (wave % 4) * 64;
    auto chunk_off = [&](int row, int chunk) { return row * SLAB + ((chunk ^ (row & 7)) << 4); };
    int stage = 0, s = 0;
    if (SHAPE == 0) {
        const int l32 = lane & 31, lhalf = lane >> 5;
        v16i acc[2][4];
        for (int i = 0; i < 2; i++)
            for (int j = 0; j < 4; j++)
                for (int v = 0; v < 16; v++) acc[i][j][v] = 0;
        v4i fw[2][2], fx[2][4];
        auto load_frags = [&](int buf, int stg, int ks) {
            const char *sx = lds + stg * 65536 + wave_r * SLAB, *sw = lds + stg * 65536 + (256 + wave_o) * SLAB;
            for (int i = 0; i < 2; i++) fw[buf][i] = *(const v4i *)(sw + chunk_off(i * 32 + l32, 2 * ks + lhalf));
            for (int j = 0; j < 4; j++) fx[buf][j] = *(const v4i *)(sx + chunk_off(j * 32 + l32, 2 * ks + lhalf));
        };
        load_frags(0, 0, 0);
        if (!FROM_LDS) load_frags(1, 0, 1);
        for (int it = 0; it < iters; it++) {
            const int next = stage ^ 1;
#pragma unroll
            for (int ks = 0; ks < 4; ks++) {
                const int cur = ks & 1;
                if (FROM_LDS) load_frags(cur ^ 1, ks + 1 < 4 ? stage : next, ks + 1 < 4 ? ks + 1 : 0);
#pragma unroll
                for (int i = 0; i < 2; i++)
#pragma unroll
                    for (int j = 0; j < 4; j++)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw[cur][i], fx[cur][j], acc[i][j], 0, 0, 0);
            }
            stage = next;
        }
        for (int i = 0; i < 2; i++)
            for (int j = 0; j < 4; j++)
                for (int v = 0; v < 16; v++) s += acc[i][j][v];
    } else {
        const int l16 = lane & 15, lq = lane >> 4;
        v4i acc[4][8];
        for (int i = 0; i < 4; i++)
            for (int j = 0; j < 8; j++)
                for (int v = 0; v < 4; v++) acc[i][j][v] = 0;
        v4i fw[2][4], fx[2][8];
        auto load_frags = [&](int buf, int stg, int ks) {
            const char *sx = lds + stg * 65536 + wave_r * SLAB, *sw = lds + stg * 65536 + (256 + wave_o) * SLAB;
            for (int i = 0; i < 4; i++) fw[buf][i] = *(const v4i *)(sw + chunk_off(i * 16 + l16, 4 * ks + lq));
            for (int j = 0; j < 8; j++) fx[buf][j] = *(const v4i *)(sx + chunk_off(j * 16 + l16, 4 * ks + lq));
        };
        load_frags(0, 0, 0);
        if (!FROM_LDS) load_frags(1, 0, 1);
        for (int it = 0; it < iters; it++) {
            const int next = stage ^ 1;
#pragma unroll
            for (int ks = 0; ks < 2; ks++) {
                const int cur = ks & 1;
                if (FROM_LDS) load_frags(cur ^ 1, ks + 1 < 2 ? stage : next, ks + 1 < 2 ? ks + 1 : 0);
#pragma unroll
                for (int i = 0; i < 4; i++)
#pragma unroll
                    for (int j = 0; j < 8; j++)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fw[cur][i], fx[cur][j], acc[i][j], 0, 0, 0);
            }
            stage = next;
        }
        for (int i = 0; i < 4; i++)
            for (int j = 0; j < 8; j++)
                for (int v = 0; v < 4; v++) s += acc[i][j][v];
    }
    if (s == 0x12345678) out[0] = s;
}

template <int SHAPE, bool FROM_LDS>
static void run_mfma(int cus, int *dout, const char *name) {
    CK(hipFuncSetAttribute((const void *)k_mfma<SHAPE, FROM_LDS>, hipFuncAttributeMaxDynamicSharedMemorySize, 131072));
    const int iters = 3000;
    for (int rnd = 0; rnd < 2; rnd++) {
        float ms = best_ms([&] { k_mfma<SHAPE, FROM_LDS><<<cus, 512, 131072>>>(iters, dout, rnd); });
        const double ops = (double)cus * 8 * iters * 2.0 * 128 * 64 * 128;
        printf("mfma i8 %-9s fragments %-13s operands %-12s: %7.1f TOP/s\n", name, FROM_LDS ? "from LDS" : "in registers",
               rnd ? "random bytes" : "all zero", ops / ms / 1e9);
    }
}

int main(int argc, char **argv) {
    hipDeviceProp_t prop;
    CK(hipGetDeviceProperties(&prop, 0));
    const int cus = prop.multiProcessorCount;
    printf("device %s, %d CUs, clock %d kHz, LDS per workgroup %zu B, L2 %d B\n", prop.gcnArchName, cus, prop.clockRate,
           prop.sharedMemPerBlock, prop.l2CacheSize);
    int *dout;
    CK(hipMalloc(&dout, 64));
    const char *what = argc > 1 ? argv[1] : "all";
    const bool all = !strcmp(what, "all");
    if (all || !strcmp(what, "hbm")) probe_hbm(cus, dout);
    if (all || !strcmp(what, "l2lds")) probe_l2lds(cus, dout);
    if (all || !strcmp(what, "lds")) {
        const int iters = 20000, blocks = cus * 4;
        float ms = best_ms([&] { k_ldsread<<<blocks, 256, 32768>>>(iters, dout); });
        const double bytes = (double)blocks * 256 * iters * 8 * 16;
        printf("lds ds_read_b128, 16 waves/CU: %6.1f TB/s = %5.1f B/clk/CU at %d MHz\n", bytes / ms / 1e9,
               bytes / (ms * 1e-3) / cus / (prop.clockRate * 1e3), prop.clockRate / 1000);
    }
    if (all || !strcmp(what, "mfma")) {
        run_mfma<0, false>(cus, dout, "32x32x32");
        run_mfma<0, true>(cus, dout, "32x32x32");
        run_mfma<1, false>(cus, dout, "16x16x64");
        run_mfma<1, true>(cus, dout, "16x16x64");
    }
    CK(hipFree(dout));
    return 0;
}
