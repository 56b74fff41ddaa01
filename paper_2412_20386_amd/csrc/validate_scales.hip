// Debug validator for the device-resident scale vectors of the quantized linear (Sec. 5.1: the
// per-token steps Delta_X and per-output-channel steps Delta_W; Sec. 2.4: the smoothing vector s).
// The hot-path kernels never inspect these values; a step that is zero, negative, infinite or NaN
// silently produces garbage codes.  This entry point counts such entries on the device and reports
// them to the host.  It is the one call of the library that synchronises its stream.
//
// Two launches: `count_bad_scales` gives every workgroup one block of kBlockElems consecutive
// entries of the concatenated index space [s_tok | m | s_w] and writes that block's three counts to
// partial[block]; `sum_bad_scales` (one workgroup) adds the partial counts up.  No atomics, and
// nothing has to be zeroed beforehand: every partial slot that is read was written by this call.
#include <mutex>

#include "common.hpp"

namespace {

constexpr int kThreads = 256;
constexpr int kBlockElems = PTQ4VM_VALIDATE_BLOCK;  // entries per workgroup and per partial slot

struct Counts {
    int v[4];  // bad entries of s_tok, m, s_w; v[3] unused (16-byte slots)
};

__device__ __forceinline__ bool bad_scale(float v) { return !(v > 0.0f && v < __builtin_inff()); }

__global__ __launch_bounds__(kThreads) void count_bad_scales(const float *__restrict__ s_tok, int64_t L,
                                                             const float *__restrict__ m, int64_t K,
                                                             const float *__restrict__ s_w, int64_t N,
                                                             Counts *__restrict__ partial) {
    __shared__ int red[kThreads / 64][3];
    const int64_t lo = (int64_t)blockIdx.x * kBlockElems;
    int bad[3] = {0, 0, 0};
    for (int i = threadIdx.x; i < kBlockElems; i += kThreads) {
        const int64_t e = lo + i;
        if (e < L) {
            bad[0] += bad_scale(s_tok[e]);
        } else if (e < L + K) {
            bad[1] += bad_scale(m[e - L]);
        } else if (e < L + K + N) {
            bad[2] += bad_scale(s_w[e - L - K]);
        }
    }
#pragma unroll
    for (int c = 0; c < 3; c++) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) bad[c] += __shfl_xor(bad[c], off, 64);
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6][c] = bad[c];
    }
    __syncthreads();
    if (threadIdx.x < 4) {
        int sum = 0;
        if (threadIdx.x < 3)
            for (int w = 0; w < kThreads / 64; w++) sum += red[w][threadIdx.x];
        partial[blockIdx.x].v[threadIdx.x] = sum;
    }
}

__global__ __launch_bounds__(kThreads) void sum_bad_scales(const Counts *__restrict__ partial, int64_t blocks,
                                                           int32_t *__restrict__ bad_counts) {
    __shared__ int red[kThreads / 64][3];
    int bad[3] = {0, 0, 0};
    for (int64_t b = threadIdx.x; b < blocks; b += kThreads) {
        const Counts c = partial[b];
        bad[0] += c.v[0], bad[1] += c.v[1], bad[2] += c.v[2];
    }
#pragma unroll
    for (int c = 0; c < 3; c++) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) bad[c] += __shfl_xor(bad[c], off, 64);
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6][c] = bad[c];
    }
    __syncthreads();
    if (threadIdx.x < 3) {
        int sum = 0;
        for (int w = 0; w < kThreads / 64; w++) sum += red[w][threadIdx.x];
        bad_counts[threadIdx.x] = sum;
    }
}

}  // namespace

namespace ptq4vm {

// Host half shared by both entry points.
int validate_scales_args(const float *s_tok, int64_t L, const float *m, int64_t K, const float *s_w, int64_t N,
                         const int32_t *bad_counts, int64_t *blocks) {
    if (!bad_counts) return PTQ4VM_ERR_NULL;
    if (L < 0 || K < 0 || N < 0) return PTQ4VM_ERR_SHAPE;
    if ((L > 0 && !s_tok) || (K > 0 && !m) || (N > 0 && !s_w)) return PTQ4VM_ERR_NULL;
    if (L > PTQ4VM_VALIDATE_MAX_ELEMS || K > PTQ4VM_VALIDATE_MAX_ELEMS || N > PTQ4VM_VALIDATE_MAX_ELEMS ||
        L + K + N > PTQ4VM_VALIDATE_MAX_ELEMS)
        return PTQ4VM_ERR_SHAPE;
    if (!aligned_to(s_tok, 4) || !aligned_to(m, 4) || !aligned_to(s_w, 4) || !aligned_to(bad_counts, 4))
        return PTQ4VM_ERR_ALIGN;
    *blocks = ceil_div(L + K + N, kBlockElems);
    return PTQ4VM_OK;
}

// Enqueues both kernels with `partial` (device, blocks slots of 16 bytes): afterwards, in stream order,
// bad_counts holds the three counts.
int validate_scales_enqueue(const float *s_tok, int64_t L, const float *m, int64_t K, const float *s_w, int64_t N,
                            int32_t *bad_counts, void *partial, int64_t blocks, hipStream_t stream) {
    if (blocks == 0) blocks = 1;  // all three vectors empty: one workgroup writes three zeros
    count_bad_scales<<<dim3((unsigned)blocks), dim3(kThreads), 0, stream>>>(s_tok, L, m, K, s_w, N,
                                                                          static_cast<Counts *>(partial));
    const int rc = check_launch("count_bad_scales");
    if (rc != PTQ4VM_OK) return rc;
    sum_bad_scales<<<dim3(1), dim3(kThreads), 0, stream>>>(static_cast<const Counts *>(partial), blocks, bad_counts);
    return check_launch("sum_bad_scales");
}

// Enqueues the kernels, copies the three counts to the host, waits for the stream and turns a non-zero
// count into PTQ4VM_ERR_VALUE.
int validate_scales_run(const float *s_tok, int64_t L, const float *m, int64_t K, const float *s_w, int64_t N,
                        int32_t *bad_counts, void *partial, int64_t blocks, hipStream_t stream) {
    const int rc = validate_scales_enqueue(s_tok, L, m, K, s_w, N, bad_counts, partial, blocks, stream);
    if (rc != PTQ4VM_OK) return rc;
    int32_t host_counts[3] = {0, 0, 0};
    hipError_t err = hipMemcpyAsync(host_counts, bad_counts, sizeof(host_counts), hipMemcpyDeviceToHost, stream);
    if (err != hipSuccess) return record_hip_error(err, "validate_scales: copy of the counts");
    err = hipStreamSynchronize(stream);
    if (err != hipSuccess) return record_hip_error(err, "validate_scales: stream synchronisation");
    return (host_counts[0] | host_counts[1] | host_counts[2]) ? PTQ4VM_ERR_VALUE : PTQ4VM_OK;
}

}  // namespace ptq4vm

extern "C" int ptq4vm_validate_scales(const float *s_tok, int64_t L, const float *m, int64_t K, const float *s_w,
                                      int64_t N, int32_t *bad_counts, void *workspace, int64_t workspace_bytes,
                                      void *stream_) {
    int64_t blocks = 0;
    const int rc = ptq4vm::validate_scales_args(s_tok, L, m, K, s_w, N, bad_counts, &blocks);
    if (rc != PTQ4VM_OK) return rc;
    if (!workspace) return PTQ4VM_ERR_NULL;
    if (workspace_bytes < PTQ4VM_VALIDATE_WORKSPACE_BYTES(L, K, N)) return PTQ4VM_ERR_SHAPE;
    if (!ptq4vm::aligned_to(workspace, 16)) return PTQ4VM_ERR_ALIGN;
    return ptq4vm::validate_scales_run(s_tok, L, m, K, s_w, N, bad_counts, workspace, blocks,
                                       static_cast<hipStream_t>(stream_));
}

// ---- the variant that allocates nothing: the partial counts live in a device array of the library itself

namespace {

constexpr int64_t kStaticSlots = PTQ4VM_VALIDATE_STATIC_MAX_ELEMS / PTQ4VM_VALIDATE_BLOCK + 1;
static __device__ __align__(256) unsigned char scratch[16 * kStaticSlots];

// In host code `scratch` is only a handle for the symbol: each GPU holds its own copy of the array at its own
// address, asked for once per device (with that device current) and kept.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_of_device[kMaxDevices] = {};

int scratch_of_current_device(void **out) {
    int device = -1;
    hipError_t err = hipGetDevice(&device);
    if (err != hipSuccess) return ptq4vm::record_hip_error(err, "hipGetDevice");
    if (device < 0 || device >= kMaxDevices)
        return ptq4vm::record_hip_error(hipErrorInvalidDevice, "validate_scales_static: device ordinal beyond the table");
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_of_device[device]) {
        void *ptr = nullptr;
        err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (err != hipSuccess || !ptr)
            return ptq4vm::record_hip_error(err == hipSuccess ? hipErrorInvalidSymbol : err, "hipGetSymbolAddress(scratch)");
        g_scratch_of_device[device] = ptr;
    }
    *out = g_scratch_of_device[device];
    return PTQ4VM_OK;
}

}  // namespace

extern "C" int ptq4vm_validate_scales_static(const float *s_tok, int64_t L, const float *m, int64_t K, const float *s_w,
                                             int64_t N, int32_t *bad_counts, void *stream_) {
    int64_t blocks = 0;
    int rc = ptq4vm::validate_scales_args(s_tok, L, m, K, s_w, N, bad_counts, &blocks);
    if (rc != PTQ4VM_OK) return rc;
    if (L + K + N > PTQ4VM_VALIDATE_STATIC_MAX_ELEMS) return PTQ4VM_ERR_SHAPE;  // more partial counts than the array holds
    void *partial = nullptr;
    rc = scratch_of_current_device(&partial);
    if (rc != PTQ4VM_OK) return rc;
    return ptq4vm::validate_scales_enqueue(s_tok, L, m, K, s_w, N, bad_counts, partial, blocks,
                                           static_cast<hipStream_t>(stream_));
}
