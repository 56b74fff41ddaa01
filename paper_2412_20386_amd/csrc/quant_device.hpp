// Device helpers shared by the quantizing kernels of libptq4vm (gfx950): the hardware fp32 -> int32
// conversion with defined behaviour for specials, and the byte packing of four int8 codes.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ptq4vm {

// fp32 -> int32 conversion with the hardware's defined behaviour for specials
// (NaN -> 0, out-of-range saturates), which a C++ cast leaves undefined.
__device__ __forceinline__ int cvt_i32_f32(float v) {
    int i;
    asm("v_cvt_i32_f32 %0, %1" : "=v"(i) : "v"(v));
    return i;
}

// The low bytes of four ints as one dword, a in the lowest byte.
__device__ __forceinline__ uint32_t pack4(int a, int b, int c, int d) {
    const uint32_t lo = __builtin_amdgcn_perm((uint32_t)b, (uint32_t)a, 0x0c0c0400u);  // a.b0 | b.b0 << 8
    const uint32_t hi = __builtin_amdgcn_perm((uint32_t)d, (uint32_t)c, 0x0c0c0400u);
    return __builtin_amdgcn_perm(hi, lo, 0x05040100u);
}

// Store of quantized codes that the next kernel (the linear) reads.  Written at device scope (the `sc1` form of the
// store: through the XCD's L2 to the memory side), the lines are found in the memory-side cache by the consumer,
// whichever XCD it runs on; a non-temporal store streams them past it.  The quantizer itself runs at the same rate
// either way; quantizer + linear on 24 rotating buffer sets: in_proj 166.5 -> 153.0 us, out_proj 110.5 -> 102.9 us
// (ordinary write-back stores: 157.7 / 104.8 us, and the quantizer alone 5-8 % slower).
// 4-, 8- and 16-byte values; `ptr` aligned to the size.
template <typename T>
__device__ __forceinline__ void store_for_next_kernel(T *ptr, const T &value) {
    static_assert(sizeof(T) == 4 || sizeof(T) == 8 || sizeof(T) == 16, "one dword, two or four");
    if constexpr (sizeof(T) == 4) {
        __hip_atomic_store(reinterpret_cast<uint32_t *>(ptr), __builtin_bit_cast(uint32_t, value), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    } else if constexpr (sizeof(T) == 8) {
        __hip_atomic_store(reinterpret_cast<uint64_t *>(ptr), __builtin_bit_cast(uint64_t, value), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    } else {
        // No 16-byte form that the compiler can be asked for, so the instruction is written out.  The compiler does
        // not look inside: the two wait states that a store of more than 8 bytes needs before its data registers may
        // be rewritten (left out, a stray dword showed up in the stored codes) follow it here as s_nop 1.
        asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" ::"v"(ptr), "v"(value) : "memory");
    }
}

}  // namespace ptq4vm
