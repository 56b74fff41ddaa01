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

}  // namespace ptq4vm
