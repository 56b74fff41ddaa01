// Host-side helpers shared by the entry points of libptq4vm: status codes, the thread-local
// HIP error text, argument checks.  No device code here.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/ptq4vm.h"

namespace ptq4vm {

// Records the text of a failed HIP call for ptq4vm_last_hip_error() and returns PTQ4VM_ERR_HIP.
int record_hip_error(hipError_t err, const char *what);

inline bool aligned_to(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// Every launch goes through this: catches configuration errors (bad grid, too much LDS)
// right after the enqueue without synchronising.
inline int check_launch(const char *what) {
    hipError_t err = hipGetLastError();
    return err == hipSuccess ? PTQ4VM_OK : record_hip_error(err, what);
}

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Raises a kernel's dynamic-LDS limit (needed above 64 KiB).  The setting belongs to the current
// device's copy of the function, so it is applied on every launch rather than cached in a flag:
// a host-side table update, negligible next to the launch itself, and correct for any number of
// devices and threads.
inline int set_lds_limit(const void *kernel, int bytes, const char *what) {
    hipError_t err = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    return err == hipSuccess ? PTQ4VM_OK : record_hip_error(err, what);
}

}  // namespace ptq4vm
