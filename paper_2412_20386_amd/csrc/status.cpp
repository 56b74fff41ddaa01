// Status strings, version and the thread-local HIP error text of libptq4vm.
#include <stdio.h>

#include "common.hpp"

namespace ptq4vm {

static thread_local char g_hip_error[256] = "";

int record_hip_error(hipError_t err, const char *what) {
    snprintf(g_hip_error, sizeof(g_hip_error), "%s: %s (%d)", what, hipGetErrorString(err), (int)err);
    return PTQ4VM_ERR_HIP;
}

}  // namespace ptq4vm

extern "C" {

const char *ptq4vm_status_string(int status) {
    switch (status) {
        case PTQ4VM_OK: return "ok";
        case PTQ4VM_ERR_NULL: return "a required pointer is NULL";
        case PTQ4VM_ERR_SHAPE: return "invalid size";
        case PTQ4VM_ERR_STRIDE: return "leading dimension smaller than the row width";
        case PTQ4VM_ERR_ALIGN: return "misaligned base pointer";
        case PTQ4VM_ERR_HIP: return "HIP runtime error";
        case PTQ4VM_ERR_VALUE: return "a scale is not a finite number greater than zero";
        default: return "unknown status";
    }
}

const char *ptq4vm_last_hip_error(void) { return ptq4vm::g_hip_error; }

int ptq4vm_version(void) { return 0 * 10000 + 1 * 100 + 0; }

}  // extern "C"
