// Internal helpers of the EASGD HIP library (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <cstdarg>
#include <cstddef>
#include <cstdint>
// the C ABI is the only thing exported from the shared library
#pragma GCC visibility push(default)
#include "../../include/easgd.h"
#pragma GCC visibility pop

namespace easgd {

// Records a formatted message for easgd_last_error() and returns `code`.
int fail(int code, const char *fmt, ...);
void clear_error();

// Number of compute units of the current device (cached per device).
int num_cus();

struct Options {
    long update_blocks_per_cu = 0;
    long update_nontemporal = 1;
    long update_groups = 4;
    long gemm_tile = 0;
};
Options &options();

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline int check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(EASGD_ELAUNCH, "%s: %s", what, hipGetErrorString(e));
    return EASGD_OK;
}

}  // namespace easgd
