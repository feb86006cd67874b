// Internal helpers of the EASGD HIP library (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <atomic>
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

// Launch-shape options: process-wide, each one an atomic word, so that a host thread that sets one while another
// thread is inside a call is no data race (the running call may see the old or the new value of each option).
struct Options {
    std::atomic<long> update_blocks_per_cu{0};
    std::atomic<long> update_nontemporal{1};
    std::atomic<long> update_groups{4};
    std::atomic<long> gemm_tile{0};
    std::atomic<long> round_overlap{1};
    std::atomic<long> gemm_xcd{1};
    std::atomic<long> gemm_pair{1};
    std::atomic<long> mlp_head{1};
};
Options &options();

// Kernel launches issued by the library in this process (easgd_launch_count, a measurement aid).
std::atomic<unsigned long long> &launch_counter();
#define EASGD_LAUNCH(...)                                                          \
    do {                                                                           \
        easgd::launch_counter().fetch_add(1, std::memory_order_relaxed);           \
        hipLaunchKernelGGL(__VA_ARGS__);                                           \
    } while (0)

// Steps (2)-(5) of a round on the parameter range [0, N) of every replica (defined with the
// elastic update kernels); V == nullptr selects Eq. (1), otherwise Eq. (5),(6).
int elastic_range(float *W, float *V, const float *G, float *Wc, int P, size_t N, size_t ld,
                  float eta, float rho, float delta, void *stream);

// Eq. (2) alone, ahead of the worker rules: Wc[j] <- Wc[j] + alpha * sum_i (W_i[j] - Wc[j]), ascending i;
// the time-t center is saved to old[0..N).
int center_range(const float *W, float *Wc, float *old, int P, size_t N, size_t ld, float alpha, void *stream);

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
// natural alignment of the element type (a NULL pointer passes: it is checked separately)
inline bool aligned_to(const void *p, size_t bytes) { return (reinterpret_cast<uintptr_t>(p) & (bytes - 1)) == 0; }

inline int check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(EASGD_ELAUNCH, "%s: %s", what, hipGetErrorString(e));
    return EASGD_OK;
}

}  // namespace easgd
