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
    std::atomic<long> update_nontemporal{2};
    std::atomic<long> update_groups{0};
    std::atomic<long> update_layout{2};
    std::atomic<long> gemm_tile{0};
    std::atomic<long> round_overlap{1};
    std::atomic<long> gemm_xcd{1};
    std::atomic<long> gemm_pair{1};
    std::atomic<long> mlp_head{1};
    std::atomic<long> round_single_launch{0};
    std::atomic<long> round_spin_limit{0};
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
// the time-t center is saved to old[0..N).  beside: the launch runs on a stream of its own beside matrix products
// (then it takes one block per compute unit, see the definition).
int center_range(const float *W, float *Wc, float *old, int P, size_t N, size_t ld, float alpha, void *stream, bool beside = false);

// Where the streaming update kernels find their parameters.  A block of 256 threads handles GROUPS groups of four
// consecutive parameters per thread: thread `tid` of block `t` owns groups first(t, tid) + q * STRIDE, q < GROUPS.
//   DIES = false: block t owns the contiguous run [t*GROUPS*256, (t+1)*GROUPS*256) (GROUPS*4 KiB per fp32 row).
//   DIES = true:  workgroups go to the eight dies in turn by block index, so eight consecutive blocks run one per
//     die.  They share a super-tile of 8*GROUPS*256 groups and interleave in pieces of 64 groups (1 KiB of an
//     fp32 row, one wavefront's 128-bit access): piece p (p < 4*GROUPS) of block x (x = t % 8) is piece
//     8*p + x of the super-tile.  Every die then touches every eighth KiB of every stream instead of runs of
//     GROUPS*4 KiB, which spreads each die's requests evenly over the memory channels whatever physical pages
//     the operands sit in: measured at P = 16, N = 61 M with momentum 5.4 -> 6.4 TB/s in the usual
//     placement of the operands, 6.0 -> 6.7 TB/s for the plain rule at P = 8.
template <int GROUPS, bool DIES>
struct TileMap {
    static constexpr size_t STRIDE = DIES ? 2048 : 256;
    static constexpr size_t SUPER = (size_t)8 * GROUPS * 256;
    __host__ __device__ static size_t tiles(size_t n4)
    {
        return DIES ? 8 * ((n4 + SUPER - 1) / SUPER) : (n4 + (size_t)GROUPS * 256 - 1) / ((size_t)GROUPS * 256);
    }
    __device__ static size_t first(size_t t, unsigned tid)
    {
        if (DIES) return (t >> 3) * SUPER + ((((size_t)(tid >> 6) << 3) + (t & 7)) << 6) + (tid & 63);
        return t * ((size_t)GROUPS * 256) + tid;
    }
    // the largest group index block t touches (thread 255, its last group)
    __device__ static size_t last(size_t t) { return first(t, 255) + (size_t)(GROUPS - 1) * STRIDE; }
};

// Launch shape of a streaming update over N parameters per row: groups per thread (1, 2, 4 or 8), the tile map and
// the grid.  `wide`: the kernel streams three arrays per worker (momentum), for which longer runs per thread pay.
struct UpdateShape {
    int groups;
    bool dies;
    size_t blocks;
};
UpdateShape update_shape(size_t N, bool wide);

// Whether a streaming update that moves `bytes` per round uses non-temporal loads and stores
// (EASGD_OPT_UPDATE_NONTEMPORAL; chosen per call by default).  Measured on replicas of 0.37 to 6.8 GB per round:
// above about half a gigabyte the streaming forms are 2-16 % faster; below it plain accesses are 10-15 % faster,
// because part of what one round writes is still in the last-level cache (256 MB) when the next reader comes.
bool update_nontemporal(size_t bytes);

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
