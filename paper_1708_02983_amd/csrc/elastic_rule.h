// The worker rules of the elastic update, shared by the streaming update kernels and by the
// matrix-product epilogue that applies them to a freshly computed gradient tile.
#pragma once
#include <hip/hip_runtime.h>

namespace easgd {

// One worker's rule applied to T = float or a float vector.  Returns d = w - c (time-t values).
template <bool MOM, typename T>
__device__ __forceinline__ T worker_rule(T &w, T &v, T g, T c, float eta, float rho, float alpha, float delta)
{
    const T d = w - c;
    if constexpr (MOM) {
        v = delta * v - eta * g;              // Eq. (5)
        w = (w + v) - alpha * d;              // Eq. (6)
    } else {
        w = w - eta * (g + rho * d);          // Eq. (1)
    }
    return d;
}

// Eq. (2) alone, ahead of the worker rules, for block `block` of 256 threads (T = float or a vector of 4 floats;
// the last of n_blocks blocks also owns the N % 4 tail of the vector form):
//   Wc[j] <- c + alpha * sum_i (W_i[j] - c)  with c = Wc[j], workers in ascending order (the order of the fused
// update kernels), and the time-t value c saved to old[j] for the worker rules that run later in the round.
// W is read with ordinary loads: the same values are needed again soon.
template <typename T>
__device__ __forceinline__ void center_rule_block(const float *__restrict__ Wp, float *__restrict__ Wcp,
                                                  float *__restrict__ oldp, int P, size_t N, size_t ld, float alpha,
                                                  size_t block, size_t n_blocks, int tid)
{
    constexpr size_t LANES = sizeof(T) / sizeof(float);
    const T *__restrict__ W = (const T *)Wp;
    T *__restrict__ Wc = (T *)Wcp;
    T *__restrict__ old = (T *)oldp;
    const size_t n = N / LANES, ldt = ld / LANES;
    const size_t j = block * 256 + (size_t)tid;
    if (j < n) {
        const T c = Wc[j];
        T acc = c - c;
        int i = 0;
        for (; i + 4 <= P; i += 4) {
            T w[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) w[u] = W[(size_t)(i + u) * ldt + j];
#pragma unroll
            for (int u = 0; u < 4; ++u) acc += w[u] - c;
        }
        for (; i < P; ++i) acc += W[(size_t)i * ldt + j] - c;
        old[j] = c;
        Wc[j] = c + alpha * acc;
    }
    const size_t tail = N - n * LANES;        // only for the vector form
    if (block == n_blocks - 1 && (size_t)tid < tail) {
        const size_t k = n * LANES + (size_t)tid;
        const float c = Wcp[k];
        float acc = 0.f;
        for (int i = 0; i < P; ++i) acc += Wp[(size_t)i * ld + k] - c;
        oldp[k] = c;
        Wcp[k] = c + alpha * acc;
    }
}

// What a launch needs to run the center rule on extra blocks of its grid (blocks == 0: none).
struct CenterJob {
    const float *W;
    float *Wc, *old;
    size_t N, ld;
    int P, vec;
    float alpha;
    unsigned blocks, first_block;           // the job's blocks are [first_block, first_block + blocks) of the grid
};

}  // namespace easgd
