// The worker rules of the elastic update, shared by the streaming update kernels and by the
// matrix-product epilogue that applies them to a freshly computed gradient tile.
#pragma once
#include <hip/hip_runtime.h>

namespace easgd {

// Marks a loaded value as needed at this point, whatever the compiler can prove about its later uses.  The
// streaming tiles call it on a worker's values after the last load of that worker in the tile that holds the end
// of a row: lanes past the end store nothing, and the loads of such a lane would otherwise move behind the branch
// that skips its stores, where they are waited for one after the other.
template <typename T>
__device__ __forceinline__ void keep_loaded(T &x) { asm volatile("" : "+v"(x)); }

// s*a + c with one rounding (T = float or a float vector, s a scalar).  The rules below spell out which of their
// products are fused: left to the compiler the choice depends on the surrounding code (a product with two uses is
// computed once and then not fused), and kernels that must give the same bits would not.
template <typename T>
__device__ __forceinline__ T fma_s(float s, T a, T c) { return __builtin_elementwise_fma((T)s, a, c); }

// One worker's rule applied to T = float or a float vector.  Returns d = w - c (time-t values).
template <bool MOM, typename T>
__device__ __forceinline__ T worker_rule(T &w, T &v, T g, T c, float eta, float rho, float alpha, float delta)
{
    const T d = w - c;
    if constexpr (MOM) {
        v = fma_s(delta, v, -(eta * g));      // Eq. (5)
        w = fma_s(-alpha, d, w + v);          // Eq. (6)
    } else {
        w = fma_s(-eta, fma_s(rho, d, g), w); // Eq. (1)
    }
    return d;
}

// ---- bfloat16 storage of gradients and momentum buffers (an extension; the paper keeps fp32 throughout) ----
// bfloat16 = the upper 16 bits of an fp32.  Widening is exact.  Narrowing rounds to nearest, ties to even; beyond
// the largest finite value it gives infinity; a NaN becomes 0x7FC0 with the input's sign.
__device__ __forceinline__ float bf16_widen(unsigned short b) { return __uint_as_float((unsigned)b << 16); }

__device__ __forceinline__ unsigned short bf16_narrow(float x)
{
    const unsigned u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)(((u >> 16) & 0x8000u) | 0x7fc0u);
    // adds just under half a unit of the kept part, and one more if the kept part is odd: ties go to even
    return (unsigned short)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

// One worker's rule on one parameter whose momentum is stored as bfloat16 (g: the gradient as fp32).
// Eq. (5) decides a stored code, so its arithmetic is pinned: fl(fl(delta*v) - fl(eta*g)), no fused
// multiply-add, then narrowed; Eq. (6) adds V_{t+1} as stored.  Returns d = w - c (time-t values).
template <bool MOM>
__device__ __forceinline__ float worker_rule_bf16(float &w, unsigned short &v16, float g, float c,
                                                  float eta, float rho, float alpha, float delta)
{
    const float d = w - c;
    if constexpr (MOM) {
        float cand;
        {
#pragma clang fp contract(off)
            const float dv = delta * bf16_widen(v16);
            const float eg = eta * g;
            cand = dv - eg;                   // Eq. (5), each operation rounded on its own
        }
        v16 = bf16_narrow(cand);
        w = fma_s(-alpha, d, w + bf16_widen(v16));   // Eq. (6) with V_{t+1} as stored
    } else {
        w = fma_s(-eta, fma_s(rho, d, g), w); // Eq. (1)
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
        Wc[j] = fma_s(alpha, acc, c);
    }
    const size_t tail = N - n * LANES;        // only for the vector form
    if (block == n_blocks - 1 && (size_t)tid < tail) {
        const size_t k = n * LANES + (size_t)tid;
        const float c = Wcp[k];
        float acc = 0.f;
        for (int i = 0; i < P; ++i) acc += Wp[(size_t)i * ld + k] - c;
        oldp[k] = c;
        Wcp[k] = fma_s(alpha, acc, c);
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
