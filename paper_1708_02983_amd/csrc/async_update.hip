// The asynchronous forms of the elastic exchange that the paper compares Sync EASGD with (Section 2.6 and
// Algorithm 1, "Original EASGD"; Section 5.1, "Async EASGD", "Async MEASGD", "Hogwild EASGD"), on replicas that
// share one memory.
//
// async_easgd_round: the master serves ONE worker at a time, in a given schedule (rank order for Original
//   EASGD, arrival order for Async EASGD).  Per turn of worker i, from the values at the start of the turn:
//       W_i <- W_i - eta*(g_i + rho*(W_i - Wc))   (or Eq. (5),(6) with momentum),   Wc <- Wc + eta*rho*(W_i - Wc).
//   The turns of a parameter are independent of every other parameter, so the serial master becomes a serial
//   loop inside the thread that owns the parameter: the center stays in a register for the whole schedule and
//   each turn streams one worker's rows.  Same skeleton, tile map and byte count per turn as the synchronous
//   kernel; the result is that of the turns taken one after the other, bit for bit.
//
// hogwild_easgd_round: no order and no lock.  Every (worker, tile) pair is a block of its own; it reads the
//   center as it finds it, applies the worker rule, and adds eta*rho*(W_i - Wc) to the center with a
//   floating-point atomic, while the blocks of the other workers do the same to the same elements.  Which value
//   of the center a worker sees, and the order of the additions, vary from run to run: the result is not
//   reproducible, which is the point of the comparison.  What every interleaving leaves unchanged: the momentum
//   buffers, and sum_i W_i + Wc (a worker loses exactly what it gives the center).
#include "common.h"
#include "elastic_rule.h"

namespace easgd {

typedef float f32x4 __attribute__((ext_vector_type(4)));

// the schedule travels in the kernel arguments
struct Schedule {
    int n;
    unsigned char worker[EASGD_MAX_SCHEDULE];
};

template <bool NT, typename T>
__device__ __forceinline__ T ld_stream(const T *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}

template <bool NT, typename T>
__device__ __forceinline__ void st_stream(T *p, T v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// One tile of the 128-bit path (the structure of the synchronous kernel's tile: thread-owned groups
// j0 + q*STRIDE; FULL = every group of the block lies inside the row; no load is guarded in either form: lanes
// past the end of the row read its last group and store nothing).
template <bool MOM, int GROUPS, size_t STRIDE, bool FULL>
__device__ __forceinline__ void async_tile(f32x4 *__restrict__ W, f32x4 *__restrict__ V, const f32x4 *__restrict__ G,
                                           f32x4 *__restrict__ Wc, const Schedule &sch, size_t n4, size_t ld4, size_t j0,
                                           float eta, float rho, float alpha, float delta)
{
    f32x4 c[GROUPS];
    size_t jl[GROUPS];
#pragma unroll
    for (int q = 0; q < GROUPS; ++q) {
        const size_t j = j0 + (size_t)q * STRIDE;
        jl[q] = (FULL || j < n4) ? j : n4 - 1;
        c[q] = Wc[jl[q]];
    }
    for (int t = 0; t < sch.n; ++t) {                    // the master's turns, one worker each, in schedule order
        const size_t row = (size_t)sch.worker[t] * ld4;
        f32x4 w[GROUPS], g[GROUPS], v[GROUPS];
#pragma unroll
        for (int q = 0; q < GROUPS; ++q) {
            w[q] = ld_stream<true>(W + row + jl[q]);
            g[q] = ld_stream<true>(G + row + jl[q]);
            if constexpr (MOM) v[q] = ld_stream<true>(V + row + jl[q]);
        }
        if constexpr (!FULL) {
#pragma unroll
            for (int q = 0; q < GROUPS; ++q) {
                keep_loaded(w[q]);
                keep_loaded(g[q]);
                if constexpr (MOM) keep_loaded(v[q]);
            }
        }
        __builtin_amdgcn_sched_barrier(0);               // loads | arithmetic | stores
#pragma unroll
        for (int q = 0; q < GROUPS; ++q) {
            const f32x4 d = worker_rule<MOM>(w[q], v[q], g[q], c[q], eta, rho, alpha, delta);   // d = W_i - Wc at the start
            c[q] = fma_s(alpha, d, c[q]);                                                           // Eq. (2), one worker
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q = 0; q < GROUPS; ++q) {
            if (FULL || j0 + (size_t)q * STRIDE < n4) {
                st_stream<true>(W + row + jl[q], w[q]);
                if constexpr (MOM) st_stream<true>(V + row + jl[q], v[q]);
            }
        }
        // a worker that comes up again later in the schedule must find these stores done
        if (t + 1 < sch.n) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    }
#pragma unroll
    for (int q = 0; q < GROUPS; ++q)
        if (FULL || j0 + (size_t)q * STRIDE < n4) Wc[jl[q]] = c[q];
}

// One parameter, every turn (the scalar path and the N % 4 tail).
template <bool MOM>
__device__ __forceinline__ void async_scalar(float *__restrict__ W, float *__restrict__ V, const float *__restrict__ G,
                                             float *__restrict__ Wc, const Schedule &sch, size_t j, size_t ld,
                                             float eta, float rho, float alpha, float delta)
{
    float c = Wc[j];
    for (int t = 0; t < sch.n; ++t) {
        const size_t k = (size_t)sch.worker[t] * ld + j;
        float w = W[k], v = MOM ? V[k] : 0.f;
        const float d = worker_rule<MOM>(w, v, G[k], c, eta, rho, alpha, delta);
        c = fma_s(alpha, d, c);
        W[k] = w;
        if constexpr (MOM) V[k] = v;
    }
    Wc[j] = c;
}

template <bool MOM, int GROUPS, bool DIES>
__device__ __forceinline__ void async_vec4_body(float *__restrict__ Wp, float *__restrict__ Vp, const float *__restrict__ Gp,
                                                float *__restrict__ Wcp, const Schedule &sch, size_t N, size_t ld,
                                                float eta, float rho, float alpha, float delta)
{
    typedef TileMap<GROUPS, DIES> Map;
    f32x4 *__restrict__ W = (f32x4 *)Wp;
    f32x4 *__restrict__ V = (f32x4 *)Vp;
    const f32x4 *__restrict__ G = (const f32x4 *)Gp;
    f32x4 *__restrict__ Wc = (f32x4 *)Wcp;
    const size_t n4 = N / 4, ld4 = ld / 4;
    const size_t n_tiles = Map::tiles(n4);
    for (size_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        const size_t j0 = Map::first(t, threadIdx.x);
        if (Map::last(t) < n4) async_tile<MOM, GROUPS, Map::STRIDE, true>(W, V, G, Wc, sch, n4, ld4, j0, eta, rho, alpha, delta);
        else async_tile<MOM, GROUPS, Map::STRIDE, false>(W, V, G, Wc, sch, n4, ld4, j0, eta, rho, alpha, delta);
    }
    const size_t tail = N - n4 * 4;
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x < tail)
        async_scalar<MOM>(Wp, Vp, Gp, Wcp, sch, n4 * 4 + threadIdx.x, ld, eta, rho, alpha, delta);
}

template <bool MOM, int GROUPS>
__global__ __launch_bounds__(256) void async_vec4_kernel(float *__restrict__ W, float *__restrict__ V, const float *__restrict__ G,
                                                         float *__restrict__ Wc, Schedule sch, size_t N, size_t ld,
                                                         float eta, float rho, float alpha, float delta)
{
    async_vec4_body<MOM, GROUPS, false>(W, V, G, Wc, sch, N, ld, eta, rho, alpha, delta);
}

// die-interleaved tiles, one wavefront per SIMD (the large-N form of the synchronous kernel)
template <bool MOM, int GROUPS>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void async_vec4_dies_kernel(float *__restrict__ W, float *__restrict__ V, const float *__restrict__ G,
                            float *__restrict__ Wc, Schedule sch, size_t N, size_t ld,
                            float eta, float rho, float alpha, float delta)
{
    async_vec4_body<MOM, GROUPS, true>(W, V, G, Wc, sch, N, ld, eta, rho, alpha, delta);
}

template <bool MOM>
__global__ __launch_bounds__(256) void async_scalar_kernel(float *__restrict__ W, float *__restrict__ V, const float *__restrict__ G,
                                                           float *__restrict__ Wc, Schedule sch, size_t N, size_t ld,
                                                           float eta, float rho, float alpha, float delta)
{
    for (size_t j = (size_t)blockIdx.x * 256 + threadIdx.x; j < N; j += (size_t)gridDim.x * 256)
        async_scalar<MOM>(W, V, G, Wc, sch, j, ld, eta, rho, alpha, delta);
}

template <bool MOM>
static int async_round(float *W, float *V, const float *G, float *Wc, int P, size_t N, size_t ld,
                       const int *order, int n_order, float eta, float rho, float delta, void *stream)
{
    const char *name = "async_easgd_round";
    if (!W || !G || !Wc || (n_order > 0 && !order)) return fail(EASGD_EINVAL, "%s: NULL pointer", name);
    if (P < 1 || P > 256) return fail(EASGD_EINVAL, "%s: P must be in [1, 256], got %d", name, P);
    if (N == 0) return fail(EASGD_EINVAL, "%s: N must be >= 1", name);
    if (ld < N) return fail(EASGD_EINVAL, "%s: ld (%zu) < N (%zu)", name, ld, N);
    if (n_order < 0 || n_order > EASGD_MAX_SCHEDULE)
        return fail(EASGD_EINVAL, "%s: a schedule holds 0 to %d turns, got %d (longer schedules: several calls)", name, EASGD_MAX_SCHEDULE, n_order);
    if (!aligned_to(W, 4) || !aligned_to(G, 4) || !aligned_to(Wc, 4) || !aligned_to(V, 4))
        return fail(EASGD_EINVAL, "%s: fp32 pointers must be 4-byte aligned", name);
    Schedule sch;
    sch.n = n_order;
    for (int t = 0; t < n_order; ++t) {
        if (order[t] < 0 || order[t] >= P) return fail(EASGD_EINVAL, "%s: order[%d] = %d is not a worker index in [0, %d)", name, t, order[t], P);
        sch.worker[t] = (unsigned char)order[t];
    }
    clear_error();
    if (n_order == 0) return EASGD_OK;                   // nobody is served: nothing to do
    hipStream_t s = static_cast<hipStream_t>(stream);
    const float alpha = eta * rho;
    const bool vec = aligned16(W) && aligned16(G) && aligned16(Wc) && (!MOM || aligned16(V)) && (ld % 4 == 0);
    const UpdateShape shape = update_shape(N, MOM);
    size_t blocks = vec ? shape.blocks : (N + 255) / 256;
    if (blocks > 0x7fffffffu) blocks = 0x7fffffffu;      // grid-stride loops cover the rest
    const dim3 grid((unsigned)blocks);
#define EASGD_ASYNC(GR)                                                                                                       \
    do {                                                                                                                      \
        if (shape.dies) EASGD_LAUNCH((async_vec4_dies_kernel<MOM, GR>), grid, dim3(256), 0, s, W, V, G, Wc, sch, N, ld, eta, rho, alpha, delta); \
        else EASGD_LAUNCH((async_vec4_kernel<MOM, GR>), grid, dim3(256), 0, s, W, V, G, Wc, sch, N, ld, eta, rho, alpha, delta);               \
    } while (0)
    if (!vec) EASGD_LAUNCH((async_scalar_kernel<MOM>), grid, dim3(256), 0, s, W, V, G, Wc, sch, N, ld, eta, rho, alpha, delta);
    else if (shape.groups >= 4) EASGD_ASYNC(4);
    else if (shape.groups == 2) EASGD_ASYNC(2);
    else EASGD_ASYNC(1);
#undef EASGD_ASYNC
    return check_launch(name);
}

// ---- Hogwild EASGD ----
// Block (worker i, tile): 256 threads, GROUPS 128-bit groups each.  Blocks are numbered worker-fastest, so the
// blocks that work on the same tile of the center at the same time are those of different workers.
template <bool MOM, int GROUPS>
__global__ __launch_bounds__(256) void hogwild_vec4_kernel(float *__restrict__ Wp, float *__restrict__ Vp, const float *__restrict__ Gp,
                                                           float *__restrict__ Wcp, int P, size_t N, size_t ld,
                                                           float eta, float rho, float alpha, float delta)
{
    f32x4 *__restrict__ W = (f32x4 *)Wp;
    f32x4 *__restrict__ V = (f32x4 *)Vp;
    const f32x4 *__restrict__ G = (const f32x4 *)Gp;
    const size_t n4 = N / 4, ld4 = ld / 4;
    const size_t n_tiles = (n4 + (size_t)GROUPS * 256 - 1) / ((size_t)GROUPS * 256) + 1;   // the last tile is the scalar tail's
    const size_t total = n_tiles * (size_t)P;
    for (size_t id = blockIdx.x; id < total; id += gridDim.x) {
        const size_t tile = id / (size_t)P;
        const int i = (int)(id - tile * (size_t)P);
        const size_t row = (size_t)i * ld4;
        if (tile + 1 == n_tiles) {                       // N % 4 tail elements
            const size_t j = n4 * 4 + threadIdx.x;
            if (j < N) {
                const size_t k = (size_t)i * ld + j;
                float w = Wp[k], v = MOM ? Vp[k] : 0.f;
                const float c = __hip_atomic_load(&Wcp[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const float d = worker_rule<MOM>(w, v, Gp[k], c, eta, rho, alpha, delta);
                Wp[k] = w;
                if constexpr (MOM) Vp[k] = v;
                (void)unsafeAtomicAdd(&Wcp[j], alpha * d);
            }
            continue;
        }
#pragma unroll
        for (int q = 0; q < GROUPS; ++q) {
            const size_t j = tile * ((size_t)GROUPS * 256) + (size_t)q * 256 + threadIdx.x;
            if (j < n4) {
                f32x4 w = ld_stream<true>(W + row + j), g = ld_stream<true>(G + row + j), v = w, c;
                if constexpr (MOM) v = ld_stream<true>(V + row + j);
                // the center as this worker finds it: whatever the other workers have added so far
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    c[e] = __hip_atomic_load(&Wcp[4 * j + e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const f32x4 d = worker_rule<MOM>(w, v, g, c, eta, rho, alpha, delta);
                st_stream<true>(W + row + j, w);
                if constexpr (MOM) st_stream<true>(V + row + j, v);
                // lock-free master: the one-worker form of Eq. (2) as an atomic addition, no lock around read and add
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    (void)unsafeAtomicAdd(&Wcp[4 * j + e], alpha * d[e]);      // the hardware's fp32 add at the L2 / memory side
            }
        }
    }
}

template <bool MOM>
__global__ __launch_bounds__(256) void hogwild_scalar_kernel(float *__restrict__ W, float *__restrict__ V, const float *__restrict__ G,
                                                             float *__restrict__ Wc, int P, size_t N, size_t ld,
                                                             float eta, float rho, float alpha, float delta)
{
    const size_t total = N * (size_t)P;
    for (size_t id = (size_t)blockIdx.x * 256 + threadIdx.x; id < total; id += (size_t)gridDim.x * 256) {
        const size_t j = id % N;
        const size_t k = (id / N) * ld + j;
        float w = W[k], v = MOM ? V[k] : 0.f;
        const float c = __hip_atomic_load(&Wc[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const float d = worker_rule<MOM>(w, v, G[k], c, eta, rho, alpha, delta);
        W[k] = w;
        if constexpr (MOM) V[k] = v;
        (void)unsafeAtomicAdd(&Wc[j], alpha * d);
    }
}

template <bool MOM>
static int hogwild_round(float *W, float *V, const float *G, float *Wc, int P, size_t N, size_t ld,
                         float eta, float rho, float delta, void *stream)
{
    const char *name = "hogwild_easgd_round";
    if (!W || !G || !Wc) return fail(EASGD_EINVAL, "%s: NULL pointer", name);
    if (P < 1) return fail(EASGD_EINVAL, "%s: P must be >= 1, got %d", name, P);
    if (N == 0) return fail(EASGD_EINVAL, "%s: N must be >= 1", name);
    if (ld < N) return fail(EASGD_EINVAL, "%s: ld (%zu) < N (%zu)", name, ld, N);
    if (!aligned_to(W, 4) || !aligned_to(G, 4) || !aligned_to(Wc, 4) || !aligned_to(V, 4))
        return fail(EASGD_EINVAL, "%s: fp32 pointers must be 4-byte aligned", name);
    clear_error();
    hipStream_t s = static_cast<hipStream_t>(stream);
    const float alpha = eta * rho;
    const bool vec = aligned16(W) && aligned16(G) && aligned16(Wc) && (!MOM || aligned16(V)) && (ld % 4 == 0);
    if (vec) {
        constexpr int GROUPS = 2;
        size_t blocks = ((N / 4 + (size_t)GROUPS * 256 - 1) / ((size_t)GROUPS * 256) + 1) * (size_t)P;
        if (blocks > 0x7fffffffu) blocks = 0x7fffffffu;
        EASGD_LAUNCH((hogwild_vec4_kernel<MOM, GROUPS>), dim3((unsigned)blocks), dim3(256), 0, s, W, V, G, Wc, P, N, ld, eta, rho, alpha, delta);
    } else {
        size_t blocks = (N * (size_t)P + 255) / 256;
        if (blocks > 0x7fffffffu) blocks = 0x7fffffffu;
        EASGD_LAUNCH((hogwild_scalar_kernel<MOM>), dim3((unsigned)blocks), dim3(256), 0, s, W, V, G, Wc, P, N, ld, eta, rho, alpha, delta);
    }
    return check_launch(name);
}

}  // namespace easgd

extern "C" {

int async_easgd_round(float *W, float *V, const float *G, float *Wc, int P, size_t N, size_t ld,
                      const int *order, int n_order, float eta, float rho, float delta, void *stream)
{
    return V ? easgd::async_round<true>(W, V, G, Wc, P, N, ld, order, n_order, eta, rho, delta, stream)
             : easgd::async_round<false>(W, nullptr, G, Wc, P, N, ld, order, n_order, eta, rho, 0.0f, stream);
}

int hogwild_easgd_round(float *W, float *V, const float *G, float *Wc, int P, size_t N, size_t ld,
                        float eta, float rho, float delta, void *stream)
{
    return V ? easgd::hogwild_round<true>(W, V, G, Wc, P, N, ld, eta, rho, delta, stream)
             : easgd::hogwild_round<false>(W, nullptr, G, Wc, P, N, ld, eta, rho, 0.0f, stream);
}

}  // extern "C"
