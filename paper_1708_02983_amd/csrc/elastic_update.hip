// Fused elastic exchange-and-update of one Sync EASGD round
// (Section 5.1 steps (2)-(5); worker rule Eq. (1) or Eq. (5),(6); center rule Eq. (2)).
//
// All P replicas and the center live in one HBM, so the paper's broadcast of
// the center is one read of Wc[j] kept in registers and its tree reduction over
// the workers is a register sum in ascending worker order.  Every operand is
// read once and every result written once: this kernel is a pure HBM stream of
// N*(12P+8) bytes (EASGD) or N*(20P+8) bytes (momentum).
//
// A block of 256 threads owns GROUPS*256 groups of four consecutive parameters
// and walks the workers one at a time: for worker i every thread issues its
// GROUPS 128-bit loads of W_i and G_i (and V_i) back to back, applies the rule
// and stores.  At any moment a block touches the streams of ONE worker;
// measured on MI355X this is 2-5 % faster than having every thread interleave
// several workers (HBM efficiency drops as more address streams are active at
// once).  Which groups a block owns is the TileMap of common.h: for large N the
// eight dies interleave at 1 KiB granularity inside super-tiles instead of
// each streaming contiguous runs of its own, worth 10-18 % of bandwidth.
#include "common.h"
#include "elastic_rule.h"

namespace easgd {

typedef float f32x4 __attribute__((ext_vector_type(4)));

template <bool NT, typename T>
__device__ __forceinline__ T stream_load(const T *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}

template <bool NT, typename T>
__device__ __forceinline__ void stream_store(T *p, T v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// T-wide groups [0, n_groups) of every row; rows are `ld_groups` groups apart.
template <bool MOM, bool NT, int UNROLL, typename T>
__device__ __forceinline__ void elastic_group(T *__restrict__ W, T *__restrict__ V, const T *__restrict__ G,
                                              T *__restrict__ Wc, int P, size_t j, size_t ld_groups,
                                              float eta, float rho, float alpha, float delta)
{
    const T c = Wc[j];
    T acc = c - c;                            // zero of type T
    int i = 0;
    for (; i + UNROLL <= P; i += UNROLL) {
        T w[UNROLL], g[UNROLL], v[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const size_t k = (size_t)(i + u) * ld_groups + j;
            w[u] = stream_load<NT>(W + k);
            g[u] = stream_load<NT>(G + k);
            if constexpr (MOM) v[u] = stream_load<NT>(V + k);
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const size_t k = (size_t)(i + u) * ld_groups + j;
            acc += worker_rule<MOM>(w[u], v[u], g[u], c, eta, rho, alpha, delta);   // ascending i
            stream_store<NT>(W + k, w[u]);
            if constexpr (MOM) stream_store<NT>(V + k, v[u]);
        }
    }
    for (; i < P; ++i) {
        const size_t k = (size_t)i * ld_groups + j;
        T w = stream_load<NT>(W + k), g = stream_load<NT>(G + k), v = w;
        if constexpr (MOM) v = stream_load<NT>(V + k);
        acc += worker_rule<MOM>(w, v, g, c, eta, rho, alpha, delta);
        stream_store<NT>(W + k, w);
        if constexpr (MOM) stream_store<NT>(V + k, v);
    }
    Wc[j] = fma_s(alpha, acc, c);                 // Eq. (2)
}

// One tile of the 128-bit path: thread-owned groups j0 + q*STRIDE.  FULL: every group of the block lies inside the
// row (the block-uniform common case).  No load is conditional in either form, so all 2*GROUPS (3*GROUPS) loads of
// a worker are in flight together: in the tile that holds the end of the row, lanes whose group lies past it read
// the row's last group instead and store nothing.  (A guarded load is a merge of two definitions and is waited
// for at the merge: one round trip to memory per group and worker, in a block that the whole launch then waits
// for when N is small enough that every block is resident at once.)
template <bool MOM, bool NT, int GROUPS, size_t STRIDE, bool FULL>
__device__ __forceinline__ void elastic_tile(f32x4 *__restrict__ W, f32x4 *__restrict__ V, const f32x4 *__restrict__ G,
                                             f32x4 *__restrict__ Wc, int P, size_t n4, size_t ld4, size_t j0,
                                             float eta, float rho, float alpha, float delta)
{
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    f32x4 c[GROUPS], acc[GROUPS];
    size_t jl[GROUPS];                                // the group this lane loads: its own, or the row's last one
#pragma unroll
    for (int q = 0; q < GROUPS; ++q) {
        const size_t j = j0 + (size_t)q * STRIDE;
        jl[q] = (FULL || j < n4) ? j : n4 - 1;
        c[q] = Wc[jl[q]];                             // the "broadcast" of the center, once per parameter
        acc[q] = zero;
    }
    for (int i = 0; i < P; ++i) {                     // ascending worker order: fixed summation order
        const size_t row = (size_t)i * ld4;
        f32x4 w[GROUPS], g[GROUPS], v[GROUPS];
        // stream by stream (the gradients, then the replica, then the momentum buffer; the stores likewise), not group
        // by group: consecutive requests of a wavefront then walk one array, 0.5-0.9 % faster at N = 61 M
#pragma unroll
        for (int q = 0; q < GROUPS; ++q) g[q] = stream_load<NT>(G + row + jl[q]);
#pragma unroll
        for (int q = 0; q < GROUPS; ++q) w[q] = stream_load<NT>(W + row + jl[q]);
        if constexpr (MOM) {
#pragma unroll
            for (int q = 0; q < GROUPS; ++q) v[q] = stream_load<NT>(V + row + jl[q]);
        }
        if constexpr (!FULL) {
#pragma unroll
            for (int q = 0; q < GROUPS; ++q) {
                keep_loaded(g[q]);
                keep_loaded(w[q]);
                if constexpr (MOM) keep_loaded(v[q]);
            }
        }
        // Three phases per worker, kept apart by scheduling barriers: every load is issued before the first result
        // is used, and every store after the last result is computed.  Left alone the scheduler pairs loads with
        // the arithmetic of earlier groups and drips the stores out between waits; bursts of reads followed by
        // bursts of writes stream 5-10 % faster (measured at P = 16, N = 61 M).
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q = 0; q < GROUPS; ++q) acc[q] += worker_rule<MOM>(w[q], v[q], g[q], c[q], eta, rho, alpha, delta);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (FULL) {
#pragma unroll
            for (int q = 0; q < GROUPS; ++q) stream_store<NT>(W + row + jl[q], w[q]);
            if constexpr (MOM) {
#pragma unroll
                for (int q = 0; q < GROUPS; ++q) stream_store<NT>(V + row + jl[q], v[q]);
            }
        } else {
#pragma unroll
            for (int q = 0; q < GROUPS; ++q) {
                if (j0 + (size_t)q * STRIDE < n4) {
                    stream_store<NT>(W + row + jl[q], w[q]);
                    if constexpr (MOM) stream_store<NT>(V + row + jl[q], v[q]);
                }
            }
        }
    }
#pragma unroll
    for (int q = 0; q < GROUPS; ++q)
        if (FULL || j0 + (size_t)q * STRIDE < n4) Wc[jl[q]] = fma_s(alpha, acc[q], c[q]);   // Eq. (2)
}

// 128-bit path.  The N % 4 tail elements are handled as scalars by the last block.
template <bool MOM, bool NT, int GROUPS, bool DIES>
__device__ __forceinline__ void elastic_vec4_body(float *__restrict__ Wp, float *__restrict__ Vp,
                                                  const float *__restrict__ Gp, float *__restrict__ Wcp,
                                                  int P, size_t N, size_t ld,
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
        if (Map::last(t) < n4)                        // uniform for the block
            elastic_tile<MOM, NT, GROUPS, Map::STRIDE, true>(W, V, G, Wc, P, n4, ld4, j0, eta, rho, alpha, delta);
        else
            elastic_tile<MOM, NT, GROUPS, Map::STRIDE, false>(W, V, G, Wc, P, n4, ld4, j0, eta, rho, alpha, delta);
    }
    const size_t tail = N - n4 * 4;
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x < tail)
        elastic_group<MOM, false, 1, float>(Wp, Vp, Gp, Wcp, P, n4 * 4 + threadIdx.x, ld, eta, rho, alpha, delta);
}

// Contiguous tiles (small N, or by option).
template <bool MOM, bool NT, int GROUPS>
__global__ __launch_bounds__(256) void elastic_vec4_kernel(float *__restrict__ W, float *__restrict__ V,
                                                           const float *__restrict__ G, float *__restrict__ Wc,
                                                           int P, size_t N, size_t ld,
                                                           float eta, float rho, float alpha, float delta)
{
    elastic_vec4_body<MOM, NT, GROUPS, false>(W, V, G, Wc, P, N, ld, eta, rho, alpha, delta);
}

// Die-interleaved tiles, the large-N kernel.  One wavefront per SIMD, i.e. one block per compute unit: with
// 2*GROUPS (3*GROUPS) KiB of loads per wavefront in flight that is enough to cover the latency, and the fewer,
// longer bursts of reads and of writes per compute unit stream 4 % faster than four blocks per compute unit
// (measured: P = 8 6.45 -> 6.75 TB/s, P = 16 with momentum 6.05 -> 6.3 TB/s at N = 61 M).
template <bool MOM, bool NT, int GROUPS>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void elastic_vec4_dies_kernel(float *__restrict__ W, float *__restrict__ V, const float *__restrict__ G,
                              float *__restrict__ Wc, int P, size_t N, size_t ld,
                              float eta, float rho, float alpha, float delta)
{
    elastic_vec4_body<MOM, NT, GROUPS, true>(W, V, G, Wc, P, N, ld, eta, rho, alpha, delta);
}

// Small-N path (few parameters, several workers): the one-thread-per-group kernel above would leave most of
// the chip idle, so the workers are split over the four wavefronts of a block instead.  A block owns 64 groups;
// wavefront v applies the worker rule for workers v, v+4, v+8, ... (ascending) and keeps a partial sum of
// W_i - Wc in registers; the partial sums meet in LDS and wavefront 0 adds them in the fixed order
// v = 0, 1, 2, 3 before it applies Eq. (2).  The result is reproducible from run to run.
template <bool MOM>
__global__ __launch_bounds__(256) void elastic_split_kernel(float *__restrict__ Wp, float *__restrict__ Vp,
                                                            const float *__restrict__ Gp, float *__restrict__ Wcp,
                                                            int P, size_t N, size_t ld,
                                                            float eta, float rho, float alpha, float delta)
{
    __shared__ f32x4 partial[4][64];
    f32x4 *__restrict__ W = (f32x4 *)Wp;
    f32x4 *__restrict__ V = (f32x4 *)Vp;
    const f32x4 *__restrict__ G = (const f32x4 *)Gp;
    f32x4 *__restrict__ Wc = (f32x4 *)Wcp;
    const size_t n4 = N / 4, ld4 = ld / 4;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t j = (size_t)blockIdx.x * 64 + lane;
    const bool live = j < n4;
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    const f32x4 c = live ? Wc[j] : zero;
    f32x4 acc = zero;
    if (live) {
        for (int i = wave; i < P; i += 4) {
            const size_t k = (size_t)i * ld4 + j;
            f32x4 w = W[k], g = G[k], v = w;
            if constexpr (MOM) v = V[k];
            acc += worker_rule<MOM>(w, v, g, c, eta, rho, alpha, delta);
            W[k] = w;
            if constexpr (MOM) V[k] = v;
        }
    }
    partial[wave][lane] = acc;
    __syncthreads();
    if (wave == 0 && live) {
        const f32x4 sum = ((partial[0][lane] + partial[1][lane]) + partial[2][lane]) + partial[3][lane];
        Wc[j] = fma_s(alpha, sum, c);             // Eq. (2)
    }
    const size_t tail = N - n4 * 4;
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x < tail)
        elastic_group<MOM, false, 1, float>(Wp, Vp, Gp, Wcp, P, n4 * 4 + threadIdx.x, ld, eta, rho, alpha, delta);
}

// Scalar path for operands that are not 16-byte aligned or ld % 4 != 0.
template <bool MOM>
__global__ __launch_bounds__(256) void elastic_scalar_kernel(float *__restrict__ W, float *__restrict__ V,
                                                             const float *__restrict__ G, float *__restrict__ Wc,
                                                             int P, size_t N, size_t ld,
                                                             float eta, float rho, float alpha, float delta)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t j = (size_t)blockIdx.x * blockDim.x + threadIdx.x; j < N; j += stride)
        elastic_group<MOM, false, 4, float>(W, V, G, Wc, P, j, ld, eta, rho, alpha, delta);
}

template <bool MOM, bool NT, bool DIES>
static void launch_vec4(int groups, dim3 grid, hipStream_t s, float *W, float *V, const float *G, float *Wc,
                        int P, size_t N, size_t ld, float eta, float rho, float alpha, float delta)
{
#define EASGD_VEC4(GR)                                                                                                   \
    do {                                                                                                                 \
        if (DIES) EASGD_LAUNCH((elastic_vec4_dies_kernel<MOM, NT, GR>), grid, dim3(256), 0, s, W, V, G, Wc, P, N, ld, eta, rho, alpha, delta); \
        else EASGD_LAUNCH((elastic_vec4_kernel<MOM, NT, GR>), grid, dim3(256), 0, s, W, V, G, Wc, P, N, ld, eta, rho, alpha, delta);          \
    } while (0)
    switch (groups) {
    case 1: EASGD_VEC4(1); break;
    case 2: EASGD_VEC4(2); break;
    case 4: EASGD_VEC4(4); break;
    default: EASGD_VEC4(8); break;
    }
#undef EASGD_VEC4
}

template <bool MOM>
static int elastic_round(float *W, float *V, const float *G, float *Wc, int P, size_t N, size_t ld,
                         float eta, float rho, float delta, void *stream)
{
    const char *name = MOM ? "measgd_round" : "easgd_sync_round";
    if (!W || !G || !Wc || (MOM && !V)) return fail(EASGD_EINVAL, "%s: NULL pointer", name);
    if (P < 1) return fail(EASGD_EINVAL, "%s: P must be >= 1, got %d", name, P);
    if (N == 0) return fail(EASGD_EINVAL, "%s: N must be >= 1", name);
    if (ld < N) return fail(EASGD_EINVAL, "%s: ld (%zu) < N (%zu)", name, ld, N);
    if (!aligned_to(W, 4) || !aligned_to(G, 4) || !aligned_to(Wc, 4) || !aligned_to(V, 4))
        return fail(EASGD_EINVAL, "%s: fp32 pointers must be 4-byte aligned", name);
    clear_error();

    hipStream_t s = static_cast<hipStream_t>(stream);
    const float alpha = eta * rho;            // elastic coefficient of workers and center
    const bool vec = aligned16(W) && aligned16(G) && aligned16(Wc) && (!MOM || aligned16(V)) && (ld % 4 == 0);
    // vector path: groups per thread, tile map and grid (the scalar tail rides on the last block)
    const UpdateShape shape = update_shape(N, MOM);
    size_t blocks = vec ? shape.blocks : (N + 255) / 256;
    if (blocks > 0x7fffffffu) blocks = 0x7fffffffu;    // grid-stride loop covers the rest
    const dim3 grid((unsigned)blocks);
    const int groups = shape.groups;
    // few parameters and several workers: split the workers over the wavefronts of a block
    const bool split = vec && P >= 4 && (N / 4 + 255) / 256 < (size_t)(2 * num_cus());
    if (split) {
        const dim3 split_grid((unsigned)((N / 4 + 63) / 64 > 0 ? (N / 4 + 63) / 64 : 1));
        EASGD_LAUNCH((elastic_split_kernel<MOM>), split_grid, dim3(256), 0, s, W, V, G, Wc, P, N, ld, eta, rho, alpha, delta);
    } else if (vec) {
        const bool nt = update_nontemporal(N * ((MOM ? 20 : 12) * (size_t)P + 8));
        if (shape.dies && nt) launch_vec4<MOM, true, true>(groups, grid, s, W, V, G, Wc, P, N, ld, eta, rho, alpha, delta);
        else if (shape.dies) launch_vec4<MOM, false, true>(groups, grid, s, W, V, G, Wc, P, N, ld, eta, rho, alpha, delta);
        else if (nt) launch_vec4<MOM, true, false>(groups, grid, s, W, V, G, Wc, P, N, ld, eta, rho, alpha, delta);
        else launch_vec4<MOM, false, false>(groups, grid, s, W, V, G, Wc, P, N, ld, eta, rho, alpha, delta);
    } else {
        EASGD_LAUNCH((elastic_scalar_kernel<MOM>), grid, dim3(256), 0, s, W, V, G, Wc, P, N, ld, eta, rho, alpha, delta);
    }
    return check_launch(name);
}

// Eq. (2) alone as a kernel of its own (see center_rule_block).
template <typename T>
__global__ __launch_bounds__(256) void center_rule_kernel(const float *__restrict__ Wp, float *__restrict__ Wcp,
                                                          float *__restrict__ oldp, int P, size_t N, size_t ld, float alpha)
{
    center_rule_block<T>(Wp, Wcp, oldp, P, N, ld, alpha, blockIdx.x, gridDim.x, threadIdx.x);
}

// The same with a grid of any size: block x does the work of blocks x, x + gridDim.x, ... of the kernel above.
template <typename T>
__global__ __launch_bounds__(256) void center_rule_walk_kernel(const float *__restrict__ Wp, float *__restrict__ Wcp,
                                                               float *__restrict__ oldp, int P, size_t N, size_t ld,
                                                               float alpha, unsigned n_blocks)
{
    for (unsigned b = blockIdx.x; b < n_blocks; b += gridDim.x)
        center_rule_block<T>(Wp, Wcp, oldp, P, N, ld, alpha, b, n_blocks, threadIdx.x);
}

int center_range(const float *W, float *Wc, float *old, int P, size_t N, size_t ld, float alpha, void *stream, bool beside)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool vec = aligned16(W) && aligned16(Wc) && aligned16(old) && (ld % 4 == 0);
    const size_t units = vec ? N / 4 : N;
    const size_t blocks = units / 256 + 1;    // the last block also owns the scalar tail
    if (blocks > 0x7fffffffu) return fail(EASGD_ERANGE, "center rule: N too large");
    // Beside the matrix products of forward propagation (on the library's second stream): one block per compute
    // unit that walks the parameter range.  A forward launch leaves each SIMD the registers of about one more
    // small wavefront; thousands of short blocks keep competing for that slot with each other and with the
    // products' own block turnover, one resident block per compute unit just streams.  Measured at P = 32,
    // N = 10.5 M: the two forward launches 2 x 381 -> 2 x 340 us (308 us alone), the round 2.37 -> 2.27 ms;
    // 192 to 256 blocks are equal, 288 and more or 128 and fewer are slower than the short blocks.
    const size_t cus = (size_t)num_cus();
    if (beside && blocks > 4 * cus) {
        if (vec) EASGD_LAUNCH((center_rule_walk_kernel<f32x4>), dim3((unsigned)cus), dim3(256), 0, s, W, Wc, old, P, N, ld, alpha, (unsigned)blocks);
        else EASGD_LAUNCH((center_rule_walk_kernel<float>), dim3((unsigned)cus), dim3(256), 0, s, W, Wc, old, P, N, ld, alpha, (unsigned)blocks);
        return check_launch("center rule");
    }
    if (vec) EASGD_LAUNCH((center_rule_kernel<f32x4>), dim3((unsigned)blocks), dim3(256), 0, s, W, Wc, old, P, N, ld, alpha);
    else EASGD_LAUNCH((center_rule_kernel<float>), dim3((unsigned)blocks), dim3(256), 0, s, W, Wc, old, P, N, ld, alpha);
    return check_launch("center rule");
}

// ---- synchronous data-parallel SGD on the replicas (Section 2.3; the partitioned form of Section 6.2) ----
// Every replica moves by the SUM of all workers' gradients: s = g_0 + g_1 + ... (ascending, one thread per
// parameter group, so the order is fixed), then W_i <- W_i - eta*s, or with momentum Eq. (3),(4)
// V_i <- mu*V_i - eta*s, W_i <- W_i + V_i.  Same streaming skeleton as the elastic update: the gradients of
// all workers are read first (they must all be known before any replica moves), then each replica is
// read and written once.
template <bool MOM, typename T>
__device__ __forceinline__ void sgd_rule(T &w, T &v, T s, float eta, float mu)
{
    if constexpr (MOM) {
        v = fma_s(mu, v, -(eta * s));         // Eq. (3)
        w = w + v;                            // Eq. (4)
    } else {
        w = fma_s(-eta, s, w);
    }
}

// One tile of the 128-bit path (FULL as in elastic_tile).
template <bool MOM, bool NT, int GROUPS, size_t STRIDE, bool FULL>
__device__ __forceinline__ void sync_sgd_tile(f32x4 *__restrict__ W, f32x4 *__restrict__ V, const f32x4 *__restrict__ G,
                                              int P, size_t n4, size_t ld4, size_t j0, float eta, float mu)
{
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    f32x4 s[GROUPS];
    size_t jl[GROUPS];                                // loads past the end of the row read its last group instead
#pragma unroll
    for (int q = 0; q < GROUPS; ++q) {
        const size_t j = j0 + (size_t)q * STRIDE;
        jl[q] = (FULL || j < n4) ? j : n4 - 1;
        s[q] = zero;
    }
    for (int i = 0; i < P; ++i) {                     // ascending worker order: fixed summation order
        const size_t row = (size_t)i * ld4;
        f32x4 g[GROUPS];
#pragma unroll
        for (int q = 0; q < GROUPS; ++q) g[q] = stream_load<NT>(G + row + jl[q]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q = 0; q < GROUPS; ++q) s[q] += g[q];
    }
    for (int i = 0; i < P; ++i) {
        const size_t row = (size_t)i * ld4;
        f32x4 w[GROUPS], v[GROUPS];
#pragma unroll
        for (int q = 0; q < GROUPS; ++q) {
            w[q] = stream_load<NT>(W + row + jl[q]);
            if constexpr (MOM) v[q] = stream_load<NT>(V + row + jl[q]);
        }
        if constexpr (!FULL) {
#pragma unroll
            for (int q = 0; q < GROUPS; ++q) {
                keep_loaded(w[q]);
                if constexpr (MOM) keep_loaded(v[q]);
            }
        }
        __builtin_amdgcn_sched_barrier(0);            // loads | arithmetic | stores, as in elastic_tile
#pragma unroll
        for (int q = 0; q < GROUPS; ++q) sgd_rule<MOM>(w[q], v[q], s[q], eta, mu);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (FULL) {
#pragma unroll
            for (int q = 0; q < GROUPS; ++q) stream_store<NT>(W + row + jl[q], w[q]);
            if constexpr (MOM) {
#pragma unroll
                for (int q = 0; q < GROUPS; ++q) stream_store<NT>(V + row + jl[q], v[q]);
            }
        } else {
#pragma unroll
            for (int q = 0; q < GROUPS; ++q) {
                if (j0 + (size_t)q * STRIDE < n4) {
                    stream_store<NT>(W + row + jl[q], w[q]);
                    if constexpr (MOM) stream_store<NT>(V + row + jl[q], v[q]);
                }
            }
        }
    }
}

template <bool MOM, bool NT, int GROUPS, bool DIES>
__device__ __forceinline__ void sync_sgd_vec4_body(float *__restrict__ Wp, float *__restrict__ Vp,
                                                   const float *__restrict__ Gp, int P, size_t N, size_t ld,
                                                   float eta, float mu)
{
    typedef TileMap<GROUPS, DIES> Map;
    f32x4 *__restrict__ W = (f32x4 *)Wp;
    f32x4 *__restrict__ V = (f32x4 *)Vp;
    const f32x4 *__restrict__ G = (const f32x4 *)Gp;
    const size_t n4 = N / 4, ld4 = ld / 4;
    const size_t n_tiles = Map::tiles(n4);
    for (size_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        const size_t j0 = Map::first(t, threadIdx.x);
        if (Map::last(t) < n4) sync_sgd_tile<MOM, NT, GROUPS, Map::STRIDE, true>(W, V, G, P, n4, ld4, j0, eta, mu);
        else sync_sgd_tile<MOM, NT, GROUPS, Map::STRIDE, false>(W, V, G, P, n4, ld4, j0, eta, mu);
    }
    const size_t tail = N - n4 * 4;
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x < tail) {
        const size_t k = n4 * 4 + threadIdx.x;
        float s = 0.f;
        for (int i = 0; i < P; ++i) s += Gp[(size_t)i * ld + k];
        for (int i = 0; i < P; ++i) {
            float w = Wp[(size_t)i * ld + k], v = MOM ? Vp[(size_t)i * ld + k] : 0.f;
            sgd_rule<MOM>(w, v, s, eta, mu);
            Wp[(size_t)i * ld + k] = w;
            if constexpr (MOM) Vp[(size_t)i * ld + k] = v;
        }
    }
}

template <bool MOM, bool NT, int GROUPS>
__global__ __launch_bounds__(256) void sync_sgd_vec4_kernel(float *__restrict__ W, float *__restrict__ V,
                                                            const float *__restrict__ G, int P, size_t N, size_t ld,
                                                            float eta, float mu)
{
    sync_sgd_vec4_body<MOM, NT, GROUPS, false>(W, V, G, P, N, ld, eta, mu);
}

// die-interleaved tiles, one wavefront per SIMD (see elastic_vec4_dies_kernel)
template <bool MOM, bool NT, int GROUPS>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void sync_sgd_vec4_dies_kernel(float *__restrict__ W, float *__restrict__ V, const float *__restrict__ G,
                               int P, size_t N, size_t ld, float eta, float mu)
{
    sync_sgd_vec4_body<MOM, NT, GROUPS, true>(W, V, G, P, N, ld, eta, mu);
}

// Any alignment: one thread per parameter.
template <bool MOM>
__global__ __launch_bounds__(256) void sync_sgd_scalar_kernel(float *__restrict__ W, float *__restrict__ V,
                                                              const float *__restrict__ G, int P, size_t N, size_t ld,
                                                              float eta, float mu)
{
    for (size_t k = (size_t)blockIdx.x * 256 + threadIdx.x; k < N; k += (size_t)gridDim.x * 256) {
        float s = 0.f;
        for (int i = 0; i < P; ++i) s += G[(size_t)i * ld + k];
        for (int i = 0; i < P; ++i) {
            float w = W[(size_t)i * ld + k], v = MOM ? V[(size_t)i * ld + k] : 0.f;
            sgd_rule<MOM>(w, v, s, eta, mu);
            W[(size_t)i * ld + k] = w;
            if constexpr (MOM) V[(size_t)i * ld + k] = v;
        }
    }
}

template <bool MOM, bool NT, bool DIES>
static void launch_sync_sgd(int groups, dim3 grid, hipStream_t s, float *W, float *V, const float *G, int P, size_t N,
                            size_t ld, float eta, float mu)
{
#define EASGD_SGD(GR)                                                                                              \
    do {                                                                                                           \
        if (DIES) EASGD_LAUNCH((sync_sgd_vec4_dies_kernel<MOM, NT, GR>), grid, dim3(256), 0, s, W, V, G, P, N, ld, eta, mu); \
        else EASGD_LAUNCH((sync_sgd_vec4_kernel<MOM, NT, GR>), grid, dim3(256), 0, s, W, V, G, P, N, ld, eta, mu);          \
    } while (0)
    if (groups >= 8) EASGD_SGD(8);
    else if (groups == 4) EASGD_SGD(4);
    else if (groups == 2) EASGD_SGD(2);
    else EASGD_SGD(1);
#undef EASGD_SGD
}

template <bool MOM>
static int sync_sgd(float *W, float *V, const float *G, int P, size_t N, size_t ld, float eta, float mu, void *stream)
{
    const char *name = "sync_sgd_round";
    if (!W || !G) return fail(EASGD_EINVAL, "%s: NULL pointer", name);
    if (P < 1) return fail(EASGD_EINVAL, "%s: P must be >= 1, got %d", name, P);
    if (N == 0) return fail(EASGD_EINVAL, "%s: N must be >= 1", name);
    if (ld < N) return fail(EASGD_EINVAL, "%s: ld (%zu) < N (%zu)", name, ld, N);
    if (!aligned_to(W, 4) || !aligned_to(G, 4) || !aligned_to(V, 4))
        return fail(EASGD_EINVAL, "%s: fp32 pointers must be 4-byte aligned", name);
    clear_error();
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool vec = aligned16(W) && aligned16(G) && (!MOM || aligned16(V)) && (ld % 4 == 0);
    const UpdateShape shape = update_shape(N, MOM);
    size_t blocks = vec ? shape.blocks : (N + 255) / 256;
    if (blocks > 0x7fffffffu) blocks = 0x7fffffffu;    // grid-stride loops cover the rest
    const dim3 grid((unsigned)blocks);
    const bool nt = update_nontemporal(N * (MOM ? 20 : 12) * (size_t)P);
    if (!vec) EASGD_LAUNCH((sync_sgd_scalar_kernel<MOM>), grid, dim3(256), 0, s, W, V, G, P, N, ld, eta, mu);
    else if (shape.dies && nt) launch_sync_sgd<MOM, true, true>(shape.groups, grid, s, W, V, G, P, N, ld, eta, mu);
    else if (shape.dies) launch_sync_sgd<MOM, false, true>(shape.groups, grid, s, W, V, G, P, N, ld, eta, mu);
    else if (nt) launch_sync_sgd<MOM, true, false>(shape.groups, grid, s, W, V, G, P, N, ld, eta, mu);
    else launch_sync_sgd<MOM, false, false>(shape.groups, grid, s, W, V, G, P, N, ld, eta, mu);
    return check_launch(name);
}

int elastic_range(float *W, float *V, const float *G, float *Wc, int P, size_t N, size_t ld,
                  float eta, float rho, float delta, void *stream)
{
    return V ? elastic_round<true>(W, V, G, Wc, P, N, ld, eta, rho, delta, stream)
             : elastic_round<false>(W, nullptr, G, Wc, P, N, ld, eta, rho, 0.0f, stream);
}

}  // namespace easgd

extern "C" {

int easgd_sync_round(float *W, const float *G, float *Wc, int P, size_t N, size_t ld,
                     float eta, float rho, void *stream)
{
    return easgd::elastic_round<false>(W, nullptr, G, Wc, P, N, ld, eta, rho, 0.0f, stream);
}

int measgd_round(float *W, float *V, const float *G, float *Wc, int P, size_t N, size_t ld,
                 float eta, float rho, float delta, void *stream)
{
    return easgd::elastic_round<true>(W, V, G, Wc, P, N, ld, eta, rho, delta, stream);
}

int sync_sgd_round(float *W, float *V, const float *G, int P, size_t N, size_t ld, float eta, float delta, void *stream)
{
    return V ? easgd::sync_sgd<true>(W, V, G, P, N, ld, eta, delta, stream)
             : easgd::sync_sgd<false>(W, nullptr, G, P, N, ld, eta, 0.0f, stream);
}

}  // extern "C"
