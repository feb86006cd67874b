// The fused elastic exchange-and-update (Section 5.1 steps (2)-(5); Eq. (1), (2), (5), (6)) with the
// gradients and the momentum buffers STORED as bfloat16 -- an extension: the paper keeps everything in
// fp32 and only names low precision as future work (Section 3.2).  Replicas and center stay fp32 and
// all arithmetic is fp32; what changes is the HBM stream: N*(10P+8) bytes per round instead of
// N*(12P+8) (EASGD), N*(14P+8) instead of N*(20P+8) (momentum), N*(16P+8) when only the momentum
// buffers are stored in 16 bits and the gradients arrive as fp32 (as easgd_grad writes them).
//
// The format, its rounding and the worker rule are in elastic_rule.h (worker_rule_bf16), shared with the
// matrix-product epilogue of the whole-round call.
//
// Same skeleton as elastic_vec4_kernel: a block owns GROUPS*256 groups of four consecutive parameters
// and walks the workers in ascending order (fixed summation order for Eq. (2)).
#include "common.h"
#include "elastic_rule.h"

namespace easgd {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16x4 __attribute__((ext_vector_type(4)));

// A gradient element as fp32: GT = unsigned short (bfloat16 storage) or float.
__device__ __forceinline__ float grad_value(unsigned short g) { return bf16_widen(g); }
__device__ __forceinline__ float grad_value(float g) { return g; }

template <bool MOM, typename GT>
__device__ __forceinline__ void scalar_param(float *__restrict__ W, unsigned short *__restrict__ V,
                                             const GT *__restrict__ G, float *__restrict__ Wc,
                                             int P, size_t j, size_t ld, float eta, float rho, float alpha, float delta)
{
    const float c = Wc[j];
    float acc = 0.f;
    for (int i = 0; i < P; ++i) {             // ascending worker order
        const size_t k = (size_t)i * ld + j;
        float w = W[k];
        unsigned short v = 0;
        if constexpr (MOM) v = V[k];
        acc += worker_rule_bf16<MOM>(w, v, grad_value(G[k]), c, eta, rho, alpha, delta);
        W[k] = w;
        if constexpr (MOM) V[k] = v;
    }
    Wc[j] = fma_s(alpha, acc, c);                 // Eq. (2)
}

template <bool NT, typename T>
__device__ __forceinline__ T lp_load(const T *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}

template <bool NT, typename T>
__device__ __forceinline__ void lp_store(T *p, T v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

template <typename T> struct Vec4;
template <> struct Vec4<float> { typedef f32x4 type; };
template <> struct Vec4<unsigned short> { typedef u16x4 type; };

// One tile: 128-bit accesses to the fp32 rows, 64-bit accesses to the bfloat16 rows.  FULL: every group of the block
// lies inside the row (block-uniform).  No load is guarded in either form (lanes past the end of the row read its
// last group and store nothing), so all loads of a worker are in flight together.  Group by group here: with rows
// of two widths the stream-by-stream order of elastic_tile measured 1 % slower.
// GT: storage type of the gradients (unsigned short = bfloat16, or float when only V is stored in 16 bits).
template <bool MOM, bool NT, int GROUPS, size_t STRIDE, bool FULL, typename GT>
__device__ __forceinline__ void elastic_bf16_tile(f32x4 *__restrict__ W, u16x4 *__restrict__ V,
                                                  const typename Vec4<GT>::type *__restrict__ G, f32x4 *__restrict__ Wc,
                                                  int P, size_t n4, size_t ld4, size_t j0,
                                                  float eta, float rho, float alpha, float delta)
{
    typedef typename Vec4<GT>::type g4;
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    f32x4 c[GROUPS], acc[GROUPS];
    size_t jl[GROUPS];
#pragma unroll
    for (int q = 0; q < GROUPS; ++q) {
        const size_t j = j0 + (size_t)q * STRIDE;
        jl[q] = (FULL || j < n4) ? j : n4 - 1;
        c[q] = Wc[jl[q]];
        acc[q] = zero;
    }
    for (int i = 0; i < P; ++i) {
        const size_t row = (size_t)i * ld4;
        f32x4 w[GROUPS];
        g4 g[GROUPS];
        u16x4 v[GROUPS];
#pragma unroll
        for (int q = 0; q < GROUPS; ++q) {
            w[q] = lp_load<NT>(W + row + jl[q]);
            g[q] = lp_load<NT>(G + row + jl[q]);
            if constexpr (MOM) v[q] = lp_load<NT>(V + row + jl[q]);
        }
        if constexpr (!FULL) {
#pragma unroll
            for (int q = 0; q < GROUPS; ++q) {
                keep_loaded(w[q]);
                keep_loaded(g[q]);
                if constexpr (MOM) keep_loaded(v[q]);
            }
        }
        __builtin_amdgcn_sched_barrier(0);            // loads | arithmetic | stores, as in elastic_tile
#pragma unroll
        for (int q = 0; q < GROUPS; ++q) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float we = w[q][e];
                unsigned short ve = 0;
                if constexpr (MOM) ve = v[q][e];
                acc[q][e] += worker_rule_bf16<MOM>(we, ve, grad_value(g[q][e]), c[q][e], eta, rho, alpha, delta);
                w[q][e] = we;
                if constexpr (MOM) v[q][e] = ve;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q = 0; q < GROUPS; ++q) {
            if (FULL || j0 + (size_t)q * STRIDE < n4) {
                lp_store<NT>(W + row + jl[q], w[q]);
                if constexpr (MOM) lp_store<NT>(V + row + jl[q], v[q]);
            }
        }
    }
#pragma unroll
    for (int q = 0; q < GROUPS; ++q)
        if (FULL || j0 + (size_t)q * STRIDE < n4) Wc[jl[q]] = fma_s(alpha, acc[q], c[q]);   // Eq. (2)
}

// The N % 4 tail rides on the last block.
template <bool MOM, bool NT, int GROUPS, bool DIES, typename GT>
__device__ __forceinline__ void elastic_bf16_vec4_body(float *__restrict__ Wp, unsigned short *__restrict__ Vp,
                                                       const GT *__restrict__ Gp,
                                                       float *__restrict__ Wcp, int P, size_t N, size_t ld,
                                                       float eta, float rho, float alpha, float delta)
{
    typedef typename Vec4<GT>::type g4;
    typedef TileMap<GROUPS, DIES> Map;
    f32x4 *__restrict__ W = (f32x4 *)Wp;
    u16x4 *__restrict__ V = (u16x4 *)Vp;
    const g4 *__restrict__ G = (const g4 *)Gp;
    f32x4 *__restrict__ Wc = (f32x4 *)Wcp;
    const size_t n4 = N / 4, ld4 = ld / 4;
    const size_t n_tiles = Map::tiles(n4);
    for (size_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        const size_t j0 = Map::first(t, threadIdx.x);
        if (Map::last(t) < n4)
            elastic_bf16_tile<MOM, NT, GROUPS, Map::STRIDE, true, GT>(W, V, G, Wc, P, n4, ld4, j0, eta, rho, alpha, delta);
        else
            elastic_bf16_tile<MOM, NT, GROUPS, Map::STRIDE, false, GT>(W, V, G, Wc, P, n4, ld4, j0, eta, rho, alpha, delta);
    }
    const size_t tail = N - n4 * 4;
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x < tail)
        scalar_param<MOM, GT>(Wp, Vp, Gp, Wcp, P, n4 * 4 + threadIdx.x, ld, eta, rho, alpha, delta);
}

template <bool MOM, bool NT, int GROUPS, typename GT>
__global__ __launch_bounds__(256) void elastic_bf16_vec4_kernel(float *__restrict__ W, unsigned short *__restrict__ V,
                                                                const GT *__restrict__ G, float *__restrict__ Wc,
                                                                int P, size_t N, size_t ld,
                                                                float eta, float rho, float alpha, float delta)
{
    elastic_bf16_vec4_body<MOM, NT, GROUPS, false, GT>(W, V, G, Wc, P, N, ld, eta, rho, alpha, delta);
}

// die-interleaved tiles, one wavefront per SIMD (one block per compute unit), as elastic_vec4_dies_kernel
template <bool MOM, bool NT, int GROUPS, typename GT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void elastic_bf16_vec4_dies_kernel(float *__restrict__ W, unsigned short *__restrict__ V, const GT *__restrict__ G,
                                   float *__restrict__ Wc, int P, size_t N, size_t ld,
                                   float eta, float rho, float alpha, float delta)
{
    elastic_bf16_vec4_body<MOM, NT, GROUPS, true, GT>(W, V, G, Wc, P, N, ld, eta, rho, alpha, delta);
}

// Any alignment: one thread per parameter.
template <bool MOM, typename GT>
__global__ __launch_bounds__(256) void elastic_bf16_scalar_kernel(float *__restrict__ W, unsigned short *__restrict__ V,
                                                                  const GT *__restrict__ G,
                                                                  float *__restrict__ Wc, int P, size_t N, size_t ld,
                                                                  float eta, float rho, float alpha, float delta)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t j = (size_t)blockIdx.x * blockDim.x + threadIdx.x; j < N; j += stride)
        scalar_param<MOM, GT>(W, V, G, Wc, P, j, ld, eta, rho, alpha, delta);
}

template <bool MOM, bool NT, bool DIES, typename GT>
static void launch_bf16(int groups, dim3 grid, hipStream_t s, float *W, unsigned short *V, const GT *G,
                        float *Wc, int P, size_t N, size_t ld, float eta, float rho, float alpha, float delta)
{
#define EASGD_BF16(GR)                                                                                                        \
    do {                                                                                                                      \
        if (DIES) EASGD_LAUNCH((elastic_bf16_vec4_dies_kernel<MOM, NT, GR, GT>), grid, dim3(256), 0, s, W, V, G, Wc, P, N, ld, eta, rho, alpha, delta); \
        else EASGD_LAUNCH((elastic_bf16_vec4_kernel<MOM, NT, GR, GT>), grid, dim3(256), 0, s, W, V, G, Wc, P, N, ld, eta, rho, alpha, delta);          \
    } while (0)
    switch (groups) {
    case 1: EASGD_BF16(1); break;
    case 2: EASGD_BF16(2); break;
    case 4: EASGD_BF16(4); break;
    default: EASGD_BF16(8); break;
    }
#undef EASGD_BF16
}

inline bool aligned8(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 7u) == 0; }

template <bool MOM, typename GT>
static int elastic_round_bf16(const char *name, float *W, unsigned short *V, const GT *G, float *Wc, int P, size_t N,
                              size_t ld, float eta, float rho, float delta, void *stream)
{
    if (!W || !G || !Wc || (MOM && !V)) return fail(EASGD_EINVAL, "%s: NULL pointer", name);
    if (P < 1) return fail(EASGD_EINVAL, "%s: P must be >= 1, got %d", name, P);
    if (N == 0) return fail(EASGD_EINVAL, "%s: N must be >= 1", name);
    if (ld < N) return fail(EASGD_EINVAL, "%s: ld (%zu) < N (%zu)", name, ld, N);
    if (!aligned_to(W, 4) || !aligned_to(Wc, 4) || !aligned_to(G, sizeof(GT)) || !aligned_to(V, 2))
        return fail(EASGD_EINVAL, "%s: fp32 pointers must be 4-byte aligned, bfloat16 pointers 2-byte aligned", name);
    clear_error();

    hipStream_t s = static_cast<hipStream_t>(stream);
    const float alpha = eta * rho;
    const bool g_aligned = sizeof(GT) == 4 ? aligned16(G) : aligned8(G);
    const bool vec = aligned16(W) && aligned16(Wc) && g_aligned && (!MOM || aligned8(V)) && (ld % 4 == 0);
    const UpdateShape shape = update_shape(N, MOM);
    size_t blocks = vec ? shape.blocks : (N + 255) / 256;
    if (blocks > 0x7fffffffu) blocks = 0x7fffffffu;    // grid-stride loops cover the rest
    const dim3 grid((unsigned)blocks);
    const bool nt = update_nontemporal(N * ((8 + sizeof(GT) + (MOM ? 4 : 0)) * (size_t)P + 8));
    if (!vec)
        EASGD_LAUNCH((elastic_bf16_scalar_kernel<MOM, GT>), grid, dim3(256), 0, s, W, V, G, Wc, P, N, ld, eta, rho, alpha, delta);
    else if (shape.dies && nt)
        launch_bf16<MOM, true, true, GT>(shape.groups, grid, s, W, V, G, Wc, P, N, ld, eta, rho, alpha, delta);
    else if (shape.dies)
        launch_bf16<MOM, false, true, GT>(shape.groups, grid, s, W, V, G, Wc, P, N, ld, eta, rho, alpha, delta);
    else if (nt)
        launch_bf16<MOM, true, false, GT>(shape.groups, grid, s, W, V, G, Wc, P, N, ld, eta, rho, alpha, delta);
    else
        launch_bf16<MOM, false, false, GT>(shape.groups, grid, s, W, V, G, Wc, P, N, ld, eta, rho, alpha, delta);
    return check_launch(name);
}

}  // namespace easgd

extern "C" {

int easgd_sync_round_bf16(float *W, const uint16_t *G, float *Wc, int P, size_t N, size_t ld,
                          float eta, float rho, void *stream)
{
    return easgd::elastic_round_bf16<false, uint16_t>("easgd_sync_round_bf16", W, nullptr, G, Wc, P, N, ld, eta, rho, 0.0f, stream);
}

int measgd_round_bf16(float *W, uint16_t *V, const uint16_t *G, float *Wc, int P, size_t N, size_t ld,
                      float eta, float rho, float delta, void *stream)
{
    return easgd::elastic_round_bf16<true, uint16_t>("measgd_round_bf16", W, V, G, Wc, P, N, ld, eta, rho, delta, stream);
}

int measgd_round_bf16v(float *W, uint16_t *V, const float *G, float *Wc, int P, size_t N, size_t ld,
                       float eta, float rho, float delta, void *stream)
{
    return easgd::elastic_round_bf16<true, float>("measgd_round_bf16v", W, V, G, Wc, P, N, ld, eta, rho, delta, stream);
}

}  // extern "C"
