// Measurement aids: plain streaming kernels of known traffic.  They are used to
// measure this GPU's attainable HBM bandwidth (the ceiling the elastic update is
// compared with) and to calibrate hardware byte counters; and a bare matrix-core loop of
// known flops, the ceiling the gradient's products are compared with.  Not part of the method.
#include "common.h"

namespace easgd {

typedef float f32x4 __attribute__((ext_vector_type(4)));

// The probes use the update kernels' die-interleaved tile map with four groups per thread (TileMap<4, true>:
// eight consecutive blocks, one per die, interleave in 1 KiB pieces inside a super-tile), so that they measure
// what a plain stream reaches with the same access pattern; the grid is a multiple of 8 blocks.
typedef TileMap<4, true> ProbeMap;

// dst[j] = src[j]: n4 128-bit groups, 4n bytes read + 4n bytes written
__global__ __launch_bounds__(256) void stream_copy_kernel(f32x4 *__restrict__ dst, const f32x4 *__restrict__ src, size_t n4)
{
    for (size_t t = blockIdx.x; t < ProbeMap::tiles(n4); t += gridDim.x) {
        const size_t j0 = ProbeMap::first(t, threadIdx.x);
        if (ProbeMap::last(t) < n4) {
            f32x4 x[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) x[q] = __builtin_nontemporal_load(src + j0 + q * ProbeMap::STRIDE);
#pragma unroll
            for (int q = 0; q < 4; ++q) __builtin_nontemporal_store(x[q], dst + j0 + q * ProbeMap::STRIDE);
        } else {
            for (int q = 0; q < 4; ++q) {
                const size_t j = j0 + q * ProbeMap::STRIDE;
                if (j < n4) __builtin_nontemporal_store(__builtin_nontemporal_load(src + j), dst + j);
            }
        }
    }
}

// a[j] = b[j] + s*c[j]: two reads and one write per element, the mix of the EASGD update
__global__ __launch_bounds__(256) void stream_triad_kernel(f32x4 *__restrict__ a, const f32x4 *__restrict__ b,
                                                           const f32x4 *__restrict__ c, float s, size_t n4)
{
    for (size_t t = blockIdx.x; t < ProbeMap::tiles(n4); t += gridDim.x) {
        const size_t j0 = ProbeMap::first(t, threadIdx.x);
        if (ProbeMap::last(t) < n4) {
            f32x4 x[4], y[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                x[q] = __builtin_nontemporal_load(b + j0 + q * ProbeMap::STRIDE);
                y[q] = __builtin_nontemporal_load(c + j0 + q * ProbeMap::STRIDE);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) __builtin_nontemporal_store(x[q] + s * y[q], a + j0 + q * ProbeMap::STRIDE);
        } else {
            for (int q = 0; q < 4; ++q) {
                const size_t j = j0 + q * ProbeMap::STRIDE;
                if (j < n4) __builtin_nontemporal_store(__builtin_nontemporal_load(b + j) + s * __builtin_nontemporal_load(c + j), a + j);
            }
        }
    }
}

// a[j] = c[j] + s*d[j], b[j] = d[j] + s*e[j]: three reads and two writes per element, the mix of the momentum update
__global__ __launch_bounds__(256) void stream_mix32_kernel(f32x4 *__restrict__ a, f32x4 *__restrict__ b,
                                                           const f32x4 *__restrict__ c, const f32x4 *__restrict__ d,
                                                           const f32x4 *__restrict__ e, float s, size_t n4)
{
    for (size_t t = blockIdx.x; t < ProbeMap::tiles(n4); t += gridDim.x) {
        const size_t j0 = ProbeMap::first(t, threadIdx.x);
        if (ProbeMap::last(t) < n4) {
            f32x4 x[4], y[4], z[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                x[q] = __builtin_nontemporal_load(c + j0 + q * ProbeMap::STRIDE);
                y[q] = __builtin_nontemporal_load(d + j0 + q * ProbeMap::STRIDE);
                z[q] = __builtin_nontemporal_load(e + j0 + q * ProbeMap::STRIDE);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                __builtin_nontemporal_store(x[q] + s * y[q], a + j0 + q * ProbeMap::STRIDE);
                __builtin_nontemporal_store(y[q] + s * z[q], b + j0 + q * ProbeMap::STRIDE);
            }
        } else {
            for (int q = 0; q < 4; ++q) {
                const size_t j = j0 + q * ProbeMap::STRIDE;
                if (j < n4) {
                    const f32x4 x = __builtin_nontemporal_load(c + j), y = __builtin_nontemporal_load(d + j),
                                z = __builtin_nontemporal_load(e + j);
                    __builtin_nontemporal_store(x + s * y, a + j);
                    __builtin_nontemporal_store(y + s * z, b + j);
                }
            }
        }
    }
}

static int probe_grid(size_t n4, dim3 &grid)
{
    size_t blocks = ProbeMap::tiles(n4);
    if (blocks > 0x7ffffff8u) blocks = 0x7ffffff8u;     // a multiple of 8; the kernels' loops cover the rest
    grid = dim3((unsigned)blocks);
    return 0;
}

// The matrix-core yardstick: blocks of four wavefronts that do nothing but the inner loop of the 64x64x32 products,
// v_mfma_f32_32x32x2_f32 on one accumulator tile per wavefront, over one 32-deep slab of operands that sits in LDS
// (A[k][m] = probe_value(64k + m), B[k][n] = probe_value(1000 + 64k + n), pitch 64 + 4 as in the products).
// LDS_FETCH = false: every lane reads its 16 + 16 operand values once and multiplies from registers: the matrix
// cores alone.  LDS_FETCH = true: the operands are fetched from LDS again for every pass over the slab, two
// ds_read_b32 per MFMA as in the products: matrix cores plus their feeding, still without global memory, barriers
// or epilogues.  Each pass adds A^T B to the accumulators; out gets the 16 accumulator values of every lane
// (out[block][register][thread]).
__device__ __forceinline__ float probe_value(int i) { return (float)((i * 37 + 11) % 64 - 32) * 0.03125f; }

// MODE 0: operands in registers; 1: fetched from LDS; 2: as 1, and every pass also does what a slab of the products'
// K loop does besides its MFMAs: 16 KB of operands requested from global memory one pass ahead (four 128-bit loads
// per thread, a different 16 KB piece of `src` every pass), stored to LDS, one barrier.  The loaded values go to an
// LDS region of their own and do not enter the products, so out is the same in all modes.
template <int MODE>
__global__ __launch_bounds__(256) void mfma_probe_kernel(float *__restrict__ out, int iters,
                                                         const f32x4 *__restrict__ src, unsigned src_pieces)
{
    typedef float f32x16 __attribute__((ext_vector_type(16)));
    constexpr bool LDS_FETCH = MODE >= 1, FEED = MODE == 2;
    constexpr int PITCH = 68;
    __shared__ float lds[2 * 32 * PITCH];
    __shared__ f32x4 staged[FEED ? 1024 : 1];
    for (int i = threadIdx.x; i < 2 * 32 * 64; i += 256) {
        const int op = i / 2048, k = (i % 2048) / 64, x = i % 64;
        lds[(op * 32 + k) * PITCH + x] = probe_value(op * 1000 + k * 64 + x);
    }
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // lane l supplies A[k = 2*step + l/32][m = l%32] and B[k][n = l%32] of its wavefront's 32x32 tile
    const float *la = lds + (lane >> 5) * PITCH + (wave >> 1) * 32 + (lane & 31);
    const float *lb = lds + (32 + (lane >> 5)) * PITCH + (wave & 1) * 32 + (lane & 31);
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    float ra[16], rb[16];
#pragma unroll
    for (int st = 0; st < 16; ++st) {
        ra[st] = la[2 * st * PITCH];
        rb[st] = lb[2 * st * PITCH];
    }
    // piece p of src is 1024 groups of four floats; block x reads pieces (977 x + pass) mod src_pieces, the next
    // piece's number kept by scalar increments (no division in the loop)
    unsigned p_next = (blockIdx.x * 977u) % src_pieces;
    auto next_piece = [&]() {
        const f32x4 *at = src + (size_t)p_next * 1024 + threadIdx.x;
        p_next = (p_next + 1 == src_pieces) ? 0u : p_next + 1;
        return at;
    };
    // Two register stages, as in the products: at the top of a pass the piece two passes ahead is requested into
    // the stage that is free, half way through the pass the piece requested a pass and a half ago moves from the
    // other stage to LDS, and the pass ends in a barrier.
    f32x4 r0[4], r1[4];
    if constexpr (FEED) {
        const f32x4 *at = next_piece();
#pragma unroll
        for (int q = 0; q < 4; ++q) r1[q] = at[q * 256];
    }
    float a = ra[0], b = rb[0];
    auto pass = [&](f32x4 (&refill)[4], f32x4 (&arrived)[4]) {
        if constexpr (LDS_FETCH) asm volatile("" ::: "memory");      // the slab is read again on every pass
        if constexpr (FEED) {
            const f32x4 *at = next_piece();
#pragma unroll
            for (int q = 0; q < 4; ++q) refill[q] = at[q * 256];
        }
#pragma unroll
        for (int st = 0; st < 16; ++st) {
            const int nx = (st + 1) & 15;
            float an = ra[nx], bn = rb[nx];
            if constexpr (LDS_FETCH) {       // the next step's operands are requested before this step's MFMA, as in the products
                an = la[2 * nx * PITCH];
                bn = lb[2 * nx * PITCH];
                __builtin_amdgcn_sched_barrier(0);
            }
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
            a = an;
            b = bn;
            if constexpr (FEED) {
                if (st == 7) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) staged[q * 256 + threadIdx.x] = arrived[q];
                }
            }
        }
        if constexpr (FEED) __syncthreads();
    };
    int it = 0;
    for (; it + 1 < iters; it += 2) {
        pass(r0, r1);
        pass(r1, r0);
    }
    if (it < iters) pass(r0, r1);
    if constexpr (FEED) acc[0] += 0.f * staged[(threadIdx.x * 5) & 1023][0];      // keeps the staging alive; adds zero
    float *o = out + (size_t)blockIdx.x * 4096 + threadIdx.x;     // [block][register][thread]: coalesced stores
#pragma unroll
    for (int r = 0; r < 16; ++r) o[r * 256] = acc[r];
}

}  // namespace easgd

extern "C" {

int easgd_stream_copy(float *dst, const float *src, size_t n, void *stream)
{
    using namespace easgd;
    if (!dst || !src || n == 0 || (n & 3u) || !aligned16(dst) || !aligned16(src))
        return fail(EASGD_EINVAL, "easgd_stream_copy: need non-NULL 16-byte aligned pointers and n %% 4 == 0, n > 0");
    clear_error();
    dim3 grid;
    probe_grid(n / 4, grid);
    EASGD_LAUNCH(stream_copy_kernel, grid, dim3(256), 0, static_cast<hipStream_t>(stream), (f32x4 *)dst, (const f32x4 *)src, n / 4);
    return check_launch("easgd_stream_copy");
}

int easgd_stream_triad(float *a, const float *b, const float *c, size_t n, float s, void *stream)
{
    using namespace easgd;
    if (!a || !b || !c || n == 0 || (n & 3u) || !aligned16(a) || !aligned16(b) || !aligned16(c))
        return fail(EASGD_EINVAL, "easgd_stream_triad: need non-NULL 16-byte aligned pointers and n %% 4 == 0, n > 0");
    clear_error();
    dim3 grid;
    probe_grid(n / 4, grid);
    EASGD_LAUNCH(stream_triad_kernel, grid, dim3(256), 0, static_cast<hipStream_t>(stream), (f32x4 *)a, (const f32x4 *)b, (const f32x4 *)c, s, n / 4);
    return check_launch("easgd_stream_triad");
}

int easgd_stream_mix32(float *a, float *b, const float *c, const float *d, const float *e, size_t n, float s, void *stream)
{
    using namespace easgd;
    if (!a || !b || !c || !d || !e || n == 0 || (n & 3u) || !aligned16(a) || !aligned16(b) || !aligned16(c) ||
        !aligned16(d) || !aligned16(e))
        return fail(EASGD_EINVAL, "easgd_stream_mix32: need non-NULL 16-byte aligned pointers and n %% 4 == 0, n > 0");
    clear_error();
    dim3 grid;
    probe_grid(n / 4, grid);
    EASGD_LAUNCH(stream_mix32_kernel, grid, dim3(256), 0, static_cast<hipStream_t>(stream), (f32x4 *)a, (f32x4 *)b,
                 (const f32x4 *)c, (const f32x4 *)d, (const f32x4 *)e, s, n / 4);
    return check_launch("easgd_stream_mix32");
}

int easgd_mfma_probe(float *out, size_t out_len, int iters, int mode, int blocks_per_cu, const float *src, size_t src_len,
                     unsigned *blocks, void *stream)
{
    using namespace easgd;
    if (!out || !aligned_to(out, 4)) return fail(EASGD_EINVAL, "easgd_mfma_probe: out must be a non-NULL fp32 pointer");
    if (iters < 1 || iters > (1 << 20)) return fail(EASGD_EINVAL, "easgd_mfma_probe: iters must be in [1, 2^20], got %d", iters);
    if (mode < 0 || mode > 2) return fail(EASGD_EINVAL, "easgd_mfma_probe: mode must be 0, 1 or 2, got %d", mode);
    if (blocks_per_cu < 1 || blocks_per_cu > 8)
        return fail(EASGD_EINVAL, "easgd_mfma_probe: blocks_per_cu must be in [1, 8], got %d", blocks_per_cu);
    if (mode == 2 && (!src || !aligned16(src) || src_len < 4096 || src_len / 4096 > 0x7fffffffu))
        return fail(EASGD_EINVAL, "easgd_mfma_probe: mode 2 needs a 16-byte aligned src of at least 4096 floats");
    const unsigned n = (unsigned)blocks_per_cu * (unsigned)num_cus();
    if (out_len < (size_t)n * 4096)
        return fail(EASGD_EINVAL, "easgd_mfma_probe: out holds %zu floats, %zu needed", out_len, (size_t)n * 4096);
    clear_error();
    if (blocks) *blocks = n;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const f32x4 *src4 = reinterpret_cast<const f32x4 *>(src);
    const unsigned pieces = mode == 2 ? (unsigned)(src_len / 4096) : 1u;
    if (mode == 2) EASGD_LAUNCH(mfma_probe_kernel<2>, dim3(n), dim3(256), 0, s, out, iters, src4, pieces);
    else if (mode == 1) EASGD_LAUNCH(mfma_probe_kernel<1>, dim3(n), dim3(256), 0, s, out, iters, src4, pieces);
    else EASGD_LAUNCH(mfma_probe_kernel<0>, dim3(n), dim3(256), 0, s, out, iters, src4, pieces);
    return check_launch("easgd_mfma_probe");
}

}  // extern "C"
