// Measurement aids: plain streaming kernels of known traffic.  They are used to
// measure this GPU's attainable HBM bandwidth (the ceiling the elastic update is
// compared with) and to calibrate hardware byte counters.  Not part of the method.
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

}  // extern "C"
