// A whole Sync EASGD round of a single-layer network (softmax regression) in ONE launch
// (Section 5.1 steps (1)-(5); Eq. (1) or Eq. (5),(6) for the workers, Eq. (2) for the center).
//
// Such a round is bound by launch boundaries, not by arithmetic: as two dependent launches (forward + softmax,
// then the weight-gradient product with the elastic epilogue) it spends more time between the kernels than in
// them.  Here one grid of at most one block per compute unit does both phases with a grid-wide barrier between:
//
//   phase A  every block takes (worker, four sample rows) items: logits, softmax cross-entropy, dZ -> workspace
//   barrier  all dZ are known and nobody reads W any more
//   phase B  every block takes slices of SN rows of the packed (d_in+1) x C matrix [W ; b]; thread (q, c) owns
//            the element (n0 + q, c) of EVERY worker: for workers in ascending order it forms the gradient
//            g = sum_r [X 1][r][n] dZ[r][c] (r ascending in four interleaved chains, fixed order), applies the
//            worker rule and adds W_i - Wc to its sum; then it applies Eq. (2).  The time-t center never leaves
//            the thread's registers, so no copy of it is needed, and the sum over workers has the order of the
//            streaming update kernels.
//
// The barrier is a count of arrivals in device memory that belongs to the library, one word per (device, stream)
// that has used this path, so that rounds on different streams never share one; it only ever grows (modulo 2^32),
// and the host, which knows how many blocks every launch on the stream adds, tells each launch the value to wait
// for.  What the blocks hand each other across the barrier (dZ, the row losses) is written and read with
// device-scope atomic accesses, which are served by the level of the memory hierarchy that all eight dies share,
// so the barrier needs no cache write-back or invalidation (a device-scope release/acquire pair would write back
// and invalidate each die's whole L2: tens of microseconds in a round that takes ten).  All blocks are resident at
// once (the grid is at most one block per compute unit and a block needs a third of a unit's LDS), so the wait
// ends; it is bounded all the same: a block that gives up marks the round by writing NaN into its share of the
// center, the replicas, the gradient and the losses, and counts itself in a word the host can read
// (easgd_round_barrier_timeouts).
#include "persistent_round.h"
#include "mlp_head.h"
#include <mutex>

namespace easgd {

typedef float f32x4 __attribute__((ext_vector_type(4)));

static constexpr int XS_FLOATS = 6144;       // LDS for the [X 1] slices of a pass (24 KiB)
static constexpr int DS_FLOATS = 6144;       // LDS for the dZ rows of a pass (24 KiB)
static constexpr int MAX_PASS_WORKERS = 8;   // workers whose replica values a thread holds in registers per pass
static constexpr int MAX_STREAMS = 64;       // streams per device that can use this path at the same time

// barrier words of one stream: [0] arrivals (only ever grows), [2] blocks that gave up waiting (ever)
static __device__ unsigned barrier_words[MAX_STREAMS][4];

// Rows of the packed matrix a block of 256 threads covers at a time: a multiple of 4, one thread per element.
__host__ __device__ static inline int slice_rows(int C) { return (256 / C) & ~3; }

bool softmax_round_fits(int d_in, int C, int b, int P)
{
    if (C < 1 || C > 16 || d_in < 1 || b < 1 || P < 1) return false;
    const int SN = slice_rows(C);
    if ((long)b * SN > XS_FLOATS || (long)b * C > DS_FLOATS) return false;
    // beyond this the round is no longer bound by launch boundaries and the matrix-core path wins
    return (long)P * b <= 2048 && (long)(d_in + 1) * C <= (1 << 17);
}

// Grid-wide barrier for a grid whose blocks are all resident: every block adds one to words[0] and waits until
// the count has reached `target` (the count before the launch plus the number of blocks; wrap-around is fine).
// Returns false if the wait was given up.
__device__ __forceinline__ bool grid_barrier(unsigned *words, unsigned target, unsigned spin_limit)
{
    __shared__ int passed;
    __builtin_amdgcn_s_waitcnt(0);                       // every memory operation of this wavefront has completed ...
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();                                     // ... before thread 0 announces the block
    if (threadIdx.x == 0) {
        int ok = 1;
        __hip_atomic_fetch_add(&words[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        unsigned spins = 0;
        while ((int)(__hip_atomic_load(&words[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) < 0) {
            if (++spins > spin_limit) {
                ok = 0;
                __hip_atomic_fetch_add(&words[2], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
        passed = ok;
    }
    __syncthreads();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    return passed != 0;
}

// MOMK: 0 = Eq. (1); 1 = Eq. (5),(6); 2 = Eq. (5),(6) with the momentum buffers stored as bfloat16
template <int CP, int MOMK>
__global__ __launch_bounds__(256) void softmax_round_kernel(HeadArgs h, SoftmaxRound u, unsigned *words, unsigned target, unsigned spin_limit)
{
    __shared__ float part[4][HEAD_ROWS * CP];
    __shared__ float dzs[HEAD_ROWS][CP];
    __shared__ __attribute__((aligned(16))) float xs[XS_FLOATS];
    __shared__ float ds[DS_FLOATS];
    const int tid = threadIdx.x;
    const int P = u.P, b = u.b, C = u.C, d_in = u.d_in;

    // ---- phase A: forward propagation and softmax cross-entropy ----
    const unsigned items = (unsigned)P * (unsigned)((b + HEAD_ROWS - 1) / HEAD_ROWS);
    for (unsigned it = blockIdx.x; it < items; it += gridDim.x) {
        head_block<HEAD_ROWS, CP, true, true>(h, it, part, dzs);
        __syncthreads();                                 // part and dzs are free again
    }

    // ---- phase B set-up: what does not depend on the other blocks is fetched before the barrier ----
    const int rows = d_in + 1;                           // rows of the packed matrix; the last one is the bias
    const int SN = slice_rows(C);
    const int n_slices = (rows + SN - 1) / SN;
    int wch = XS_FLOATS / (b * SN);
    if (wch > DS_FLOATS / (b * C)) wch = DS_FLOATS / (b * C);
    if (wch > MAX_PASS_WORKERS) wch = MAX_PASS_WORKERS;
    if (wch > P) wch = P;
    const int q = tid / C, c = tid - q * C;
    const bool update = u.W != nullptr;
    const bool x_vec = (d_in & 3) == 0 && (reinterpret_cast<uintptr_t>(u.X) & 15u) == 0;
    // [X 1] of workers w0 .. w0+nw-1, columns n0 .. n0+SN-1 -> xs[(worker, row)][column].  Loads are issued in
    // batches from clamped (always valid) addresses, so that a batch is in flight together.
    auto load_xs = [&](int n0, int w0, int nw) {
        const float *__restrict__ Xp = u.X + (size_t)w0 * b * d_in;
        constexpr int U = 6;
        if (x_vec && n0 + SN <= d_in) {                  // uniform: whole 128-bit chunks inside X
            const int per_row = SN / 4, total = nw * b * per_row;
            for (int base = tid; base < total; base += 256 * U) {
                f32x4 v[U];
#pragma unroll
                for (int k = 0; k < U; ++k) {
                    const int idx = min(base + 256 * k, total - 1), wr = idx / per_row, kq = idx - wr * per_row;
                    v[k] = *reinterpret_cast<const f32x4 *>(Xp + (size_t)wr * d_in + n0 + 4 * kq);
                }
#pragma unroll
                for (int k = 0; k < U; ++k)
                    if (base + 256 * k < total) *reinterpret_cast<f32x4 *>(xs + 4 * (base + 256 * k)) = v[k];
            }
        } else {
            const int total = nw * b * SN;
            for (int base = tid; base < total; base += 256 * 2 * U) {
                float v[2 * U];
#pragma unroll
                for (int k = 0; k < 2 * U; ++k) {
                    const int idx = min(base + 256 * k, total - 1), wr = idx / SN, nn = n0 + (idx - wr * SN);
                    const float x = Xp[(size_t)wr * d_in + min(nn, d_in - 1)];
                    v[k] = nn < d_in ? x : (nn == d_in ? 1.f : 0.f);
                }
#pragma unroll
                for (int k = 0; k < 2 * U; ++k)
                    if (base + 256 * k < total) xs[base + 256 * k] = v[k];
            }
        }
    };
    const bool has_slice = (int)blockIdx.x < n_slices;
    if (has_slice) load_xs((int)blockIdx.x * SN, 0, wch);

    const bool passed = grid_barrier(words, target, spin_limit);

    // the workers' mean losses (the order of mean_loss_kernel): wavefront 0 of block w, lanes over rows
    if (u.loss && tid < 64) {
        for (int w = blockIdx.x; w < P; w += gridDim.x) {
            float acc = 0.f;
            for (int r = tid; r < b; r += 64)
                acc += __hip_atomic_load(&h.row_loss[(size_t)w * b + r], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
            if (tid == 0) u.loss[w] = passed ? acc / (float)b : __builtin_nanf("");
        }
    }

    // ---- phase B: weight and bias gradients, worker rule, center rule ----
    for (int slice = blockIdx.x; slice < n_slices; slice += gridDim.x) {
        const int n0 = slice * SN, n = n0 + q;
        const bool live = q < SN && n < rows;
        const size_t e = (size_t)n * C + c;              // the thread's element of the packed matrix
        // the center at time t, read once (a local step has rho = 0: the center is not read at all)
        const float cen = (live && update && u.write_center) ? u.Wc[e] : 0.f;
        float acc = 0.f;
        if (!passed) {                                   // the barrier was given up: mark the round, compute nothing
            const float bad = __builtin_nanf("");
            if (live && update) {
                for (int w = 0; w < P; ++w) u.W[(size_t)w * u.ld + e] = bad;
                if (u.write_center) u.Wc[e] = bad;
            }
            if (live && u.G)
                for (int w = 0; w < P; ++w) u.G[(size_t)w * u.ld + e] = bad;
            if (live && u.G16)
                for (int w = 0; w < P; ++w) u.G16[(size_t)w * u.ld + e] = 0x7fc0;
            continue;
        }
        for (int w0 = 0; w0 < P; w0 += wch) {
            const int nw = min(wch, P - w0);
            const bool first = slice == (int)blockIdx.x && w0 == 0;      // its xs was loaded before the barrier
            if (!first) __syncthreads();                 // the previous pass is done with xs and ds
            float wv[MAX_PASS_WORKERS], vv[MAX_PASS_WORKERS];
            unsigned short v16[MAX_PASS_WORKERS];
#pragma unroll
            for (int wi = 0; wi < MAX_PASS_WORKERS; ++wi) {
                wv[wi] = 0.f; vv[wi] = 0.f; v16[wi] = 0;
                if (live && update && wi < nw) {
                    wv[wi] = u.W[(size_t)(w0 + wi) * u.ld + e];
                    if constexpr (MOMK == 1) vv[wi] = u.V[(size_t)(w0 + wi) * u.ld + e];
                    if constexpr (MOMK == 2) v16[wi] = u.V16[(size_t)(w0 + wi) * u.ld + e];
                }
            }
            {
                float *dzp = h.dz + (size_t)w0 * b * C;
                const int total = nw * b * C;
                constexpr int U = 10;
                for (int base = tid; base < total; base += 256 * U) {
                    float v[U];
#pragma unroll
                    for (int k = 0; k < U; ++k)
                        v[k] = __hip_atomic_load(&dzp[min(base + 256 * k, total - 1)], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
                    for (int k = 0; k < U; ++k)
                        if (base + 256 * k < total) ds[base + 256 * k] = v[k];
                }
            }
            if (!first) load_xs(n0, w0, nw);
            __syncthreads();
            if (live) {
#pragma unroll
                for (int wi = 0; wi < MAX_PASS_WORKERS; ++wi) {
                    if (wi < nw) {
                        const float *xp = xs + (size_t)wi * b * SN + q, *dp = ds + (size_t)wi * b * C + c;
                        float g0 = 0.f, g1 = 0.f, g2 = 0.f, g3 = 0.f;
                        int r = 0;
                        for (; r + 4 <= b; r += 4) {
                            g0 = fmaf(xp[(r + 0) * SN], dp[(r + 0) * C], g0);
                            g1 = fmaf(xp[(r + 1) * SN], dp[(r + 1) * C], g1);
                            g2 = fmaf(xp[(r + 2) * SN], dp[(r + 2) * C], g2);
                            g3 = fmaf(xp[(r + 3) * SN], dp[(r + 3) * C], g3);
                        }
                        for (; r < b; ++r) g0 = fmaf(xp[r * SN], dp[r * C], g0);
                        const float g = (g0 + g1) + (g2 + g3);
                        const size_t at = (size_t)(w0 + wi) * u.ld + e;
                        if (u.G) u.G[at] = g;
                        if (u.G16) u.G16[at] = bf16_narrow(g);
                        if (update) {                                          // workers in ascending order
                            if constexpr (MOMK == 2) acc += worker_rule_bf16<true>(wv[wi], v16[wi], g, cen, u.eta, u.rho, u.alpha, u.delta);
                            else acc += worker_rule<MOMK == 1>(wv[wi], vv[wi], g, cen, u.eta, u.rho, u.alpha, u.delta);
                            u.W[at] = wv[wi];
                            if constexpr (MOMK == 1) u.V[at] = vv[wi];
                            if constexpr (MOMK == 2) u.V16[at] = v16[wi];
                        }
                    }
                }
            }
        }
        if (live && update && u.write_center) u.Wc[e] = fma_s(u.alpha, acc, cen);   // Eq. (2)
    }
}

// ---- host side ----
// Per device: which stream owns which barrier words, and how many arrivals the launches enqueued on it so far
// add up to (the value its counter has when they have all run).
struct StreamSlots {
    hipStream_t streams[MAX_STREAMS];
    unsigned arrivals[MAX_STREAMS];
    int used = 0;
    unsigned *base = nullptr;        // device address of barrier_words on this device
    bool tried = false;
};
static std::mutex slots_mutex;       // held from the slot look-up to the launch, so that the targets handed out for
static StreamSlots slots[64];        // a stream follow the order of its launches

// Slot of (current device, stream), or -1 when there is none to give.  Call with slots_mutex held.
static int slot_for(StreamSlots &t, hipStream_t s)
{
    if (!t.tried) {
        t.tried = true;
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(barrier_words)) == hipSuccess) t.base = static_cast<unsigned *>(p);
        else (void)hipGetLastError();
    }
    if (!t.base) return -1;
    for (int k = 0; k < t.used; ++k)
        if (t.streams[k] == s) return k;
    if (t.used == MAX_STREAMS) return -1;
    t.streams[t.used] = s;
    t.arrivals[t.used] = 0;
    return t.used++;
}

template <int CP>
static void launch_cp(const HeadArgs &h, const SoftmaxRound &u, unsigned blocks, unsigned *words, unsigned target, unsigned limit, hipStream_t s)
{
    if (u.V16) EASGD_LAUNCH((softmax_round_kernel<CP, 2>), dim3(blocks), dim3(256), 0, s, h, u, words, target, limit);
    else if (u.V) EASGD_LAUNCH((softmax_round_kernel<CP, 1>), dim3(blocks), dim3(256), 0, s, h, u, words, target, limit);
    else EASGD_LAUNCH((softmax_round_kernel<CP, 0>), dim3(blocks), dim3(256), 0, s, h, u, words, target, limit);
}

int softmax_round_launch(const SoftmaxRound &u, void *stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    // a launch whose blocks wait for each other is not something to record into a graph
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &cap) != hipSuccess) {
        (void)hipGetLastError();
        return 1;
    }
    if (cap != hipStreamCaptureStatusNone) return 1;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        (void)hipGetLastError();
        return 1;
    }

    HeadArgs h = {};
    h.A = u.X; h.Wl = u.W_in; h.w_ws = u.ld; h.y = u.y;
    h.dz = u.dz; h.row_loss = u.row_loss; h.da = nullptr;
    h.d_in = u.d_in; h.C = u.C; h.b = u.b; h.P = u.P;
    const unsigned items = (unsigned)u.P * (unsigned)((u.b + HEAD_ROWS - 1) / HEAD_ROWS);
    const unsigned n_slices = (unsigned)((u.d_in + 1 + slice_rows(u.C) - 1) / slice_rows(u.C));
    unsigned blocks = items > n_slices ? items : n_slices;
    const unsigned cus = (unsigned)num_cus();
    if (blocks > cus) blocks = cus;                      // one block per compute unit at most: all resident at once
    long limit = options().round_spin_limit;
    if (limit <= 0) limit = 1L << 22;                    // some seconds; a round takes microseconds

    std::lock_guard<std::mutex> guard(slots_mutex);
    StreamSlots &t = slots[dev];
    const int k = slot_for(t, s);
    if (k < 0) return 1;
    unsigned *words = t.base + 4 * k;
    const unsigned target = t.arrivals[k] + blocks;      // modulo 2^32, like the counter
    if (u.C <= 4) launch_cp<4>(h, u, blocks, words, target, (unsigned)limit, s);
    else if (u.C <= 8) launch_cp<8>(h, u, blocks, words, target, (unsigned)limit, s);
    else if (u.C <= 12) launch_cp<12>(h, u, blocks, words, target, (unsigned)limit, s);
    else launch_cp<16>(h, u, blocks, words, target, (unsigned)limit, s);
    // a launch that was refused adds nothing to the counter (the caller reports the error)
    if (hipPeekAtLastError() == hipSuccess) t.arrivals[k] = target;
    return 0;
}

}  // namespace easgd

extern "C" long easgd_round_barrier_timeouts(void *stream)
{
    using namespace easgd;
    hipStream_t s = static_cast<hipStream_t>(stream);
    unsigned *words = nullptr;
    {
        int dev = -1;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return fail(EASGD_ELAUNCH, "easgd_round_barrier_timeouts: no current device");
        std::lock_guard<std::mutex> guard(slots_mutex);
        const StreamSlots &t = slots[dev];
        for (int k = 0; k < t.used; ++k)
            if (t.streams[k] == s) words = t.base + 4 * k;
    }
    if (!words) return 0;                                // this stream never took the single-launch path
    unsigned n = 0;
    if (hipMemcpyAsync(&n, words + 2, sizeof(n), hipMemcpyDeviceToHost, s) != hipSuccess || hipStreamSynchronize(s) != hipSuccess) {
        const hipError_t e = hipGetLastError();
        return fail(EASGD_ELAUNCH, "easgd_round_barrier_timeouts: %s", hipGetErrorString(e));
    }
    clear_error();
    return (long)n;
}
