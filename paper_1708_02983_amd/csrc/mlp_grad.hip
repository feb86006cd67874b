// Step (1) of a Sync EASGD round (Section 5.1): the minibatch gradient of every
// worker at its own weights, for a dense ReLU MLP with softmax cross-entropy
// (forward / backward propagation of Section 2.2), written straight into the
// packed gradient buffer (the packed single-buffer layout of Section 5.2).
//
// Per layer l (d_in = dims[l], d_out = dims[l+1]) the packed block is the
// (d_in+1) x d_out matrix [W_l ; b_l], so with a ones column appended to the
// layer input A_l the three products are
//   forward   Z_l      = [A_l 1] * [W_l ; b_l]                (b x d_out),  A_{l+1} = relu(Z_l)
//   weights   [dW;db]  = [A_l 1]^T * dZ_l                     ((d_in+1) x d_out, contiguous in G)
//   inputs    dZ_{l-1} = (dZ_l * W_l^T) masked by A_l > 0     (b x d_in)
// The last layer's logits are produced as split-K partial sums that the softmax
// kernel adds in ascending split order, so every sum has a fixed order; a last
// layer of at most 16 classes instead takes one launch for its forward product,
// the softmax and its input-gradient product (mlp_head_kernel).
//
// The same sequence of launches also serves the whole round in one call
// (easgd_mlp_round, steps (1)-(5)): Eq. (2) runs ahead of backward propagation
// (on extra blocks of the first forward launch, on a second stream, or as a
// kernel of its own), the input-gradient product of a layer runs before its
// weight-gradient product, and that product applies the worker rule Eq. (1) /
// Eq. (5),(6) to the layer's slice of every replica in its epilogue.
#include "gemm_mfma.h"
#include "mlp_head.h"
#include "persistent_round.h"
#include <mutex>

// The workspace of easgd_grad_static: device memory that belongs to the library, one copy per GPU, held from
// the moment the library is loaded on that GPU until the process ends.  In host code this name is only a
// stand-in for the symbol; the device address is looked up once per device (static_scratch below).
static __device__ __align__(256) unsigned char scratch[EASGD_STATIC_SCRATCH_BYTES];

namespace easgd {

static constexpr int MAX_LAYERS = 8;
static constexpr int MAX_CLASSES = 1024;
static constexpr int MAX_SPLITS = 16;

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct GradPlan {
    size_t N = 0;
    size_t off[MAX_LAYERS] = {0};       // packed offset of layer l
    size_t act_off[MAX_LAYERS] = {0};   // workspace offset (bytes) of A_l, l = 1..L-1
    size_t logits_off = 0, rowloss_off = 0, dz_off[3] = {0, 0, 0};
    size_t bytes = 0;
    int splits = 1, k_per_split = 0;
    size_t center_off = 0, round_bytes = 0;
};

// Slab depth of the 128x32 tile (logits, narrow weight gradients).  These products are latency-bound: a block has
// a handful of slabs and little to multiply per slab, so fewer, deeper slabs win (32 against 16: the logits of a
// 2048-wide layer 26 -> 19 us, a whole 784-10 round 25.8 -> 23.2 us).
static constexpr int SPLIT_BK = 32;

static bool make_plan(const int *dims, int L, int P, int b, GradPlan &pl)
{
    if (!dims || L < 1 || L > MAX_LAYERS || P < 1 || b < 1) return false;
    for (int l = 0; l <= L; ++l)
        if (dims[l] < 1) return false;
    size_t n = 0;
    for (int l = 0; l < L; ++l) {
        pl.off[l] = n;
        n += (size_t)dims[l] * dims[l + 1] + dims[l + 1];
    }
    pl.N = n;
    // split the long, skinny logits product over K so that enough blocks run
    const int K = dims[L - 1] + 1;
    int splits = (K + 127) / 128;
    if (splits > MAX_SPLITS) splits = MAX_SPLITS;
    if (splits < 1) splits = 1;
    int kps = (K + splits - 1) / splits;
    kps = (kps + SPLIT_BK - 1) / SPLIT_BK * SPLIT_BK;
    pl.k_per_split = kps;
    pl.splits = (K + kps - 1) / kps;

    size_t o = 0, widest = 0;
    for (int l = 1; l < L; ++l) {
        pl.act_off[l] = o;
        o += align_up((size_t)P * b * dims[l] * sizeof(float), 256);
    }
    for (int l = 1; l <= L; ++l) widest = dims[l] > (int)widest ? dims[l] : widest;
    pl.logits_off = o;
    o += align_up((size_t)pl.splits * P * b * dims[L] * sizeof(float), 256);
    pl.rowloss_off = o;
    o += align_up((size_t)P * b * sizeof(float), 256);
    for (int q = 0; q < 3; ++q) {
        pl.dz_off[q] = o;
        o += align_up((size_t)P * b * widest * sizeof(float), 256);
    }
    pl.bytes = o;
    pl.center_off = o;                   // whole-round call only: the center at time t
    pl.round_bytes = o + align_up(pl.N * sizeof(float), 256);
    return true;
}

// Softmax cross-entropy on the logits of all workers: one wavefront per sample row, the classes
// spread over the lanes.  Sums use fixed shuffle trees and fixed orders.
//   zpart [splits][rows][C] partial logits (added in ascending split order)
//   dz [rows][C] <- (softmax - onehot)/b;   row_loss[rows] <- -log softmax(label)
__global__ __launch_bounds__(256) void softmax_xent_kernel(const float *__restrict__ zpart, const int *__restrict__ y,
                                                           float *__restrict__ dz, float *__restrict__ row_loss,
                                                           int rows, int b, int C, int splits, size_t split_stride)
{
    const int lane = threadIdx.x & 63;
    const size_t row = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= (size_t)rows) return;
    const float inv_b = 1.0f / (float)b;
    const int label = y[row];
    float z[MAX_CLASSES / 64];               // up to 16 classes per lane
    float zmax = -INFINITY;
#pragma unroll
    for (int q = 0; q < MAX_CLASSES / 64; ++q) {
        const int c = lane + 64 * q;
        float v = -INFINITY;
        if (c < C) {
            v = 0.f;
            for (int s = 0; s < splits; ++s) v += zpart[s * split_stride + row * C + c];
        }
        z[q] = v;
        zmax = fmaxf(zmax, v);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) zmax = fmaxf(zmax, __shfl_xor(zmax, o));
    float sum = 0.f, zlabel = 0.f;           // zlabel: shifted logit of the true class (one lane holds it)
#pragma unroll
    for (int q = 0; q < MAX_CLASSES / 64; ++q) {
        const int c = lane + 64 * q;
        if (c < C) {
            if (c == label) zlabel = z[q] - zmax;
            z[q] = expf(z[q] - zmax);
            sum += z[q];
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) zlabel += __shfl_xor(zlabel, o);
    const float inv_sum = 1.0f / sum;
#pragma unroll
    for (int q = 0; q < MAX_CLASSES / 64; ++q) {
        const int c = lane + 64 * q;
        if (c < C) dz[row * C + c] = (z[q] * inv_sum - (c == label ? 1.f : 0.f)) * inv_b;
    }
    if (lane == 0) row_loss[row] = logf(sum) - zlabel;
}

// loss[w] = mean of the worker's b row losses: lane l adds rows l, l+64, ... in order, then a fixed shuffle tree.
__global__ __launch_bounds__(64) void mean_loss_kernel(const float *__restrict__ row_loss, float *__restrict__ loss, int b)
{
    const int w = blockIdx.x, lane = threadIdx.x;
    float acc = 0.f;
    for (int r = lane; r < b; r += 64) acc += row_loss[(size_t)w * b + r];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
    if (lane == 0) loss[w] = acc / (float)b;
}

// One launch for the head of the network; the grid may be extended by blocks that run the center rule (h.ctr).
template <int ROWS, int CP, bool ONE_PASS, int NT = 4>
__global__ __launch_bounds__(256) void mlp_head_kernel(HeadArgs h)
{
    __shared__ float part[4][ROWS * CP];
    __shared__ float dzs[ROWS][CP];
    if (h.ctr.blocks > 0 && blockIdx.x >= h.ctr.first_block) {         // uniform for the block
        const size_t cb = blockIdx.x - h.ctr.first_block;
        if (h.ctr.vec) center_rule_block<f32x4>(h.ctr.W, h.ctr.Wc, h.ctr.old, h.ctr.P, h.ctr.N, h.ctr.ld, h.ctr.alpha, cb, h.ctr.blocks, threadIdx.x);
        else center_rule_block<float>(h.ctr.W, h.ctr.Wc, h.ctr.old, h.ctr.P, h.ctr.N, h.ctr.ld, h.ctr.alpha, cb, h.ctr.blocks, threadIdx.x);
        return;
    }
    head_block<ROWS, CP, ONE_PASS, false, NT>(h, blockIdx.x, part, dzs);
}

// Whether the head of a network with these layer widths takes the single-launch path.
static bool head_fits(const int *dims, int L) { return dims[L] <= HEAD_MAX_C; }

template <int CP>
static void launch_head_cp(const HeadArgs &h, unsigned blocks, hipStream_t s)
{
    if (h.d_in <= 1024) EASGD_LAUNCH((mlp_head_kernel<HEAD_ROWS, CP, true>), dim3(blocks), dim3(256), 0, s, h);
    else if (h.d_in <= 2048) EASGD_LAUNCH((mlp_head_kernel<HEAD_ROWS, CP, true, 8>), dim3(blocks), dim3(256), 0, s, h);
    else EASGD_LAUNCH((mlp_head_kernel<HEAD_ROWS, CP, false>), dim3(blocks), dim3(256), 0, s, h);
}

static unsigned head_blocks(int P, int b) { return (unsigned)P * (unsigned)((b + HEAD_ROWS - 1) / HEAD_ROWS); }

static void launch_head(HeadArgs h, hipStream_t s)
{
    unsigned blocks = head_blocks(h.P, h.b);
    if (h.ctr.blocks > 0) {
        h.ctr.first_block = blocks;
        blocks += h.ctr.blocks;
    }
    if (h.C <= 4) launch_head_cp<4>(h, blocks, s);
    else if (h.C <= 8) launch_head_cp<8>(h, blocks, s);
    else if (h.C <= 12) launch_head_cp<12>(h, blocks, s);
    else launch_head_cp<16>(h, blocks, s);
}

// ---- GEMM dispatch -------------------------------------------------------

enum Kind { FWD, DW, DA };

// Fills in the tile counts and the die-aware block numbering of a product; returns its number of blocks.
template <int BM, int BN>
static unsigned place_blocks(GemmArgs &a)
{
    a.tiles_m = (a.M + BM - 1) / BM;
    a.tiles_n = (a.N + BN - 1) / BN;
    size_t total = (size_t)a.tiles_m * a.tiles_n * a.splits * a.P;
    a.xcd_chunk = 0;
    a.die_workers = 0;
    a.band_log2 = 0;
    a.band_tiles = 0;
    if (options().gemm_xcd && total >= 64) {
        total = (total + 7) / 8 * 8;
        a.xcd_chunk = (int)(total / 8);
        // a product with an elastic epilogue (it has a center): interleave the workers of a die
        const long order = options().gemm_xcd;
        if (a.center && a.splits == 1 && a.P % 8 == 0 && (order == 1 || order == 3)) {
            a.die_workers = a.P / 8;
            // bands of 8 (4, 2) tile columns when the tile columns divide into them
            if (order == 1 && a.tiles_m > 1)
                a.band_log2 = a.tiles_n % 8 == 0 ? 3 : a.tiles_n % 4 == 0 ? 2 : a.tiles_n % 2 == 0 ? 1 : 0;
            a.band_tiles = a.tiles_m << a.band_log2;
        }
    }
    // the kernel's divisions by multiplication: exact while dividend * divisor < 2^32
    auto magic = [&](size_t dividend_max, int d) -> unsigned {
        if (d <= 1 || dividend_max * (size_t)d >= ((size_t)1 << 32)) return 0u;
        return (unsigned)((((size_t)1 << 32) + (size_t)d - 1) / (size_t)d);
    };
    const size_t tiles = (size_t)a.tiles_m * a.tiles_n;
    a.magic_tiles = magic(total, (int)tiles);
    a.magic_tiles_n = magic(tiles, a.tiles_n);
    a.magic_die = magic(total / 8 + 1, a.die_workers);
    a.magic_band = magic(tiles, a.band_tiles);
    return (unsigned)total;
}

// Two products of backward propagation in one launch (gemm_pair_kernel).
// (i) the input-gradient product of layer l (64x64 tiles) with the weight-gradient product of a narrow layer
//     l+1 (128x32 tile): the few blocks of the second fill wave slots the first leaves idle;
// (ii) the weight-gradient products of two layers (64x64 tiles both): one launch boundary and one tail less.
template <int EPI, bool VEC_DW>
static void launch_pair_da_narrow_dw(GemmArgs da, GemmArgs dw, hipStream_t s)
{
    const unsigned n0 = place_blocks<64, 64>(da), n1 = place_blocks<128, 32>(dw);
    EASGD_LAUNCH((gemm_pair_kernel<64, 64, 32, 2, 2, K_CONTIG, K_CONTIG, true, EPI_MASK,
                                         128, 32, SPLIT_BK, 4, 1, MN_CONTIG, MN_CONTIG, VEC_DW, EPI>),
                       dim3(n0 + n1), dim3(256), 0, s, da, dw, n0);
}

template <int EPI>
static void launch_pair_dw_dw(GemmArgs d0, GemmArgs d1, hipStream_t s)
{
    const unsigned n0 = place_blocks<64, 64>(d0), n1 = place_blocks<64, 64>(d1);
    EASGD_LAUNCH((gemm_pair_kernel<64, 64, 32, 2, 2, MN_CONTIG, MN_CONTIG, true, EPI,
                                         64, 64, 32, 2, 2, MN_CONTIG, MN_CONTIG, true, EPI>),
                       dim3(n0 + n1), dim3(256), 0, s, d0, d1, n0);
}

template <int BM, int BN, int BK, int WM, int WN, int AL, int BL, int EPI, int MT = 32>
static void launch_tile(const GemmArgs &a_in, bool vec, hipStream_t s)
{
    GemmArgs a = a_in;
    size_t total = place_blocks<BM, BN>(a);
    static_assert(WM * WN * 64 == 256, "the center rule's extra blocks assume 256 threads");
    if (a.ctr.blocks > 0) {
        a.ctr.first_block = (unsigned)total;
        total += a.ctr.blocks;
    }
    const dim3 grid((unsigned)total), block(WM * WN * 64);
    if (vec) EASGD_LAUNCH((gemm_mfma_kernel<BM, BN, BK, WM, WN, AL, BL, true, EPI, MT>), grid, block, 0, s, a);
    else EASGD_LAUNCH((gemm_mfma_kernel<BM, BN, BK, WM, WN, AL, BL, false, EPI, MT>), grid, block, 0, s, a);
}

// A batch that is not a multiple of 32 rows wastes matrix-core time in 32-row MFMA tiles (b = 100: 128 rows are
// multiplied, 28 % more than stored).  The 16x16x4 instruction has the same rate, so a block tile of 3, 5 or 7 x 16
// rows by 128 columns (four wavefronts side by side, 3, 5 or 7 x 2 accumulators each) multiplies 48, 80 or 112
// rows per tile.  It is chosen for the products whose M is the batch (forward, input gradient) when one of the
// three heights covers M with fewer rows than 32-row tiles do and still gives every compute unit about two
// blocks.  Returns that height, or 0.
static int tile16_rows(int M, int N, int P, int splits)
{
    if (N <= 32) return 0;
    long best_rows = (long)((M + 31) / 32) * 32;
    int best = 0;
    for (int bm : {112, 80, 48}) {
        const long rows = (long)((M + bm - 1) / bm) * bm;
        if (rows < best_rows) {
            best_rows = rows;
            best = bm;
        }
    }
    if (best == 0) return 0;
    return (size_t)((M + best - 1) / best) * ((N + 127) / 128) * splits * P >= (size_t)(2 * num_cus()) ? best : 0;
}

// Picks the tile shape.  Outputs at most 32 wide use a 128x32 tile.  Otherwise 64x64 blocks (four per
// compute unit, so that the epilogue of one overlaps the products of the others) unless the caller asks
// for the large tile and it still gives every compute unit about two blocks: that pays for the long-K
// forward products, not for the short-K weight gradients with their heavy epilogues.
template <int AL, int BL, int EPI>
static void launch_gemm(const GemmArgs &a, bool vec, bool large_ok, hipStream_t s)
{
    if (a.N <= 32) {
        launch_tile<128, 32, SPLIT_BK, 4, 1, AL, BL, EPI>(a, vec, s);
        return;
    }
    const size_t big = (size_t)((a.M + 127) / 128) * ((a.N + 127) / 128) * a.splits * a.P;
    long tile = options().gemm_tile;
    if constexpr (AL == K_CONTIG && (EPI == EPI_NONE || EPI == EPI_RELU || EPI == EPI_MASK)) {
        int bm16 = (tile == 0) ? tile16_rows(a.M, a.N, a.P, a.splits) : 0;
        if (tile == 4) bm16 = a.M <= 48 ? 48 : a.M <= 80 ? 80 : 112;    // forced: the smallest height that covers M, else 112
        if (bm16 == 112) launch_tile<112, 128, 32, 1, 4, AL, BL, EPI, 16>(a, vec, s);
        else if (bm16 == 80) launch_tile<80, 128, 32, 1, 4, AL, BL, EPI, 16>(a, vec, s);
        else if (bm16 == 48) launch_tile<48, 128, 32, 1, 4, AL, BL, EPI, 16>(a, vec, s);
        if (bm16) return;
    }
    if (tile == 4) tile = 0;            // the weight-gradient products have no 16-row form
    if (tile == 0) tile = (large_ok && big >= (size_t)(2 * num_cus())) ? 1 : 2;
    if (tile == 1) launch_tile<128, 128, 16, 2, 2, AL, BL, EPI>(a, vec, s);
    else if (tile == 2) launch_tile<64, 64, 32, 2, 2, AL, BL, EPI>(a, vec, s);
    else launch_tile<128, 64, 32, 2, 2, AL, BL, EPI>(a, vec, s);
}

static inline bool mult4(size_t x) { return (x & 3u) == 0; }

// Whether the launch of a forward product (M x N per worker, P workers, `splits` K splits) leaves room on the
// chip for extra blocks that do bandwidth-bound work beside it.  Mirrors launch_gemm: the 128x32 and 64x64
// tiles use few enough registers and LDS for four blocks per compute unit, the 128x128 tile for two, and it
// is chosen exactly when its blocks already fill those.
static bool forward_launch_has_room(int M, int N, int P, int splits)
{
    const size_t cus = (size_t)num_cus();
    if (N <= 32) return (size_t)((M + 127) / 128) * splits * P <= 3 * cus;
    long tile = options().gemm_tile;
    if (tile == 4 || (tile == 0 && tile16_rows(M, N, P, splits) != 0)) return false;
    const size_t big = (size_t)((M + 127) / 128) * ((N + 127) / 128) * splits * P;
    if (tile == 0) tile = (big >= 2 * cus) ? 1 : 2;
    if (tile != 2) return false;
    return (size_t)((M + 63) / 64) * ((N + 63) / 64) * splits * P <= 3 * cus;
}

// Elastic update fused into the backward pass.  Eq. (2) runs first and saves the time-t
// center in the workspace for the worker rules; the worker rule is the epilogue of each
// layer's weight-gradient product, which runs after the layer's input-gradient product, the
// last reader of W_l at time t.
struct ElasticStep {
    float *W, *V, *Wc;
    float eta, rho, delta;
    unsigned short *V16;    // momentum buffers stored as bfloat16 (then V is null), or null
};

static int grad_impl(const char *name, const int *dims, int n_layers, const float *W, size_t ld, const float *X,
                     const int32_t *y, int P, int b, float *G, float *loss, void *workspace, size_t workspace_bytes,
                     void *stream, const ElasticStep *step, unsigned short *G16 = nullptr);

// A second stream per device (default priority) with the two events that order it against the caller's
// stream: `fork` is recorded on the caller's stream when the round starts, `join` on the second stream when
// the center rule is done.  Created on first use and kept until the process ends; whole-round calls hold
// `side_mutex`, so that two host threads never interleave their record/wait pairs.
struct SideLane {
    hipStream_t stream = nullptr;
    hipEvent_t fork = nullptr, join = nullptr;
    bool tried = false, ok = false;
};
static std::mutex side_mutex;
static constexpr int MAX_DEVICES = 64;
static SideLane side_lanes[MAX_DEVICES];

static SideLane *side_lane()       // call with side_mutex held; nullptr when no lane can be made
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
    SideLane &ln = side_lanes[dev];
    if (!ln.tried) {
        ln.tried = true;
        ln.ok = hipStreamCreateWithFlags(&ln.stream, hipStreamNonBlocking) == hipSuccess &&
                hipEventCreateWithFlags(&ln.fork, hipEventDisableTiming) == hipSuccess &&
                hipEventCreateWithFlags(&ln.join, hipEventDisableTiming) == hipSuccess;
        if (!ln.ok) (void)hipGetLastError();
    }
    return ln.ok ? &ln : nullptr;
}

// Device address of `scratch` on the current device, looked up on the first call per device (with that device
// current) and kept; nullptr (and the error string set) when the lookup fails.
static void *static_scratch(const char *name)
{
    static std::mutex lookup_mutex;
    static void *ptrs[MAX_DEVICES] = {nullptr};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) {
        (void)hipGetLastError();
        fail(EASGD_ELAUNCH, "%s: no current device", name);
        return nullptr;
    }
    std::lock_guard<std::mutex> guard(lookup_mutex);
    if (!ptrs[dev]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            (void)hipGetLastError();
            fail(EASGD_ELAUNCH, "%s: address of the static workspace: %s", name, hipGetErrorString(e));
            return nullptr;
        }
        ptrs[dev] = p;
    }
    return ptrs[dev];
}

}  // namespace easgd

extern "C" {

size_t easgd_mlp_num_params(const int *dims, int n_layers)
{
    easgd::GradPlan pl;
    if (!easgd::make_plan(dims, n_layers, 1, 1, pl)) return 0;
    return pl.N;
}

size_t easgd_grad_workspace_bytes(const int *dims, int n_layers, int P, int b)
{
    easgd::GradPlan pl;
    if (!easgd::make_plan(dims, n_layers, P, b, pl)) return 0;
    return pl.bytes;
}

size_t easgd_mlp_round_workspace_bytes(const int *dims, int n_layers, int P, int b)
{
    easgd::GradPlan pl;
    if (!easgd::make_plan(dims, n_layers, P, b, pl)) return 0;
    return pl.round_bytes;
}

int easgd_grad(const int *dims, int n_layers, const float *W, size_t ld, const float *X, const int32_t *y,
               int P, int b, float *G, float *loss, void *workspace, size_t workspace_bytes, void *stream)
{
    return easgd::grad_impl("easgd_grad", dims, n_layers, W, ld, X, y, P, b, G, loss, workspace, workspace_bytes,
                            stream, nullptr);
}

int easgd_grad_static(const int *dims, int n_layers, const float *W, size_t ld, const float *X, const int32_t *y,
                      int P, int b, float *G, float *loss, void *stream)
{
    easgd::GradPlan pl;
    if (!easgd::make_plan(dims, n_layers, P, b, pl))
        return easgd::fail(EASGD_EINVAL, "easgd_grad_static: need 1 <= n_layers <= %d, all dims >= 1, P >= 1, b >= 1", easgd::MAX_LAYERS);
    if (pl.bytes > (size_t)EASGD_STATIC_SCRATCH_BYTES)
        return easgd::fail(EASGD_EWORKSPACE, "easgd_grad_static: this shape needs %zu bytes of workspace, the static workspace holds %zu; "
                           "use easgd_grad with a workspace of the caller", pl.bytes, (size_t)EASGD_STATIC_SCRATCH_BYTES);
    void *ws = easgd::static_scratch("easgd_grad_static");
    if (!ws) return EASGD_ELAUNCH;
    return easgd::grad_impl("easgd_grad_static", dims, n_layers, W, ld, X, y, P, b, G, loss, ws,
                            (size_t)EASGD_STATIC_SCRATCH_BYTES, stream, nullptr);
}

int easgd_grad_bf16(const int *dims, int n_layers, const float *W, size_t ld, const float *X, const int32_t *y,
                    int P, int b, uint16_t *G, float *loss, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!G) return easgd::fail(EASGD_EINVAL, "easgd_grad_bf16: NULL pointer");
    if (reinterpret_cast<uintptr_t>(G) & 1u) return easgd::fail(EASGD_EINVAL, "easgd_grad_bf16: G must be 2-byte aligned");
    return easgd::grad_impl("easgd_grad_bf16", dims, n_layers, W, ld, X, y, P, b, nullptr, loss, workspace,
                            workspace_bytes, stream, nullptr, G);
}

int easgd_mlp_round(const int *dims, int n_layers, float *W, float *V, float *Wc, size_t ld,
                    const float *X, const int32_t *y, int P, int b, float *G, float *loss,
                    float eta, float rho, float delta, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!Wc) return easgd::fail(EASGD_EINVAL, "easgd_mlp_round: NULL pointer");
    const easgd::ElasticStep step = {W, V, Wc, eta, rho, delta, nullptr};
    return easgd::grad_impl("easgd_mlp_round", dims, n_layers, W, ld, X, y, P, b, G, loss, workspace,
                            workspace_bytes, stream, &step);
}

int easgd_mlp_round_bf16v(const int *dims, int n_layers, float *W, uint16_t *V, float *Wc, size_t ld,
                          const float *X, const int32_t *y, int P, int b, float *G, float *loss,
                          float eta, float rho, float delta, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!Wc || !V) return easgd::fail(EASGD_EINVAL, "easgd_mlp_round_bf16v: NULL pointer");
    if (reinterpret_cast<uintptr_t>(V) & 1u) return easgd::fail(EASGD_EINVAL, "easgd_mlp_round_bf16v: V must be 2-byte aligned");
    const easgd::ElasticStep step = {W, nullptr, Wc, eta, rho, delta, V};
    return easgd::grad_impl("easgd_mlp_round_bf16v", dims, n_layers, W, ld, X, y, P, b, G, loss, workspace,
                            workspace_bytes, stream, &step);
}

}  // extern "C"

namespace easgd {

static int grad_impl(const char *name, const int *dims, int n_layers, const float *W, size_t ld, const float *X,
                     const int32_t *y, int P, int b, float *G, float *loss, void *workspace, size_t workspace_bytes,
                     void *stream, const ElasticStep *step, unsigned short *G16)
{
    const int L = n_layers;
    GradPlan pl;
    if (!W || !X || !y || (!G && !G16 && !step)) return fail(EASGD_EINVAL, "%s: NULL pointer", name);
    if (!make_plan(dims, L, P, b, pl))
        return fail(EASGD_EINVAL, "%s: need 1 <= n_layers <= %d, all dims >= 1, P >= 1, b >= 1", name, MAX_LAYERS);
    if (dims[L] > MAX_CLASSES) return fail(EASGD_EINVAL, "%s: at most %d classes, got %d", name, MAX_CLASSES, dims[L]);
    if (ld < pl.N) return fail(EASGD_EINVAL, "%s: ld (%zu) < N (%zu)", name, ld, pl.N);
    if (!aligned16(W) || !aligned16(G) || !aligned16(X)) return fail(EASGD_EINVAL, "%s: W, G, X must be 16-byte aligned", name);
    const size_t need_bytes = step ? pl.round_bytes : pl.bytes;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < need_bytes)
        return fail(EASGD_EWORKSPACE, "%s: workspace must be 256-byte aligned and hold %zu bytes (got %zu)", name, need_bytes, workspace_bytes);
    for (int l = 0; l < L; ++l) {
        const size_t per_worker = (size_t)(dims[l] + 1) * dims[l + 1];
        if (per_worker > 0x3fffffffull || (size_t)b * dims[l] > 0x3fffffffull || (size_t)b * dims[l + 1] > 0x3fffffffull)
            return fail(EASGD_ERANGE, "%s: layer %d exceeds 2^30-1 elements per worker", name, l);
    }
    if ((size_t)P * b * (size_t)pl.splits > 0x7fffffffull) return fail(EASGD_ERANGE, "%s: P*b too large", name);
    clear_error();

    hipStream_t s = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    auto act = [&](int l) -> const float * { return l == 0 ? X : reinterpret_cast<const float *>(ws + pl.act_off[l]); };
    float *logits = reinterpret_cast<float *>(ws + pl.logits_off);
    // dZ_l lives in buffer l % 3: the input-gradient product of layer l reads buffer l % 3 and writes (l-1) % 3
    // while the weight-gradient product of layer l+1, which may share its launch, still reads (l+1) % 3
    float *dz[3] = {reinterpret_cast<float *>(ws + pl.dz_off[0]), reinterpret_cast<float *>(ws + pl.dz_off[1]),
                    reinterpret_cast<float *>(ws + pl.dz_off[2])};
    const bool base_vec = mult4(ld);

    // a narrow last layer goes through mlp_head_kernel together with the softmax and its own input gradient
    const bool head = options().mlp_head != 0 && head_fits(dims, L);
    if (head && (size_t)P * ((b + HEAD_ROWS - 1) / HEAD_ROWS) > 0x3fffffffull) return fail(EASGD_ERANGE, "%s: P*b too large", name);

    // ---- a single-layer network small enough to be bound by launch boundaries: the whole call in one launch ----
    if (L == 1 && head && options().round_single_launch != 0 &&
        softmax_round_fits(dims[0], dims[1], b, P)) {
        SoftmaxRound r = {};
        r.X = X; r.y = y; r.W_in = W; r.G = G; r.G16 = G16;
        r.dz = dz[0]; r.row_loss = reinterpret_cast<float *>(ws + pl.rowloss_off); r.loss = loss;
        r.ld = ld; r.d_in = dims[0]; r.C = dims[1]; r.b = b; r.P = P;
        if (step) {
            r.W = step->W; r.V = step->V; r.V16 = step->V16; r.Wc = step->Wc;
            r.eta = step->eta; r.rho = step->rho; r.alpha = step->eta * step->rho; r.delta = step->delta;
            r.write_center = step->rho != 0.f;
        }
        if (softmax_round_launch(r, stream) == 0) return check_launch(name);
        // otherwise (stream under capture, no barrier words left): the separate launches below
    }

    // ---- Eq. (2); beside forward propagation when the second stream is in use ----
    // rho == 0: a local step.  Eq. (2) leaves the center as it is and Eq. (1) is a plain (momentum) SGD step, so
    // the center rule is not launched at all and the worker rule reads the center in place (times zero).
    const bool local_step = step && step->rho == 0.f;
    float *old_center = step ? reinterpret_cast<float *>(ws + pl.center_off) : nullptr;
    const float *center_t = local_step ? step->Wc : old_center;
    std::unique_lock<std::mutex> lane_guard;
    SideLane *lane = nullptr;
    bool attach_center = false;
    if (step && !local_step) {
        // Where Eq. (2) runs (EASGD_OPT_ROUND_OVERLAP): 0 = a kernel of its own on the caller's stream, 2 = the
        // same on the library's second stream, beside forward propagation, 3 = on extra blocks of the first
        // forward product's launch.  1 (default) chooses: the extra blocks when that launch leaves room on the
        // chip (they then fill idle wave slots, no stream is involved); else the second stream when the rule has
        // enough to read to be worth the tens of microseconds that ordering two streams costs; else its own kernel.
        const long overlap = options().round_overlap;
        const int splits0 = (L == 1) ? pl.splits : 1;
        const bool room = (head && L == 1) ? head_blocks(P, b) <= 3u * (unsigned)num_cus()
                                           : forward_launch_has_room(b, dims[1], P, splits0);
        attach_center = (overlap == 3) || (overlap == 1 && room);
        if (!attach_center && (overlap == 2 || (overlap == 1 && (size_t)P * pl.N >= ((size_t)1 << 24)))) {
            lane_guard = std::unique_lock<std::mutex>(side_mutex);
            lane = side_lane();
        }
        const float alpha = step->eta * step->rho;
        int rc;
        if (lane) {
            if (hipEventRecord(lane->fork, s) != hipSuccess || hipStreamWaitEvent(lane->stream, lane->fork, 0) != hipSuccess)
                return check_launch(name) != EASGD_OK ? EASGD_ELAUNCH : fail(EASGD_ELAUNCH, "%s: stream fork failed", name);
            rc = center_range(step->W, step->Wc, old_center, P, pl.N, ld, alpha, lane->stream, true);
            if (rc == EASGD_OK && hipEventRecord(lane->join, lane->stream) != hipSuccess)
                rc = fail(EASGD_ELAUNCH, "%s: stream join failed", name);
        } else if (!attach_center) {
            rc = center_range(step->W, step->Wc, old_center, P, pl.N, ld, alpha, s);
        } else {
            rc = EASGD_OK;
        }
        if (rc != EASGD_OK) return rc;
    }

    // ---- forward propagation ----
    CenterJob center_job = {};           // rides on the first launch of forward propagation when attach_center
    if (attach_center) {
        const bool cvec = aligned16(step->W) && aligned16(step->Wc) && aligned16(old_center) && (ld % 4 == 0);
        const size_t cblocks = (cvec ? pl.N / 4 : pl.N) / 256 + 1;
        if (cblocks > 0x3fffffffu) return fail(EASGD_ERANGE, "%s: N too large", name);
        center_job.W = step->W; center_job.Wc = step->Wc; center_job.old = old_center;
        center_job.N = pl.N; center_job.ld = ld; center_job.P = P; center_job.vec = cvec ? 1 : 0;
        center_job.alpha = step->eta * step->rho; center_job.blocks = (unsigned)cblocks;
    }
    for (int l = 0; l < (head ? L - 1 : L); ++l) {
        const int d_in = dims[l], d_out = dims[l + 1];
        const bool last = (l == L - 1);
        GemmArgs a = {};
        a.A = act(l); a.a_ws = (size_t)b * d_in; a.lda = d_in; a.a_lim = d_in; a.a_ones = d_in;
        a.B = W + pl.off[l]; a.b_ws = ld; a.ldb = d_out;
        a.C = last ? logits : const_cast<float *>(act(l + 1)); a.c_ws = (size_t)b * d_out; a.ldc = d_out;
        a.M = b; a.N = d_out; a.K = d_in + 1; a.P = P;
        a.splits = last ? pl.splits : 1;
        a.k_per_split = last ? pl.k_per_split : ((a.K + 63) / 64 * 64);
        a.c_ss = (size_t)P * b * d_out;
        if (l == 0) a.ctr = center_job;
        const bool vec = base_vec && mult4(d_in) && mult4(d_out) && mult4(pl.off[l]);
        if (last) launch_gemm<K_CONTIG, MN_CONTIG, EPI_NONE>(a, vec, true, s);
        else launch_gemm<K_CONTIG, MN_CONTIG, EPI_RELU>(a, vec, true, s);
    }
    float *row_loss = reinterpret_cast<float *>(ws + pl.rowloss_off);
    const int rows = P * b;
    if (head) {
        HeadArgs h = {};
        h.A = act(L - 1); h.Wl = W + pl.off[L - 1]; h.w_ws = ld; h.y = y;
        h.dz = dz[(L - 1) % 3]; h.row_loss = row_loss; h.da = L >= 2 ? dz[(L - 2) % 3] : nullptr;
        h.d_in = dims[L - 1]; h.C = dims[L]; h.b = b; h.P = P;
        if (L == 1) h.ctr = center_job;
        launch_head(h, s);
    } else {
        EASGD_LAUNCH(softmax_xent_kernel, dim3((rows + 3) / 4), dim3(256), 0, s, logits, y, dz[(L - 1) % 3], row_loss,
                           rows, b, dims[L], pl.splits, (size_t)rows * dims[L]);
    }
    if (loss) EASGD_LAUNCH(mean_loss_kernel, dim3(P), dim3(64), 0, s, row_loss, loss, b);

    // ---- backward propagation ----
    // The weight-gradient product of a layer is held back until the next product is known, because two
    // independent products can share a launch (launch_pair_*): with the input-gradient product of the layer
    // below when the held one is narrow, or with the weight-gradient product of the layer below.
    const int epi = !step ? (G16 ? EPI_STORE_BF16 : EPI_NONE) : (step->V16 ? EPI_ELASTIC_MOM_BF16 : (step->V ? EPI_ELASTIC_MOM : EPI_ELASTIC));
    const bool pairing = options().gemm_pair != 0;
    const bool tile64 = options().gemm_tile == 0 || options().gemm_tile == 2;   // wide backward products use 64x64
    struct Held { bool have = false; GemmArgs a; bool vec = false; } held;
    auto launch_dw = [&](const GemmArgs &d, bool vec) {
        if (epi == EPI_NONE) launch_gemm<MN_CONTIG, MN_CONTIG, EPI_NONE>(d, vec, false, s);
        else if (epi == EPI_STORE_BF16) launch_gemm<MN_CONTIG, MN_CONTIG, EPI_STORE_BF16>(d, vec, false, s);
        else if (epi == EPI_ELASTIC) launch_gemm<MN_CONTIG, MN_CONTIG, EPI_ELASTIC>(d, vec, false, s);
        else if (epi == EPI_ELASTIC_MOM) launch_gemm<MN_CONTIG, MN_CONTIG, EPI_ELASTIC_MOM>(d, vec, false, s);
        else launch_gemm<MN_CONTIG, MN_CONTIG, EPI_ELASTIC_MOM_BF16>(d, vec, false, s);
    };
    auto flush = [&]() {
        if (held.have) launch_dw(held.a, held.vec);
        held.have = false;
    };
    for (int l = L - 1; l >= 0; --l) {
        const int d_in = dims[l], d_out = dims[l + 1];
        const float *dz_l = dz[l % 3];
        if (l > 0 && !(head && l == L - 1)) {   // dZ_{l-1} = (dZ_l W_l^T) where A_l > 0
            GemmArgs a = {};
            a.A = dz_l; a.a_ws = (size_t)b * d_out; a.lda = d_out; a.a_lim = d_out; a.a_ones = -1;
            a.B = W + pl.off[l]; a.b_ws = ld; a.ldb = d_out;
            a.C = dz[(l - 1) % 3]; a.c_ws = (size_t)b * d_in; a.ldc = d_in;
            a.mask = act(l); a.mask_ws = (size_t)b * d_in; a.ldmask = d_in;
            a.M = b; a.N = d_in; a.K = d_out; a.P = P;
            a.splits = 1; a.k_per_split = (a.K + 63) / 64 * 64;
            const bool vec = base_vec && mult4(d_out) && mult4(pl.off[l]);
            // sharing costs the input-gradient blocks some occupancy (the kernel takes the larger register count
            // of its two halves), so it is done only when their launch leaves wave slots idle anyway
            const bool room = (size_t)((a.M + 63) / 64) * ((a.N + 63) / 64) * P <= (size_t)3 * num_cus();
            if (held.have && pairing && held.a.N <= 32 && vec && tile64 && a.N > 32 && room) {
                if (epi == EPI_NONE) {
                    if (held.vec) launch_pair_da_narrow_dw<EPI_NONE, true>(a, held.a, s);
                    else launch_pair_da_narrow_dw<EPI_NONE, false>(a, held.a, s);
                } else if (epi == EPI_STORE_BF16) {
                    if (held.vec) launch_pair_da_narrow_dw<EPI_STORE_BF16, true>(a, held.a, s);
                    else launch_pair_da_narrow_dw<EPI_STORE_BF16, false>(a, held.a, s);
                } else if (epi == EPI_ELASTIC) {
                    if (held.vec) launch_pair_da_narrow_dw<EPI_ELASTIC, true>(a, held.a, s);
                    else launch_pair_da_narrow_dw<EPI_ELASTIC, false>(a, held.a, s);
                } else if (epi == EPI_ELASTIC_MOM) {
                    if (held.vec) launch_pair_da_narrow_dw<EPI_ELASTIC_MOM, true>(a, held.a, s);
                    else launch_pair_da_narrow_dw<EPI_ELASTIC_MOM, false>(a, held.a, s);
                } else {
                    if (held.vec) launch_pair_da_narrow_dw<EPI_ELASTIC_MOM_BF16, true>(a, held.a, s);
                    else launch_pair_da_narrow_dw<EPI_ELASTIC_MOM_BF16, false>(a, held.a, s);
                }
                held.have = false;
            } else {
                flush();
                launch_gemm<K_CONTIG, K_CONTIG, EPI_MASK>(a, vec, false, s);
            }
        }
        // the first kernel that changes W waits for the center rule, which reads W at time t
        if (step && lane && l == L - 1 && hipStreamWaitEvent(s, lane->join, 0) != hipSuccess)
            return fail(EASGD_ELAUNCH, "%s: stream join failed", name);
        // [dW_l ; db_l] = [A_l 1]^T dZ_l, stored at the layer's place in the packed gradient
        GemmArgs d = {};
        d.A = act(l); d.a_ws = (size_t)b * d_in; d.lda = d_in; d.a_lim = d_in; d.a_ones = d_in;
        d.B = dz_l; d.b_ws = (size_t)b * d_out; d.ldb = d_out;
        d.C = G ? G + pl.off[l] : nullptr; d.c_ws = ld; d.ldc = d_out;
        d.C16 = G16 ? G16 + pl.off[l] : nullptr;
        d.M = d_in + 1; d.N = d_out; d.K = b; d.P = P;
        d.splits = 1; d.k_per_split = (d.K + 63) / 64 * 64;
        if (step) {
            d.Wt = step->W + pl.off[l];
            d.Vt = step->V ? step->V + pl.off[l] : nullptr;
            d.Vt16 = step->V16 ? step->V16 + pl.off[l] : nullptr;
            d.center = center_t + pl.off[l];
            d.eta = step->eta; d.rho = step->rho; d.alpha = step->eta * step->rho; d.delta = step->delta;
        }
        const bool vec = mult4(d_in) && mult4(d_out);
        if (held.have) {     // two weight-gradient products in a row (no input-gradient product for layer 0)
            if (pairing && tile64 && held.vec && vec && held.a.N > 32 && d.N > 32) {
                if (epi == EPI_NONE) launch_pair_dw_dw<EPI_NONE>(held.a, d, s);
                else if (epi == EPI_STORE_BF16) launch_pair_dw_dw<EPI_STORE_BF16>(held.a, d, s);
                else if (epi == EPI_ELASTIC) launch_pair_dw_dw<EPI_ELASTIC>(held.a, d, s);
                else if (epi == EPI_ELASTIC_MOM) launch_pair_dw_dw<EPI_ELASTIC_MOM>(held.a, d, s);
                else launch_pair_dw_dw<EPI_ELASTIC_MOM_BF16>(held.a, d, s);
                held.have = false;
                continue;
            }
            flush();
        }
        held.have = true; held.a = d; held.vec = vec;
    }
    flush();
    return check_launch(name);
}

}  // namespace easgd

// One product of forward / backward propagation alone, through the same tile selection and kernels as the gradient.
extern "C" int easgd_layer_product(int kind, int d_in, int d_out, int P, int b, const float *A, const float *Wl, size_t ld,
                                   const float *dZ, float *out, size_t out_ws, int relu, void *stream)
{
    using namespace easgd;
    const char *name = "easgd_layer_product";
    if (kind < 0 || kind > 2 || d_in < 1 || d_out < 1 || P < 1 || b < 1) return fail(EASGD_EINVAL, "%s: bad kind or size", name);
    if (!A || !out || (kind != 1 && !Wl) || (kind != 0 && !dZ)) return fail(EASGD_EINVAL, "%s: NULL pointer", name);
    if (!aligned16(A) || !aligned16(out) || !aligned16(dZ) || !aligned_to(Wl, 4))
        return fail(EASGD_EINVAL, "%s: A, dZ, out must be 16-byte aligned, Wl 4-byte aligned", name);
    const size_t out_need = kind == 0 ? (size_t)b * d_out : kind == 1 ? (size_t)(d_in + 1) * d_out : (size_t)b * d_in;
    if (out_ws < out_need) return fail(EASGD_EINVAL, "%s: out_ws (%zu) below one worker's result (%zu)", name, out_ws, out_need);
    if (kind != 1 && ld < (size_t)(d_in + 1) * d_out) return fail(EASGD_EINVAL, "%s: ld below one layer block", name);
    if ((size_t)(d_in + 1) * d_out > 0x3fffffffull || (size_t)b * d_in > 0x3fffffffull || (size_t)b * d_out > 0x3fffffffull ||
        (size_t)P * b > 0x7fffffffull)
        return fail(EASGD_ERANGE, "%s: an operand exceeds 2^30-1 elements per worker", name);
    clear_error();
    hipStream_t s = static_cast<hipStream_t>(stream);
    GemmArgs a = {};
    a.P = P; a.splits = 1;
    if (kind == 0) {            // Z = [A 1] [W ; b]
        a.A = A; a.a_ws = (size_t)b * d_in; a.lda = d_in; a.a_lim = d_in; a.a_ones = d_in;
        a.B = Wl; a.b_ws = ld; a.ldb = d_out;
        a.C = out; a.c_ws = out_ws; a.ldc = d_out;
        a.M = b; a.N = d_out; a.K = d_in + 1;
        a.k_per_split = (a.K + 63) / 64 * 64;
        const bool vec = mult4(ld) && mult4(d_in) && mult4(d_out) && aligned16(Wl);
        if (relu) launch_gemm<K_CONTIG, MN_CONTIG, EPI_RELU>(a, vec, true, s);
        else launch_gemm<K_CONTIG, MN_CONTIG, EPI_NONE>(a, vec, true, s);
    } else if (kind == 1) {     // [dW ; db] = [A 1]^T dZ
        a.A = A; a.a_ws = (size_t)b * d_in; a.lda = d_in; a.a_lim = d_in; a.a_ones = d_in;
        a.B = dZ; a.b_ws = (size_t)b * d_out; a.ldb = d_out;
        a.C = out; a.c_ws = out_ws; a.ldc = d_out;
        a.M = d_in + 1; a.N = d_out; a.K = b;
        a.k_per_split = (a.K + 63) / 64 * 64;
        launch_gemm<MN_CONTIG, MN_CONTIG, EPI_NONE>(a, mult4(d_in) && mult4(d_out), false, s);
    } else {                    // dA = (dZ W^T) where A > 0
        a.A = dZ; a.a_ws = (size_t)b * d_out; a.lda = d_out; a.a_lim = d_out; a.a_ones = -1;
        a.B = Wl; a.b_ws = ld; a.ldb = d_out;
        a.C = out; a.c_ws = out_ws; a.ldc = d_in;
        a.mask = A; a.mask_ws = (size_t)b * d_in; a.ldmask = d_in;
        a.M = b; a.N = d_in; a.K = d_out;
        a.k_per_split = (a.K + 63) / 64 * 64;
        launch_gemm<K_CONTIG, K_CONTIG, EPI_MASK>(a, mult4(ld) && mult4(d_out) && aligned16(Wl), false, s);
    }
    return check_launch(name);
}
