// Batched fp32 GEMM on the CDNA matrix cores (v_mfma_f32_32x32x2_f32, or
// v_mfma_f32_16x16x4_f32 where a ragged batch would waste rows of a 32-row tile) for the
// forward / backward passes of the per-worker dense models (Section 5.1 step (1),
// Section 2.2).  One launch covers all P workers: every worker multiplies its
// own operands, so the worker index is one more block coordinate.
//
//   C[w][m][n] = epilogue( sum_k A[w](m,k) * B[w](k,n) )
//
// Operand storage is described per operand:
//   K_CONTIG   element (x,k) at ptr[x*ld + k]      (row-major M x K, or N x K)
//   MN_CONTIG  element (x,k) at ptr[k*ld + x]      (row-major K x M, or K x N)
// A may be augmented by a vector of ones at index a_ones along its contiguous
// axis.  With the packed layout "weight matrix, then bias" this turns the bias
// add of the forward pass and the bias gradient of the backward pass into one
// more row of the same matrix product.
//
// Tiling: a block of WAVES_M x WAVES_N wavefronts owns a BM x BN tile of C; each
// wavefront owns (BM/WAVES_M) x (BN/WAVES_N) of it as 32x32 (MT = 32) or 16x16 (MT = 16) MFMA accumulators.
// K is walked in slabs of BK with a prefetch distance of two slabs: global ->
// registers (two stages) -> LDS (two buffers) -> MFMA operands.
// LDS holds both operands k-major ([k][m] and [k][n], padded row pitch) so an
// MFMA operand fetch is one conflict-free ds_read_b32 per lane.
#pragma once
#include "common.h"
#include <type_traits>
#include "elastic_rule.h"

namespace easgd {

enum { K_CONTIG = 0, MN_CONTIG = 1 };
// EPI_ELASTIC / EPI_ELASTIC_MOM: the product is a gradient tile g; the epilogue applies the worker rule
// Eq. (1) / Eq. (5),(6) to the matching tile of the replica (and momentum buffer) in place, with the
// time-t center read from `center`; g itself is stored only when C is not null.
// EPI_STORE_BF16: the product is narrowed to bfloat16 (round to nearest even) and stored at C16 instead of C.
enum { EPI_NONE = 0, EPI_RELU = 1, EPI_MASK = 2, EPI_ELASTIC = 3, EPI_ELASTIC_MOM = 4, EPI_ELASTIC_MOM_BF16 = 5,
       EPI_STORE_BF16 = 6 };

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct GemmArgs {
    const float *A, *B, *mask;
    float *C;
    unsigned short *C16;                // EPI_STORE_BF16: the result as bfloat16, indexed like C
    size_t a_ws, b_ws, c_ws, mask_ws;   // worker strides (elements)
    size_t c_ss;                        // split stride of C (elements); split s writes C + s*c_ss
    int lda, ldb, ldc, ldmask;
    int M, N, K;
    int a_lim;                          // number of stored elements of A along its contiguous axis
    int a_ones;                         // index along that axis that reads as 1.0f, or -1
    int k_per_split;                    // multiple of BK; splits = ceil(K / k_per_split)
    int splits;
    int tiles_m, tiles_n;
    int P;
    int xcd_chunk;                      // 0 = plain block order; else grid/8 (see the kernel)
    int die_workers;                    // > 0 (needs xcd_chunk > 0, splits == 1, P == 8 * die_workers): a die walks its
                                        // workers' tiles tile by tile, the workers of a tile next to each other
    int band_log2;                      // > 0 (needs die_workers > 0, tiles_n a multiple of 2^band_log2): that walk goes
                                        // through C in bands of 2^band_log2 tile columns, down each band row by row
    int band_tiles;                     // tiles_m << band_log2
    // ceil(2^32 / d) for the divisors of the block -> tile mapping (tiles per worker, tiles_n, die_workers, band_tiles),
    // or 0 where the host could not guarantee that the product form is exact (then the kernel divides)
    unsigned magic_tiles, magic_tiles_n, magic_die, magic_band;
    // elastic epilogues: replica / momentum tiles indexed like C (worker stride c_ws, row stride ldc);
    // the center has the row stride ldc and no worker stride
    float *Wt, *Vt;
    unsigned short *Vt16;               // EPI_ELASTIC_MOM_BF16: the momentum tiles stored as bfloat16
    const float *center;
    float eta, rho, alpha, delta;
    // extra blocks at the end of the grid that run the center rule beside the product (bandwidth-bound
    // work in the shadow of matrix-core-bound work, without a second stream); ctr.blocks == 0: none
    CenterJob ctr;
};

// n / d for 0 <= n, d >= 1, with magic = ceil(2^32 / d) when n * d < 2^32 (then the high half of n * magic is the
// quotient), magic = 0 otherwise.  A 32-bit division costs some thirty instructions of which most go through the
// vector unit, where they queue behind the MFMAs of the other wavefronts of the SIMD; every block of a short product
// pays for three of them before it can issue its first load.
__device__ __forceinline__ int fast_div(int n, int d, unsigned magic)
{
    if (d == 1) return n;
    if (magic == 0) return n / d;
    return (int)__umulhi((unsigned)n, magic);
}

// Four elements idx0..idx0+3 along the contiguous axis of a row that starts at `row`.
// Elements at or beyond `lim` read as 0, except index `ones` which reads as 1.
template <bool VEC>
__device__ __forceinline__ f32x4 fetch4(const float *row, int idx0, int lim, int ones, bool row_valid)
{
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (!row_valid) return v;
    if (VEC && idx0 + 3 < lim) return *reinterpret_cast<const f32x4 *>(row + idx0);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int idx = idx0 + q;
        if (idx < lim) v[q] = row[idx];
        else if (idx == ones) v[q] = 1.0f;
    }
    return v;
}

// LDS floats of one block of a tile configuration (both operands, two buffers each).
template <int BM, int BN, int BK, int A_LAYOUT, int B_LAYOUT>
constexpr int gemm_lds_floats()
{
    constexpr int PAD_K = (BK == 32) ? 1 : 2;
    constexpr int PITCH_A = BM + (A_LAYOUT == K_CONTIG ? PAD_K : 4), PITCH_B = BN + (B_LAYOUT == K_CONTIG ? PAD_K : 4);
    return 2 * BK * PITCH_A + 2 * BK * PITCH_B;
}

// The work of block `bid` of one product.  `lds` is the calling kernel's buffer of at least
// gemm_lds_floats<...>() floats, 16-byte aligned: kernels that carry two products lend the same buffer to both.
template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, int A_LAYOUT, int B_LAYOUT, bool VEC, int EPI, int MT = 32, bool ALONE = false>
__device__ __forceinline__ void gemm_block(const GemmArgs &p, const unsigned bid, float *__restrict__ lds)
{
    constexpr int NTHREADS = WAVES_M * WAVES_N * 64;
    constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
    constexpr int TM = WTM / MT, TN = WTN / MT;
    static_assert(MT == 32 || MT == 16, "MFMA tile");
    // LDS row pitch: +4 keeps 128-bit row stores aligned for operands that arrive m/n-contiguous; operands that
    // arrive k-contiguous are scattered as scalars (lane -> k quad fastest), which is conflict-free when
    // 4*pitch = 32/(BK/4) mod 32, i.e. pitch = 1 mod 8 for BK = 32 and pitch = 2 mod 8 for BK = 16
    constexpr int PAD_K = (BK == 32) ? 1 : 2;
    constexpr int PITCH_A = BM + (A_LAYOUT == K_CONTIG ? PAD_K : 4), PITCH_B = BN + (B_LAYOUT == K_CONTIG ? PAD_K : 4);
    static_assert(BK == 16 || BK == 32, "slab depth");
    static_assert(BM % 8 == 0 && BN % 8 == 0, "tile shape");
    constexpr int CHUNKS_A = BM * BK / 4, CHUNKS_B = BN * BK / 4;
    constexpr int IT_A = (CHUNKS_A + NTHREADS - 1) / NTHREADS, IT_B = (CHUNKS_B + NTHREADS - 1) / NTHREADS;
    static_assert(WTM % MT == 0 && WTN % MT == 0 && BK % 4 == 0, "tile shape");

    float (*As)[BK * PITCH_A] = reinterpret_cast<float (*)[BK * PITCH_A]>(lds);
    float (*Bs)[BK * PITCH_B] = reinterpret_cast<float (*)[BK * PITCH_B]>(lds + 2 * BK * PITCH_A);
    static_assert((2 * BK * PITCH_A) % 4 == 0, "B tiles must stay 16-byte aligned");

    // block -> (worker, split, tile_m, tile_n)
    // Workgroups go to the eight accelerator dies (XCDs, each with its own L2) in turn, by block index.
    // With xcd_chunk > 0 the grid is a multiple of 8 and block b works on the logical index
    // (b % 8) * xcd_chunk + b / 8: each die then owns a run of consecutive tiles, i.e. whole workers,
    // so that an operand panel shared by the tiles of a worker is fetched into one L2 only.
    const int tiles = p.tiles_m * p.tiles_n;
    int id = (int)bid;
    if (p.xcd_chunk > 0) {
        id = (id & 7) * p.xcd_chunk + (id >> 3);
        if (id >= tiles * p.splits * p.P) return;
    }
    int tile, split, w;
    if (p.die_workers > 0) {
        // Elastic epilogues read the time-t center tile, which all workers share: with the tiles of a die's workers
        // interleaved, the die fetches each center tile once instead of once per worker.
        const int q = (int)(bid >> 3);
        tile = fast_div(q, p.die_workers, p.magic_die);
        split = 0;
        w = (int)(bid & 7) * p.die_workers + (q - tile * p.die_workers);
    } else {
        const int rest = fast_div(id, tiles, p.magic_tiles);
        tile = id - rest * tiles;
        if (p.splits == 1) {
            split = 0;
            w = rest;
        } else {
            split = rest % p.splits;
            w = rest / p.splits;
        }
    }
    int tile_m, tile_n;
    if (p.band_log2 > 0) {
        // The blocks a die runs at the same time are a few dozen consecutive tiles of each of its workers.  In
        // row-major tile order those are one row of tiles: one panel of A and every panel of B, so B is swept
        // again for each row of tiles, and what streams through the L2 in between (the replica and momentum
        // tiles of the epilogue) has evicted it by then.  Walking bands of 2^band_log2 tile columns row by row
        // makes the concurrent tiles a near-square patch that shares a few panels of each operand.
        const int band = fast_div(tile, p.band_tiles, p.magic_band);
        const int rem = tile - band * p.band_tiles;
        tile_m = rem >> p.band_log2;
        tile_n = (band << p.band_log2) + (rem & ((1 << p.band_log2) - 1));
    } else {
        tile_m = fast_div(tile, p.tiles_n, p.magic_tiles_n);
        tile_n = tile - tile_m * p.tiles_n;
    }
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int k_begin = split * p.k_per_split;
    const int k_end = min(p.K, k_begin + p.k_per_split);

    const float *__restrict__ A = p.A + (size_t)w * p.a_ws;
    const float *__restrict__ B = p.B + (size_t)w * p.b_ws;
    const int b_lim = (B_LAYOUT == MN_CONTIG) ? p.N : p.K;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / WAVES_N) * WTM, wn0 = (wave % WAVES_N) * WTN;

    // ---- per-thread loader geometry (constant over the K loop) ----
    // chunk c = tid + it*NTHREADS is four consecutive elements along the operand's contiguous axis
    const float *a_src[IT_A], *b_src[IT_B];   // source of the chunk in the slab that starts at k = 0
    int a_dst[IT_A], b_dst[IT_B];             // LDS offset of the chunk's first element
    bool a_ok[IT_A], b_ok[IT_B];              // false: the chunk lies outside the stored matrix (its address was
                                              // clamped); zeros are stored instead, or 1 where the ones vector sits
    int a_krel[IT_A], b_krel[IT_B];           // k of the chunk's first element relative to the slab start
#pragma unroll
    for (int it = 0; it < IT_A; ++it) {
        const int c = tid + it * NTHREADS;
        if (A_LAYOUT == K_CONTIG) {
            const int kq = c % (BK / 4), m = c / (BK / 4);
            a_ok[it] = (m0 + m < p.M);
            a_src[it] = A + (size_t)min(m0 + m, p.M - 1) * p.lda + 4 * kq;
            a_dst[it] = 4 * kq * PITCH_A + m;
            a_krel[it] = 4 * kq;
        } else {
            // with 128-bit loads a_lim is a multiple of 4, so a chunk is entirely inside or entirely outside
            const int mq = c % (BM / 4), k = c / (BM / 4), m = m0 + 4 * mq;
            a_ok[it] = (m + 3 < p.a_lim);
            a_src[it] = A + (size_t)k * p.lda + (a_ok[it] ? m : 0);
            a_dst[it] = k * PITCH_A + 4 * mq;
            a_krel[it] = k;
        }
    }
#pragma unroll
    for (int it = 0; it < IT_B; ++it) {
        const int c = tid + it * NTHREADS;
        if (B_LAYOUT == K_CONTIG) {
            const int kq = c % (BK / 4), n = c / (BK / 4);
            b_ok[it] = (n0 + n < p.N);
            b_src[it] = B + (size_t)min(n0 + n, p.N - 1) * p.ldb + 4 * kq;
            b_dst[it] = 4 * kq * PITCH_B + n;
            b_krel[it] = 4 * kq;
        } else {
            const int nq = c % (BN / 4), k = c / (BN / 4), n = n0 + 4 * nq;
            b_ok[it] = (n + 3 < b_lim);
            b_src[it] = B + (size_t)k * p.ldb + (b_ok[it] ? n : 0);
            b_dst[it] = k * PITCH_B + 4 * nq;
            b_krel[it] = k;
        }
    }
    const size_t a_kstep = (A_LAYOUT == K_CONTIG) ? 1 : (size_t)p.lda;   // address step per unit of k
    const size_t b_kstep = (B_LAYOUT == K_CONTIG) ? 1 : (size_t)p.ldb;

    // Interior slabs: plain 128-bit loads, no lane diverges (chunks outside the matrix were clamped above).
    auto load_fast = [&](int k0, f32x4 (&ra)[IT_A], f32x4 (&rb)[IT_B]) {
#pragma unroll
        for (int it = 0; it < IT_A; ++it)
            if (CHUNKS_A % NTHREADS == 0 || tid + it * NTHREADS < CHUNKS_A)
                ra[it] = *reinterpret_cast<const f32x4 *>(a_src[it] + (size_t)k0 * a_kstep);
#pragma unroll
        for (int it = 0; it < IT_B; ++it)
            if (CHUNKS_B % NTHREADS == 0 || tid + it * NTHREADS < CHUNKS_B)
                rb[it] = *reinterpret_cast<const f32x4 *>(b_src[it] + (size_t)k0 * b_kstep);
    };
    // The last slab of the K range when it is only partly inside the operands (128-bit path): a chunk is
    // either entirely inside or entirely outside along k (all limits are multiples of 4), so chunks outside
    // are loaded from a clamped, valid address and replaced when they are stored to LDS: by zeros, or by
    // the 1 of the ones vector.
    const int a_klim = min(p.a_lim, k_end);   // K_CONTIG A: elements at k >= a_klim are not stored
    const int b_klim = min(b_lim, k_end);
    bool ta_ok[IT_A], tb_ok[IT_B];
    auto load_tail = [&](int k0, f32x4 (&ra)[IT_A], f32x4 (&rb)[IT_B]) {
#pragma unroll
        for (int it = 0; it < IT_A; ++it) {
            if (CHUNKS_A % NTHREADS != 0 && tid + it * NTHREADS >= CHUNKS_A) continue;
            ta_ok[it] = (A_LAYOUT == K_CONTIG) ? (k0 + a_krel[it] + 3 < a_klim) : (k0 + a_krel[it] < k_end);
            const int k_eff = ta_ok[it] ? k0 : ((A_LAYOUT == K_CONTIG) ? -a_krel[it] : k0 - a_krel[it]);
            ra[it] = *reinterpret_cast<const f32x4 *>(a_src[it] + (ptrdiff_t)k_eff * (ptrdiff_t)a_kstep);
        }
#pragma unroll
        for (int it = 0; it < IT_B; ++it) {
            if (CHUNKS_B % NTHREADS != 0 && tid + it * NTHREADS >= CHUNKS_B) continue;
            tb_ok[it] = (B_LAYOUT == K_CONTIG) ? (k0 + b_krel[it] + 3 < b_klim) : (k0 + b_krel[it] < k_end);
            const int k_eff = tb_ok[it] ? k0 : ((B_LAYOUT == K_CONTIG) ? -b_krel[it] : k0 - b_krel[it]);
            rb[it] = *reinterpret_cast<const f32x4 *>(b_src[it] + (ptrdiff_t)k_eff * (ptrdiff_t)b_kstep);
        }
    };
    // replaces the chunks of the tail slab that lie outside along k (called on the registers before store_lds)
    auto fix_tail = [&](int k0, f32x4 (&ra)[IT_A], f32x4 (&rb)[IT_B]) {
#pragma unroll
        for (int it = 0; it < IT_A; ++it) {
            if (CHUNKS_A % NTHREADS != 0 && tid + it * NTHREADS >= CHUNKS_A) continue;
            if (!ta_ok[it]) {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    ra[it][q] = (A_LAYOUT == K_CONTIG && k0 + a_krel[it] + q == p.a_ones && p.a_ones < k_end) ? 1.f : 0.f;
            }
        }
#pragma unroll
        for (int it = 0; it < IT_B; ++it) {
            if (CHUNKS_B % NTHREADS != 0 && tid + it * NTHREADS >= CHUNKS_B) continue;
            if (!tb_ok[it]) rb[it] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    };
    // Edge slabs and edge tiles: every element guarded (zero fill, ones vector).
    auto load_guarded = [&](int k0, f32x4 (&ra)[IT_A], f32x4 (&rb)[IT_B]) {
#pragma unroll
        for (int it = 0; it < IT_A; ++it) {
            const int c = tid + it * NTHREADS;
            if (CHUNKS_A % NTHREADS != 0 && c >= CHUNKS_A) continue;
            if (A_LAYOUT == K_CONTIG) {
                const int kq = c % (BK / 4), m = m0 + c / (BK / 4);
                ra[it] = fetch4<VEC>(A + (size_t)m * p.lda, k0 + 4 * kq, min(p.a_lim, k_end), p.a_ones < k_end ? p.a_ones : -1, m < p.M);
            } else {
                const int mq = c % (BM / 4), k = k0 + c / (BM / 4);
                ra[it] = fetch4<VEC>(A + (size_t)k * p.lda, m0 + 4 * mq, p.a_lim, p.a_ones, k < k_end);
            }
        }
#pragma unroll
        for (int it = 0; it < IT_B; ++it) {
            const int c = tid + it * NTHREADS;
            if (CHUNKS_B % NTHREADS != 0 && c >= CHUNKS_B) continue;
            if (B_LAYOUT == K_CONTIG) {
                const int kq = c % (BK / 4), n = n0 + c / (BK / 4);
                rb[it] = fetch4<VEC>(B + (size_t)n * p.ldb, k0 + 4 * kq, min(b_lim, k_end), -1, n < p.N);
            } else {
                const int nq = c % (BN / 4), k = k0 + c / (BN / 4);
                rb[it] = fetch4<VEC>(B + (size_t)k * p.ldb, n0 + 4 * nq, b_lim, -1, k < k_end);
            }
        }
    };

    auto store_lds = [&](int buf, const f32x4 (&ra)[IT_A], const f32x4 (&rb)[IT_B], bool clamped) {
#pragma unroll
        for (int it = 0; it < IT_A; ++it) {
            if (CHUNKS_A % NTHREADS != 0 && tid + it * NTHREADS >= CHUNKS_A) continue;
            f32x4 v = ra[it];
            if (A_LAYOUT == K_CONTIG) {
                if (clamped && !a_ok[it]) v = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int q = 0; q < 4; ++q) As[buf][a_dst[it] + q * PITCH_A] = v[q];
            } else {
                if (clamped && !a_ok[it]) {
                    // only the one tile that holds the ones vector comes here: its position is worked out on the spot
                    const int m_chunk = m0 + 4 * ((tid + it * NTHREADS) % (BM / 4));
#pragma unroll
                    for (int q = 0; q < 4; ++q) v[q] = (m_chunk + q == p.a_ones) ? 1.f : 0.f;
                }
                *reinterpret_cast<f32x4 *>(&As[buf][a_dst[it]]) = v;
            }
        }
#pragma unroll
        for (int it = 0; it < IT_B; ++it) {
            if (CHUNKS_B % NTHREADS != 0 && tid + it * NTHREADS >= CHUNKS_B) continue;
            f32x4 v = rb[it];
            if (B_LAYOUT == K_CONTIG) {
                if (clamped && !b_ok[it]) v = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int q = 0; q < 4; ++q) Bs[buf][b_dst[it] + q * PITCH_B] = v[q];
            } else {
                if (clamped && !b_ok[it]) v = f32x4{0.f, 0.f, 0.f, 0.f};
                *reinterpret_cast<f32x4 *>(&Bs[buf][b_dst[it]]) = v;
            }
        }
    };

    constexpr int ACC_REGS = MT * MT / 64;
    typedef float acc_t __attribute__((ext_vector_type(ACC_REGS)));
    acc_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < ACC_REGS; ++r) acc[i][j][r] = 0.f;

    // MFMA operand fetch.  32x32x2: lane l supplies A[m = l%32][k = l/32] and B[k = l/32][n = l%32] of a k pair.
    // 16x16x4: lane l supplies A[m = l%16] and B[n = l%16] at the k of its slot l/16.  Which k of the slab the
    // four slots of one MFMA take is free as long as both operands agree; here MFMA j of a slab takes
    // k = j, j + BK/4, j + BK/2, j + 3BK/4, with slots 0 and 1 (the lanes whose LDS reads are served together)
    // BK/2 rows apart: for an operand that arrived k-contiguous (row pitch 1 mod 8 at BK = 32, 2 mod 8 at
    // BK = 16) those two rows start 16 banks apart, so its reads do not collide.
    constexpr int KSTEP = (MT == 32) ? 2 : 4;           // k consumed per MFMA
    const int frag_k = (MT == 32) ? (lane >> 5) : (BK / 2) * ((lane >> 4) & 1) + (BK / 4) * (lane >> 5);
    const int frag_x = lane & (MT - 1);
    // multiply the slab held in LDS buffer `buf`; k_left = number of valid k in it
    // `mid` runs after half of the full slab's MFMAs have been issued (used to move the next slab registers -> LDS
    // while the matrix pipeline is busy)
    auto multiply_slab = [&](int buf, int k_left, auto &&mid) {
        const float *as = &As[buf][frag_k * PITCH_A + wm0 + frag_x];
        const float *bs = &Bs[buf][frag_k * PITCH_B + wn0 + frag_x];
        // step st: k pair 2*st of the slab (32x32x2), or rows st, st + BK/4, ... (16x16x4)
        auto fetch = [&](int st, float (&a)[TM], float (&b)[TN]) {
            const int kk = (MT == 32) ? 2 * st : st;
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = as[kk * PITCH_A + i * MT];
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = bs[kk * PITCH_B + j * MT];
        };
        auto multiply = [&](const float (&a)[TM], const float (&b)[TN]) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    if constexpr (MT == 32) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
                    else acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[i], b[j], acc[i][j], 0, 0, 0);
                }
        };
        constexpr int STEPS = BK / KSTEP;
        if (k_left >= BK) {
            // operands are fetched from LDS DIST steps ahead of the MFMAs that use them, so the LDS
            // latency hides behind the matrix pipeline (one step ahead = 4 MFMAs when a wave owns 2x2
            // tiles; two steps ahead when it owns a single tile)
            constexpr int DIST = (TM * TN == 1) ? 2 : 1;
            float a[DIST + 1][TM], b[DIST + 1][TN];
#pragma unroll
            for (int d = 0; d < DIST; ++d) fetch(d, a[d], b[d]);
#pragma unroll
            for (int st = 0; st < STEPS; ++st) {
                if (st + DIST < STEPS) fetch(st + DIST, a[(st + DIST) % (DIST + 1)], b[(st + DIST) % (DIST + 1)]);
                __builtin_amdgcn_sched_barrier(0);      // keep the LDS reads ahead of the MFMAs below
                multiply(a[st % (DIST + 1)], b[st % (DIST + 1)]);
                __builtin_amdgcn_sched_barrier(0);
                if (st == STEPS / 2 - 1) {
                    mid();
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        } else {
            // short slab: stop at the last step that holds data (the rest of the slab is zero); with 16x16x4
            // step st holds k = st and three rows further down, so the steps below k_left are the ones to take
            const int n_steps = (MT == 32) ? (k_left + 1) / 2 : min(k_left, STEPS);
            for (int st = 0; st < n_steps; ++st) {
                float a[TM], b[TN];
                fetch(st, a, b);
                multiply(a, b);
            }
            mid();
        }
    };
    auto nothing = [] {};

    // All slabs of a block go through the 128-bit pipeline when the operands allow 128-bit loads; the
    // last slab may be partial (n_full counts the slabs that lie fully inside both operands along k).
    const int n_slabs = (k_end - k_begin + BK - 1) / BK;
    int n_full = 0, n_pipe = 0;
    {
        // 128-bit loads need the limits along the contiguous axes to be multiples of 4 (the host only sets VEC then)
        const bool vec_ok = VEC && (p.a_lim & 3) == 0 && (b_lim & 3) == 0 &&
                            (A_LAYOUT != K_CONTIG || (a_klim & 3) == 0) && (B_LAYOUT != K_CONTIG || (b_klim & 3) == 0);
        int k_lim = k_end;
        if (A_LAYOUT == K_CONTIG) k_lim = min(k_lim, a_klim);
        if (B_LAYOUT == K_CONTIG) k_lim = min(k_lim, b_klim);
        if (vec_ok) {
            n_pipe = n_slabs;
            n_full = k_lim > k_begin ? (k_lim - k_begin) / BK : 0;
        }
    }
    auto load_slab = [&](int s, f32x4 (&ra)[IT_A], f32x4 (&rb)[IT_B]) {
        if (s < n_full) load_fast(k_begin + s * BK, ra, rb);
        else load_tail(k_begin + s * BK, ra, rb);
    };
    // Most tiles have nothing to replace on the way to LDS; the replacement is one select per element and slab on
    // the vector unit, which the MFMAs of the SIMD then wait for.
    // Rows of A beyond M and columns of B beyond N only reach elements of C that are never stored, so whatever the
    // clamped loads brought for them may stay; the one thing that has to be replaced is the ones vector, which
    // sits in the tile of an m/n-contiguous A that holds row a_ones.
    const bool inner_tile = !(A_LAYOUT == MN_CONTIG && p.a_ones >= m0 && p.a_ones < m0 + BM);      // uniform
    auto store_full = [&](int buf, f32x4 (&ra)[IT_A], f32x4 (&rb)[IT_B]) {      // a slab fully inside along k
        if (inner_tile) store_lds(buf, ra, rb, false);
        else store_lds(buf, ra, rb, true);
    };
    auto store_slab = [&](int buf, int s, f32x4 (&ra)[IT_A], f32x4 (&rb)[IT_B]) {
        if (s >= n_full) fix_tail(k_begin + s * BK, ra, rb);
        store_full(buf, ra, rb);
    };
    auto k_in_slab = [&](int s) { return min(BK, k_end - (k_begin + s * BK)); };

    // Two register stages R0/R1 and two LDS buffers: slab s sits in stage s%2 while in flight and in LDS
    // buffer s%2 while it is multiplied.  In the steady state the loads of slab s+2 are issued, slab s is
    // multiplied and, half way through its MFMAs, slab s+1 moves registers -> LDS: a prefetch distance of two slabs,
    // one barrier per slab.
    f32x4 ra0[IT_A], rb0[IT_B], ra1[IT_A], rb1[IT_B];
    int s_done = 0;
    // The narrow tile with the worker rule in its epilogue (the weight gradient of a last layer of a few classes; a
    // softmax regression has nothing else) is a chain of round trips to memory on a chip that is otherwise idle:
    // operands, then the replica, center and momentum tiles.  Its epilogue's tiles are requested here, before the
    // operands, so that the two trips become one.  (The wide tiles do not do this: their launches fill the chip, and
    // requests made this early only queue ahead of the operand loads of the blocks that share the compute unit; nor
    // does a narrow product that shares its launch with a wide one, ALONE = false: the registers would cost the wide
    // product a block per compute unit.)
    constexpr bool ELASTIC_EPI = (EPI == EPI_ELASTIC || EPI == EPI_ELASTIC_MOM || EPI == EPI_ELASTIC_MOM_BF16);
    constexpr bool EARLY_TILES = ALONE && ELASTIC_EPI && BN == 32 && TM == 1 && TN == 1 && MT == 32;
    float pre_w[EARLY_TILES ? 16 : 1], pre_c[EARLY_TILES ? 16 : 1], pre_v[EARLY_TILES ? 16 : 1];
    unsigned pre_v16[EARLY_TILES ? 16 : 1];     // one 32-bit register per code: loads into the halves of a shared register
                                                // would each wait for the other
    if constexpr (EARLY_TILES) {
        const int n = n0 + wn0 + (lane & 31);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            // unconditional loads: a lane whose element lies outside C reads the last row or column instead
            const int m = min(m0 + wm0 + 8 * (r / 4) + 4 * (lane >> 5) + (r % 4), p.M - 1);
            const size_t at = (size_t)m * p.ldc + min(n, p.N - 1);
            pre_w[r] = (p.Wt + (size_t)w * p.c_ws)[at];
            pre_c[r] = p.center[at];
            pre_v[r] = (EPI == EPI_ELASTIC_MOM) ? (p.Vt + (size_t)w * p.c_ws)[at] : 0.f;
            pre_v16[r] = (EPI == EPI_ELASTIC_MOM_BF16) ? (unsigned)(p.Vt16 + (size_t)w * p.c_ws)[at] : 0u;
        }
    }
    if (n_pipe >= 2) {
        load_slab(0, ra0, rb0);
        load_slab(1, ra1, rb1);
        store_slab(0, 0, ra0, rb0);
        __syncthreads();
        int s = 0;
        // The steady state proper: every slab it loads or stores lies fully inside the operands, so it contains
        // nothing of the partial-slab handling (which the compiler otherwise folds into the loop as selects and
        // per-lane address arithmetic on every slab; the vector unit is what the MFMAs wait for).
        // (one copy of the loop per kind of tile, so that the kind is not a branch, and a register merge, per slab)
        auto steady = [&](auto clamp) {
            for (; s + 3 < n_full; s += 2) {
                load_fast(k_begin + (s + 2) * BK, ra0, rb0);
                multiply_slab(0, BK, [&] { store_lds(1, ra1, rb1, decltype(clamp)::value); });
                __syncthreads();
                load_fast(k_begin + (s + 3) * BK, ra1, rb1);
                multiply_slab(1, BK, [&] { store_lds(0, ra0, rb0, decltype(clamp)::value); });
                __syncthreads();
            }
        };
        if (inner_tile) steady(std::false_type{});
        else steady(std::true_type{});
        // the same with the partial last slab allowed (at most one more trip)
        for (; s + 3 < n_pipe; s += 2) {
            load_slab(s + 2, ra0, rb0);
            multiply_slab(0, BK, [&] { store_slab(1, s + 1, ra1, rb1); });
            __syncthreads();
            load_slab(s + 3, ra1, rb1);
            multiply_slab(1, BK, [&] { store_slab(0, s + 2, ra0, rb0); });
            __syncthreads();
        }
        // two or three slabs are left: s (in LDS 0), s+1 (in R1), and s+2 if n_pipe is odd
        const bool three = (s + 2 < n_pipe);
        if (three) load_slab(s + 2, ra0, rb0);
        multiply_slab(0, BK, [&] { store_slab(1, s + 1, ra1, rb1); });
        __syncthreads();
        if (three) {
            multiply_slab(1, BK, [&] { store_slab(0, s + 2, ra0, rb0); });
            __syncthreads();
            multiply_slab(0, k_in_slab(s + 2), nothing);
        } else {
            multiply_slab(1, k_in_slab(s + 1), nothing);
        }
        __syncthreads();
        s_done = n_pipe;
    }
    // Otherwise (operands that do not allow 128-bit loads, or a single slab).  Kernels built for such operands take
    // two slabs per trip, both requested before the first is waited for, so that a short product (K = the minibatch:
    // two to four slabs) pays one round trip to memory per pair of slabs instead of one per slab.  The kernels of the
    // 128-bit path only come here with a single slab, and keep the plain loop: the second register stage in this
    // path costs them registers that the center rule's wavefronts need to run beside them (cfg3's forward launch:
    // 228 -> 246 registers, the round 2.37 -> 2.51 ms).
    if constexpr (!VEC) {
        for (int s = s_done; s < n_slabs; s += 2) {
            const int k0 = k_begin + s * BK;
            const bool two = s + 1 < n_slabs;                 // uniform; slab s is then a full one
            load_guarded(k0, ra0, rb0);
            if (two) load_guarded(k0 + BK, ra1, rb1);
            store_lds(0, ra0, rb0, false);
            __syncthreads();
            if (two) {
                multiply_slab(0, BK, [&] { store_lds(1, ra1, rb1, false); });
                __syncthreads();
                multiply_slab(1, k_end - (k0 + BK), nothing);
            } else {
                multiply_slab(0, k_end - k0, nothing);
            }
            __syncthreads();
        }
    } else {
        for (int s = s_done; s < n_slabs; ++s) {
            const int k0 = k_begin + s * BK;
            load_guarded(k0, ra0, rb0);
            store_lds(0, ra0, rb0, false);
            __syncthreads();
            multiply_slab(0, k_end - k0, nothing);
            __syncthreads();
        }
    }

    // epilogue: accumulator register r of lane l is C[8*(r/4) + 4*(l/32) + r%4][l%32] of its 32x32 tile.
    // Addresses are split into a block-uniform row pointer (scalar arithmetic) and one 32-bit lane offset
    // that is computed once; tiles that lie fully inside C skip the per-element bounds checks.
    constexpr bool ELASTIC = ELASTIC_EPI;
    constexpr bool MOM = (EPI == EPI_ELASTIC_MOM);
    constexpr bool MOM16 = (EPI == EPI_ELASTIC_MOM_BF16);
    constexpr bool OUT16 = (EPI == EPI_STORE_BF16);
    const bool keep = !OUT16 && (!ELASTIC || p.C != nullptr);                         // uniform
    float *__restrict__ C = keep ? p.C + (size_t)w * p.c_ws + (size_t)split * p.c_ss : nullptr;
    unsigned short *__restrict__ C16 = OUT16 ? p.C16 + (size_t)w * p.c_ws + (size_t)split * p.c_ss : nullptr;
    const float *__restrict__ mask = (EPI == EPI_MASK) ? p.mask + (size_t)w * p.mask_ws : nullptr;
    float *__restrict__ Wr = ELASTIC ? p.Wt + (size_t)w * p.c_ws : nullptr;
    float *__restrict__ Vr = MOM ? p.Vt + (size_t)w * p.c_ws : nullptr;
    unsigned short *__restrict__ Vr16 = MOM16 ? p.Vt16 + (size_t)w * p.c_ws : nullptr;
    const float *__restrict__ Cc = ELASTIC ? p.center : nullptr;
    const int wave_m = __builtin_amdgcn_readfirstlane(m0 + wm0), wave_n = __builtin_amdgcn_readfirstlane(n0 + wn0);
    const int frag_r = 4 * (lane / MT);     // first row of the lane's accumulator registers inside an MFMA tile
    const unsigned lane_c = (unsigned)frag_r * (unsigned)p.ldc + (unsigned)frag_x;
    const unsigned lane_mask = (unsigned)frag_r * (unsigned)p.ldmask + (unsigned)frag_x;
    if constexpr (MT == 16) {
        // 16x16 accumulators: register r of lane l is C[4*(l/16) + r][l%16] of its tile.  The block tile is as
        // tall as the ragged batch rounded up to 16 rows, so the last rows of tiles are the common case here, not
        // an edge: a row of tiles that lies inside C (block-uniform test) stores without bounds checks, the one
        // that straddles the last row of C checks rows only.
        static_assert(!ELASTIC && !OUT16, "the 16x16 tiles serve the forward and input-gradient products");
        const bool cols_inside = (n0 + BN <= p.N);                                    // uniform
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int mt = wave_m + i * 16;                                           // uniform
            if (mt >= p.M) break;
            const bool inside = cols_inside && mt + 16 <= p.M;
            // all mask values of the row of tiles in flight together: none of the loads is conditional (a lane whose
            // element lies outside C reads the last row or column instead, and stores nothing)
            float gate[TN][4];
            if (EPI == EPI_MASK) {
                if (inside) {
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int r = 0; r < 4; ++r) gate[j][r] = (mask + (size_t)(mt + r) * p.ldmask + wave_n + j * 16)[lane_mask];
                } else {
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const int m = min(mt + frag_r + r, p.M - 1), n = min(wave_n + j * 16 + frag_x, p.N - 1);
                            gate[j][r] = mask[(size_t)m * p.ldmask + n];
                        }
                }
            }
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float v = acc[i][j][r];
                    if (EPI == EPI_RELU) v = fmaxf(v, 0.f);
                    if (EPI == EPI_MASK) v = (gate[j][r] > 0.f) ? v : 0.f;
                    if (inside || (mt + frag_r + r < p.M && wave_n + j * 16 + frag_x < p.N))
                        (C + (size_t)(mt + r) * p.ldc + wave_n + j * 16)[lane_c] = v;
                }
        }
        return;
    }
    if (m0 + BM <= p.M && n0 + BN <= p.N) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int n = wave_n + j * 32;                                        // uniform
                if constexpr (ELASTIC) {
                    // with momentum the tile goes through in two halves of eight values per lane: three arrays of
                    // sixteen in flight put the kernel over the registers that four blocks per compute unit leave
                    // (147 against 123; cfg3 round 2.25 -> 2.23 ms with the fourth block)
                    constexpr int HALF = ((MOM || MOM16) && !EARLY_TILES) ? 8 : 16;
#pragma unroll
                    for (int r0 = 0; r0 < 16; r0 += HALF) {
                        float wv[HALF], cv[HALF], vv[HALF];
                        unsigned short v16[HALF];
#pragma unroll
                        for (int q = 0; q < HALF; ++q) {  // all loads of the half first, so that they overlap
                            const int r = r0 + q;
                            if constexpr (EARLY_TILES) {        // requested before the K loop
                                wv[q] = pre_w[r]; cv[q] = pre_c[r]; vv[q] = pre_v[r]; v16[q] = (unsigned short)pre_v16[r];
                                continue;
                            }
                            const size_t row = (size_t)(wave_m + i * 32 + 8 * (r / 4) + (r % 4)) * p.ldc + n;
                            wv[q] = (Wr + row)[lane_c];
                            cv[q] = (Cc + row)[lane_c];
                            vv[q] = MOM ? (Vr + row)[lane_c] : 0.f;
                            v16[q] = MOM16 ? (Vr16 + row)[lane_c] : (unsigned short)0;
                        }
#pragma unroll
                        for (int q = 0; q < HALF; ++q) {
                            const int r = r0 + q;
                            const size_t row = (size_t)(wave_m + i * 32 + 8 * (r / 4) + (r % 4)) * p.ldc + n;
                            const float g = acc[i][j][r];
                            if constexpr (MOM16) worker_rule_bf16<true>(wv[q], v16[q], g, cv[q], p.eta, p.rho, p.alpha, p.delta);
                            else worker_rule<MOM>(wv[q], vv[q], g, cv[q], p.eta, p.rho, p.alpha, p.delta);
                            (Wr + row)[lane_c] = wv[q];
                            if (MOM) (Vr + row)[lane_c] = vv[q];
                            if (MOM16) (Vr16 + row)[lane_c] = v16[q];
                            if (keep) (C + row)[lane_c] = g;
                        }
                    }
                    continue;
                }
                float gate[16];
                if (EPI == EPI_MASK) {      // all mask loads of the tile first, so that they overlap
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int m = wave_m + i * 32 + 8 * (r / 4) + (r % 4);
                        gate[r] = (mask + (size_t)m * p.ldmask + n)[lane_mask];
                    }
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = wave_m + i * 32 + 8 * (r / 4) + (r % 4);            // uniform
                    float v = acc[i][j][r];
                    if (EPI == EPI_RELU) v = fmaxf(v, 0.f);
                    if (EPI == EPI_MASK) v = (gate[r] > 0.f) ? v : 0.f;
                    if constexpr (OUT16) (C16 + (size_t)m * p.ldc + n)[lane_c] = bf16_narrow(v);
                    else (C + (size_t)m * p.ldc + n)[lane_c] = v;
                }
            }
    } else {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int n = n0 + wn0 + j * 32 + frag_x;
                if constexpr (ELASTIC) {
                    // Three passes over the tile, as in the full-tile path: every load, then the rule, then every
                    // store.  Written element by element (load, rule, store, next element) the stores to the replica
                    // keep the next element's loads from the same array behind them, and a narrow layer, all of whose
                    // tiles are edge tiles, pays sixteen round trips to memory in a row.
                    float wv[16], cv[16], vv[16];
                    unsigned short v16[16];
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        if constexpr (EARLY_TILES) {        // requested before the K loop
                            wv[r] = pre_w[r]; cv[r] = pre_c[r]; vv[r] = pre_v[r]; v16[r] = (unsigned short)pre_v16[r];
                            continue;
                        }
                        // unconditional loads: a lane whose element lies outside C reads the last row or column
                        const int m = min(m0 + wm0 + i * 32 + 8 * (r / 4) + frag_r + (r % 4), p.M - 1);
                        const size_t at = (size_t)m * p.ldc + min(n, p.N - 1);
                        wv[r] = Wr[at];
                        cv[r] = Cc[at];
                        vv[r] = MOM ? Vr[at] : 0.f;
                        v16[r] = MOM16 ? Vr16[at] : (unsigned short)0;
                    }
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        if constexpr (MOM16) worker_rule_bf16<true>(wv[r], v16[r], acc[i][j][r], cv[r], p.eta, p.rho, p.alpha, p.delta);
                        else worker_rule<MOM>(wv[r], vv[r], acc[i][j][r], cv[r], p.eta, p.rho, p.alpha, p.delta);
                    }
                    // One branch on the column for the whole pass, and none on the rows unless the tile is ragged
                    // there too: behind every per-element branch the compiler waits for all outstanding memory
                    // operations, the previous element's stores included.
                    auto store_at = [&](int r, size_t at) {
                        Wr[at] = wv[r];
                        if (MOM) Vr[at] = vv[r];
                        if (MOM16) Vr16[at] = v16[r];
                        if (keep) C[at] = acc[i][j][r];
                    };
                    if (n < p.N) {
                        if (m0 + BM <= p.M) {                                           // uniform
#pragma unroll
                            for (int r = 0; r < 16; ++r)
                                store_at(r, (size_t)(m0 + wm0 + i * 32 + 8 * (r / 4) + frag_r + (r % 4)) * p.ldc + n);
                        } else {
#pragma unroll
                            for (int r = 0; r < 16; ++r) {
                                const int m = m0 + wm0 + i * 32 + 8 * (r / 4) + frag_r + (r % 4);
                                if (m < p.M) store_at(r, (size_t)m * p.ldc + n);
                            }
                        }
                    }
                    continue;
                }
                float gate[16];
                if (EPI == EPI_MASK) {      // unconditional loads (clamped into the matrix), all in flight together
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int m = min(m0 + wm0 + i * 32 + 8 * (r / 4) + frag_r + (r % 4), p.M - 1);
                        gate[r] = mask[(size_t)m * p.ldmask + min(n, p.N - 1)];
                    }
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = m0 + wm0 + i * 32 + 8 * (r / 4) + frag_r + (r % 4);
                    if (m < p.M && n < p.N) {
                        float v = acc[i][j][r];
                        const size_t at = (size_t)m * p.ldc + n;
                        if (EPI == EPI_RELU) v = fmaxf(v, 0.f);
                        if (EPI == EPI_MASK) v = (gate[r] > 0.f) ? v : 0.f;
                        if constexpr (OUT16) C16[at] = bf16_narrow(v);
                        else C[at] = v;
                    }
                }
            }
    }
}

// One product per launch; the grid may be extended by blocks that run the center rule (p.ctr).
template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, int A_LAYOUT, int B_LAYOUT, bool VEC, int EPI, int MT = 32>
__global__ __launch_bounds__(WAVES_M *WAVES_N * 64, 2) void gemm_mfma_kernel(GemmArgs p)
{
    __shared__ __attribute__((aligned(16))) float lds[gemm_lds_floats<BM, BN, BK, A_LAYOUT, B_LAYOUT>()];
    if (p.ctr.blocks > 0 && blockIdx.x >= p.ctr.first_block) {         // uniform for the block
        const size_t b = blockIdx.x - p.ctr.first_block;
        if (p.ctr.vec) center_rule_block<f32x4>(p.ctr.W, p.ctr.Wc, p.ctr.old, p.ctr.P, p.ctr.N, p.ctr.ld, p.ctr.alpha, b, p.ctr.blocks, threadIdx.x);
        else center_rule_block<float>(p.ctr.W, p.ctr.Wc, p.ctr.old, p.ctr.P, p.ctr.N, p.ctr.ld, p.ctr.alpha, b, p.ctr.blocks, threadIdx.x);
        return;
    }
    gemm_block<BM, BN, BK, WAVES_M, WAVES_N, A_LAYOUT, B_LAYOUT, VEC, EPI, MT, true>(p, blockIdx.x, lds);
}

// Two independent products in one launch: blocks [0, n0) work on p0 with the first configuration, the rest on
// p1 with the second.  The products of backward propagation are short, so sharing a launch saves a launch
// boundary and lets the blocks of one fill the wave slots and the tail the other leaves idle.  Both
// configurations use 256 threads; the LDS buffer is the larger of the two needs.
template <int BM0, int BN0, int BK0, int WM0, int WN0, int AL0, int BL0, bool VEC0, int EPI0,
          int BM1, int BN1, int BK1, int WM1, int WN1, int AL1, int BL1, bool VEC1, int EPI1>
__global__ __launch_bounds__(256, 2) void gemm_pair_kernel(GemmArgs p0, GemmArgs p1, unsigned n0)
{
    static_assert(WM0 * WN0 == 4 && WM1 * WN1 == 4, "both products use 256 threads");
    constexpr int L0 = gemm_lds_floats<BM0, BN0, BK0, AL0, BL0>(), L1 = gemm_lds_floats<BM1, BN1, BK1, AL1, BL1>();
    __shared__ __attribute__((aligned(16))) float lds[L0 > L1 ? L0 : L1];
    if (blockIdx.x < n0) gemm_block<BM0, BN0, BK0, WM0, WN0, AL0, BL0, VEC0, EPI0>(p0, blockIdx.x, lds);
    else gemm_block<BM1, BN1, BK1, WM1, WN1, AL1, BL1, VEC1, EPI1>(p1, blockIdx.x - n0, lds);
}

}  // namespace easgd
