// The last layer of the network for a few sample rows of one worker: forward product, softmax cross-entropy and
// input-gradient product (Section 2.2), on the vector ALUs.  Shared by mlp_head_kernel and by the single-launch
// round of a single-layer network.
#pragma once
#include "common.h"
#include "elastic_rule.h"

namespace easgd {

// ---- the head of the network in one launch ---------------------------------
// With few classes the last layer is latency-bound however it is tiled: its logits product has only P*b*C outputs
// with a long K, and the input-gradient product that follows has K = C.  For C <= HEAD_MAX_C this kernel does
// the last layer's forward product, the softmax cross-entropy and the last layer's input-gradient product
// (Section 2.2) for HEAD_ROWS sample rows of one worker per block.  Thread t owns the columns n = t, t+256, ...
// of the layer input: it loads rows n of W_L (C values each) and A[r][n] of the block's rows once, into
// registers, and uses them for both products:
//   z[r][c]  = sum_n A[r][n] W_L[n][c] + b_L[c]   per thread ascending n, then a fixed exchange tree over the
//                                                  lanes, then the four wavefronts in ascending order, then b_L
//   dz[r][c] = (softmax(z[r])[c] - [c == y_r]) / b,   row_loss[r] = -log softmax(z[r])[y_r]   16 lanes per row, one
//                                                  class each; maximum and sum by fixed xor trees
//   da[r][n] = sum_c dz[r][c] W_L[n][c] (ascending c), zero where A[r][n] <= 0
// Blocks are numbered worker-fastest, so that with P a multiple of 8 all blocks of a worker run on one die and
// share its copy of W_L in that die's L2.
static constexpr int HEAD_MAX_C = 16;
static constexpr int HEAD_ROWS = 4;

struct HeadArgs {
    const float *A;         // A_{L-1}: [P][b][d_in]
    const float *Wl;        // [W_L ; b_L] of worker 0: (d_in+1) x C row-major; worker stride w_ws elements
    const int *y;           // [P*b] labels
    float *dz;              // [P*b][C]
    float *row_loss;        // [P*b]
    float *da;              // dZ_{L-2}: [P][b][d_in]
    size_t w_ws;
    int d_in, C, b, P;
    CenterJob ctr;          // optional extra blocks that run the center rule (single-layer networks)
};

// Partials a lane holds before step `step` of the exchange tree that starts from n per lane.
static constexpr int head_tree_count(int n, int step)
{
    for (int q = 0; q < step; ++q)
        if (n % 2 == 0) n /= 2;
    return n;
}

// Steps STEP..5 of the exchange tree on the first CNT entries of v (see mlp_head_kernel).
template <int N, int CNT, int STEP>
__device__ __forceinline__ void head_tree(float (&v)[N], int lane, int &base, bool &writer)
{
    if constexpr (STEP < 6) {
        constexpr int m = 32 >> STEP;
        const bool up = (lane & m) != 0;
        if constexpr (CNT % 2 == 0) {
            constexpr int half = CNT / 2;
#pragma unroll
            for (int i = 0; i < half; ++i) {
                const float keep = up ? v[i + half] : v[i];
                const float send = up ? v[i] : v[i + half];
                v[i] = keep + __shfl_xor(send, m);
            }
            base += up ? half : 0;
            head_tree<N, half, STEP + 1>(v, lane, base, writer);
        } else {
#pragma unroll
            for (int i = 0; i < CNT; ++i) v[i] += __shfl_xor(v[i], m);
            writer = writer && !up;
            head_tree<N, CNT, STEP + 1>(v, lane, base, writer);
        }
    }
}

// CP: class count rounded up to a multiple of 4; NT: columns per thread and pass; ONE_PASS: d_in <= 256 * NT, every
// thread keeps its operands in registers between the two products instead of loading them again (NT = 4 up to
// 1024 columns, NT = 8 up to 2048: one burst of loads per block instead of four dependent ones; the per-thread
// order of the sums is the same, ascending n).
// The work of block `bid` (HEAD_ROWS rows of one worker); part and dzs are the calling kernel's LDS.
// SHARE: dz and row_loss are read by other blocks of the same launch, so they are stored with device-scope
// atomic stores (which go to the level of the memory hierarchy that all dies share) instead of plain ones.
template <int ROWS, int CP, bool ONE_PASS, bool SHARE = false, int NT = 4>
__device__ __forceinline__ void head_block(const HeadArgs &h, const unsigned bid, float (&part)[4][ROWS * CP], float (&dzs)[ROWS][CP])
{
    constexpr int CNT = ROWS * CP;           // partial logits per thread
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int w = bid % h.P;
    const int r0 = (bid / h.P) * ROWS;
    const int C = h.C, K = h.d_in;
    const int rows_here = min(ROWS, h.b - r0);
    const float *__restrict__ Wg = h.Wl + (size_t)w * h.w_ws;
    const float *__restrict__ Am = h.A + ((size_t)w * h.b + r0) * (size_t)K;

    float wv[NT][CP], gate[ROWS][NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
#pragma unroll
        for (int c = 0; c < CP; ++c) wv[j][c] = 0.f;
#pragma unroll
        for (int rr = 0; rr < ROWS; ++rr) gate[rr][j] = 0.f;
    }
    auto load = [&](int n0) {
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const int n = n0 + 256 * j;
            const bool ok = n < K;
#pragma unroll
            for (int rr = 0; rr < ROWS; ++rr) gate[rr][j] = (ok && rr < rows_here) ? Am[(size_t)rr * K + n] : 0.f;
#pragma unroll
            for (int c = 0; c < CP; ++c) wv[j][c] = (ok && c < C) ? Wg[(size_t)n * C + c] : 0.f;
        }
    };

    // partial logits of the thread's columns
    float v[CNT];
#pragma unroll
    for (int i = 0; i < CNT; ++i) v[i] = 0.f;
    for (int n0 = tid; n0 < K; n0 += 256 * NT) {
        load(n0);
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int rr = 0; rr < ROWS; ++rr)
#pragma unroll
                for (int c = 0; c < CP; ++c) v[rr * CP + c] = fmaf(gate[rr][j], wv[j][c], v[rr * CP + c]);
    }
    // exchange tree over the lanes, partner distance 32, 16, ..., 1: while a lane's count of partials is even it
    // keeps one half of them and receives the partner's sums of the same half; once it is odd, both partners add
    // the other's partials to all of theirs.  Each partial ends up summed over the 64 lanes in a fixed order.
    {
        int base = 0;
        bool writer = true;
        head_tree<CNT, CNT, 0>(v, lane, base, writer);
        if (writer) {
#pragma unroll
            for (int i = 0; i < head_tree_count(CNT, 6); ++i) part[wave][base + i] = v[i];
        }
    }
    __syncthreads();

    // softmax cross-entropy: 16 lanes per sample row, one class each; maximum and sum over the row's lanes by
    // fixed xor trees
    static_assert(ROWS * 16 <= 64 && CP <= 16, "the rows of a block share one wavefront");
    if (tid < ROWS * 16) {
        const int rr = tid >> 4, c = tid & 15;
        const bool row_ok = rr < rows_here, live = row_ok && c < C;
        const size_t grow = (size_t)w * h.b + r0 + (row_ok ? rr : 0);
        const int label = h.y[grow];
        float z = -INFINITY;
        if (live) {
            const int i = rr * CP + c;
            z = (((part[0][i] + part[1][i]) + part[2][i]) + part[3][i]) + Wg[(size_t)K * C + c];
        }
        float zmax = z;
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) zmax = fmaxf(zmax, __shfl_xor(zmax, o));
        const float e = live ? expf(z - zmax) : 0.f;
        float sum = e;
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
        float zlabel = (live && c == label) ? z - zmax : 0.f;     // one lane of the row holds it
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) zlabel += __shfl_xor(zlabel, o);
        const float d = live ? (e / sum - (c == label ? 1.f : 0.f)) / (float)h.b : 0.f;
        if (live) {
            if constexpr (SHARE) __hip_atomic_store(&h.dz[grow * (size_t)C + c], d, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            else h.dz[grow * (size_t)C + c] = d;
        }
        if (c < CP) dzs[rr][c] = d;
        if (row_ok && c == 0) {
            if constexpr (SHARE) __hip_atomic_store(&h.row_loss[grow], logf(sum) - zlabel, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            else h.row_loss[grow] = logf(sum) - zlabel;
        }
    }
    if (!h.da) return;                                                         // uniform
    __syncthreads();

    // input gradient of the last layer for the block's rows
    float *__restrict__ da = h.da + ((size_t)w * h.b + r0) * (size_t)K;
    for (int n0 = tid; n0 < K; n0 += 256 * NT) {
        if (!ONE_PASS) load(n0);
#pragma unroll
        for (int rr = 0; rr < ROWS; ++rr) {
            if (rr < rows_here) {
                float d[CP];
#pragma unroll
                for (int c = 0; c < CP; ++c) d[c] = dzs[rr][c];
#pragma unroll
                for (int j = 0; j < NT; ++j) {
                    const int n = n0 + 256 * j;
                    float o = 0.f;
#pragma unroll
                    for (int c = 0; c < CP; ++c) o = fmaf(d[c], wv[j][c], o);
                    if (n < K) da[(size_t)rr * K + n] = gate[rr][j] > 0.f ? o : 0.f;
                }
            }
        }
    }
}

}  // namespace easgd
