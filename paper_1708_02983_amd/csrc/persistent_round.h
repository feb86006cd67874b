// Single-launch round of a single-layer network (internal interface; see persistent_round.hip).
#pragma once
#include "common.h"

namespace easgd {

struct SoftmaxRound {
    const float *X;             // [P][b][d_in]
    const int *y;               // [P][b]
    const float *W_in;          // replicas as read by forward propagation: [P][ld], packed (d_in+1) x C
    float *W, *V, *Wc;          // the same replicas, momentum buffers (or null) and center for the update;
                                // W == null: gradient only
    unsigned short *V16;        // momentum buffers stored as bfloat16 (then V is null), or null
    float *G;                   // [P][ld] gradient out, or null
    unsigned short *G16;        // [P][ld] gradient out as bfloat16 (round to nearest even), or null
    float *dz, *row_loss;       // workspace: [P*b][C], [P*b]
    float *loss;                // [P] mean loss per worker, or null
    size_t ld;
    int d_in, C, b, P;
    float eta, rho, alpha, delta;
    int write_center;           // 0: a local step (rho == 0), the center is neither read for Eq. (2) nor written
};

// Whether a network of this shape takes the single-launch path at all (sizes only).
bool softmax_round_fits(int d_in, int C, int b, int P);

// Enqueues the round on `stream`.  Returns 0 when launched, 1 when this call cannot take the path (the stream is
// being captured, or no barrier words are left for it): the caller then uses separate launches.
int softmax_round_launch(const SoftmaxRound &r, void *stream);

}  // namespace easgd
