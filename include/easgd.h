/*
 * easgd.h -- C ABI of the MI355X (gfx950) Sync EASGD hot-path library.
 *
 * One Sync EASGD round (paper Section 5.1, steps (1)-(5)) for P worker
 * replicas that all live in ONE GPU's memory:
 *
 *   step (1)      easgd_grad        every worker's minibatch gradient dW^i_t at W^i_t
 *   steps (2)-(5) easgd_sync_round  broadcast of the center, reduction over the
 *                                   workers, worker rule Eq. (1), center rule Eq. (2)
 *                 measgd_round      the same with the momentum worker rule Eq. (5),(6)
 *   steps (1)-(5) easgd_mlp_round   the whole round in one call, the update fused into
 *                                   backward propagation
 *   extension     *_bf16, *_bf16v   the same updates with gradients and/or momentum buffers
 *                                   stored as bfloat16 (fp32 replicas, center and arithmetic)
 *
 * Conventions shared by every entry point
 *   - every pointer marked DEVICE is a device (HBM) pointer owned by the caller;
 *     the library never allocates or frees device memory and never keeps a caller's
 *     pointer after the call returns;
 *   - calls are asynchronous on `stream` (a hipStream_t passed as void*, NULL =
 *     the default stream); no host synchronisation happens inside;
 *   - the return value is an easgd_status and easgd_last_error() describes the reason
 *     (thread-local string).  EASGD_EINVAL, EASGD_EWORKSPACE and EASGD_ERANGE are found
 *     before anything is launched: the buffers are untouched.  EASGD_ELAUNCH is what the
 *     HIP runtime reports when a launch, an event or a stream wait fails; the calls that
 *     issue several kernels (easgd_grad*, easgd_mlp_round*) check once at their end, so
 *     earlier kernels of the call may already be queued and the outputs are then undefined;
 *   - fp32 pointers must be 4-byte aligned and bfloat16 pointers 2-byte aligned
 *     (EASGD_EINVAL otherwise); stricter alignment selects the fast paths, see each call;
 *   - buffers of one call must not overlap each other;
 *   - process-wide state: the launch-shape options below, a launch counter, and per device
 *     what easgd_mlp_round and easgd_grad_static create on first use (described there);
 *   - all floating point is IEEE fp32 (storage and arithmetic), except the *_bf16 / *_bf16v entry points,
 *     which keep fp32 arithmetic and store gradients and momentum buffers as bfloat16;
 *   - replica matrices are [P][ld] row-major: row i is worker i, its first N
 *     entries are the parameters, entries [N, ld) are padding that is never
 *     read or written.
 *
 * Packed parameter layout of a replica (the packed single-buffer idea of
 * Section 5.2): for layer l = 0..L-1 in order, the weight matrix
 * W_l[dims[l]][dims[l+1]] row-major followed by the bias b_l[dims[l+1]];
 * N = sum_l (dims[l]*dims[l+1] + dims[l+1]).
 */
#ifndef EASGD_H
#define EASGD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    EASGD_OK         =  0,
    EASGD_EINVAL     = -1,   /* NULL pointer, P < 1, N == 0, ld < N, b < 1, bad dims, bad option */
    EASGD_ELAUNCH    = -2,   /* the HIP runtime refused a launch (hipGetLastError text in last_error) */
    EASGD_EWORKSPACE = -3,   /* workspace NULL, misaligned or smaller than easgd_grad_workspace_bytes */
    EASGD_ERANGE     = -4    /* a size exceeds what the kernels index (see each call) */
} easgd_status;

/*
 * Steps (2)-(5) of a Sync EASGD round, fused (Section 5.1; Eq. (1), Eq. (2)):
 *
 *   for every parameter j:   c = Wc[j]                                (the broadcast of Wc_t)
 *     for every worker i:    d_i = W[i][j] - c                        (time-t values)
 *                            W[i][j] <- W[i][j] - eta*(G[i][j] + rho*d_i)        Eq. (1)
 *     Wc[j] <- c + eta*rho * (d_0 + d_1 + ... + d_{P-1})                         Eq. (2)
 *
 * The sum over the workers is taken in a fixed order (ascending i by one thread;
 * for small N with P >= 4 the workers are split over four wavefronts whose
 * partial sums are added in a fixed order), so results are bitwise reproducible
 * from run to run and independent of the launch-shape options.  The arithmetic is
 * fp32 with the fused multiply-adds fixed in the source, the same in every kernel of
 * the library that applies these rules (fma = one rounding):
 *   Eq. (1)  W <- fma(-eta, fma(rho, d, G), W)          Eq. (2)  Wc <- fma(eta*rho, sum, c)
 *   Eq. (5)  V <- fma(delta, V, -(eta*G))               Eq. (6)  W  <- fma(-(eta*rho), d, W + V)
 *
 *   W   DEVICE in/out [P][ld]   worker replicas W^i_t -> W^i_{t+1}
 *   G   DEVICE in     [P][ld]   worker gradients dW^i_t (never written)
 *   Wc  DEVICE in/out [N]       center weights Wc_t -> Wc_{t+1}
 *   P >= 1, N >= 1, ld >= N (elements).
 *
 * Fast path: W, G, Wc 16-byte aligned and ld % 4 == 0 (128-bit accesses; N need
 * not be a multiple of 4).  Otherwise a scalar kernel computes the same values.
 * Errors: EASGD_EINVAL, EASGD_ELAUNCH.
 */
int easgd_sync_round(float *W, const float *G, float *Wc,
                     int P, size_t N, size_t ld,
                     float eta, float rho, void *stream);

/*
 * The same round with the momentum worker rule (Eq. (5), Eq. (6)); the center
 * keeps Eq. (2).  delta is the momentum rate (the paper's mu).
 *
 *     V[i][j] <- delta*V[i][j] - eta*G[i][j]                                     Eq. (5)
 *     W[i][j] <- W[i][j] + V[i][j](new) - eta*rho*d_i                            Eq. (6)
 *
 *   V   DEVICE in/out [P][ld]   momentum buffers V^i_t -> V^i_{t+1}
 * Other arguments, alignment rule and errors as for easgd_sync_round.
 */
int measgd_round(float *W, float *V, const float *G, float *Wc,
                 int P, size_t N, size_t ld,
                 float eta, float rho, float delta, void *stream);

/*
 * The asynchronous exchanges that the paper compares Sync EASGD with, on the same replicas (comparison points:
 * the deterministic fused round above is the method).
 *
 * async_easgd_round: the master serves ONE worker at a time (Section 2.6 and Algorithm 1, "Original EASGD",
 * in rank order; Section 5.1, "Async EASGD" / "Async MEASGD", in the order in which workers arrive).  A
 * schedule is the sequence of workers served, order[0 .. n_order).  Per turn of worker i = order[t], from the
 * values at the start of the turn:
 *     d = W[i][j] - Wc[j]
 *     W[i][j] <- W[i][j] - eta*(G[i][j] + rho*d)                       Eq. (1)
 *       (V != NULL:  V[i][j] <- delta*V[i][j] - eta*G[i][j];  W[i][j] <- W[i][j] + V[i][j] - eta*rho*d    Eq. (5),(6))
 *     Wc[j]   <- Wc[j] + eta*rho*d                                     Eq. (2) for one worker
 * One launch for the whole schedule: the thread that owns parameter j takes the turns one after the other with
 * the center in a register, so the result is that of n_order separate one-worker exchanges, bit for bit, and is
 * reproducible.  A worker may come up more than once; its gradient row is used as it is each time.
 *   order  HOST in [n_order]   worker indices in [0, P); copied before the call returns
 *   0 <= n_order <= EASGD_MAX_SCHEDULE (longer schedules: several calls); P <= 256.
 *   HBM traffic N*(12*n_order + 8) bytes (Eq. (1)), N*(20*n_order + 8) bytes (Eq. (5),(6)).
 *
 * hogwild_easgd_round: Section 5.1, "Hogwild EASGD" -- all P workers exchange with the center at the same time
 * and nothing orders them: each worker reads the center as it finds it, applies Eq. (1) (Eq. (5),(6)) with that
 * value and adds eta*rho*(W[i][j] - Wc[j]) to the center with a floating-point atomic add.  Which center value a
 * worker sees and the order of the additions vary from run to run: W and Wc are NOT reproducible (that is what
 * the comparison is about).  Every interleaving gives the same V, and leaves sum_i W[i][j] + Wc[j] equal to its
 * value before the call minus eta * sum_i G[i][j] (plus sum_i V[i][j] (new) with momentum), up to rounding.
 *   Wc must be ordinary device memory (the hardware's fp32 atomic add is used).
 * Other arguments, alignment rule (a scalar kernel serves operands that are not 16-byte aligned) and errors as
 * for easgd_sync_round / measgd_round.
 */
#define EASGD_MAX_SCHEDULE 256
int async_easgd_round(float *W, float *V, const float *G, float *Wc, int P, size_t N, size_t ld,
                      const int *order, int n_order, float eta, float rho, float delta, void *stream);
int hogwild_easgd_round(float *W, float *V, const float *G, float *Wc, int P, size_t N, size_t ld,
                        float eta, float rho, float delta, void *stream);

/*
 * The two rounds above with the gradients (and the momentum buffers) STORED as bfloat16 -- an
 * extension: the paper keeps fp32 throughout and names low precision only as future work (Section 3.2).
 * Replicas and center stay fp32, all arithmetic is fp32; the HBM stream shrinks from N*(12P+8) to
 * N*(10P+8) bytes per round (Eq. (1)) and from N*(20P+8) to N*(14P+8) bytes (Eq. (5),(6)).
 *
 * A bfloat16 is the upper 16 bits of an IEEE fp32, passed as uint16_t.  Widening is exact.  Narrowing
 * rounds to nearest, ties to even; values beyond the largest finite bfloat16 become infinity; a NaN
 * becomes 0x7FC0 with the input's sign.  With g = widened G[i][j], v = widened V[i][j]:
 *
 *     V[i][j] <- narrow( fl(fl(delta*v) - fl(eta*g)) )       Eq. (5): three fp32 operations, each
 *                                                            rounded on its own (no fused multiply-add),
 *                                                            so the stored code is reproducible anywhere
 *     W[i][j] <- W[i][j] + widened V[i][j](new) - eta*rho*d_i                    Eq. (6)
 *     easgd_sync_round_bf16:  W[i][j] <- W[i][j] - eta*(g + rho*d_i)             Eq. (1)
 *     Wc as in easgd_sync_round                                                  Eq. (2)
 *
 *   W   DEVICE in/out [P][ld] fp32;  Wc  DEVICE in/out [N] fp32
 *   G   DEVICE in     [P][ld] bfloat16 (never written);  V  DEVICE in/out [P][ld] bfloat16
 *   ld counts elements and is the same for W, G and V.
 * Fast path: W, Wc 16-byte aligned, G, V 8-byte aligned, ld % 4 == 0; otherwise a scalar kernel
 * computes the same values.  The sum of Eq. (2) is taken in ascending worker order by one thread.
 * Errors: EASGD_EINVAL, EASGD_ELAUNCH.
 */
int easgd_sync_round_bf16(float *W, const uint16_t *G, float *Wc,
                          int P, size_t N, size_t ld,
                          float eta, float rho, void *stream);
int measgd_round_bf16(float *W, uint16_t *V, const uint16_t *G, float *Wc,
                      int P, size_t N, size_t ld,
                      float eta, float rho, float delta, void *stream);
/*
 * measgd_round_bf16 for gradients that arrive as fp32 (what easgd_grad writes): only the momentum buffers
 * are stored as bfloat16; g in Eq. (5) above is G[i][j] itself.  N*(16P+8) bytes per round.
 * G DEVICE in [P][ld] fp32, 16-byte aligned for the fast path; everything else as for measgd_round_bf16.
 */
int measgd_round_bf16v(float *W, uint16_t *V, const float *G, float *Wc,
                       int P, size_t N, size_t ld,
                       float eta, float rho, float delta, void *stream);

/*
 * Synchronous data-parallel SGD on the same replicas, the method's point of comparison (Section 2.3,
 * "Data Parallelism": the gradients of all workers are summed, W <- W - eta * sum_i dW^i, and every worker
 * receives the new W; Section 6.2: on a partitioned chip every partition receives the gradient sum and
 * updates its own copy).  With momentum buffers the sum drives Eq. (3),(4).
 *
 *   for every parameter j:   s = G[0][j] + G[1][j] + ... + G[P-1][j]          (ascending i, fixed order)
 *     for every worker i:    W[i][j] <- W[i][j] - eta*s                       (V == NULL)
 *                            V[i][j] <- delta*V[i][j] - eta*s;  W[i][j] <- W[i][j] + V[i][j]   Eq. (3),(4)
 *
 *   W  DEVICE in/out [P][ld];  V  DEVICE in/out [P][ld] or NULL;  G  DEVICE in [P][ld]
 * Replicas that start equal stay equal bit for bit.  Alignment rule and errors as for easgd_sync_round.
 */
int sync_sgd_round(float *W, float *V, const float *G,
                   int P, size_t N, size_t ld,
                   float eta, float delta, void *stream);

/*
 * Step (1) of the round (Section 5.1; forward/backward propagation of Section
 * 2.2) for a dense ReLU multilayer perceptron with softmax cross-entropy loss,
 * averaged over the b samples of each worker's minibatch.  Worker i uses its
 * own weights W[i] and its own minibatch (X[i], y[i]); all P workers are
 * processed by batched fp32 MFMA matrix products.
 *
 *   dims        HOST   in  [n_layers+1]  layer widths, e.g. {784,1024,1024,10};
 *                                        hidden layers use ReLU, the last layer is linear
 *   W           DEVICE in  [P][ld]       packed replicas (layout above)
 *   X           DEVICE in  [P][b][dims[0]] row-major inputs
 *   y           DEVICE in  [P][b]        int32 labels in [0, dims[n_layers])
 *   G           DEVICE out [P][ld]       packed gradients; every one of the N valid
 *                                        entries of every row is overwritten
 *   loss        DEVICE out [P]           mean loss of each worker, or NULL
 *   workspace   DEVICE     scratch of at least easgd_grad_workspace_bytes(...)
 *                                        bytes, 256-byte aligned; contents undefined after
 *
 * Requirements: 1 <= n_layers <= 8, every dims[l] >= 1, dims[n_layers] <= 1024,
 * P >= 1, b >= 1, ld >= N, W/G/X 16-byte aligned.  The ReLU derivative at exactly 0 is 0.
 * Errors: EASGD_EINVAL, EASGD_EWORKSPACE, EASGD_ERANGE (an operand above 2^30-1
 * elements per worker), EASGD_ELAUNCH.
 */
size_t easgd_grad_workspace_bytes(const int *dims, int n_layers, int P, int b);

int easgd_grad(const int *dims, int n_layers,
               const float *W, size_t ld,
               const float *X, const int32_t *y, int P, int b,
               float *G, float *loss,
               void *workspace, size_t workspace_bytes, void *stream);

/*
 * easgd_grad for callers that cannot allocate device memory or hand over a workspace: code that runs
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The workspace is an
 * array of EASGD_STATIC_SCRATCH_BYTES bytes in the library's own device image: every GPU the library runs
 * on holds one copy of it from the first use of the library on that GPU until the process ends.  The call
 * itself allocates and frees nothing (no hipMalloc / hipFree, no allocating library routine); its first
 * call on a device looks up the device address of that array (hipGetSymbolAddress) and keeps it.
 *
 * Same arguments, kernels, results (bit for bit) and errors as easgd_grad, without `workspace` and
 * `workspace_bytes`.  A shape whose easgd_grad_workspace_bytes(...) exceeds EASGD_STATIC_SCRATCH_BYTES is
 * rejected with EASGD_EWORKSPACE before anything is launched (use easgd_grad then).  The array keeps the
 * contents of the last call; nothing in it has to start at zero, every part is written before it is read.
 * All calls on one GPU share the one array: calls that overlap in time on the same GPU (different
 * streams, or different host threads) race on it and must be serialised by the caller.
 */
#define EASGD_STATIC_SCRATCH_BYTES (64u << 20)

int easgd_grad_static(const int *dims, int n_layers,
                      const float *W, size_t ld,
                      const float *X, const int32_t *y, int P, int b,
                      float *G, float *loss, void *stream);

/*
 * easgd_grad with the gradients stored as bfloat16 (an extension; format and rounding as described for
 * measgd_round_bf16): every product is accumulated in fp32 exactly as in easgd_grad and narrowed once when it
 * is stored, so G[i][j] here is the narrowed value of what easgd_grad writes.  G DEVICE out [P][ld] bfloat16,
 * not NULL, 2-byte aligned (8-byte aligned if measgd_round_bf16 is to take its fast path on it).
 * Everything else as for easgd_grad.
 */
int easgd_grad_bf16(const int *dims, int n_layers,
                    const float *W, size_t ld,
                    const float *X, const int32_t *y, int P, int b,
                    uint16_t *G, float *loss,
                    void *workspace, size_t workspace_bytes, void *stream);

/*
 * A whole Sync EASGD round in one call: steps (1)-(5) of Section 5.1 for the
 * multilayer perceptron of easgd_grad, with the elastic update fused into
 * backward propagation (the overlap of steps that Section 5.1 allows).
 * Eq. (2) runs first and keeps a copy of the time-t center for the rest of
 * the round; the worker rule Eq. (1) (Eq. (5),(6) when V != NULL) is applied to
 * layer l's slice of every replica by the kernel that computes that layer's
 * weight gradient, straight from the accumulators, once no later product of
 * the round reads W_l.  Every parameter is updated exactly once from time-t values and the
 * workers are summed in ascending order, so the result equals easgd_grad
 * followed by easgd_sync_round / measgd_round to rounding.
 *
 *   W   DEVICE in/out [P][ld]   replicas W^i_t -> W^i_{t+1}
 *   V   DEVICE in/out [P][ld]   momentum buffers, or NULL for the plain rule Eq. (1)
 *   Wc  DEVICE in/out [N]       center weights
 *   G   DEVICE out    [P][ld]   the gradients dW^i_t of this round, or NULL when the
 *                               caller does not need them (they are then never stored)
 *   delta is ignored when V == NULL; the other arguments are those of easgd_grad
 *   and easgd_sync_round, with the same requirements; the workspace must hold
 *   easgd_mlp_round_workspace_bytes(...) bytes.
 *   rho == 0 makes the call a local step: with rho = 0 Eq. (1) (Eq. (5),(6)) is a plain
 *   (momentum) SGD step of every worker and Eq. (2) leaves the center as it is, so no
 *   exchange is launched and Wc is not written.  A caller who wants workers to
 *   exchange only every tau-th round (a communication period; an extension, the
 *   paper's Sync EASGD exchanges in every round) passes rho = 0 in the rounds between.
 *
 * Library state: when the center rule is placed on a second stream (EASGD_OPT_ROUND_OVERLAP 2, or 1
 * with P*N >= 2^24 and a first forward launch that fills the chip) the first such call on a device
 * creates one non-blocking stream of default priority and two events for that device, which live
 * until the process ends, and calls from several host threads are serialised on a mutex around
 * their record/wait pair.  A caller that wants to capture the call in a HIP graph makes one eager
 * call with the same shape first, so that the stream is not created under capture (or sets
 * EASGD_OPT_ROUND_OVERLAP to 0 or 3, which keep the call on the caller's stream).
 *
 * With EASGD_OPT_ROUND_SINGLE_LAUNCH set to 1 (default 0) a single-layer network (softmax regression) of at
 * most 16 classes with b <= 256 and P*b <= 2048 takes ONE launch for the whole call (the gradient entry
 * points take the same launch without the update): forward propagation and softmax, a
 * barrier over the grid, then gradient, worker rule and center rule per parameter with the workers in
 * ascending order.  The gradient's sum over the minibatch has another (fixed) order there than in the
 * matrix-product kernels, so results agree with the separate launches to rounding, not bit for bit.
 * The barrier is a count of arrivals in device memory that belongs to the library, one per (device,
 * stream) that has taken this path, at most 64 streams per device; a call on a stream under capture, or
 * on a 65th stream, takes the separate launches instead.  All blocks of the grid are resident at once,
 * so the wait ends; it is bounded all the same (EASGD_OPT_ROUND_SPIN_LIMIT): a block that gives up
 * writes NaN into its share of W, Wc, G and loss instead of a result, and easgd_round_barrier_timeouts
 * counts it.
 * Errors: as easgd_grad.
 */
size_t easgd_mlp_round_workspace_bytes(const int *dims, int n_layers, int P, int b);

int easgd_mlp_round(const int *dims, int n_layers,
                    float *W, float *V, float *Wc, size_t ld,
                    const float *X, const int32_t *y, int P, int b,
                    float *G, float *loss,
                    float eta, float rho, float delta,
                    void *workspace, size_t workspace_bytes, void *stream);

/*
 * easgd_mlp_round with the momentum buffers stored as bfloat16 (an extension; format, rounding and the
 * arithmetic of Eq. (5) as described for measgd_round_bf16v, the gradient being the fp32 value the
 * matrix product has just accumulated).  V DEVICE in/out [P][ld] bfloat16, not NULL, 2-byte aligned.
 * Results equal easgd_grad followed by measgd_round_bf16v.  Everything else as for easgd_mlp_round.
 */
int easgd_mlp_round_bf16v(const int *dims, int n_layers,
                          float *W, uint16_t *V, float *Wc, size_t ld,
                          const float *X, const int32_t *y, int P, int b,
                          float *G, float *loss,
                          float eta, float rho, float delta,
                          void *workspace, size_t workspace_bytes, void *stream);

/*
 * One matrix product of forward / backward propagation (Section 2.2) alone, for all P workers, through the
 * tile selection and the MFMA kernels that easgd_grad uses for it (a testing aid: integer-valued operands
 * make every product and partial sum exact in fp32, so the result can be checked bit for bit).
 * For one layer with d_in inputs and d_out outputs, [W ; b] its packed (d_in+1) x d_out block:
 *
 *   kind 0  forward           out[w] = [A[w] 1] [W[w] ; b[w]]          b x d_out   (max(., 0) when relu != 0)
 *   kind 1  weight gradient   out[w] = [A[w] 1]^T dZ[w]                (d_in+1) x d_out, i.e. [dW ; db]
 *   kind 2  input gradient    out[w] = (dZ[w] W[w]^T) where A[w] > 0, else 0      b x d_in
 *
 *   A    DEVICE in  [P][b][d_in]     layer input (kind 2: only its sign is used)
 *   Wl   DEVICE in  worker w's block at Wl + w*ld (kinds 0, 2; ignored for kind 1)
 *   dZ   DEVICE in  [P][b][d_out]    (kinds 1, 2; ignored for kind 0)
 *   out  DEVICE out worker w's result at out + w*out_ws, row-major with the widths above
 * A, dZ, out 16-byte aligned.  Errors: EASGD_EINVAL, EASGD_ERANGE, EASGD_ELAUNCH.
 */
int easgd_layer_product(int kind, int d_in, int d_out, int P, int b,
                        const float *A, const float *Wl, size_t ld, const float *dZ,
                        float *out, size_t out_ws, int relu, void *stream);

/* Number of parameters N of the packed layout for `dims`; 0 on invalid input. */
size_t easgd_mlp_num_params(const int *dims, int n_layers);

/*
 * Launch-shape knobs (performance only).  Process-wide; each is one atomic word, so setting one from
 * a host thread while another thread is inside a call is safe, and that call may use the old or the
 * new value.  The results of the update entry points never depend on them (the worker sum has one
 * fixed order).  EASGD_OPT_GEMM_TILE changes the slab depth of the matrix products and with it the
 * order of their k sums: gradients then agree to rounding (about 1e-6 normwise), not bit for bit;
 * the other matrix-product options change block order and launch grouping only (same bits).
 * Returns EASGD_EINVAL for an unknown option or an out-of-range value.
 */
typedef enum {
    EASGD_OPT_UPDATE_BLOCKS_PER_CU = 1,  /* 0 = one block per tile (default); k>0 = persistent grid of k*CUs blocks */
    EASGD_OPT_UPDATE_NONTEMPORAL   = 2,  /* 1 = streaming (non-temporal) loads/stores for W, G, V, 0 = plain, 2 = chosen per call
                                            (default): streaming when the round moves more than 512 MiB, plain below that,
                                            where much of what a round writes is still in the caches for the next reader */
    EASGD_OPT_UPDATE_GROUPS        = 3,  /* 128-bit groups per thread and worker: 1, 2, 4 or 8; 0 = chosen per call (default): 4, fewer
                                            when N is small */
    EASGD_OPT_GEMM_TILE            = 4,  /* block tile of the wide matrix products of easgd_grad: 0 = chosen per product (default),
                                            1 = 128x128, 2 = 64x64, 3 = 128x64, 4 = 48, 80 or 112 rows by 128 columns in 16x16x4 matrix
                                            instructions for the products whose rows are the minibatch (chosen by default when
                                            one of these heights covers b with fewer rows than b rounded up to 32, e.g. b = 100) */
    EASGD_OPT_ROUND_OVERLAP        = 5,  /* easgd_mlp_round, where the center rule runs: 0 = a kernel of its own on the caller's
                                            stream; 2 = the same on a second stream of the library, beside forward propagation;
                                            3 = on extra blocks of the first forward product's launch; 1 = chosen per call
                                            (default): 3 when that launch leaves room on the chip, else 2 when P*N >= 2^24
                                            (below which ordering two streams costs more than it hides), else 0 */
    EASGD_OPT_GEMM_XCD             = 6,  /* 1 = the blocks of a matrix product are renumbered so that each of the eight dies
                                            works on whole workers, and in products that apply the worker rule a die walks
                                            its workers tile by tile, so that it fetches each tile of the center once, going
                                            through the result in bands of up to eight tile columns, so that the tiles it
                                            works on at one time share their operand panels (default); 3 = the same walk in
                                            row-major tile order; 2 = whole workers per die only; 0 = plain block order */
    EASGD_OPT_GEMM_PAIR            = 7,  /* 1 = independent products of backward propagation share a launch where their tile
                                            shapes allow (default), 0 = one launch per product */
    EASGD_OPT_MLP_HEAD             = 8,  /* 1 = a last layer of at most 16 classes takes one launch for its forward product, the
                                            softmax cross-entropy and its input-gradient product (default), 0 = three launches
                                            (split-K product, softmax, product) */
    EASGD_OPT_UPDATE_LAYOUT        = 9,  /* which parameters a block of the streaming update kernels owns: 0 = a contiguous run of
                                            groups*1024 parameters; 1 = eight consecutive blocks (one per die) interleave in pieces
                                            of 1 KiB inside a super-tile, so that every die's requests spread over all memory
                                            channels; 2 = chosen per call (default): 1 when N is large enough for 4 groups */
    EASGD_OPT_ROUND_SINGLE_LAUNCH  = 10, /* 1 = easgd_grad, easgd_grad_static, easgd_grad_bf16, easgd_mlp_round and
                                            easgd_mlp_round_bf16v take ONE launch for a single-layer network of at most 16
                                            classes with b <= 256 and P*b <= 2048 (both phases of the round in one grid with
                                            a grid-wide barrier between; see easgd_mlp_round); 0 = separate launches
                                            (default: measured on MI355X the barrier over the eight dies costs what the
                                            launch boundary it replaces costs) */
    EASGD_OPT_ROUND_SPIN_LIMIT     = 11  /* polls after which a block of that launch gives up waiting at the barrier;
                                            0 = 2^22 (default; some seconds) */
} easgd_option;

int easgd_set_option(int option, long value);
long easgd_get_option(int option);

/*
 * Measurement aids (not part of the method): plain streaming kernels of known
 * traffic, used to measure the attainable HBM bandwidth of the device and to
 * calibrate hardware byte counters.  All pointers DEVICE, 16-byte aligned,
 * n > 0 and n % 4 == 0 elements; asynchronous on `stream`.
 *   easgd_stream_copy   dst[j] = src[j]            reads 4n bytes, writes 4n bytes
 *   easgd_stream_triad  a[j] = b[j] + s*c[j]       reads 8n bytes, writes 4n bytes
 * Errors: EASGD_EINVAL, EASGD_ELAUNCH.
 */
int easgd_stream_copy(float *dst, const float *src, size_t n, void *stream);
int easgd_stream_triad(float *a, const float *b, const float *c, size_t n, float s, void *stream);
/*   easgd_stream_mix32  a[j] = c[j] + s*d[j], b[j] = d[j] + s*e[j]   reads 12n bytes, writes 8n bytes
 *                       (three reads and two writes per element: the mix of the momentum update) */
int easgd_stream_mix32(float *a, float *b, const float *c, const float *d, const float *e, size_t n, float s, void *stream);

/*
 * Measurement aid: the attainable rate of the fp32 matrix instruction the products use (32x32x2), without the
 * products' epilogues.  blocks_per_cu x (compute units) blocks of four wavefronts each run `iters` passes over one
 * 32-deep slab of operands held in LDS; a pass is 16 matrix instructions per wavefront on one accumulator tile, as
 * in the 64x64x32 tiles of easgd_grad.  mode 0: operands stay in registers (the matrix cores alone); mode 1: every
 * instruction's operands are fetched from LDS again (matrix cores plus their feeding); mode 2: as 1, and every pass
 * also requests 16 KB from global memory one pass ahead, stores it to LDS and ends in a barrier, which is what a
 * slab of the products' K loop does besides its matrix instructions (the loaded values are not multiplied).
 * Flops per launch: blocks x 4 x iters x 16 x 4096.
 *   out     DEVICE out  [blocks][16][256]  accumulator register r of thread t of a block at [r][t] (every pass adds
 *                       the same 64x64 product, so out = iters x that product in every mode: lets a test check that
 *                       the flops were really done)
 *   out_len elements available at out;  blocks  HOST out, may be NULL: the number of blocks launched
 *   src     DEVICE in   [src_len] floats, 16-byte aligned, src_len >= 4096: what mode 2 reads, in pieces of 4096
 *                       floats, block x piece (977 x + pass) mod (src_len / 4096); ignored (may be NULL) otherwise
 *   iters in [1, 2^20], blocks_per_cu in [1, 8].  Errors: EASGD_EINVAL, EASGD_ELAUNCH.
 */
int easgd_mfma_probe(float *out, size_t out_len, int iters, int mode, int blocks_per_cu, const float *src, size_t src_len,
                     unsigned *blocks, void *stream);

/* Number of blocks that ever gave up waiting at the barrier of a single-launch round on `stream` of the
 * current device (0 unless something kept part of a grid from running for seconds).  Synchronises `stream`.
 * Returns the count, or a negative easgd_status. */
long easgd_round_barrier_timeouts(void *stream);

/* Measurement aid: number of kernel launches the library has issued in this process so far
 * (the difference across a call is the number of launches of that call). */
unsigned long long easgd_launch_count(void);

/* Message for the last error returned on the calling thread ("" if none). */
const char *easgd_last_error(void);

/* Library version: major*10000 + minor*100 + patch. */
int easgd_version(void);

#ifdef __cplusplus
}
#endif
#endif /* EASGD_H */
