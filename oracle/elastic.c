/*
 * CPU ORACLE -- test infrastructure, not the product.
 *
 * Slow, plain evaluation of one Sync EASGD round's exchange-and-update,
 * written from the paper's update rules:
 *
 *   worker, Eq. (1):   W^i_{t+1} = W^i_t - eta * ( dW^i_t + rho * (W^i_t - Wc_t) )
 *   center, Eq. (2):   Wc_{t+1}  = Wc_t  + eta * sum_i rho * (W^i_t - Wc_t)
 *   momentum worker, Eq. (5),(6):
 *                      V^i_{t+1} = mu * V^i_t - eta * dW^i_t
 *                      W^i_{t+1} = W^i_t + V^i_{t+1} - eta * rho * (W^i_t - Wc_t)
 *   (the momentum variant keeps Eq. (2) for the center, Section 5.1 "Async MEASGD").
 *
 * The five steps of Sync EASGD (Section 5.1) collapse, on one memory, to:
 * read Wc_t (the "broadcast"), sum the time-t differences over the workers
 * (the "reduce"), apply Eq. (1) to every worker and Eq. (2) to the center.
 * Both rules use the time-t values of W^i and Wc.
 *
 * State is stored as fp32 (the same bits the GPU library is given); every
 * right-hand side is evaluated in double and rounded once when stored.
 *
 * Only tests/, the smoke check and the benchmark's cpu_baseline leg may call
 * this file.  It shares no code with the HIP library.
 *
 * The elastic coefficient of the center is a separate argument so that the
 * "conserved only when both coefficients match" property can be tested; the
 * paper's Eq. (2) is center_coef = eta * rho.
 */
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Number of threads the loops below use from now on (n < 1: all cores again); for timing only. */
void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    omp_set_num_threads(n >= 1 ? n : omp_get_num_procs());
#else
    (void)n;
#endif
}

/* W, G: [P][ld] (first N entries of each row are valid); Wc: [N]. In place on W, Wc. */
void oracle_easgd_round(float *W, const float *G, float *Wc,
                        int P, size_t N, size_t ld,
                        double eta, double rho, double center_coef)
{
    long long j;
#pragma omp parallel for schedule(static)
    for (j = 0; j < (long long)N; ++j) {
        const double c = (double)Wc[j];          /* Wc_t, seen by every worker */
        double sum_diff = 0.0;                   /* sum_i (W^i_t - Wc_t) */
        for (int i = 0; i < P; ++i) {
            const double w = (double)W[(size_t)i * ld + j];
            const double g = (double)G[(size_t)i * ld + j];
            const double diff = w - c;
            sum_diff += diff;
            W[(size_t)i * ld + j] = (float)(w - eta * (g + rho * diff));     /* Eq. (1) */
        }
        Wc[j] = (float)(c + center_coef * sum_diff);                         /* Eq. (2) */
    }
}

/* V: [P][ld] momentum buffers, in place. mu is the momentum rate. */
void oracle_measgd_round(float *W, float *V, const float *G, float *Wc,
                         int P, size_t N, size_t ld,
                         double eta, double rho, double mu, double center_coef)
{
    long long j;
#pragma omp parallel for schedule(static)
    for (j = 0; j < (long long)N; ++j) {
        const double c = (double)Wc[j];
        double sum_diff = 0.0;
        for (int i = 0; i < P; ++i) {
            const size_t k = (size_t)i * ld + j;
            const double w = (double)W[k];
            const double g = (double)G[k];
            const double diff = w - c;
            sum_diff += diff;
            /* Eq. (5); Eq. (6) uses V_{t+1} as it is stored, i.e. as an fp32 value */
            const float v_new = (float)(mu * (double)V[k] - eta * g);
            V[k] = v_new;
            W[k] = (float)(w + (double)v_new - eta * rho * diff);            /* Eq. (6) */
        }
        Wc[j] = (float)(c + center_coef * sum_diff);                         /* Eq. (2) */
    }
}

/*
 * Synchronous data-parallel SGD on P replicas that share one memory.
 *
 * Section 2.3 ("Data Parallelism"): the gradients of all workers are summed and the weights move by
 *     W_{t+1} = W_t - eta * sum_i dW^i_t ,
 * after which every worker holds the new W.  Section 6.2 (the partitioned chip) is the replicated form
 * of the same rule: every partition receives the gradient sum and updates its own copy of the weights.
 * With momentum the sum drives Eq. (3),(4):  V_{t+1} = mu * V_t - eta * sum_i dW^i_t ;  W_{t+1} = W_t + V_{t+1}.
 *
 * W, G (and V, or NULL for the plain rule): [P][ld], first N entries of a row valid.  In place on W and V.
 * The sum is taken over the workers in ascending order, in double.
 */
void oracle_sync_sgd_round(float *W, float *V, const float *G,
                           int P, size_t N, size_t ld, double eta, double mu)
{
    long long j;
#pragma omp parallel for schedule(static)
    for (j = 0; j < (long long)N; ++j) {
        double sum_g = 0.0;
        for (int i = 0; i < P; ++i) sum_g += (double)G[(size_t)i * ld + j];
        for (int i = 0; i < P; ++i) {
            const size_t k = (size_t)i * ld + j;
            if (V) {
                const float v_new = (float)(mu * (double)V[k] - eta * sum_g);     /* Eq. (3) */
                V[k] = v_new;
                W[k] = (float)((double)W[k] + (double)v_new);                      /* Eq. (4) */
            } else {
                W[k] = (float)((double)W[k] - eta * sum_g);
            }
        }
    }
}

/*
 * The master interacting with ONE worker at a time (Section 2.6, Algorithm 1 "Original EASGD", and Section 5.1
 * "Async EASGD" / "Async MEASGD").  For the worker j whose turn it is, the loop body of Algorithm 1 does, with the
 * weights W^j and the center Wc as they are when the turn starts:
 *     worker:  W^j  <- W^j - eta * ( dW^j + rho * (W^j - Wc) )                 Eq. (1)
 *              (with momentum, Eq. (5),(6):  V^j <- mu V^j - eta dW^j ;  W^j <- W^j + V^j - eta rho (W^j - Wc))
 *     master:  Wc   <- Wc + eta * rho * (W^j - Wc)                              the one-worker form of Eq. (2)
 * Both right-hand sides use the values from the start of the turn (the master fetches W^j before the worker
 * updates it).  Original EASGD takes the turns in rank order (j = t mod P), Async EASGD in the order in which the
 * workers arrive (first come, first served); either way the master serves one worker at a time, so a schedule
 * is a sequence of worker indices, given here as `order[0..n_order)`.  A worker may come up more than once; its
 * gradient row is used as it is each time.
 *
 * W, G (and V, or NULL for the plain rule): [P][ld], first N entries of a row valid; Wc: [N].  In place.
 * State is fp32, every right-hand side is evaluated in double and rounded once when stored (the center is
 * stored, i.e. rounded, after every turn: the next worker sees what is in memory).
 */
void oracle_async_easgd(float *W, float *V, const float *G, float *Wc,
                        int P, size_t N, size_t ld, const int *order, int n_order,
                        double eta, double rho, double mu, double center_coef)
{
    (void)P;
    for (int t = 0; t < n_order; ++t) {
        const int j = order[t];
        long long p;
#pragma omp parallel for schedule(static)
        for (p = 0; p < (long long)N; ++p) {
            const size_t k = (size_t)j * ld + (size_t)p;
            const double w = (double)W[k], c = (double)Wc[p], g = (double)G[k];
            const double diff = w - c;
            if (V) {
                const float v_new = (float)(mu * (double)V[k] - eta * g);           /* Eq. (5) */
                V[k] = v_new;
                W[k] = (float)(w + (double)v_new - eta * rho * diff);              /* Eq. (6) */
            } else {
                W[k] = (float)(w - eta * (g + rho * diff));                        /* Eq. (1) */
            }
            Wc[p] = (float)(c + center_coef * diff);                               /* Eq. (2), one worker */
        }
    }
}
