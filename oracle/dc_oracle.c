/* CPU oracle for the DropCompute batched step-time computation.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the checker the GPU library is compared
 * against; the library never links, loads or calls it.  It shares no code with the HIP
 * path and is written from the paper's definitions:
 *
 *   - completion time of micro-batch m on worker n: T_n^(m) = sum_{j<=m} t_n^(j)   (Section 4.3)
 *   - a micro-batch counts as completed iff T_n^(m) < tau (strict)                 (Section 4.3, M~ definition;
 *                                                                                    Algorithm 2, Appendix C.1)
 *   - compute time of an iteration: T = max_n T_n^(M)                              (Section 4.2)
 *   - iteration time under a threshold: min{tau, T} + T^c                          (Section 4.3)
 *   - effective speedup of one iteration, S = M~ (T + T^c) / (M (min{tau,T} + T^c)) (Section 4.4, eq:auto_eff)
 *   - reduction over iterations and choice of tau                                  (Appendix C.1, Algorithm 2)
 *
 * Counts, completion times and step times are int64 integer arithmetic on integer-microsecond
 * latencies, so they are exact and independent of summation order.  Integer outputs are
 * un-normalised sums over trials:
 *   step_sum[k] = sum_i ( min(tau_k, T_i) + comm )
 *   done_sum[k] = sum_i sum_n #{ m : T_{i,n}^(m) < tau_k }       ( = N * sum_i M~_i(tau_k) )
 *
 * Pinned by tests/test_oracle_pins.py (hand-worked example, closed forms, brute force,
 * invariants).
 */
#include <stdint.h>
#include <stdlib.h>

enum { DCO_OK = 0, DCO_ERR_INVALID_ARG = 1, DCO_ERR_NEGATIVE_LATENCY = 2 };

static int check_args(const int32_t* lat, int64_t T, int64_t N, int64_t M, const int64_t* taus, int64_t K,
                      int64_t comm, const int64_t* a, const int64_t* b) {
    if (T < 1 || N < 1 || M < 1 || K < 0 || comm < 0) return DCO_ERR_INVALID_ARG;
    if (!lat || (K > 0 && (!taus || !a || !b))) return DCO_ERR_INVALID_ARG;
    for (int64_t k = 0; k < K; ++k) if (taus[k] < 0) return DCO_ERR_INVALID_ARG;
    return DCO_OK;
}

static int has_negative(const int32_t* lat, int64_t count) {
    for (int64_t i = 0; i < count; ++i) if (lat[i] < 0) return 1;
    return 0;
}

/* Completion times T_n^(m), m = 1..M, of one worker in one iteration (Section 4.3); returns T_n = T_n^(M). */
static int64_t completion_times(const int32_t* t, int64_t M, int64_t* out) {
    int64_t elapsed = 0;
    for (int64_t m = 0; m < M; ++m) {
        elapsed += t[m];
        out[m] = elapsed;
    }
    return elapsed;
}

/* How many of a worker's completion times lie strictly below tau (Section 4.3, the indicator inside M~). */
static int64_t completed_below(const int64_t* done_at, int64_t M, int64_t tau) {
    int64_t count = 0;
    for (int64_t m = 0; m < M; ++m) count += done_at[m] < tau;
    return count;
}

/* The definition, every (iteration, worker, micro-batch, threshold) combination evaluated: O(K*T*N*M).
 * Per iteration: every worker's completion times, the count of those below each threshold summed over the
 * workers (N * M~(tau), Section 4.3), the slowest worker's total (Section 4.2), and the step time
 * min{tau, T} + T^c (Section 4.3). */
int dc_oracle_simulate_literal(const int32_t* lat, int64_t T, int64_t N, int64_t M,
                               const int64_t* taus, int64_t K, int64_t comm,
                               int64_t* step_sum, int64_t* done_sum) {
    int rc = check_args(lat, T, N, M, taus, K, comm, step_sum, done_sum);
    if (rc) return rc;
    if (has_negative(lat, T * N * M)) return DCO_ERR_NEGATIVE_LATENCY;
    int64_t* done_at = (int64_t*)malloc((size_t)M * sizeof(int64_t));
    if (!done_at) return DCO_ERR_INVALID_ARG;
    for (int64_t k = 0; k < K; ++k) step_sum[k] = done_sum[k] = 0;
    for (int64_t i = 0; i < T; ++i) {
        int64_t slowest = 0;                                        /* T = max_n T_n */
        for (int64_t n = 0; n < N; ++n) {
            const int64_t total = completion_times(lat + (i * N + n) * M, M, done_at);
            if (total > slowest) slowest = total;
            for (int64_t k = 0; k < K; ++k) done_sum[k] += completed_below(done_at, M, taus[k]);
        }
        for (int64_t k = 0; k < K; ++k) step_sum[k] += (taus[k] < slowest ? taus[k] : slowest) + comm;
    }
    free(done_at);
    return DCO_OK;
}

/* Same result in O(T*N*(M+K)) for large inputs: thresholds sorted once; per worker the
 * completion times are non-decreasing (latencies >= 0), so one forward walk over both
 * sorted lists gives, for every threshold, how many completion times lie below it.
 * Must equal dc_oracle_simulate_literal bit for bit (tests/test_oracle_pins.py). */
typedef struct { int64_t tau; int64_t pos; } tau_entry;

static int cmp_tau(const void* x, const void* y) {
    const tau_entry* a = (const tau_entry*)x; const tau_entry* b = (const tau_entry*)y;
    if (a->tau != b->tau) return a->tau < b->tau ? -1 : 1;
    return a->pos < b->pos ? -1 : (a->pos > b->pos ? 1 : 0);
}

int dc_oracle_simulate_sorted(const int32_t* lat, int64_t T, int64_t N, int64_t M,
                              const int64_t* taus, int64_t K, int64_t comm,
                              int64_t* step_sum, int64_t* done_sum) {
    int rc = check_args(lat, T, N, M, taus, K, comm, step_sum, done_sum);
    if (rc) return rc;
    if (has_negative(lat, T * N * M)) return DCO_ERR_NEGATIVE_LATENCY;
    if (K == 0) return DCO_OK;
    tau_entry* order = (tau_entry*)malloc((size_t)K * sizeof(tau_entry));
    int64_t* done_sorted = (int64_t*)calloc((size_t)K, sizeof(int64_t));
    int64_t* step_sorted = (int64_t*)calloc((size_t)K, sizeof(int64_t));
    if (!order || !done_sorted || !step_sorted) { free(order); free(done_sorted); free(step_sorted); return DCO_ERR_INVALID_ARG; }
    for (int64_t k = 0; k < K; ++k) { order[k].tau = taus[k]; order[k].pos = k; }
    qsort(order, (size_t)K, sizeof(tau_entry), cmp_tau);

    for (int64_t i = 0; i < T; ++i) {
        int64_t slowest = 0;
        for (int64_t n = 0; n < N; ++n) {
            const int32_t* t = lat + (i * N + n) * M;
            int64_t elapsed = 0;
            int64_t k = 0;                  /* thresholds order[0..k) are <= elapsed */
            for (int64_t m = 0; m < M; ++m) {
                elapsed += t[m];
                /* thresholds passed by this completion time were beaten by exactly m micro-batches */
                while (k < K && order[k].tau <= elapsed) { done_sorted[k] += m; ++k; }
            }
            for (; k < K; ++k) done_sorted[k] += M;   /* threshold above the worker's total */
            if (elapsed > slowest) slowest = elapsed;
        }
        for (int64_t k = 0; k < K; ++k)
            step_sorted[k] += (order[k].tau < slowest ? order[k].tau : slowest) + comm;
    }
    for (int64_t k = 0; k < K; ++k) {
        step_sum[order[k].pos] = step_sorted[k];
        done_sum[order[k].pos] = done_sorted[k];
    }
    free(order); free(done_sorted); free(step_sorted);
    return DCO_OK;
}

/* Effective speedup per iteration, summed over the iterations given (Section 4.4, eq:auto_eff, applied to each
 * iteration as Algorithm 2 of Appendix C.1 does; the caller divides by the number of iterations for the mean):
 *   S_i(tau) = M~_i(tau) (T_i + T_i^c) / (M (min{tau, T_i} + T_i^c)),
 *   M~_i(tau) = (1/N) sum_n #{ m : T_{i,n}^(m) < tau }          (Section 4.3),   T_i = max_n T_{i,n}   (Section 4.2).
 * The count is an exact integer, divided once; the ratio and the sum over iterations are float64, iterations
 * added in order.  comm[i] is T_i^c (one value per iteration).
 * Returns DCO_ERR_INVALID_ARG if some iteration has min(tau, T_i) + T_i^c = 0 (the ratio is undefined). */
int dc_oracle_per_step_speedup_sums(const int32_t* lat, int64_t T, int64_t N, int64_t M,
                                    const int64_t* taus, int64_t K, const int64_t* comm, double* s_sum) {
    if (T < 1 || N < 1 || M < 1 || K < 0 || !lat || !comm || (K > 0 && (!taus || !s_sum))) return DCO_ERR_INVALID_ARG;
    for (int64_t k = 0; k < K; ++k) if (taus[k] < 0) return DCO_ERR_INVALID_ARG;
    for (int64_t i = 0; i < T; ++i) if (comm[i] < 0) return DCO_ERR_INVALID_ARG;
    if (has_negative(lat, T * N * M)) return DCO_ERR_NEGATIVE_LATENCY;
    int64_t* done_at = (int64_t*)malloc((size_t)(N * M) * sizeof(int64_t));      /* one iteration's completion times */
    if (!done_at) return DCO_ERR_INVALID_ARG;
    for (int64_t k = 0; k < K; ++k) s_sum[k] = 0.0;
    int status = DCO_OK;
    for (int64_t i = 0; i < T && status == DCO_OK; ++i) {
        int64_t slowest = 0;
        for (int64_t n = 0; n < N; ++n) {
            const int64_t total = completion_times(lat + (i * N + n) * M, M, done_at + n * M);
            if (total > slowest) slowest = total;
        }
        for (int64_t k = 0; k < K; ++k) {
            const int64_t tau = taus[k];
            const int64_t step = (tau < slowest ? tau : slowest) + comm[i];
            if (step == 0) { status = DCO_ERR_INVALID_ARG; break; }
            const int64_t completed = completed_below(done_at, N * M, tau);      /* N * M~_i(tau) */
            const double m_tilde = (double)completed / (double)N;
            s_sum[k] += m_tilde * (double)(slowest + comm[i]) / ((double)M * (double)step);
        }
    }
    free(done_at);
    return status;
}
