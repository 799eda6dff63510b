/* CPU oracle for the DropCompute batched step-time computation.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the checker the GPU library is compared
 * against; the library never links, loads or calls it.  It shares no code with the HIP
 * path and is written directly from the paper:
 *
 *   - completion time of micro-batch m on worker n: T_n^(m) = sum_{j<=m} t_n^(j)   (Section 4.3)
 *   - a micro-batch counts as completed iff T_n^(m) < tau (strict)                 (Section 4.3, M~ definition;
 *                                                                                    Algorithm 2 inner loop)
 *   - compute time of an iteration: T = max_n T_n^(M)                              (Section 4.2)
 *   - iteration time under a threshold: min{tau, T} + T^c                          (Section 4.3)
 *   - reduction over iterations and choice of tau                                  (Appendix C.1, Algorithm 2)
 *
 * Everything is int64 integer arithmetic on integer-microsecond latencies, so results are
 * exact and independent of summation order.  Outputs are un-normalised sums over trials:
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

/* The definition, loop for loop: thresholds, iterations, workers, micro-batches
 * (Appendix C.1, Algorithm 2), with the per-iteration quantities kept as integers. */
int dc_oracle_simulate_literal(const int32_t* lat, int64_t T, int64_t N, int64_t M,
                               const int64_t* taus, int64_t K, int64_t comm,
                               int64_t* step_sum, int64_t* done_sum) {
    int rc = check_args(lat, T, N, M, taus, K, comm, step_sum, done_sum);
    if (rc) return rc;
    if (has_negative(lat, T * N * M)) return DCO_ERR_NEGATIVE_LATENCY;
    for (int64_t k = 0; k < K; ++k) {
        const int64_t tau = taus[k];
        int64_t steps = 0, done = 0;
        for (int64_t i = 0; i < T; ++i) {
            int64_t completed = 0;          /* N * M~_i(tau) */
            int64_t slowest = 0;            /* T_i */
            for (int64_t n = 0; n < N; ++n) {
                const int32_t* t = lat + (i * N + n) * M;
                int64_t elapsed = 0;        /* T_{i,n} */
                for (int64_t m = 0; m < M; ++m) {
                    elapsed += t[m];
                    if (elapsed < tau) completed += 1;
                }
                if (elapsed > slowest) slowest = elapsed;
            }
            steps += (tau < slowest ? tau : slowest) + comm;
            done += completed;
        }
        step_sum[k] = steps;
        done_sum[k] = done;
    }
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

/* Algorithm 2 exactly as printed (Appendix C.1): for every threshold, the effective speedup of each
 * iteration, S_i(tau) = (T_i + T_i^c) / (min(tau, T_i) + T_i^c) * M~_i(tau) / M, with M~_i(tau) built up in
 * steps of 1/N, then the mean over the I iterations.  comm[i] is T_i^c (one value per iteration).
 * float64 throughout, as a direct reading of the listing's real-valued quantities.
 * Returns DCO_ERR_INVALID_ARG if some iteration has min(tau, T_i) + T_i^c = 0 (the ratio is undefined). */
int dc_oracle_per_step_speedup(const int32_t* lat, int64_t T, int64_t N, int64_t M,
                               const int64_t* taus, int64_t K, const int64_t* comm, double* s_eff) {
    if (T < 1 || N < 1 || M < 1 || K < 0 || !lat || !comm || (K > 0 && (!taus || !s_eff))) return DCO_ERR_INVALID_ARG;
    for (int64_t k = 0; k < K; ++k) if (taus[k] < 0) return DCO_ERR_INVALID_ARG;
    for (int64_t i = 0; i < T; ++i) if (comm[i] < 0) return DCO_ERR_INVALID_ARG;
    if (has_negative(lat, T * N * M)) return DCO_ERR_NEGATIVE_LATENCY;
    for (int64_t k = 0; k < K; ++k) {
        const int64_t tau = taus[k];
        double total = 0.0;
        for (int64_t i = 0; i < T; ++i) {
            double completed = 0.0;         /* M~_i(tau) */
            int64_t slowest = 0;            /* T_i */
            for (int64_t n = 0; n < N; ++n) {
                const int32_t* t = lat + (i * N + n) * M;
                int64_t elapsed = 0;        /* T_{i,n} */
                for (int64_t m = 0; m < M; ++m) {
                    elapsed += t[m];
                    if (elapsed < tau) completed += 1.0 / (double)N;
                }
                if (elapsed > slowest) slowest = elapsed;
            }
            const int64_t capped = tau < slowest ? tau : slowest;
            if (capped + comm[i] == 0) return DCO_ERR_INVALID_ARG;
            total += (double)(slowest + comm[i]) / (double)(capped + comm[i]) * completed / (double)M;
        }
        s_eff[k] = total / (double)T;
    }
    return DCO_OK;
}
