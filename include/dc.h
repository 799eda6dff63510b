/* dc.h - C ABI of the DropCompute batched step-time simulator for AMD MI355X (gfx950).
 *
 * What is computed (DropCompute, arXiv 2306.10598):
 *   lat[t][n][m]  compute latency of micro-batch m on worker n in iteration ("trial") t,
 *                 the samples t_{i,n}^{(m)} that Algorithm 2 (Appendix C.1) takes as input;
 *   P[t][n][m]  = sum_{j<=m} lat[t][n][j], the completion time T_n^{(m)} (Section 4.3);
 *   a micro-batch is completed under threshold tau iff P < tau, strictly (Section 4.3,
 *                 definition of M~; Algorithm 2, inner loop);
 *   Tmax[t]     = max_n P[t][n][M-1], the iteration's compute time T (Section 4.2);
 *   step time   = min{tau, Tmax[t]} + comm, comm = T^c, the serial latency that includes
 *                 the all-reduce (Section 4.3);
 *   the reduction over iterations and the choice of tau follow Section 4.4 and the last
 *   lines of Algorithm 2.
 *
 * Units are integer microseconds; every sum is an exact integer, so results do not depend
 * on the order of accumulation.
 *
 * General conventions
 *   - Every function returns a dc_status (0 = DC_OK).  Nothing throws or aborts across this
 *     boundary.  On any status other than DC_OK the output buffers hold unspecified values.
 *   - Every pointer is owned by the caller.  "DEVICE" pointers are HIP device memory of the
 *     current device; "HOST" pointers are ordinary host memory.
 *   - lat must be 4-byte aligned; rows are contiguous with m fastest: element (t,n,m) is at
 *     lat[(t*N + n)*M + m].  The fastest kernels need lat 16-byte aligned and either M a multiple of 4
 *     up to 128, or 256 (best when M is a power of two), or M <= 16 with a multiple of 4 rows in all,
 *     or M <= 63 with N*M a multiple of 4 and at least 32 workers; every other M >= 1 and any 4-byte
 *     alignment takes a kernel that reads the tensor as one flat run of 16-byte vectors, with the same
 *     results at 75-90 % of that speed.
 *   - Preconditions on values, checked while streaming: every latency is >= 0
 *     (else DC_ERR_NEGATIVE_LATENCY) and <= floor((2^31-1)/M) (else DC_ERR_RANGE), which
 *     guarantees that no worker's total overflows 31 bits.
 *   - Thresholds: 0 <= tau (else DC_ERR_INVALID_ARG), any order, duplicates allowed; a
 *     threshold >= 2^31 is above every possible completion time.  1 <= T, N, M;
 *     0 <= K <= DC_MAX_THRESHOLDS (K = 0 does nothing and returns DC_OK); comm >= 0;
 *     T*N*M < 2^62.
 */
#ifndef DC_H
#define DC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DC_OK = 0,
    DC_ERR_INVALID_ARG = 1,       /* null pointer, size out of range, negative tau or comm, workspace too small */
    DC_ERR_NEGATIVE_LATENCY = 2,  /* some lat < 0 */
    DC_ERR_RANGE = 3,             /* some lat > floor((2^31-1)/M) */
    DC_ERR_DEVICE = 4,            /* a HIP call failed (see dc_last_device_error) */
    DC_ERR_NOMEM = 5              /* device or host allocation failed */
} dc_status;

#define DC_MAX_THRESHOLDS 65536

/* Step-time and completed-micro-batch sums for K thresholds (Sections 4.2-4.3; the loops of
 * Algorithm 2 with the per-iteration quantities kept as integers):
 *   out_step[k] = sum_t ( min(taus[k], Tmax[t]) + comm )
 *   out_done[k] = sum_t sum_n #{ m : P[t][n][m] < taus[k] }      ( = N * sum_t M~_t(taus[k]) )
 * lat: DEVICE, int32 [T][N][M], read only.  taus: HOST, K int64.  out_step, out_done: HOST,
 * K int64 each, in the caller's threshold order.
 * Runs on the null stream of the current device and returns after the results are on the
 * host.  Uses a workspace that the library allocates on first use, keeps per process and
 * grows when needed (dc_shutdown frees it); the synchronous entry points share it, so calls of theirs from
 * several threads are serialised.  The *_async entry points and dc_simulate_static hold no lock while they
 * enqueue and may be called from several threads at once, each call with a workspace of its own. */
int dc_simulate(const int32_t* lat, int64_t T, int64_t N, int64_t M,
                const int64_t* taus, int64_t K, int64_t comm,
                int64_t* out_step, int64_t* out_done);

/* Bytes of DEVICE workspace that dc_simulate_async needs for these sizes (0 if they are invalid). */
size_t dc_workspace_bytes(int64_t T, int64_t N, int64_t M, int64_t K);

/* Same computation, enqueued on `stream` (a hipStream_t passed as void*; NULL = null stream)
 * without synchronising and without allocating.  taus_dev, out_step_dev, out_done_dev: DEVICE,
 * K int64 each; the two outputs may also be pinned host memory that the device can write (hipHostMalloc): the
 * last kernel then delivers the sums without a separate copy, valid once the stream has been waited for.  workspace_dev: DEVICE, 256-byte aligned, at least dc_workspace_bytes(T,N,M,K)
 * bytes, contents irrelevant on entry; it must not be used by another call until this one has
 * finished on the stream.  The return value covers only what the host can check (arguments,
 * launch errors); value errors found on the device (negative tau, negative or too large
 * latency) are recorded in the workspace and read back with dc_workspace_status. */
int dc_simulate_async(const int32_t* lat, int64_t T, int64_t N, int64_t M,
                      const int64_t* taus_dev, int64_t K, int64_t comm,
                      int64_t* out_step_dev, int64_t* out_done_dev,
                      void* workspace_dev, size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory or carry a workspace around (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): dc_simulate_async with the workspace
 * replaced by a fixed array of DC_STATIC_SCRATCH_BYTES that is part of the library's device code (one per
 * GPU, held until the process ends).  The call allocates nothing, on the device or on the host, and never
 * synchronises.  lat, taus_dev, out_step_dev, out_done_dev, stream: as for dc_simulate_async.
 * out_status_dev: DEVICE, one int32, may be NULL; when the work has finished on the stream it holds the
 * dc_status of the value checks made on the device (DC_OK, DC_ERR_INVALID_ARG for a negative threshold,
 * DC_ERR_NEGATIVE_LATENCY, DC_ERR_RANGE).
 * Sizes whose workspace (dc_workspace_bytes) exceeds DC_STATIC_SCRATCH_BYTES are refused with
 * DC_ERR_INVALID_ARG before anything is enqueued (dc_last_device_error says how much was needed); the five
 * workloads of the benchmark need up to 12.1 MB, and a pass with 4095 thresholds needs 33 MB and is refused.
 * Every call on one GPU uses that GPU's array and starts by clearing what it needs cleared: calls on one GPU
 * whose work overlaps in time (two streams, or two threads) race on it and give wrong results; calls that
 * follow one another on a stream are fine.  The first call on a device looks up the array's address, which
 * must not happen while a stream is being captured: call once eagerly before capturing. */
#define DC_STATIC_SCRATCH_BYTES (16u << 20)
int dc_simulate_static(const int32_t* lat, int64_t T, int64_t N, int64_t M,
                       const int64_t* taus_dev, int64_t K, int64_t comm,
                       int64_t* out_step_dev, int64_t* out_done_dev, int32_t* out_status_dev, void* stream);

/* The same two calls for a tensor whose trials are not adjacent: element (t,n,m) is at
 * lat[t*trial_stride + n*M + m], trial_stride >= N*M elements (else DC_ERR_INVALID_ARG).  This is how the first
 * N' of N workers of a resident tensor [T][N][M] are simulated without a copy (lat, N', trial_stride = N*M), or
 * the workers n0 .. n0+N'-1 (lat + n0*M): the slab of the latency samples that one worker group holds before the
 * one-time synchronisation of Section 4.4, and the way a scale sweep over the number of workers reads one tensor.
 * Everything else as dc_simulate / dc_simulate_async; dc_workspace_bytes(T, N, M, K) bytes of workspace suffice.
 * Trials that do not start on 16-byte boundaries (trial_stride not a multiple of 4) take the kernel for any alignment. */
int dc_simulate_strided(const int32_t* lat, int64_t T, int64_t N, int64_t M, int64_t trial_stride,
                        const int64_t* taus, int64_t K, int64_t comm, int64_t* out_step, int64_t* out_done);
int dc_simulate_strided_async(const int32_t* lat, int64_t T, int64_t N, int64_t M, int64_t trial_stride,
                              const int64_t* taus_dev, int64_t K, int64_t comm,
                              int64_t* out_step_dev, int64_t* out_done_dev,
                              void* workspace_dev, size_t workspace_bytes, void* stream);

/* Waits for `stream` and returns the dc_status that the last dc_simulate_async using
 * workspace_dev recorded on the device (DC_OK, DC_ERR_INVALID_ARG for a negative threshold,
 * DC_ERR_NEGATIVE_LATENCY, DC_ERR_RANGE) or DC_ERR_DEVICE if the stream reports an error. */
int dc_workspace_status(const void* workspace_dev, void* stream);

/* Throughput, effective speedup and the best threshold (Section 4.4; Algorithm 2, last line).
 * HOST only, no GPU work.  Inputs are dc_simulate's outputs for the same taus, T, N, M.
 *   out_thr[k]  = done_sum[k] / step_sum[k]       completed micro-batches per microsecond over all
 *                                                 workers, N*M~/(min{tau,T}+T^c) with iteration means
 *   out_seff[k] = out_thr[k] * base_step_sum / (T*N*M)   S_eff(tau_k): ratio to the no-drop
 *                 throughput N*M/(T+T^c); base_step_sum = sum_t (Tmax[t] + comm), i.e. out_step
 *                 of any threshold above every worker total.  With base_step_sum = 0 the
 *                 S_eff values are NaN.
 *   *out_best_k = argmax_k out_thr[k], decided exactly by 128-bit integer cross-multiplication;
 *                 among exact ties the largest tau wins (fewest dropped micro-batches), then the
 *                 lowest index.
 * out_thr and out_seff may be NULL.  K >= 1 and every step_sum[k] > 0, else DC_ERR_INVALID_ARG. */
int dc_select_tau(const int64_t* step_sum, const int64_t* done_sum, const int64_t* taus, int64_t K,
                  int64_t T, int64_t N, int64_t M, int64_t base_step_sum,
                  double* out_thr, double* out_seff, int64_t* out_best_k);

/* Effective speedup exactly as Algorithm 2 (Appendix C.1) prints it: the mean over iterations of the
 * per-iteration ratio
 *   S_t(tau) = (Tmax[t] + c_t) / (min(tau, Tmax[t]) + c_t) * done_t(tau) / (N*M),
 *   done_t(tau) = sum_n #{ m : P[t][n][m] < tau },          out_seff[k] = (1/T) sum_t S_t(taus[k]),
 * with c_t = comm_per_trial[t] (the listing's per-iteration T_i^c) or, when comm_per_trial is NULL, the
 * constant comm.  float64; the sum over iterations is taken in a fixed order, so repeated calls give
 * identical bits.  (dc_select_tau's S_eff is the ratio of iteration means instead; the two differ by a
 * covariance term of order N^-1/2, Appendix C.2.)
 * lat: DEVICE int32 [T][N][M].  taus: HOST K int64.  comm_per_trial: HOST T int64 (each >= 0) or NULL.
 * out_seff: HOST K doubles, caller's threshold order.  Extra preconditions: N*M < 2^31, and
 * min(tau, Tmax[t]) + c_t > 0 for every iteration and threshold (else DC_ERR_INVALID_ARG: the ratio is
 * undefined).  Same stream, workspace caching and error rules as dc_simulate. */
int dc_speedup_per_step(const int32_t* lat, int64_t T, int64_t N, int64_t M,
                        const int64_t* taus, int64_t K, int64_t comm, const int64_t* comm_per_trial,
                        double* out_seff);

/* The best threshold under Algorithm 2's own convention (Appendix C.1, last line): tau* = argmax_tau S_eff(tau)
 * with S_eff the mean of per-iteration speedups, i.e. dc_speedup_per_step's output.  HOST only, no GPU work.
 * seff, taus: HOST, K values each (same order).  *out_best_k = index of the largest seff; among equal values the
 * largest tau wins (fewest dropped micro-batches: every threshold above all worker totals gives exactly 1), then
 * the lowest index, the same rule as dc_select_tau.  K >= 1, no NaN, taus >= 0, else DC_ERR_INVALID_ARG. */
int dc_select_tau_per_step(const double* seff, const int64_t* taus, int64_t K, int64_t* out_best_k);

/* Bytes of DEVICE workspace that dc_speedup_per_step_async needs (0 if the sizes are invalid). */
size_t dc_speedup_workspace_bytes(int64_t T, int64_t N, int64_t M, int64_t K);

/* Same, enqueued on `stream` without synchronising or allocating.  taus_dev: DEVICE K int64;
 * comm_per_trial_dev: DEVICE T int64 or NULL; out_seff_dev: K doubles in any memory the device can write
 * (device memory, or pinned host memory: the last kernel then delivers the result without a copy);
 * workspace as for dc_simulate_async (at least dc_speedup_workspace_bytes bytes); device-side value
 * errors are read back with dc_workspace_status. */
int dc_speedup_per_step_async(const int32_t* lat, int64_t T, int64_t N, int64_t M,
                              const int64_t* taus_dev, int64_t K, int64_t comm,
                              const int64_t* comm_per_trial_dev, double* out_seff_dev,
                              void* workspace_dev, size_t workspace_bytes, void* stream);

/* Exact first and second moments of all T*N*M latencies (one streaming pass): the mu and sigma^2 of a single
 * micro-batch that the closed forms of Sections 4.2-4.3 take (one distribution for all workers, Appendix C.2,
 * first assumption; population variance).
 *   *out_sum = sum lat;  out_sumsq[0], out_sumsq[1] = low and high 64 bits of sum lat^2 (exact integers);
 *   *out_mean = sum / n;  *out_variance = (sumsq*n - sum^2) / n^2,  n = T*N*M.
 * lat: DEVICE.  All outputs HOST, each may be NULL.  DC_ERR_NEGATIVE_LATENCY if some lat < 0.  The sum is kept in
 * 64 bits: DC_ERR_RANGE when n times the bitwise OR of all latencies (an upper bound of the largest) reaches 2^63,
 * i.e. when it cannot be shown that the sum stayed below 2^63 (never for n <= 2^32).
 * Null stream, synchronous, cached workspace as dc_simulate. */
int dc_moments(const int32_t* lat, int64_t T, int64_t N, int64_t M,
               int64_t* out_sum, uint64_t* out_sumsq, double* out_mean, double* out_variance);

/* Per-worker statistics of the compute time T_n = sum_m lat[t][n][m] over the T iterations (one streaming pass):
 * the empirical mean and variance of each worker's iteration time, from which the paper's iteration-time figure
 * redraws every T_n from a normal distribution (Section 4.3, "simulation" curve).  For worker n:
 *   out_sum[n] = sum_t T_n;  out_sumsq[2n], out_sumsq[2n+1] = low and high 64 bits of sum_t T_n^2 (exact);
 *   out_mean[n] = sum / T;   out_variance[n] = (sumsq*T - sum^2) / T^2  (population variance).
 * lat: DEVICE.  Outputs HOST arrays of N (out_sumsq: 2N), each may be NULL.  The accumulators live in LDS, 2560
 * workers at a time: more workers take one pass over their rows of lat per 2560.  Latency preconditions and errors
 * as dc_simulate.  Null stream, synchronous, cached workspace.
 * dc_worker_moments_strided: trials trial_stride >= N*M elements apart, as dc_simulate_strided. */
int dc_worker_moments(const int32_t* lat, int64_t T, int64_t N, int64_t M,
                      int64_t* out_sum, uint64_t* out_sumsq, double* out_mean, double* out_variance);
int dc_worker_moments_strided(const int32_t* lat, int64_t T, int64_t N, int64_t M, int64_t trial_stride,
                              int64_t* out_sum, uint64_t* out_sumsq, double* out_mean, double* out_variance);

/* Closed-form estimates from (mu, sigma2) of one micro-batch latency (Sections 4.2-4.4, Appendix C.2):
 *   out_edone[k] = sum_{m=1..M} Phi((taus[k] - m*mu) / sqrt(m*sigma2))     expected completed micro-batches per
 *                  worker, the CLT estimate of M~ (Section 4.3); for sigma2 = 0 the count #{m : m*mu < tau}
 *   *out_et      = sqrt(M*sigma2) * ((1-g)*PhiInv(1 - 1/N) + g*PhiInv(1 - 1/(e*N))) + M*mu, g = Euler's constant:
 *                  expected compute time of the slowest of N workers (Section 4.2; without T^c; needs N >= 2)
 *   out_seff[k]  = out_edone[k]/M * (ET + comm) / (min(taus[k], ET) + comm)  Section 4.4's S_eff with the
 *                  estimates plugged in, where ET = mean_tmax if mean_tmax >= 0 (the measured mean iteration
 *                  time: "analytical given E[T]" of Appendix C.2), else *out_et.  comm is added to ET in the
 *                  numerator because T = max_n T_n excludes T^c in Sections 4.2-4.4.
 *   *out_best_k  = argmax_k out_edone[k] / (taus[k] + comm)                  Appendix C.2, "Finding tau*";
 *                  exact float ties go to the largest tau, then the lowest index
 * The sum over m runs on the GPU (fixed order); everything else is O(K) host arithmetic.  taus: HOST, K int64 >= 0.
 * out_edone: HOST K doubles (required if K > 0); out_seff, out_et, out_best_k may be NULL.
 * mu >= 0, sigma2 >= 0 finite; N >= 2; else DC_ERR_INVALID_ARG. */
int dc_analytic_curves(double mu, double sigma2, int64_t N, int64_t M, const int64_t* taus, int64_t K,
                       int64_t comm, double mean_tmax,
                       double* out_edone, double* out_seff, double* out_et, int64_t* out_best_k);

/* Optional kernel timing for benchmarks.  enable = 1: every entry point that streams lat brackets its
 * streaming kernel (the single pass over lat) with HIP events on the stream it runs on; enable = 2:
 * also the whole enqueued sequence (two more event records per call); 0: off.  The setting is per process; the
 * events belong to the workspace a call runs in (the library's own for the synchronous entry points), so calls on
 * different streams, each with its own workspace, are timed independently (up to 16 workspaces are remembered).
 * dc_workspace_kernel_ms waits for the events of the last timed call in workspace_dev and returns the elapsed
 * milliseconds (scan_ms: streaming kernel(s) only; total_ms: all kernels of the call, needs enable = 2);
 * dc_last_kernel_ms does the same for the calling thread's last timed call.  Either pointer may be NULL.
 * DC_ERR_INVALID_ARG if the requested timing is off or no such call has been timed.  Leave timing off while a
 * stream is being captured into a graph (event records would become graph nodes whose times cannot be read back). */
int dc_set_kernel_timing(int enable);
int dc_last_kernel_ms(float* scan_ms, float* total_ms);
int dc_workspace_kernel_ms(const void* workspace_dev, float* scan_ms, float* total_ms);

/* Name of a status code; a static string, never NULL. */
const char* dc_status_string(int status);

/* Text of the last HIP error that made a call in this thread return DC_ERR_DEVICE or
 * DC_ERR_NOMEM ("" if none).  Static storage, valid until the next failing call. */
const char* dc_last_device_error(void);

/* What the current device reports about itself, for a benchmark that states the roofline it measures against (the
 * memory roofline of Section 8 of this library's measurements is bytes per second, so clock and bus width are what a
 * reader needs to check the peak figure): compute units, memory clock in kHz, memory bus width in bits, L2 size in
 * bytes.  Any pointer may be NULL.  DC_ERR_DEVICE if a query fails. */
int dc_device_info(int32_t* compute_units, int32_t* memory_clock_khz, int32_t* memory_bus_bits, int32_t* l2_bytes);

/* Frees everything the library holds (cached workspace, events).  Safe to call twice. */
void dc_shutdown(void);

#ifdef __cplusplus
}
#endif
#endif /* DC_H */
