// Shared between dc_api.hip (host logic, C ABI) and the translation units with the kernels and their launchers
// (dc_kernels.hip, dc_rows.hip, dc_rows_long.hip, dc_trial.hip, dc_workers.hip, dc_analytic.hip).
#ifndef DC_INTERNAL_H
#define DC_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

// Tuning knobs of the streaming kernel (overridable at build time with -D).
#ifndef DC_SCAN_THREADS
#define DC_SCAN_THREADS 256
#endif
#ifndef DC_SCAN_UNROLL
#define DC_SCAN_UNROLL 8                // 16-byte loads in flight per lane
#endif
#ifndef DC_FLAT_UNROLL
#define DC_FLAT_UNROLL 4                // the same for the kernel of arbitrary row lengths
#endif
#ifndef DC_FLAT_UNIT_ELEMENTS
#define DC_FLAT_UNIT_ELEMENTS 16384u    // target elements per unit of that kernel (whole rows, at least one)
#endif
#ifndef DC_UNIT_RUN
#define DC_UNIT_RUN 64u                 // units per run (power of two); halved while the tensor has too few runs for the grid
#endif
#ifndef DC_DENSE_LANES
#define DC_DENSE_LANES 48u              // lanes per load inside the threshold grid from which long rows are binned without the queue
#endif
#ifndef DC_DENSE_PERMILLE
#define DC_DENSE_PERMILLE 180u          // share of completion times inside the grid (per mille, sampled) from which
#endif                                  // long rows are streamed with DC_DENSE_BLOCKS_PER_CU blocks per compute unit
#ifndef DC_DENSE_BLOCKS_PER_CU
#define DC_DENSE_BLOCKS_PER_CU 3
#endif
#ifndef DC_LANE_ROWS_MIN_N
#define DC_LANE_ROWS_MIN_N 256u         // workers per trial from which short rows are streamed with whole rows per lane
#endif
#ifndef DC_ROWS_UNITS_PER_WAVE
#define DC_ROWS_UNITS_PER_WAVE 1ull     // the kernel with whole rows per lane: units are shortened until a wave gets this many (8: 7-10 % slower on 512 MB)
#endif
#define DC_LDS_BYTES (160u * 1024u)      // LDS of a compute unit (gfx950): the most one block can ask for
#define DC_ROWS_SHORT_MAX 12u            // row lengths up to this are built in dc_rows.hip, longer ones in dc_rows_long.hip
#ifndef DC_WAVE_TRIAL_ELEMENTS
#define DC_WAVE_TRIAL_ELEMENTS 16384u   // per-iteration pass: trials of up to this many latencies are taken by single waves
#endif
#define DC_WAVE_TRIAL_THRESHOLDS 511u   // ... when one pass holds every threshold with the waves' own histograms in LDS
#ifndef DC_SPAN_TRIALS
#define DC_SPAN_TRIALS 1                // short rows of few workers: stream the tensor as one run of rows (0: never)
#endif
#ifndef DC_ROWS_PREFETCH_MAX_V
#define DC_ROWS_PREFETCH_MAX_V 8        // rows of up to this many elements: the next chunk's loads are in flight during a chunk's arithmetic
#endif
#define DC_SAMPLE_ROWS 32               // rows of lat that the sample reads (a multiple of 4: a quarter per wave)
#ifndef DC_MAX_SCAN_BLOCKS
#define DC_MAX_SCAN_BLOCKS 2048u        // upper bound of the grid (sizes the per-block histograms in the workspace)
#endif
#define DC_SCAN_WAVES (DC_SCAN_THREADS / 64)
#define DC_REDUCE_TRIAL_BLOCKS 256u     // at most this many blocks of the reduce kernel bin the per-trial maxima
#define DC_REDUCE_SLOTS 64u             // per-block histograms added by one block of the reduce kernel
#define DC_CHUNK_THRESHOLDS 4095u      // thresholds handled by one pass over lat (LDS-resident grid)
#define DC_TRIAL_CHUNK_THRESHOLDS 2047u // same for the per-iteration speedup pass (it also keeps float64 sums in LDS)
#define DC_MAX_TRIAL_BLOCKS 2048u      // upper bound of that pass's grid (sizes its per-block sums in the workspace)
#define DC_MAX_STAT_WORKERS 2560u        // per-worker statistics keep 24 bytes per worker in LDS
#define DC_ROWS_ODD_MAX 17u             // longest odd row of which a lane holds four in registers, and the longest row of
#define DC_ROWS_EVEN_MAX 30u            // 4k+2 elements of which it holds two (the instantiations of dc_scan_rows_kernel)
#define DC_ROW_LANE_MIN_M 17u           // shortest row of the kernel with one row per lane ...
#define DC_ROW_LANE_MIN_M_MANY 25u      // ... with 256 workers or more (shorter ones are kernel 3's or stream faster in the flat pass)
#define DC_ROW_LANE_MAX_M 63u           // longest row of the kernel with one row per lane (16 KiB of LDS per wave)
#define DC_ROW_LANE_MIN_N 32u           // fewer workers leave most of a wave's 64 rows empty
#define DC_TAU_CLAMP 0x80000000u       // thresholds at or above 2^31 exceed every completion time

#define DC_FLAG_NEGATIVE_TAU 1u
#define DC_FLAG_NEGATIVE_LATENCY 2u
#define DC_FLAG_RANGE 4u
#define DC_FLAG_ZERO_STEP 8u             // some iteration has min(tau, Tmax) + comm = 0 (per-iteration speedup undefined)

namespace dc {

// row lengths that kernel is built for
// (rows of 12 and 16 elements only over trials of few workers: with long delays in the data the kernel with whole rows
// per load streams them 10-35 % faster, without them 5 % slower)
inline bool lane_rows_length(uint32_t M) {
    return (M <= 15u && M != 12u) || ((M & 1u) && M <= DC_ROWS_ODD_MAX) || ((M & 3u) == 2u && M <= DC_ROWS_EVEN_MAX);
}
// longer rows that are no multiple of 4: one row per lane, read word by word from the wave's copy of the chunk in LDS
inline bool row_lane_length(uint32_t M) { return M >= DC_ROW_LANE_MIN_M && M <= DC_ROW_LANE_MAX_M && (M & 3u) != 0u; }

// Rows that one wave of the kernels with whole rows per lane takes at a time (a chunk): a lane holds 16 rows of one
// element, 8 of two, otherwise 4 (2 of the longer even rows); one_row: the kernel in which it holds one.
inline uint32_t lane_rows_chunk_rows(uint32_t M, bool one_row) {
    if (one_row) return 64u;
    return M == 1u ? 1024u : M == 2u ? 512u : (M > 16u && (M & 3u) == 2u) ? 128u : 256u;
}
// 16-byte vectors that a lane holds per chunk when they pass through LDS: its four rows, or two of the longer even rows
inline uint32_t lane_rows_vectors(uint32_t M) { return (M > 16u && (M & 3u) == 2u) ? M / 2u : M; }

// Everything the host decides about one call: which streaming kernel, how the tensor is cut
// into units, and where each array sits in the workspace.
struct Plan {
    uint32_t T, N, M, K;
    uint64_t elements;          // T*N*M
    uint64_t stride;            // elements from one trial to the next (N*M when the tensor is contiguous)
    uint64_t extent;            // elements from the first one of the tensor to its last: (T-1)*stride + N*M
    bool vec4;                  // 16-byte loads, whole rows per load (M a multiple of 4 up to 128, or 256; lat 16-byte aligned)
    bool lane_rows;             // every lane holds whole rows (the row lengths of lane_rows_length: N a multiple of the
                                // rows per lane and at least DC_LANE_ROWS_MIN_N, trials 16-byte aligned; or span_rows; or
                                // row_lane); never set together with vec4
    bool row_lane;              // lane_rows with one row per lane (dc_scan_row_lane_kernel: the row lengths of
                                // row_lane_length, N*M a multiple of 4, at least DC_ROW_LANE_MIN_N workers)
    bool wave_trials;           // per-iteration pass: every wave owns a trial (small trials of a contiguous tensor, K <= 511)
    uint32_t span_rows;         // lane_rows with few workers per trial on a contiguous tensor: N, and the units ignore the
                                // trials (unit_max then holds one maximum per trial); 0 otherwise
    uint32_t rows_per_load;     // vec4: whole rows per 1 KiB load when fewer than fit are taken, so that a small trial is a
                                // whole number of loads (8 workers of 20 accumulations: 8 rows of the 12 that fit); else 0
    uint32_t trials_per_unit;   // vec4 with small trials on a contiguous tensor whose N is a multiple of the rows per load:
                                // a unit is this many whole trials and unit_max holds one maximum per trial; else 0
    uint32_t per_unit;          // vec4: loads (1 KiB, 64/L rows) per unit; lane_rows: chunks per unit; otherwise rows per unit
    uint32_t units_per_trial;
    uint32_t units;             // T * units_per_trial
    uint32_t run;               // consecutive units that one block takes at a time (a multiple of DC_SCAN_WAVES)
    uint32_t grid;              // blocks of the streaming kernel (= histogram slots) for narrow threshold grids ...
    uint32_t grid_wide;         // ... and for dense ones (long rows only, else equal): both are launched, one works
    uint32_t chunk;             // thresholds per pass, <= DC_CHUNK_THRESHOLDS
    uint32_t p2;                // power of two > chunk: padded length of the LDS threshold array
    uint32_t max_latency;       // floor((2^31-1)/M)
    // byte offsets into the workspace
    size_t off_status, off_tau_sorted, off_tau_u32, off_pos, off_bins, off_unit_max, off_hist_part;
    size_t off_partial;         // per-iteration speedup pass: float64 [grid][p2]
    size_t bytes;
};

void launch_prep(const int64_t* taus, uint32_t K, int64_t* tau_sorted, uint32_t* tau_u32, uint32_t* pos,
                 uint32_t* status, unsigned long long* bins, uint32_t bins_words, const int32_t* lat,
                 uint64_t rows_total, uint32_t N, uint64_t trial_stride, uint32_t M, uint32_t sample_rows,
                 uint32_t* zero_words, uint32_t zero_count, hipStream_t stream);
void launch_scan(const Plan& p, const int32_t* lat, const uint32_t* tau_chunk, uint32_t kc, uint32_t* unit_max,
                 uint32_t* hist_part, uint32_t* status, hipStream_t stream);
void launch_reduce(const Plan& p, const uint32_t* hist_part, unsigned long long* hist_total,
                   const uint32_t* unit_max, const uint32_t* tau_chunk, uint32_t kc,
                   unsigned long long* trial_cnt, unsigned long long* trial_sum, uint32_t* status, uint32_t chunk0,
                   const int64_t* tau_sorted, const uint32_t* pos, int64_t comm, int64_t* out_step, int64_t* out_done,
                   hipStream_t stream);
int row_lane_blocks_per_cu(size_t lds);
void launch_row_lane_scan(const Plan& p, const int32_t* lat, const uint32_t* tau_chunk, uint32_t kc, uint32_t* unit_max,
                          uint32_t* hist_part, uint32_t* status, hipStream_t stream);
void launch_trial_scan(const Plan& p, const int32_t* lat, const uint32_t* tau_chunk, uint32_t kc,
                       const int64_t* comm_per_trial, int64_t comm, double* partial, uint32_t* status,
                       hipStream_t stream);
void launch_speedup_finalize(const Plan& p, const double* partial, uint32_t kc, uint32_t chunk0, const uint32_t* pos,
                             uint32_t* status, const int64_t* tau_sorted, double* out_seff, hipStream_t stream);
size_t trial_scan_lds_bytes(const Plan& p);
void launch_worker_totals(const Plan& p, const int32_t* lat, unsigned long long* partial,
                          unsigned long long* result, uint32_t* status, hipStream_t stream, hipEvent_t before,
                          hipEvent_t after);
void launch_moments(const int32_t* lat, uint64_t n, uint32_t grid, unsigned long long* partial,
                    unsigned long long* result, uint32_t* status, hipStream_t stream);
void launch_expected_done(const int64_t* taus, uint32_t K, uint32_t M, double mu, double sigma2, double* out,
                          hipStream_t stream);
void launch_export_status(const uint32_t* status, int32_t* out, hipStream_t stream);
size_t scan_lds_bytes(const Plan& p);
int rows_blocks_per_cu(const Plan& p, size_t lds);
void launch_rows_scan(const Plan& p, const int32_t* lat, const uint32_t* tau_chunk, uint32_t kc, uint32_t* unit_max,
                      uint32_t* hist_part, uint32_t* status, hipStream_t stream);
int scan_blocks_per_cu(const Plan& p);
int trial_scan_blocks_per_cu(const Plan& p);

}  // namespace dc
#endif
