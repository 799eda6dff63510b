// Device kernels of the DropCompute step-time simulator, written for gfx950 (wave64, DPP, LDS).
//
// Pipeline of one call (all on one stream):
//   dc_prep_kernel       sort the K thresholds by rank, clamp them to 32 bits, clear accumulators; for long rows
//                        also sample the tensor to choose the streaming kernel's launch shape
//   dc_scan_vec4_kernel  the single pass over lat: completion times (a segmented wave scan over the lanes of a row;
//     / dc_scan_rows     plain sums where a lane holds whole short rows; one flat scan for any other row length),
//     / dc_scan_flat     histogram of completion times over the threshold grid, per-unit or per-trial maxima
//   dc_reduce_kernel     add the per-block histograms; per-trial maximum -> binned count and sum; the last block
//                        to finish takes prefix sums over the bins -> out_step, out_done in the caller's order
//
// Counting rests on two facts.  Latencies are >= 0, so a worker's completion times
// P[m] = sum_{j<=m} lat[j] (Section 4.3) are non-decreasing.  And "P < tau_k" (strict, Section 4.3)
// for ascending thresholds means k >= b(P) with b(P) = #{k : tau_k <= P}.  So one histogram of b(P)
// and one running sum over k replace the K comparisons per element of Algorithm 2's loops, and
// elements below the smallest threshold (b = 0) need no work at all.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dc_device.h"
#include "dc_internal.h"

// ---------------------------------------------------------------------------------------------
// dc_prep_kernel: rank-sort the thresholds, clamp, validate, clear accumulators
// ---------------------------------------------------------------------------------------------

// Share of completion times at or above the smallest threshold, from `sample_rows` <= DC_SAMPLE_ROWS rows spread
// evenly over the tensor.  Rows here are 128 or 256 elements of a 16-byte aligned tensor: one 16-byte load per lane
// covers a row.  sample_begin issues every load (a wave has DC_SAMPLE_ROWS / 4 rows in flight, and its share of the
// thresholds) so that their latency passes behind other work; sample_is_dense, called later by the whole block of
// 256 threads, returns 1 if the share reaches DC_DENSE_PERMILLE.
struct Sample {
    u32x4 x[DC_SAMPLE_ROWS / 4];
    long long lowest;          // smallest threshold among those this thread read
};

__device__ __forceinline__ Sample sample_begin(const int64_t* __restrict__ taus, uint32_t K,
                                               const int32_t* __restrict__ lat, unsigned long long rows_total,
                                               uint32_t N, unsigned long long trial_stride, uint32_t M,
                                               uint32_t sample_rows) {
    constexpr int PER_WAVE = DC_SAMPLE_ROWS / 4;
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    Sample sm;
    sm.lowest = 0x7FFFFFFFFFFFFFFFll;
    for (uint32_t i = threadIdx.x; i < K; i += blockDim.x) sm.lowest = taus[i] < sm.lowest ? taus[i] : sm.lowest;
#pragma unroll
    for (int q = 0; q < PER_WAVE; ++q) {
        const uint32_t sidx = wave * PER_WAVE + (uint32_t)q;
        const unsigned long long row = rows_total / sample_rows * sidx + rows_total % sample_rows * sidx / sample_rows;
        sm.x[q] = u32x4{0u, 0u, 0u, 0u};
        const unsigned long long at = row / N * trial_stride + row % N * M;        // row = trial * N + worker
        if (sidx < sample_rows && lane < M / 4u) sm.x[q] = *(reinterpret_cast<const u32x4*>(lat + at) + lane);
    }
    return sm;
}

__device__ __forceinline__ uint32_t sample_is_dense(const Sample& sm, uint32_t M, uint32_t sample_rows) {
    constexpr int PER_WAVE = DC_SAMPLE_ROWS / 4;
    __shared__ long long wave_min[4];
    __shared__ uint32_t wave_hits[4];
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    long long lowest = sm.lowest;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const long long other = __shfl_xor(lowest, d, 64);
        lowest = other < lowest ? other : lowest;
    }
    if (lane == 0) wave_min[wave] = lowest;
    __syncthreads();
    lowest = wave_min[0];
    for (int w = 1; w < 4; ++w) lowest = wave_min[w] < lowest ? wave_min[w] : lowest;
    const uint32_t tau0 = lowest >= (long long)DC_TAU_CLAMP ? DC_TAU_CLAMP : (lowest < 0 ? 0u : (uint32_t)lowest);

    uint32_t hits = 0u;                                           // per lane; added up below
#pragma unroll
    for (int q = 0; q < PER_WAVE; ++q) {
        const u32x4 x = sm.x[q];
        const uint32_t c3 = segmented_inclusive_scan<64>(x.x + x.y + x.z + x.w, lane);
        const uint32_t c2 = c3 - x.w, c1 = c2 - x.z, c0 = c1 - x.y;
        if (wave * PER_WAVE + (uint32_t)q < sample_rows && lane < M / 4u)
            hits += (c0 >= tau0 ? 1u : 0u) + (c1 >= tau0 ? 1u : 0u) + (c2 >= tau0 ? 1u : 0u) + (c3 >= tau0 ? 1u : 0u);
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) hits += (uint32_t)__shfl_xor((int)hits, d, 64);
    if (lane == 0) wave_hits[wave] = hits;
    __syncthreads();
    const unsigned long long all = (unsigned long long)wave_hits[0] + wave_hits[1] + wave_hits[2] + wave_hits[3];
    return all * 1000ull >= (unsigned long long)DC_DENSE_PERMILLE * sample_rows * M ? 1u : 0u;
}

__global__ __launch_bounds__(256)
void dc_prep_kernel(const int64_t* __restrict__ taus, uint32_t K,
                    int64_t* __restrict__ tau_sorted, uint32_t* __restrict__ tau_u32,
                    uint32_t* __restrict__ pos, uint32_t* __restrict__ status,
                    unsigned long long* __restrict__ bins, uint32_t bins_words,
                    const int32_t* __restrict__ lat, unsigned long long rows_total, uint32_t N,
                    unsigned long long trial_stride, uint32_t M, uint32_t sample_rows,
                    uint32_t* __restrict__ zero_words, uint32_t zero_count) {
    // A block ranks 32 thresholds; the comparisons of each are split over 8 threads.
    constexpr uint32_t TILE = 1024;
    __shared__ int64_t tile[TILE];
    __shared__ uint32_t partial[8][32];
    const uint32_t gid = blockIdx.x * blockDim.x + threadIdx.x;
    const uint32_t stride = gridDim.x * blockDim.x;
    // Block 0 also looks at a sample of rows (sample_rows > 0) and tells the streaming kernel which of its two launch
    // shapes to use; its loads are issued here and used after the ranking.
    const bool sampling = blockIdx.x == 0 && sample_rows != 0u;
    Sample sm{};
    if (sampling) sm = sample_begin(taus, K, lat, rows_total, N, trial_stride, M, sample_rows);
    if (gid == 0) { status[0] = 0u; status[2] = 0u; }   // value flags (set by later kernels) and the reduce kernel's ticket
    for (uint32_t i = gid; i < bins_words; i += stride) bins[i] = 0ull;
    for (uint32_t i = gid; i < zero_count; i += stride) zero_words[i] = 0u;      // per-trial maxima built with atomics
    const uint32_t jj = threadIdx.x & 31u, part = threadIdx.x >> 5;
    const uint32_t j = blockIdx.x * 32 + jj;
    const int64_t mine = j < K ? taus[j] : 0;
    // position in ascending order = number of thresholds that sort before mine (ties by index)
    uint32_t rank = 0;
    for (uint32_t base = 0; base < K; base += TILE) {
        const uint32_t n = K - base < TILE ? K - base : TILE;
        __syncthreads();
        for (uint32_t i = threadIdx.x; i < n; i += blockDim.x) tile[i] = taus[base + i];
        __syncthreads();
#pragma unroll 8
        for (uint32_t i = part; i < n; i += 8) {
            const int64_t other = tile[i];
            rank += (other < mine) || (other == mine && base + i < j);
        }
    }
    partial[part][jj] = rank;
    __syncthreads();
    // status[1] = 1 when a large share of the sampled completion times reaches the smallest threshold
    if (sampling) {
        const uint32_t dense = sample_is_dense(sm, M, sample_rows);   // synchronises the block
        if (threadIdx.x == 0) status[1] = dense;
    }
    if (part != 0 || j >= K) return;
    rank = 0;
#pragma unroll
    for (int q = 0; q < 8; ++q) rank += partial[q][jj];
    pos[j] = rank;
    tau_sorted[rank] = mine;
    tau_u32[rank] = mine >= (int64_t)DC_TAU_CLAMP ? DC_TAU_CLAMP : (mine < 0 ? 0u : (uint32_t)mine);
    // A negative threshold is flagged by the kernel that ends the call, from tau_sorted[0]: this kernel's own
    // clearing of the status word (block 0) is not ordered against the other blocks.
}

// ---------------------------------------------------------------------------------------------
// dc_scan_vec4_kernel: the streaming pass, M = 4*L with L in {1,2,4,...,64}
// ---------------------------------------------------------------------------------------------
// A "load" is 1 KiB read by one wave (16 B per lane) = 64/L whole rows.  A "unit" is up to
// loads_per_unit consecutive loads inside one trial; waves take units round-robin.  Every wave owns
// its queue and the histogram is updated with LDS atomics, so the only block-level synchronisation
// in the loop is one barrier per unit that keeps the block's waves in step.
template <int L, int SHAPE>
__global__ __launch_bounds__(DC_SCAN_THREADS)
void dc_scan_vec4_kernel(const int32_t* __restrict__ lat, uint64_t trial_stride, uint32_t N, uint32_t units, uint32_t units_per_trial,
                         uint32_t run, uint32_t loads_per_unit, const uint32_t* __restrict__ tau_chunk, uint32_t kc, uint32_t p2,
                         uint32_t* __restrict__ unit_max, uint32_t* __restrict__ hist_part,
                         uint32_t* __restrict__ status, uint32_t max_latency, uint32_t lanes_per_row, uint32_t T,
                         uint32_t trials_per_unit, uint32_t rows_per_load) {
    extern __shared__ __align__(16) unsigned char smem[];
    if (!launch_is_chosen<SHAPE>(status)) return;
    uint4* queue_all = reinterpret_cast<uint4*>(smem);                                  // [waves][QUEUE_ITEMS]
    const GridView g = stage_grid(reinterpret_cast<uint32_t*>(queue_all + DC_SCAN_WAVES * QUEUE_ITEMS), tau_chunk, kc, p2);

    const uint32_t lane = threadIdx.x & 63u;
    const RowShape shape = row_shape<L>(lane, lanes_per_row, rows_per_load);
    const uint32_t R = shape.rows;                 // rows per load
    const uint32_t M = 4 * shape.lanes;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform by construction
    uint4* queue = queue_all + wave * QUEUE_ITEMS;
    WaveState st{0u, 0u, 0u, 0u};
    // A block takes runs of `run` consecutive units (blocks take the runs round-robin) and, inside a run, its
    // waves take four adjacent units at a time, in step: every wave streams its own contiguous unit while the
    // block as a whole moves through one contiguous stretch of the tensor.  Measured on 34 GB at M = 256: runs of
    // 64 units (2 MiB) 7.10-7.14 TB/s, runs of 4 (every block jumps ahead by the whole grid each time) 6.87-6.96.
    // Both loop bounds are the same for the whole block, so the barrier is reached by every wave the same
    // number of times; it only paces the waves (1-2 % faster than letting them drift apart).
    const UnitRuns ur = unit_runs(units, run, gridDim.x);
    for (uint32_t r = blockIdx.x; r < ur.padded; r += gridDim.x)
    for (uint32_t round = 0; round < ur.rounds; ++round) {
        const uint32_t u = r < ur.runs ? r * run + round * DC_SCAN_WAVES + wave : units;
        if (u < units && trials_per_unit > 1u) {
            // small trials (contiguous tensor, N a multiple of R): the unit is a run of whole trials, unit_max holds
            // one maximum per trial
            const uint32_t t0 = u * trials_per_unit;
            const uint32_t trials = T - t0 < trials_per_unit ? T - t0 : trials_per_unit;
            const uint32_t loads_per_trial = N / R;
            const u32x4* base = reinterpret_cast<const u32x4*>(lat + (uint64_t)t0 * trial_stride) + lane;
            stream_small_trials<L>(st, base, trials * loads_per_trial, loads_per_trial, unit_max + t0, queue, g, lane, shape);
        } else if (u < units) {
            const uint32_t t = u / units_per_trial;
            const uint32_t j = u - t * units_per_trial;
            const uint32_t row0 = j * loads_per_unit * R;
            const uint32_t rows_left = row0 < N ? N - row0 : 0u;          // (a unit past the trial's end is empty)
            const uint32_t rows = rows_left < loads_per_unit * R ? rows_left : loads_per_unit * R;
            const uint32_t nfull = rows / R;
            const u32x4* base = reinterpret_cast<const u32x4*>(lat + (uint64_t)t * trial_stride + (uint64_t)row0 * M) + lane;
            st.lane_max = 0u;
            stream_rows<L>(st, base, nfull, rows - nfull * R, queue, g, lane, shape);
            const uint32_t m = wave_max(st.lane_max);
            if (lane == 0) unit_max[u] = m;
        }
        __syncthreads();
    }
    while (st.q_count) drain(st, queue, g, lane);
    report_range(st.check, max_latency, lane, status);

    __syncthreads();
    uint32_t* out = hist_part + (uint64_t)blockIdx.x * p2;
    for (uint32_t i = threadIdx.x; i < p2; i += DC_SCAN_THREADS) out[i] = g.hist[i];
}

// ---------------------------------------------------------------------------------------------
// dc_scan_flat_kernel: any M >= 1, any 4-byte alignment of lat (the flat pass of dc_device.h)
// ---------------------------------------------------------------------------------------------
template <int MS>        // 0: rows of at least 4 elements; 1, 2, 3: rows of exactly that many
__global__ __launch_bounds__(DC_SCAN_THREADS)
void dc_scan_flat_kernel(const int32_t* __restrict__ lat, uint64_t total, uint64_t trial_stride, uint32_t N, uint32_t M, uint32_t units,
                         uint32_t units_per_trial, uint32_t run, uint32_t rows_per_unit, const uint32_t* __restrict__ tau_chunk,
                         uint32_t kc, uint32_t p2, uint32_t* __restrict__ unit_max, uint32_t* __restrict__ hist_part,
                         uint32_t* __restrict__ status, uint32_t max_latency) {
    extern __shared__ __align__(16) unsigned char smem[];
    uint4* queue_all = reinterpret_cast<uint4*>(smem);                                  // [waves][QUEUE_ITEMS]
    const GridView g = stage_grid(reinterpret_cast<uint32_t*>(queue_all + DC_SCAN_WAVES * QUEUE_ITEMS), tau_chunk, kc, p2);

    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint4* queue = queue_all + wave * QUEUE_ITEMS;
    const FlatTensor f = flat_tensor(lat, total, M);

    WaveState st{0u, 0u, 0u, 0u};
    const UnitRuns ur = unit_runs(units, run, gridDim.x);                                  // as in dc_scan_vec4_kernel
    for (uint32_t r = blockIdx.x; r < ur.padded; r += gridDim.x)                          // block-uniform bounds
    for (uint32_t round = 0; round < ur.rounds; ++round) {
        const uint32_t u = r < ur.runs ? r * run + round * DC_SCAN_WAVES + wave : units;
        if (u < units) {
            const uint32_t t = u / units_per_trial;
            const uint32_t j = u - t * units_per_trial;
            const uint32_t row0 = j * rows_per_unit;
            const uint32_t rows = (N - row0) < rows_per_unit ? (N - row0) : rows_per_unit;
            st.lane_max = 0u;
            flat_stream_unit<(MS != 0), DC_FLAT_UNROLL, MS>(st.check, f, (uint64_t)t * trial_stride + (uint64_t)row0 * M, rows * M, lane,
                                    [&](uint4 p, uint32_t vm, uint32_t, uint32_t) { flat_count(st, p, vm, queue, g, lane); });
            const uint32_t m = wave_max(st.lane_max);
            if (lane == 0) unit_max[u] = m;
        }
        __syncthreads();
    }
    while (st.q_count) drain(st, queue, g, lane);
    report_range(st.check, max_latency, lane, status);

    __syncthreads();
    uint32_t* out = hist_part + (uint64_t)blockIdx.x * p2;
    for (uint32_t i = threadIdx.x; i < p2; i += DC_SCAN_THREADS) out[i] = g.hist[i];
}

// ---------------------------------------------------------------------------------------------
// The last step of a pass, run by one block of THREADS threads once every sum is in.  Running sums over the bins
// give, for sorted threshold i of the chunk: not_done[i] = sum_{b>i} hist[b];
// below[i] = #{t : Tmax_t < tau_i} = sum_{b<=i} cnt[b];  below_sum[i] = sum_{b<=i} sum[b].  Then
//   done[i] = T*N*M - not_done[i]
//   step[i] = below_sum[i] + tau_i * (T - below[i]) + T*comm
// and results go to the caller's positions.  The accumulators are cleared for the next chunk.  They were written
// with device-scope atomics by other blocks, hence the device-scope loads.
// ---------------------------------------------------------------------------------------------
struct FinalArgs {
    unsigned long long* hist_total;
    unsigned long long* trial_cnt;
    unsigned long long* trial_sum;
    uint32_t kc, p2, chunk0, K;
    uint32_t* status;
    const int64_t* tau_sorted;
    const uint32_t* pos;
    unsigned long long T, elements;
    long long comm;
    long long* out_step;
    long long* out_done;
};

__device__ __forceinline__ unsigned long long load_device_scope(const unsigned long long* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <uint32_t THREADS>
__device__ __forceinline__ void finalize_chunk(const FinalArgs& f, long long* s_step, long long* s_done) {
    constexpr uint32_t MAX_PER = (DC_CHUNK_THRESHOLDS + 1u + THREADS - 1u) / THREADS;   // p2 <= 4096
    __shared__ unsigned long long s_a[THREADS], s_b[THREADS], s_c[THREADS];
    const uint32_t tid = threadIdx.x;
    const uint32_t per = (f.p2 + THREADS - 1) / THREADS;           // each thread owns a contiguous run of bins
    const uint32_t b0 = tid * per;
    unsigned long long h[MAX_PER], c[MAX_PER], s[MAX_PER];
    long long tau[MAX_PER];
    unsigned long long th = 0, tc = 0, ts = 0;
    // everything this step reads from device memory is requested here, in one go: a block that runs alone waits
    // a few microseconds for every dependent round trip
    const uint32_t first_pos = tid < f.K ? f.pos[tid] : 0xFFFFFFFFu;
#pragma unroll
    for (uint32_t i = 0; i < MAX_PER; ++i) {
        const uint32_t b = b0 + i;
        h[i] = i < per && b < f.p2 ? load_device_scope(&f.hist_total[b]) : 0ull;
        c[i] = i < per && b <= f.kc ? load_device_scope(&f.trial_cnt[b]) : 0ull;
        s[i] = i < per && b <= f.kc ? load_device_scope(&f.trial_sum[b]) : 0ull;
        tau[i] = i < per && b < f.kc ? f.tau_sorted[f.chunk0 + b] : 0ll;
    }
#pragma unroll
    for (uint32_t i = 0; i < MAX_PER; ++i) { th += h[i]; tc += c[i]; ts += s[i]; }
    s_a[tid] = th; s_b[tid] = tc; s_c[tid] = ts;
    __syncthreads();
    for (uint32_t d = 1; d < THREADS; d <<= 1) {                    // inclusive scan over threads
        unsigned long long xa = 0, xb = 0, xc = 0;
        if (tid >= d) { xa = s_a[tid - d]; xb = s_b[tid - d]; xc = s_c[tid - d]; }
        __syncthreads();
        s_a[tid] += xa; s_b[tid] += xb; s_c[tid] += xc;
        __syncthreads();
    }
    const unsigned long long all_hist = s_a[THREADS - 1];
    unsigned long long run_h = s_a[tid] - th, run_c = s_b[tid] - tc, run_s = s_c[tid] - ts;   // exclusive
#pragma unroll
    for (uint32_t i = 0; i < MAX_PER; ++i) {
        const uint32_t b = b0 + i;
        run_h += h[i]; run_c += c[i]; run_s += s[i];                 // inclusive up to bin b
        if (i < per && b < f.kc) {
            const unsigned long long not_done = all_hist - run_h;
            const unsigned long long tau_c = tau[i] >= (long long)DC_TAU_CLAMP ? (unsigned long long)DC_TAU_CLAMP
                                                                               : (unsigned long long)(tau[i] < 0 ? 0 : tau[i]);
            s_done[b] = (long long)(f.elements - not_done);          // the chunk's results stay in LDS until they are
            s_step[b] = (long long)(run_s + tau_c * (f.T - run_c) + f.T * (unsigned long long)f.comm);   // scattered
        }
    }
    for (uint32_t b = tid; b < f.p2; b += THREADS) {
        f.hist_total[b] = 0ull;
        if (b <= f.kc) { f.trial_cnt[b] = 0ull; f.trial_sum[b] = 0ull; }
    }
    if (tid == 0 && f.chunk0 == 0u && f.kc > 0u && tau[0] < 0) atomicOr(f.status, DC_FLAG_NEGATIVE_TAU);
    __syncthreads();
    for (uint32_t j = tid; j < f.K; j += THREADS) {
        const uint32_t p = j == tid ? first_pos : f.pos[j];
        if (p >= f.chunk0 && p < f.chunk0 + f.kc) {
            f.out_step[j] = s_step[p - f.chunk0];
            f.out_done[j] = s_done[p - f.chunk0];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// dc_reduce_kernel: (a) column sums of the per-block histograms, (b) per-trial maximum binned over the chunk's
// thresholds, (c) the final running sums.  Blocks [0, hist_blocks) do (a): block (c, g) adds slots
// [g*DC_REDUCE_SLOTS, ...) of columns [64c, 64c+64) and adds its partial sums to hist_total (cleared beforehand).
// The remaining blocks do (b), one thread per trial.  Every block then takes a ticket (status[2], cleared by the
// prep kernel and again here); the block that draws the last one knows that all sums are in and does (c).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256)
void dc_reduce_kernel(const uint32_t* __restrict__ hist_part, uint32_t narrow_slots, uint32_t wide_slots,
                      uint32_t* __restrict__ status, uint32_t col_blocks, uint32_t hist_blocks,
                      const uint32_t* __restrict__ unit_max, uint32_t units_per_trial,
                      const uint32_t* __restrict__ tau_chunk, FinalArgs f) {
    extern __shared__ unsigned long long bin_sum[];                       // (b): [p2], then the counts; (c): 2 [p2] results
    __shared__ unsigned long long part[4][64];
    __shared__ uint32_t is_last;
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t grp = threadIdx.x >> 6;
    const uint32_t p2 = f.p2, kc = f.kc;
    if (blockIdx.x < hist_blocks) {
        // histograms were written by the launch of the streaming kernel that the sample chose
        const uint32_t slots = wide_slots > narrow_slots && status[1] != 0u ? wide_slots : narrow_slots;
        const uint32_t col = (blockIdx.x % col_blocks) * 64 + lane;       // consecutive lanes, consecutive columns
        const uint32_t s0 = (blockIdx.x / col_blocks) * DC_REDUCE_SLOTS;
        const uint32_t s1 = s0 + DC_REDUCE_SLOTS < slots ? s0 + DC_REDUCE_SLOTS : slots;
        uint32_t v[DC_REDUCE_SLOTS / 4];                                  // all requested before the first is used
#pragma unroll
        for (uint32_t q = 0; q < DC_REDUCE_SLOTS / 4; ++q) {
            const uint32_t s = s0 + grp + 4u * q;
            v[q] = col < p2 && s < s1 ? hist_part[(uint64_t)s * p2 + col] : 0u;
        }
        unsigned long long acc = 0ull;
#pragma unroll
        for (uint32_t q = 0; q < DC_REDUCE_SLOTS / 4; ++q) acc += v[q];
        part[grp][lane] = acc;
        __syncthreads();
        if (grp == 0 && col < p2) {
            const unsigned long long sum = part[0][lane] + part[1][lane] + part[2][lane] + part[3][lane];
            if (sum) atomicAdd(&f.hist_total[col], sum);
        }
    } else {
        // (b) one thread per trial.  The trial maxima of a block are binned in LDS first (maxima of one
        // workload crowd into a few bins, and same-address atomics in device memory serialise), then the
        // bins that were hit go to device memory: at most one addition per bin and block.
        uint32_t* bin_cnt = reinterpret_cast<uint32_t*>(bin_sum + p2);    // [p2]
        uint32_t* tau_s = bin_cnt + p2;                                   // [p2] the pass's thresholds, for the searches
        for (uint32_t i = threadIdx.x; i < p2; i += 256) {
            bin_sum[i] = 0ull;
            bin_cnt[i] = 0u;
            tau_s[i] = i < kc ? tau_chunk[i] : 0xFFFFFFFFu;
        }
        __syncthreads();
        // The trial blocks take groups of 256 trials round-robin: with very many trials a bin then receives one
        // addition per block in device memory, not one per 256 trials (measured 141 -> 35 us at T = 524288).
        const uint32_t trial_blocks = gridDim.x - hist_blocks;
        for (uint32_t t = (blockIdx.x - hist_blocks) * 256 + threadIdx.x; t < (uint32_t)f.T; t += trial_blocks * 256) {
            uint32_t tmax = 0u;
            const uint32_t* um = unit_max + (uint64_t)t * units_per_trial;
            if ((units_per_trial & 3u) == 0u) {                           // unit_max is 256-byte aligned
                uint32_t j = 0;
                for (; j + 32u <= units_per_trial; j += 32u) {            // eight independent loads at a time
                    uint4 v[8];
#pragma unroll
                    for (uint32_t q = 0; q < 8; ++q) v[q] = *reinterpret_cast<const uint4*>(um + j + 4u * q);
#pragma unroll
                    for (uint32_t q = 0; q < 8; ++q) tmax = umax(umax(tmax, v[q].x), umax(umax(v[q].y, v[q].z), v[q].w));
                }
                for (; j < units_per_trial; j += 4u) {
                    const uint4 v = *reinterpret_cast<const uint4*>(um + j);
                    tmax = umax(umax(tmax, v.x), umax(umax(v.y, v.z), v.w));
                }
            } else {
#pragma unroll 4
                for (uint32_t j = 0; j < units_per_trial; ++j) tmax = umax(tmax, um[j]);
            }
            // b = #{i < kc : tau_i <= tmax}; the trial's step time is tmax for thresholds i >= b, tau_i below
            uint32_t lo = 0, hi = kc;
            while (lo < hi) {
                const uint32_t mid = (lo + hi) >> 1;
                if (tau_s[mid] <= tmax) lo = mid + 1; else hi = mid;
            }
            atomicAdd(&bin_cnt[lo], 1u);
            atomicAdd(&bin_sum[lo], (unsigned long long)tmax);
        }
        __syncthreads();
        for (uint32_t i = threadIdx.x; i <= kc; i += 256) {
            const uint32_t c = bin_cnt[i];
            if (c) {
                atomicAdd(&f.trial_cnt[i], (unsigned long long)c);
                atomicAdd(&f.trial_sum[i], bin_sum[i]);
            }
        }
    }
    // (c) the block that draws the last ticket finishes the pass
    __threadfence();                                   // this thread's additions are visible device-wide ...
    __syncthreads();                                   // ... for every thread of the block, before its ticket is drawn
    if (threadIdx.x == 0) {
        const uint32_t ticket = atomicAdd(&status[2], 1u);
        is_last = ticket == gridDim.x - 1u ? 1u : 0u;
    }
    __syncthreads();
    if (!is_last) return;
    __threadfence();
    if (threadIdx.x == 0) status[2] = 0u;              // next pass (kernels on a stream run one after the other)
    long long* results = reinterpret_cast<long long*>(bin_sum);   // the block's bins, if it had any, are added by now
    finalize_chunk<256>(f, results, results + p2);
}

// ---------------------------------------------------------------------------------------------
// launchers (called from dc_api.hip)
// ---------------------------------------------------------------------------------------------
namespace dc {

// sample_rows > 0: also sample that many rows of lat ([rows_total][M]) for the choice of the launch shape
void launch_prep(const int64_t* taus, uint32_t K, int64_t* tau_sorted, uint32_t* tau_u32, uint32_t* pos,
                 uint32_t* status, unsigned long long* bins, uint32_t bins_words, const int32_t* lat,
                 uint64_t rows_total, uint32_t N, uint64_t trial_stride, uint32_t M, uint32_t sample_rows,
                 uint32_t* zero_words, uint32_t zero_count, hipStream_t stream) {
    const uint32_t threads = 256;                 // 32 thresholds per block
    uint32_t blocks = (K + 31) / 32;
    if (blocks == 0) blocks = 1;
    const uint32_t clearing = (zero_count + 4095u) / 4096u;           // blocks beyond the thresholds only clear
    if (blocks < clearing) blocks = clearing < 1024u ? clearing : 1024u;
    hipLaunchKernelGGL(dc_prep_kernel, dim3(blocks), dim3(threads), 0, stream, taus, K, tau_sorted, tau_u32, pos,
                       status, bins, bins_words, lat, (unsigned long long)rows_total, N ? N : 1u,
                       (unsigned long long)trial_stride, M, sample_rows, zero_words, zero_count);
}

size_t scan_lds_bytes(const Plan& p) {
    const size_t tables = (size_t)p.p2 * 8;                       // thresholds + histogram
    if (p.row_lane) return tables + (size_t)p.p2 * 8 + (size_t)DC_SCAN_WAVES * 256u * p.M;   // + cells + every wave's 64 rows
    if (p.lane_rows)                                              // + cells + every wave's stretch for its chunk
        return tables + (size_t)p.p2 * 8 + (4u % p.M ? (size_t)DC_SCAN_WAVES * 64u * (lane_rows_vectors(p.M) | 1u) * sizeof(u32x4) : 0u);
    return tables + (size_t)p.p2 * 8 + (size_t)DC_SCAN_WAVES * QUEUE_ITEMS * sizeof(uint4);   // + cells + queues
}

template <int L>
static int resident_vec4(size_t lds) {
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, dc_scan_vec4_kernel<L, 0>, DC_SCAN_THREADS, lds) != hipSuccess) n = 0;
    return n;
}

// Blocks of the streaming kernel that one compute unit holds at a time (0 if the query fails).
int scan_blocks_per_cu(const Plan& p) {
    const size_t lds = scan_lds_bytes(p);
    int n = 0;
    if (p.row_lane) return row_lane_blocks_per_cu(lds);
    if (p.lane_rows) return rows_blocks_per_cu(p, lds);
    if (!p.vec4) {
        hipError_t e;
        switch (p.M) {
            case 1:  e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, dc_scan_flat_kernel<1>, DC_SCAN_THREADS, lds); break;
            case 2:  e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, dc_scan_flat_kernel<2>, DC_SCAN_THREADS, lds); break;
            case 3:  e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, dc_scan_flat_kernel<3>, DC_SCAN_THREADS, lds); break;
            default: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, dc_scan_flat_kernel<0>, DC_SCAN_THREADS, lds); break;
        }
        return e == hipSuccess ? n : 0;
    }
    switch (p.rows_per_load ? 0u : p.M / 4) {     // fewer rows per load than fit: the instantiation for any row length
        case 1:  return resident_vec4<1>(lds);
        case 2:  return resident_vec4<2>(lds);
        case 4:  return resident_vec4<4>(lds);
        case 8:  return resident_vec4<8>(lds);
        case 16: return resident_vec4<16>(lds);
        case 32: return resident_vec4<32>(lds);
        case 64: return resident_vec4<64>(lds);
        default: return resident_vec4<0>(lds);
    }
}

template <int L>
static void launch_vec4(const Plan& p, const int32_t* lat, const uint32_t* tau_chunk, uint32_t kc,
                        uint32_t* unit_max, uint32_t* hist_part, uint32_t* status, hipStream_t stream) {
    if (p.grid_wide > p.grid) {                     // the sample decides on the device which of the two launches works
        if constexpr (L == 8 || L == 16 || L == 32 || L == 64) {
            hipLaunchKernelGGL((dc_scan_vec4_kernel<L, 1>), dim3(p.grid), dim3(DC_SCAN_THREADS), scan_lds_bytes(p), stream,
                               lat, p.stride, p.N, p.units, p.units_per_trial, p.run, p.per_unit, tau_chunk, kc, p.p2, unit_max,
                               hist_part, status, p.max_latency, p.M / 4, p.T, p.trials_per_unit, p.rows_per_load);
            hipLaunchKernelGGL((dc_scan_vec4_kernel<L, 2>), dim3(p.grid_wide), dim3(DC_SCAN_THREADS), scan_lds_bytes(p),
                               stream, lat, p.stride, p.N, p.units, p.units_per_trial, p.run, p.per_unit, tau_chunk, kc, p.p2,
                               unit_max, hist_part, status, p.max_latency, p.M / 4, p.T, p.trials_per_unit, p.rows_per_load);
            return;
        }
    }
    hipLaunchKernelGGL((dc_scan_vec4_kernel<L, 0>), dim3(p.grid), dim3(DC_SCAN_THREADS), scan_lds_bytes(p), stream, lat,
                       p.stride, p.N, p.units, p.units_per_trial, p.run, p.per_unit, tau_chunk, kc, p.p2, unit_max, hist_part,
                       status, p.max_latency, p.M / 4, p.T, p.trials_per_unit, p.rows_per_load);
}

template <int MS>
static void launch_flat(const Plan& p, const int32_t* lat, const uint32_t* tau_chunk, uint32_t kc,
                        uint32_t* unit_max, uint32_t* hist_part, uint32_t* status, hipStream_t stream) {
    hipLaunchKernelGGL(dc_scan_flat_kernel<MS>, dim3(p.grid), dim3(DC_SCAN_THREADS), scan_lds_bytes(p), stream, lat,
                       p.extent, p.stride, p.N, p.M, p.units, p.units_per_trial, p.run, p.per_unit, tau_chunk, kc, p.p2,
                       unit_max, hist_part, status, p.max_latency);
}

void launch_scan(const Plan& p, const int32_t* lat, const uint32_t* tau_chunk, uint32_t kc, uint32_t* unit_max,
                 uint32_t* hist_part, uint32_t* status, hipStream_t stream) {
    if (p.row_lane) { launch_row_lane_scan(p, lat, tau_chunk, kc, unit_max, hist_part, status, stream); return; }
    if (p.lane_rows) { launch_rows_scan(p, lat, tau_chunk, kc, unit_max, hist_part, status, stream); return; }
    if (!p.vec4) {
        switch (p.M) {
            case 1:  launch_flat<1>(p, lat, tau_chunk, kc, unit_max, hist_part, status, stream); break;
            case 2:  launch_flat<2>(p, lat, tau_chunk, kc, unit_max, hist_part, status, stream); break;
            case 3:  launch_flat<3>(p, lat, tau_chunk, kc, unit_max, hist_part, status, stream); break;
            default: launch_flat<0>(p, lat, tau_chunk, kc, unit_max, hist_part, status, stream); break;
        }
        return;
    }
    switch (p.rows_per_load ? 0u : p.M / 4) {
        case 1:  launch_vec4<1>(p, lat, tau_chunk, kc, unit_max, hist_part, status, stream); break;
        case 2:  launch_vec4<2>(p, lat, tau_chunk, kc, unit_max, hist_part, status, stream); break;
        case 4:  launch_vec4<4>(p, lat, tau_chunk, kc, unit_max, hist_part, status, stream); break;
        case 8:  launch_vec4<8>(p, lat, tau_chunk, kc, unit_max, hist_part, status, stream); break;
        case 16: launch_vec4<16>(p, lat, tau_chunk, kc, unit_max, hist_part, status, stream); break;
        case 32: launch_vec4<32>(p, lat, tau_chunk, kc, unit_max, hist_part, status, stream); break;
        case 64: launch_vec4<64>(p, lat, tau_chunk, kc, unit_max, hist_part, status, stream); break;
        default: launch_vec4<0>(p, lat, tau_chunk, kc, unit_max, hist_part, status, stream); break;
    }
}

// One launch ends a pass: sums of the per-block histograms, binned trial maxima, then the chunk's results.
void launch_reduce(const Plan& p, const uint32_t* hist_part, unsigned long long* hist_total,
                   const uint32_t* unit_max, const uint32_t* tau_chunk, uint32_t kc,
                   unsigned long long* trial_cnt, unsigned long long* trial_sum, uint32_t* status, uint32_t chunk0,
                   const int64_t* tau_sorted, const uint32_t* pos, int64_t comm, int64_t* out_step, int64_t* out_done,
                   hipStream_t stream) {
    const uint32_t col_blocks = (p.p2 + 63) / 64;
    const uint32_t slot_groups = (p.grid_wide + DC_REDUCE_SLOTS - 1) / DC_REDUCE_SLOTS;
    const uint32_t hist_blocks = col_blocks * slot_groups;
    const uint32_t trial_groups = (p.T + 255) / 256;
    const uint32_t trial_blocks = trial_groups < DC_REDUCE_TRIAL_BLOCKS ? trial_groups : DC_REDUCE_TRIAL_BLOCKS;
    FinalArgs f;
    f.hist_total = hist_total; f.trial_cnt = trial_cnt; f.trial_sum = trial_sum;
    f.kc = kc; f.p2 = p.p2; f.chunk0 = chunk0; f.K = p.K;
    f.status = status;
    f.tau_sorted = tau_sorted; f.pos = pos;
    f.T = p.T; f.elements = p.elements; f.comm = (long long)comm;
    f.out_step = (long long*)out_step; f.out_done = (long long*)out_done;
    hipLaunchKernelGGL(dc_reduce_kernel, dim3(hist_blocks + trial_blocks), dim3(256), (size_t)p.p2 * 16, stream, hist_part,
                       p.grid, p.grid_wide, status, col_blocks, hist_blocks, unit_max, p.span_rows ? 1u : p.units_per_trial,
                       tau_chunk, f);
}

// The value flags of a finished call as a dc_status code, for callers that cannot read the workspace.
__global__ void dc_export_status_kernel(const uint32_t* __restrict__ status, int32_t* __restrict__ out) {
    const uint32_t flags = status[0];
    int32_t code = 0;                                                            // DC_OK
    if (flags & (DC_FLAG_NEGATIVE_TAU | DC_FLAG_ZERO_STEP)) code = 1;            // DC_ERR_INVALID_ARG
    else if (flags & DC_FLAG_NEGATIVE_LATENCY) code = 2;                         // DC_ERR_NEGATIVE_LATENCY
    else if (flags & DC_FLAG_RANGE) code = 3;                                    // DC_ERR_RANGE
    *out = code;
}

void launch_export_status(const uint32_t* status, int32_t* out, hipStream_t stream) {
    hipLaunchKernelGGL(dc_export_status_kernel, dim3(1), dim3(1), 0, stream, status, out);
}

}  // namespace dc
