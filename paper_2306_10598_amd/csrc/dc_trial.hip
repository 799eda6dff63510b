// Per-iteration speedup (Algorithm 2 as printed): the kernels in which a block or a wave owns a whole trial, the sum
// over blocks, and their launchers.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dc_device.h"
#include "dc_internal.h"

// ---------------------------------------------------------------------------------------------
// Per-iteration speedup (Algorithm 2 as printed): one block per trial
// ---------------------------------------------------------------------------------------------
// S_t(tau) = (Tmax_t + c_t) / (min(tau, Tmax_t) + c_t) * done_t(tau) / (N*M) needs the completed count of
// every trial separately, so here a block owns a whole trial: its histogram in LDS is the trial's,
// and when the trial is read the block turns it into S_t for every threshold of the pass and adds
// that to its running sums (float64, one owner thread per threshold, trials in a fixed order, so the
// result does not depend on timing).  The per-block sums are added by dc_speedup_finalize_kernel.

struct TrialShared {
    double* acc;          // [p2] running sums of S_t per sorted threshold
    uint32_t* wave_tot;   // [DC_SCAN_WAVES] scratch of the block-wide prefix sum
    uint32_t* block_max;  // [1] the trial's largest worker total
};

// a / b for finite a >= 0 and b >= 1: the hardware reciprocal refined twice, the quotient corrected once.  Within an ulp
// of the exact quotient at a quarter of the instructions of an IEEE division, which a trial's end pays per threshold
// (small trials spend most of their time there).
__device__ __forceinline__ double quotient(double a, double b) {
    double r = __builtin_amdgcn_rcp(b);
    r = __builtin_fma(__builtin_fma(-b, r, 1.0), r, r);
    r = __builtin_fma(__builtin_fma(-b, r, 1.0), r, r);
    const double q = a * r;
    return __builtin_fma(__builtin_fma(-b, q, a), r, q);
}

// S_t(tau) = (Tmax + c) / (min(tau, Tmax) + c) * done / (N M)  (Algorithm 2, Appendix C.1): the iteration's speedup
// at one threshold, from its step time without drops, its step time den with them, and its completed count.
__device__ __forceinline__ double trial_speedup(long long step, long long den, double done, double per_element) {
    return quotient((double)step, (double)den) * (done * per_element);
}

// After every wave has binned its share of trial t: prefix sums over the histogram, S_t per threshold.
__device__ __forceinline__ void finish_trial(const GridView& g, const TrialShared& sh, uint32_t kc, uint32_t t,
                                             const long long* __restrict__ comm_per_trial, long long comm,
                                             double elements_per_trial, uint32_t* status) {
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const double per_element = 1.0 / elements_per_trial;
    __syncthreads();                                           // histogram and block_max complete
    const uint32_t tmax = *sh.block_max;
    const uint32_t per = (g.p2 + DC_SCAN_THREADS - 1) / DC_SCAN_THREADS;
    const uint32_t b0 = threadIdx.x * per;
    uint32_t mine = 0;
    for (uint32_t i = 0; i < per; ++i) mine += (b0 + i < g.p2) ? g.hist[b0 + i] : 0u;
    uint32_t incl = segmented_inclusive_scan<64>(mine, lane);  // prefix over the wave, then over waves
    if (lane == 63) sh.wave_tot[wave] = incl;
    __syncthreads();
    uint32_t before = 0, all = 0;
#pragma unroll
    for (uint32_t w = 0; w < DC_SCAN_WAVES; ++w) {
        const uint32_t v = sh.wave_tot[w];
        before += w < wave ? v : 0u;
        all += v;
    }
    const long long c = comm_per_trial ? comm_per_trial[t] : comm;
    if (c < 0 && threadIdx.x == 0) atomicOr(status, DC_FLAG_NEGATIVE_TAU);
    uint32_t run = before + incl - mine;                       // counted elements in bins below b0
    for (uint32_t i = 0; i < per; ++i) {
        const uint32_t b = b0 + i;
        if (b >= kc) break;
        run += g.hist[b];
        const uint32_t not_done = all - run;                   // completion times at or above threshold b
        const uint32_t tau = g.tau[b];
        const long long capped = (long long)(tau < tmax ? tau : tmax);
        const long long den = capped + c;
        if (den <= 0) { atomicOr(status, DC_FLAG_ZERO_STEP); continue; }
        const double done = elements_per_trial - (double)not_done;
        sh.acc[b] += trial_speedup((long long)tmax + c, den, done, per_element);
    }
    __syncthreads();                                           // everyone has read the histogram
    for (uint32_t i = threadIdx.x; i < g.p2; i += DC_SCAN_THREADS) g.hist[i] = 0u;
    if (threadIdx.x == 0) *sh.block_max = 0u;
    __syncthreads();
}

template <int L, int SHAPE>
__global__ __launch_bounds__(DC_SCAN_THREADS)
void dc_trial_scan_vec4_kernel(const int32_t* __restrict__ lat, uint32_t T, uint32_t N,
                               const uint32_t* __restrict__ tau_chunk, uint32_t kc, uint32_t p2,
                               const long long* __restrict__ comm_per_trial, long long comm,
                               double* __restrict__ partial, uint32_t* __restrict__ status, uint32_t max_latency,
                               uint32_t lanes_per_row, uint32_t loads_per_unit) {
    if (!launch_is_chosen<SHAPE>(status)) return;         // two launch shapes for long rows, as in dc_scan_vec4_kernel
    extern __shared__ __align__(16) unsigned char smem[];
    uint4* queue_all = reinterpret_cast<uint4*>(smem);                                  // [waves][QUEUE_ITEMS]
    uint32_t* tables = reinterpret_cast<uint32_t*>(queue_all + DC_SCAN_WAVES * QUEUE_ITEMS);
    TrialShared sh;
    sh.acc = reinterpret_cast<double*>(tables + 4 * p2);                                // 8-byte aligned: p2 is even
    sh.wave_tot = reinterpret_cast<uint32_t*>(sh.acc + p2);
    sh.block_max = sh.wave_tot + DC_SCAN_WAVES;
    for (uint32_t i = threadIdx.x; i < p2; i += DC_SCAN_THREADS) sh.acc[i] = 0.0;
    if (threadIdx.x == 0) *sh.block_max = 0u;
    const GridView g = stage_grid(tables, tau_chunk, kc, p2);

    const uint32_t lane = threadIdx.x & 63u;
    const RowShape shape = row_shape<L>(lane, lanes_per_row);
    const uint32_t R = shape.rows;
    const uint32_t M = 4 * shape.lanes;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint4* queue = queue_all + wave * QUEUE_ITEMS;
    const uint32_t nfull = N / R, tail_rows = N - nfull * R;
    // The trial is cut into units of loads_per_unit loads that the block's waves take in turn, in step
    // (one barrier per round, as in dc_scan_vec4_kernel); a trailing partial load belongs to the last unit.
    const uint32_t n_units = (nfull + (tail_rows ? 1u : 0u) + loads_per_unit - 1) / loads_per_unit;
    const uint32_t tail_unit = nfull / loads_per_unit;
    const double elements_per_trial = (double)N * (double)M;

    WaveState st{0u, 0u, 0u, 0u};
    for (uint32_t t = blockIdx.x; t < T; t += gridDim.x) {
        st.lane_max = 0u;
        for (uint32_t j0 = 0; j0 < n_units; j0 += DC_SCAN_WAVES) {
            const uint32_t j = j0 + wave;
            if (j < n_units) {
                const uint32_t f0 = j * loads_per_unit;
                const uint32_t f1 = f0 + loads_per_unit < nfull ? f0 + loads_per_unit : nfull;
                const u32x4* base = reinterpret_cast<const u32x4*>(lat + ((uint64_t)t * N + (uint64_t)f0 * R) * M) + lane;
                stream_rows<L>(st, base, f1 - f0, j == tail_unit ? tail_rows : 0u, queue, g, lane, shape);
            }
            __syncthreads();
        }
        while (st.q_count) drain(st, queue, g, lane);
        const uint32_t m = wave_max(st.lane_max);
        if (lane == 0) atomicMax(sh.block_max, m);
        finish_trial(g, sh, kc, t, comm_per_trial, comm, elements_per_trial, status);
    }
    report_range(st.check, max_latency, lane, status);
    double* out = partial + (uint64_t)blockIdx.x * p2;
    for (uint32_t i = threadIdx.x; i < p2; i += DC_SCAN_THREADS) out[i] = sh.acc[i];
}

// Small trials (a few KiB to tens of KiB, which is what a few hundred workers with tens of accumulations give): the
// per-trial step above, with its block-wide barriers, then costs more than reading the trial.  Here every wave owns
// a trial of its own, with a histogram and running sums of its own in LDS, and ends it without leaving the wave:
// each lane adds up p2/64 consecutive bins, one wave scan gives the running counts, and the lane forms S_t for its
// thresholds.  Trials go to the waves of the grid round-robin and a wave adds its trials in ascending order; the
// block's four sets of sums are added in wave order at the end, so the result does not depend on timing.
struct WaveTrial {
    double* acc_all;      // [waves][p2]
    double* acc;          // this wave's
    uint32_t per, b0;     // bins per lane at a trial's end, and the lane's first
};

// LDS behind the queues: tau | block histogram (unused here) | cells | sums [waves][p2] | histograms [waves][p2].
// Returns the grid with the calling wave's histogram; synchronises the block.
__device__ __forceinline__ GridView stage_wave_trials(unsigned char* smem, const uint32_t* __restrict__ tau_chunk,
                                                      uint32_t kc, uint32_t p2, uint32_t wave, uint32_t lane, WaveTrial* wt) {
    uint32_t* tables = reinterpret_cast<uint32_t*>(reinterpret_cast<uint4*>(smem) + DC_SCAN_WAVES * QUEUE_ITEMS);
    wt->acc_all = reinterpret_cast<double*>(tables + 4 * p2);
    uint32_t* hist_all = reinterpret_cast<uint32_t*>(wt->acc_all + DC_SCAN_WAVES * p2);
    for (uint32_t i = threadIdx.x; i < DC_SCAN_WAVES * p2; i += DC_SCAN_THREADS) { wt->acc_all[i] = 0.0; hist_all[i] = 0u; }
    GridView g = stage_grid(tables, tau_chunk, kc, p2);
    wt->acc = wt->acc_all + wave * p2;
    wt->per = (p2 + 63u) / 64u;
    wt->b0 = lane * wt->per;
    g.hist = hist_all + wave * p2;
    return g;
}

// The wave's trial t is binned: S_t for every threshold of the pass, and the histogram cleared for the next trial.
__device__ __forceinline__ void finish_wave_trial(const GridView& g, const WaveTrial& wt, uint32_t kc, uint32_t t,
                                                  uint32_t tmax, const long long* __restrict__ comm_per_trial, long long comm,
                                                  double elements_per_trial, uint32_t lane, uint32_t* status) {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");                          // the wave's histogram is complete
    const double per_element = 1.0 / elements_per_trial;
    uint32_t mine = 0;
    for (uint32_t i = 0; i < wt.per; ++i) mine += (wt.b0 + i < g.p2) ? g.hist[wt.b0 + i] : 0u;
    const uint32_t incl = segmented_inclusive_scan<64>(mine, lane);
    const uint32_t all = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
    const long long c = comm_per_trial ? comm_per_trial[t] : comm;
    if (c < 0 && lane == 0) atomicOr(status, DC_FLAG_NEGATIVE_TAU);
    uint32_t run = incl - mine;                                                     // counted elements in bins below b0
    for (uint32_t i = 0; i < wt.per; ++i) {
        const uint32_t b = wt.b0 + i;
        if (b >= g.p2) break;
        const uint32_t h = g.hist[b];
        g.hist[b] = 0u;
        if (b >= kc) continue;
        run += h;
        const uint32_t not_done = all - run;                                        // completion times at or above threshold b
        const uint32_t tau = g.tau[b];
        const long long capped = (long long)(tau < tmax ? tau : tmax);
        const long long den = capped + c;
        if (den <= 0) { atomicOr(status, DC_FLAG_ZERO_STEP); continue; }
        const double done = elements_per_trial - (double)not_done;
        wt.acc[b] += trial_speedup((long long)tmax + c, den, done, per_element);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");                          // cleared before the next trial counts
}

// partial[block][i] = the four waves' sums in wave order.  Every thread of the block must call it.
__device__ __forceinline__ void write_wave_trial_sums(const WaveTrial& wt, uint32_t p2, double* __restrict__ partial) {
    __syncthreads();
    double* out = partial + (uint64_t)blockIdx.x * p2;
    for (uint32_t i = threadIdx.x; i < p2; i += DC_SCAN_THREADS) {
        double sum = wt.acc_all[i];
#pragma unroll
        for (uint32_t w = 1; w < DC_SCAN_WAVES; ++w) sum += wt.acc_all[w * p2 + i];
        out[i] = sum;
    }
}

template <int L>
__global__ __launch_bounds__(DC_SCAN_THREADS)
void dc_trial_scan_wave_kernel(const int32_t* __restrict__ lat, uint32_t T, uint32_t N,
                               const uint32_t* __restrict__ tau_chunk, uint32_t kc, uint32_t p2,
                               const long long* __restrict__ comm_per_trial, long long comm,
                               double* __restrict__ partial, uint32_t* __restrict__ status, uint32_t max_latency,
                               uint32_t lanes_per_row) {
    extern __shared__ __align__(16) unsigned char smem[];
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    WaveTrial wt;
    const GridView g = stage_wave_trials(smem, tau_chunk, kc, p2, wave, lane, &wt);
    const RowShape shape = row_shape<L>(lane, lanes_per_row);
    const uint32_t R = shape.rows;
    const uint32_t M = 4 * shape.lanes;
    uint4* queue = reinterpret_cast<uint4*>(smem) + wave * QUEUE_ITEMS;
    const uint32_t nfull = N / R, tail_rows = N - nfull * R;
    const double elements_per_trial = (double)N * (double)M;

    WaveState st{0u, 0u, 0u, 0u};
    const uint32_t step = gridDim.x * DC_SCAN_WAVES;                                // from one of the wave's trials to its next
    constexpr int U = DC_SCAN_UNROLL;
    if (tail_rows == 0u && 2u * nfull <= (uint32_t)U) {
        // Trials of one to four loads: the loads of the wave's next U / nfull trials are requested together (a trial at
        // a time leaves one load in flight and a trial's end to wait for: 1.4 TB/s on 1 KiB trials), then the trials
        // are binned and finished one after the other, in the same order as below.
        const uint64_t stride = L ? 64u : shape.active;                             // 16-byte vectors per load
        const uint32_t batch = (uint32_t)U / nfull * nfull;                         // loads per batch: whole trials
        for (uint32_t t0 = blockIdx.x * DC_SCAN_WAVES + wave; t0 < T; t0 += step * ((uint32_t)U / nfull)) {
            u32x4 x[U];
            uint32_t tl = t0, jl = 0u;                                              // wave-uniform
#pragma unroll
            for (int k = 0; k < U; ++k) {
                x[k] = u32x4{0u, 0u, 0u, 0u};
                if ((uint32_t)k < batch && tl < T) {
                    x[k] = load_rows<L>(reinterpret_cast<const u32x4*>(lat + (uint64_t)tl * N * M) + lane + (uint64_t)jl * stride, shape);
                    if (++jl == nfull) { jl = 0u; tl += step; }
                }
            }
            uint32_t t = t0, j = 0u;
            st.lane_max = 0u;
#pragma unroll
            for (int k = 0; k < U; ++k) {
                if ((uint32_t)k < batch && t < T) {
                    const u32x4 one[1] = {x[k]};
                    process_loads<L, 1>(st, one, queue, g, lane, shape);
                    if (++j == nfull) {
                        while (st.q_count) drain(st, queue, g, lane);
                        finish_wave_trial(g, wt, kc, t, wave_max(st.lane_max), comm_per_trial, comm, elements_per_trial, lane, status);
                        st.lane_max = 0u;
                        j = 0u;
                        t += step;
                    }
                }
            }
        }
    } else {
        for (uint32_t t = blockIdx.x * DC_SCAN_WAVES + wave; t < T; t += step) {
            st.lane_max = 0u;
            const u32x4* base = reinterpret_cast<const u32x4*>(lat + (uint64_t)t * N * M) + lane;
            stream_rows<L>(st, base, nfull, tail_rows, queue, g, lane, shape);
            while (st.q_count) drain(st, queue, g, lane);
            finish_wave_trial(g, wt, kc, t, wave_max(st.lane_max), comm_per_trial, comm, elements_per_trial, lane, status);
        }
    }
    report_range(st.check, max_latency, lane, status);
    write_wave_trial_sums(wt, p2, partial);
}

// The same for rows of any length and tensors of any 4-byte alignment: a trial is one unit of the flat pass.
template <bool SMALL>
__global__ __launch_bounds__(DC_SCAN_THREADS)
void dc_trial_scan_wave_flat_kernel(const int32_t* __restrict__ lat, uint32_t T, uint32_t N, uint32_t M,
                                    const uint32_t* __restrict__ tau_chunk, uint32_t kc, uint32_t p2,
                                    const long long* __restrict__ comm_per_trial, long long comm,
                                    double* __restrict__ partial, uint32_t* __restrict__ status, uint32_t max_latency) {
    extern __shared__ __align__(16) unsigned char smem[];
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    WaveTrial wt;
    const GridView g = stage_wave_trials(smem, tau_chunk, kc, p2, wave, lane, &wt);
    uint4* queue = reinterpret_cast<uint4*>(smem) + wave * QUEUE_ITEMS;
    const FlatTensor f = flat_tensor(lat, (uint64_t)T * N * M, M);
    const uint32_t per_trial = N * M;                                               // at most DC_WAVE_TRIAL_ELEMENTS
    const double elements_per_trial = (double)N * (double)M;

    WaveState st{0u, 0u, 0u, 0u};
    for (uint32_t t = blockIdx.x * DC_SCAN_WAVES + wave; t < T; t += gridDim.x * DC_SCAN_WAVES) {
        st.lane_max = 0u;
        flat_stream_unit<SMALL>(st.check, f, (uint64_t)t * per_trial, per_trial, lane,
                                [&](uint4 p, uint32_t vm, uint32_t, uint32_t) { flat_count(st, p, vm, queue, g, lane); });
        while (st.q_count) drain(st, queue, g, lane);
        finish_wave_trial(g, wt, kc, t, wave_max(st.lane_max), comm_per_trial, comm, elements_per_trial, lane, status);
    }
    report_range(st.check, max_latency, lane, status);
    write_wave_trial_sums(wt, p2, partial);
}

// Any M >= 1, any 4-byte alignment: the waves of the block take the trial's units (runs of whole rows) in
// turn, in step, with the flat pass of dc_scan_flat_kernel.
template <bool SMALL>
__global__ __launch_bounds__(DC_SCAN_THREADS)
void dc_trial_scan_flat_kernel(const int32_t* __restrict__ lat, uint32_t T, uint32_t N, uint32_t M,
                               uint32_t rows_per_unit, const uint32_t* __restrict__ tau_chunk, uint32_t kc, uint32_t p2,
                               const long long* __restrict__ comm_per_trial, long long comm,
                               double* __restrict__ partial, uint32_t* __restrict__ status, uint32_t max_latency) {
    extern __shared__ __align__(16) unsigned char smem[];
    uint4* queue_all = reinterpret_cast<uint4*>(smem);                                  // [waves][QUEUE_ITEMS]
    uint32_t* tables = reinterpret_cast<uint32_t*>(queue_all + DC_SCAN_WAVES * QUEUE_ITEMS);
    TrialShared sh;
    sh.acc = reinterpret_cast<double*>(tables + 4 * p2);
    sh.wave_tot = reinterpret_cast<uint32_t*>(sh.acc + p2);
    sh.block_max = sh.wave_tot + DC_SCAN_WAVES;
    for (uint32_t i = threadIdx.x; i < p2; i += DC_SCAN_THREADS) sh.acc[i] = 0.0;
    if (threadIdx.x == 0) *sh.block_max = 0u;
    const GridView g = stage_grid(tables, tau_chunk, kc, p2);

    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint4* queue = queue_all + wave * QUEUE_ITEMS;
    const FlatTensor f = flat_tensor(lat, (uint64_t)T * N * M, M);
    const uint32_t n_units = (N + rows_per_unit - 1) / rows_per_unit;
    const double elements_per_trial = (double)N * (double)M;

    WaveState st{0u, 0u, 0u, 0u};
    for (uint32_t t = blockIdx.x; t < T; t += gridDim.x) {
        st.lane_max = 0u;
        for (uint32_t j0 = 0; j0 < n_units; j0 += DC_SCAN_WAVES) {                        // block-uniform bound
            const uint32_t j = j0 + wave;
            if (j < n_units) {
                const uint32_t row0 = j * rows_per_unit;
                const uint32_t rows = (N - row0) < rows_per_unit ? (N - row0) : rows_per_unit;
                flat_stream_unit<SMALL>(st.check, f, ((uint64_t)t * N + row0) * M, rows * M, lane,
                                        [&](uint4 p, uint32_t vm, uint32_t, uint32_t) { flat_count(st, p, vm, queue, g, lane); });
            }
            __syncthreads();
        }
        while (st.q_count) drain(st, queue, g, lane);
        const uint32_t m = wave_max(st.lane_max);
        if (lane == 0) atomicMax(sh.block_max, m);
        finish_trial(g, sh, kc, t, comm_per_trial, comm, elements_per_trial, status);
    }
    report_range(st.check, max_latency, lane, status);
    double* out = partial + (uint64_t)blockIdx.x * p2;
    for (uint32_t i = threadIdx.x; i < p2; i += DC_SCAN_THREADS) out[i] = sh.acc[i];
}

// out_seff[j] = (sum of the per-block sums for j's sorted position) / T.  A block of 256 threads serves 8
// thresholds; the range of blocks is cut into 32 fixed slices that are summed in order (eight values requested at a
// time, added one after the other) and then combined in slice order, so the grouping of the float additions never
// changes between calls.  (32 thresholds x 8 slices per block left a handful of blocks to read several MB of sums;
// this shape took a call on 82 MB with 128 thresholds from 94 to 54 us.)
__global__ __launch_bounds__(256)
void dc_speedup_finalize_kernel(const double* __restrict__ partial, uint32_t narrow_blocks, uint32_t wide_blocks,
                                uint32_t* __restrict__ status, const int64_t* __restrict__ tau_sorted, uint32_t p2,
                                uint32_t kc, uint32_t chunk0, const uint32_t* __restrict__ pos, uint32_t K,
                                double trials, double* __restrict__ out_seff) {
    constexpr uint32_t PER_BLOCK = 8, SLICES = 32;
    __shared__ double slice_sum[SLICES][PER_BLOCK];
    if (blockIdx.x == 0 && threadIdx.x == 0 && chunk0 == 0u && tau_sorted[0] < 0) atomicOr(status, DC_FLAG_NEGATIVE_TAU);
    // per-block sums were written by the launch of the per-trial kernel that the sample chose
    const uint32_t blocks = wide_blocks > narrow_blocks && status[1] != 0u ? wide_blocks : narrow_blocks;
    const uint32_t jj = threadIdx.x % PER_BLOCK, slice = threadIdx.x / PER_BLOCK;
    const uint32_t j = blockIdx.x * PER_BLOCK + jj;
    const uint32_t p = j < K ? pos[j] : 0xFFFFFFFFu;
    const bool mine = p >= chunk0 && p < chunk0 + kc;
    const uint32_t per = (blocks + SLICES - 1) / SLICES;
    const uint32_t b0 = slice * per < blocks ? slice * per : blocks, b1 = b0 + per < blocks ? b0 + per : blocks;
    double sum = 0.0;
    if (mine) {
        const double* col = partial + (p - chunk0);
        uint32_t b = b0;
        for (; b + 8u <= b1; b += 8u) {
            double v[8];
#pragma unroll
            for (uint32_t q = 0; q < 8; ++q) v[q] = col[(uint64_t)(b + q) * p2];
#pragma unroll
            for (uint32_t q = 0; q < 8; ++q) sum += v[q];
        }
        for (; b < b1; ++b) sum += col[(uint64_t)b * p2];
    }
    slice_sum[slice][jj] = sum;
    __syncthreads();
    if (slice != 0 || !mine) return;
    sum = 0.0;
#pragma unroll
    for (uint32_t q = 0; q < SLICES; ++q) sum += slice_sum[q][jj];
    out_seff[j] = sum / trials;
}

namespace dc {

template <int L>
static int resident_trial_vec4(size_t lds) {
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, dc_trial_scan_vec4_kernel<L, 0>, DC_SCAN_THREADS, lds) != hipSuccess) n = 0;
    return n;
}

size_t trial_scan_lds_bytes(const Plan& p);

// Blocks of the per-trial kernel that one compute unit holds at a time (0 if the query fails).
template <int L>
static int resident_trial_wave(size_t lds) {
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, dc_trial_scan_wave_kernel<L>, DC_SCAN_THREADS, lds) != hipSuccess) n = 0;
    return n;
}

int trial_scan_blocks_per_cu(const Plan& p) {
    const size_t lds = trial_scan_lds_bytes(p);
    int n = 0;
    if (p.wave_trials && !p.vec4) {
        if ((p.M < 4 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, dc_trial_scan_wave_flat_kernel<true>, DC_SCAN_THREADS, lds)
                     : hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, dc_trial_scan_wave_flat_kernel<false>, DC_SCAN_THREADS, lds)) != hipSuccess) n = 0;
        return n;
    }
    if (p.wave_trials) {
        switch (p.M / 4) {
            case 1:  return resident_trial_wave<1>(lds);
            case 2:  return resident_trial_wave<2>(lds);
            case 4:  return resident_trial_wave<4>(lds);
            case 8:  return resident_trial_wave<8>(lds);
            case 16: return resident_trial_wave<16>(lds);
            case 32: return resident_trial_wave<32>(lds);
            case 64: return resident_trial_wave<64>(lds);
            default: return resident_trial_wave<0>(lds);
        }
    }
    if (!p.vec4) {
        if ((p.M < 4 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, dc_trial_scan_flat_kernel<true>, DC_SCAN_THREADS, lds)
                     : hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, dc_trial_scan_flat_kernel<false>, DC_SCAN_THREADS, lds)) != hipSuccess) n = 0;
        return n;
    }
    switch (p.M / 4) {
        case 1:  return resident_trial_vec4<1>(lds);
        case 2:  return resident_trial_vec4<2>(lds);
        case 4:  return resident_trial_vec4<4>(lds);
        case 8:  return resident_trial_vec4<8>(lds);
        case 16: return resident_trial_vec4<16>(lds);
        case 32: return resident_trial_vec4<32>(lds);
        case 64: return resident_trial_vec4<64>(lds);
        default: return resident_trial_vec4<0>(lds);
    }
}

size_t trial_scan_lds_bytes(const Plan& p) {
    if (p.wave_trials)                                                                      // grid + every wave's sums and histogram + queues
        return (size_t)p.p2 * 16 + (size_t)DC_SCAN_WAVES * p.p2 * 12 + (size_t)DC_SCAN_WAVES * QUEUE_ITEMS * sizeof(uint4);
    const size_t tables = (size_t)p.p2 * 16 + (size_t)p.p2 * 8 + (DC_SCAN_WAVES + 1) * 4;   // grid + sums + scratch
    return tables + (size_t)DC_SCAN_WAVES * QUEUE_ITEMS * sizeof(uint4);                    // + queues
}

template <int L>
static void launch_trial_vec4(const Plan& p, const int32_t* lat, const uint32_t* tau_chunk, uint32_t kc,
                              const int64_t* comm_per_trial, int64_t comm, double* partial, uint32_t* status,
                              hipStream_t stream) {
    if (p.grid_wide > p.grid) {                     // the sample decides on the device which of the two launches works
        if constexpr (L == 32 || L == 64) {
            hipLaunchKernelGGL((dc_trial_scan_vec4_kernel<L, 1>), dim3(p.grid), dim3(DC_SCAN_THREADS), trial_scan_lds_bytes(p),
                               stream, lat, p.T, p.N, tau_chunk, kc, p.p2, (const long long*)comm_per_trial, (long long)comm,
                               partial, status, p.max_latency, p.M / 4, p.per_unit);
            hipLaunchKernelGGL((dc_trial_scan_vec4_kernel<L, 2>), dim3(p.grid_wide), dim3(DC_SCAN_THREADS),
                               trial_scan_lds_bytes(p), stream, lat, p.T, p.N, tau_chunk, kc, p.p2,
                               (const long long*)comm_per_trial, (long long)comm, partial, status, p.max_latency, p.M / 4,
                               p.per_unit);
            return;
        }
    }
    hipLaunchKernelGGL((dc_trial_scan_vec4_kernel<L, 0>), dim3(p.grid), dim3(DC_SCAN_THREADS), trial_scan_lds_bytes(p),
                       stream, lat, p.T, p.N, tau_chunk, kc, p.p2, (const long long*)comm_per_trial, (long long)comm,
                       partial, status, p.max_latency, p.M / 4, p.per_unit);
}

void launch_trial_scan(const Plan& p, const int32_t* lat, const uint32_t* tau_chunk, uint32_t kc,
                       const int64_t* comm_per_trial, int64_t comm, double* partial, uint32_t* status,
                       hipStream_t stream) {
    if (p.wave_trials && !p.vec4) {
        if (p.M < 4)
            hipLaunchKernelGGL(dc_trial_scan_wave_flat_kernel<true>, dim3(p.grid), dim3(DC_SCAN_THREADS), trial_scan_lds_bytes(p),
                               stream, lat, p.T, p.N, p.M, tau_chunk, kc, p.p2, (const long long*)comm_per_trial,
                               (long long)comm, partial, status, p.max_latency);
        else
            hipLaunchKernelGGL(dc_trial_scan_wave_flat_kernel<false>, dim3(p.grid), dim3(DC_SCAN_THREADS), trial_scan_lds_bytes(p),
                               stream, lat, p.T, p.N, p.M, tau_chunk, kc, p.p2, (const long long*)comm_per_trial,
                               (long long)comm, partial, status, p.max_latency);
        return;
    }
    if (p.wave_trials) {
#define DC_WAVE_CASE(l) hipLaunchKernelGGL(dc_trial_scan_wave_kernel<l>, dim3(p.grid), dim3(DC_SCAN_THREADS), trial_scan_lds_bytes(p), \
                                           stream, lat, p.T, p.N, tau_chunk, kc, p.p2, (const long long*)comm_per_trial,              \
                                           (long long)comm, partial, status, p.max_latency, p.M / 4)
        switch (p.M / 4) {
            case 1:  DC_WAVE_CASE(1); break;
            case 2:  DC_WAVE_CASE(2); break;
            case 4:  DC_WAVE_CASE(4); break;
            case 8:  DC_WAVE_CASE(8); break;
            case 16: DC_WAVE_CASE(16); break;
            case 32: DC_WAVE_CASE(32); break;
            case 64: DC_WAVE_CASE(64); break;
            default: DC_WAVE_CASE(0); break;
        }
#undef DC_WAVE_CASE
        return;
    }
    if (!p.vec4) {
        if (p.M < 4)
            hipLaunchKernelGGL(dc_trial_scan_flat_kernel<true>, dim3(p.grid), dim3(DC_SCAN_THREADS),
                               trial_scan_lds_bytes(p), stream, lat, p.T, p.N, p.M, p.per_unit, tau_chunk, kc, p.p2,
                               (const long long*)comm_per_trial, (long long)comm, partial, status, p.max_latency);
        else
            hipLaunchKernelGGL(dc_trial_scan_flat_kernel<false>, dim3(p.grid), dim3(DC_SCAN_THREADS),
                               trial_scan_lds_bytes(p), stream, lat, p.T, p.N, p.M, p.per_unit, tau_chunk, kc, p.p2,
                               (const long long*)comm_per_trial, (long long)comm, partial, status, p.max_latency);
        return;
    }
    switch (p.M / 4) {
        case 1:  launch_trial_vec4<1>(p, lat, tau_chunk, kc, comm_per_trial, comm, partial, status, stream); break;
        case 2:  launch_trial_vec4<2>(p, lat, tau_chunk, kc, comm_per_trial, comm, partial, status, stream); break;
        case 4:  launch_trial_vec4<4>(p, lat, tau_chunk, kc, comm_per_trial, comm, partial, status, stream); break;
        case 8:  launch_trial_vec4<8>(p, lat, tau_chunk, kc, comm_per_trial, comm, partial, status, stream); break;
        case 16: launch_trial_vec4<16>(p, lat, tau_chunk, kc, comm_per_trial, comm, partial, status, stream); break;
        case 32: launch_trial_vec4<32>(p, lat, tau_chunk, kc, comm_per_trial, comm, partial, status, stream); break;
        case 64: launch_trial_vec4<64>(p, lat, tau_chunk, kc, comm_per_trial, comm, partial, status, stream); break;
        default: launch_trial_vec4<0>(p, lat, tau_chunk, kc, comm_per_trial, comm, partial, status, stream); break;
    }
}

void launch_speedup_finalize(const Plan& p, const double* partial, uint32_t kc, uint32_t chunk0, const uint32_t* pos,
                             uint32_t* status, const int64_t* tau_sorted, double* out_seff, hipStream_t stream) {
    hipLaunchKernelGGL(dc_speedup_finalize_kernel, dim3((p.K + 7) / 8), dim3(256), 0, stream, partial, p.grid,
                       p.grid_wide, status, tau_sorted, p.p2, kc, chunk0, pos, p.K, (double)p.T, out_seff);
}

}  // namespace dc
