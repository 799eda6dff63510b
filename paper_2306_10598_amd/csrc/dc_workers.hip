// Per-worker statistics of the iteration time: streaming kernels, the sum over blocks, and their launcher.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dc_device.h"
#include "dc_internal.h"

// ---------------------------------------------------------------------------------------------
// Per-worker statistics of the compute time T_n = sum_m t_n^(m): sum and sum of squares over iterations
// ---------------------------------------------------------------------------------------------
// A block owns whole trials and a wave always the same rows of each trial, so every worker's accumulators
// in LDS ([3][N]: sum, squares low word, squares high word) have one owner lane and need no atomics.

__device__ __forceinline__ void add_worker_total(unsigned long long* acc, uint32_t N, uint32_t n, uint32_t total) {
    acc[n] += total;
    const unsigned long long sq = (unsigned long long)total * total;
    const unsigned long long before = acc[N + n];
    acc[N + n] = before + sq;
    if (before + sq < before) acc[2 * N + n] += 1ull;
}

template <int L>
__global__ __launch_bounds__(DC_SCAN_THREADS)
void dc_worker_totals_vec4_kernel(const int32_t* __restrict__ lat, uint64_t trial_stride, uint32_t T, uint32_t N,
                                  unsigned long long* __restrict__ partial, uint32_t* __restrict__ status,
                                  uint32_t max_latency, uint32_t lanes_per_row, uint32_t trials_by_wave,
                                  uint32_t rows_per_load) {
    // trials_by_wave: a trial is fewer whole loads than the block has waves (8 workers of 32 accumulations are one), so
    // every wave takes whole trials of its own, the block's trials w, w + 4, ..., and keeps accumulators of its own
    // ([waves][3][N] in LDS, added up at the end); otherwise the waves share a trial's loads and one set of accumulators
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned long long* acc_all = reinterpret_cast<unsigned long long*>(smem);
    const uint32_t sets = trials_by_wave ? DC_SCAN_WAVES : 1u;
    for (uint32_t i = threadIdx.x; i < sets * 3 * N; i += DC_SCAN_THREADS) acc_all[i] = 0ull;
    __syncthreads();

    constexpr int U = DC_SCAN_UNROLL;
    const uint32_t lane = threadIdx.x & 63u;
    const RowShape shape = row_shape<L>(lane, lanes_per_row, rows_per_load);
    const uint32_t R = shape.rows, M = 4 * shape.lanes;
    const uint64_t stride = L ? 64u : shape.active;
    const bool row_end = shape.ok && shape.pos == shape.lanes - 1;      // this lane ends a row: it holds the total
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t nfull = N / R, tail_rows = N - nfull * R;
    const uint32_t lo = trials_by_wave ? 0u : (uint32_t)((uint64_t)nfull * wave / DC_SCAN_WAVES);
    const uint32_t hi = trials_by_wave ? nfull : (uint32_t)((uint64_t)nfull * (wave + 1) / DC_SCAN_WAVES);
    unsigned long long* acc = acc_all + (trials_by_wave ? wave * 3u * N : 0u);
    uint32_t check = 0u;
    const uint32_t len = hi - lo;                                   // the wave's loads per trial
    if (len >= 4u * (uint32_t)U) {
        for (uint32_t t = blockIdx.x; t < T; t += gridDim.x) {
            const u32x4* base = reinterpret_cast<const u32x4*>(lat + (uint64_t)t * trial_stride + (uint64_t)lo * R * M) + lane;
            uint32_t i = 0;
            for (; i + U <= len; i += U) {
                u32x4 x[U];
                uint32_t incl[U];
#pragma unroll
                for (int k = 0; k < U; ++k) x[k] = load_rows<L>(base + (uint64_t)(i + k) * stride, shape);
                completion_times<L, U>(x, incl, lane, shape);
#pragma unroll
                for (int k = 0; k < U; ++k) {
                    check = umax(check, umax(umax(x[k].x, x[k].y), umax(x[k].z, x[k].w)));
                    if (row_end) add_worker_total(acc, N, (lo + i + k) * R + shape.row, incl[k]);
                }
            }
            if (i < len) {                                          // the rest of the trial's loads as one batch
                const uint32_t n = len - i;                         // wave-uniform
                u32x4 x[U];
                uint32_t incl[U];
#pragma unroll
                for (int k = 0; k < U; ++k) {
                    x[k] = u32x4{0u, 0u, 0u, 0u};
                    if ((uint32_t)k < n) x[k] = load_rows<L>(base + (uint64_t)(i + k) * stride, shape);
                }
                completion_times<L, U>(x, incl, lane, shape);
#pragma unroll
                for (int k = 0; k < U; ++k) {
                    check = umax(check, umax(umax(x[k].x, x[k].y), umax(x[k].z, x[k].w)));
                    if ((uint32_t)k < n && row_end) add_worker_total(acc, N, (lo + i + k) * R + shape.row, incl[k]);
                }
            }
        }
    } else {
        // Few loads per trial (64 workers of 32 accumulations: two per wave; 200 of 64: twelve): the wave's loads
        // over all of the block's trials are taken U at a time whatever the trial they belong to, which keeps as
        // many loads in flight as long trials do.  A worker's row is always the same lane's, so two items of a
        // batch that belong to one worker are added one after the other by that lane.
        const uint32_t block_trials = blockIdx.x < T ? (T - blockIdx.x + gridDim.x - 1u) / gridDim.x : 0u;
        // the trials whose loads this wave takes: all of the block's, or every fourth from the wave's own number on
        const uint32_t my_trials = !trials_by_wave ? block_trials
                                 : block_trials > wave ? (block_trials - wave + DC_SCAN_WAVES - 1u) / DC_SCAN_WAVES : 0u;
        const uint32_t first_trial = trials_by_wave ? wave : 0u, trial_step = trials_by_wave ? DC_SCAN_WAVES : 1u;
        const uint64_t items = (uint64_t)my_trials * len;
        uint32_t at_trial = 0u, at_load = 0u;                       // the next item: which of the block's trials, which load
        for (uint64_t k0 = 0; k0 < items; k0 += U) {
            const uint32_t n = items - k0 < (uint64_t)U ? (uint32_t)(items - k0) : (uint32_t)U;      // wave-uniform
            u32x4 x[U];
            uint32_t incl[U], load_of[U];
#pragma unroll
            for (int k = 0; k < U; ++k) {
                x[k] = u32x4{0u, 0u, 0u, 0u};
                load_of[k] = at_load;
                if ((uint32_t)k < n) {
                    const uint64_t t = (uint64_t)blockIdx.x + (uint64_t)(first_trial + at_trial * trial_step) * gridDim.x;
                    const u32x4* p = reinterpret_cast<const u32x4*>(lat + t * trial_stride + (uint64_t)(lo + at_load) * R * M) + lane;
                    x[k] = load_rows<L>(p, shape);
                    if (++at_load == len) { at_load = 0u; ++at_trial; }
                }
            }
            completion_times<L, U>(x, incl, lane, shape);
#pragma unroll
            for (int k = 0; k < U; ++k) {
                check = umax(check, umax(umax(x[k].x, x[k].y), umax(x[k].z, x[k].w)));
                if ((uint32_t)k < n && row_end) add_worker_total(acc, N, (lo + load_of[k]) * R + shape.row, incl[k]);
            }
        }
    }
    for (uint32_t t = blockIdx.x; t < T; t += gridDim.x) {          // the trial's last, partial load
        const u32x4* base = reinterpret_cast<const u32x4*>(lat + (uint64_t)t * trial_stride + (uint64_t)lo * R * M) + lane;
        if (wave == DC_SCAN_WAVES - 1 && tail_rows) {
            const bool valid = lane < tail_rows * shape.lanes;
            u32x4 x[1] = {{0u, 0u, 0u, 0u}};
            if (valid) x[0] = __builtin_nontemporal_load(base + (uint64_t)(hi - lo) * stride);
            uint32_t incl[1];
            completion_times<L, 1>(x, incl, lane, shape);
            check = umax(check, umax(umax(x[0].x, x[0].y), umax(x[0].z, x[0].w)));
            if (valid && row_end) add_worker_total(acc, N, nfull * R + shape.row, incl[0]);
        }
    }
    report_range(check, max_latency, lane, status);
    __syncthreads();
    unsigned long long* out = partial + (uint64_t)blockIdx.x * 3 * N;
    if (!trials_by_wave) {
        for (uint32_t i = threadIdx.x; i < 3 * N; i += DC_SCAN_THREADS) out[i] = acc_all[i];
        return;
    }
    for (uint32_t n = threadIdx.x; n < N; n += DC_SCAN_THREADS) {  // the waves' sums, the squares in 128 bits
        unsigned long long sum = 0ull;
        unsigned __int128 sq = 0;
        for (uint32_t w = 0; w < DC_SCAN_WAVES; ++w) {
            const unsigned long long* a = acc_all + w * 3u * N;
            sum += a[n];
            sq += ((unsigned __int128)a[2u * N + n] << 64) | a[N + n];
        }
        out[n] = sum;
        out[N + n] = (unsigned long long)sq;
        out[2u * N + n] = (unsigned long long)(sq >> 64);
    }
}

// Any M >= 1, any 4-byte alignment: the flat pass; the lane that holds a row's last element holds its total.
// Wave w takes units w, w + 4, ... of every trial, so a worker's accumulators always belong to the same wave.
template <bool SMALL>
__global__ __launch_bounds__(DC_SCAN_THREADS)
void dc_worker_totals_flat_kernel(const int32_t* __restrict__ lat, uint64_t extent, uint64_t trial_stride, uint32_t T,
                                  uint32_t N, uint32_t M, uint32_t rows_per_unit, unsigned long long* __restrict__ partial,
                                  uint32_t* __restrict__ status, uint32_t max_latency) {
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned long long* acc = reinterpret_cast<unsigned long long*>(smem);
    for (uint32_t i = threadIdx.x; i < 3 * N; i += DC_SCAN_THREADS) acc[i] = 0ull;
    __syncthreads();
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const FlatTensor f = flat_tensor(lat, extent, M);
    const uint32_t n_units = (N + rows_per_unit - 1) / rows_per_unit;
    uint32_t check = 0u;
    for (uint32_t t = blockIdx.x; t < T; t += gridDim.x)
        for (uint32_t j = wave; j < n_units; j += DC_SCAN_WAVES) {
            const uint32_t row0 = j * rows_per_unit;
            const uint32_t rows = (N - row0) < rows_per_unit ? (N - row0) : rows_per_unit;
            // few waves per compute unit here (the accumulators fill the LDS), so more loads in flight per lane
            flat_stream_unit<SMALL, DC_SCAN_UNROLL>(check, f, (uint64_t)t * trial_stride + (uint64_t)row0 * M, rows * M, lane,
                                                    [&](uint4 p, uint32_t vm, uint32_t pos0, uint32_t row) {
                const uint32_t val[4] = {p.x, p.y, p.z, p.w};
                if constexpr (SMALL) {
#pragma unroll
                    for (uint32_t c = 0; c < 4; ++c) {
                        const uint32_t e = pos0 + c;                      // < 6: position counted from the first element's row head
                        if (((vm >> c) & 1u) && e % M == M - 1u) add_worker_total(acc, N, row0 + row + e / M, val[c]);
                    }
                } else {
                    const uint32_t ce = M - pos0;                         // the row of the first element ends at component ce - 1
                    if (ce <= 4u && ((vm >> (ce - 1u)) & 1u))
                        add_worker_total(acc, N, row0 + row, ce == 1u ? val[0] : ce == 2u ? val[1] : ce == 3u ? val[2] : val[3]);
                }
            });
        }
    report_range(check, max_latency, lane, status);
    __syncthreads();
    unsigned long long* out = partial + (uint64_t)blockIdx.x * 3 * N;
    for (uint32_t i = threadIdx.x; i < 3 * N; i += DC_SCAN_THREADS) out[i] = acc[i];
}

// result[3][N] = sums over blocks (the 128-bit squares with carry).  A block of 1024 threads takes 32 workers; each of
// its 32 groups of 32 threads adds every 32nd block's partial sums (32 consecutive 8-byte words per read, eight rows
// requested together: one thread after the other through 64 rows had taken 23 us, more than the streaming kernel on
// a small tensor), then the 32 partial results are added in two fixed stages.
#define DC_FINAL_SLICES 32
#define DC_FINAL_BATCH 8
__global__ __launch_bounds__(32 * DC_FINAL_SLICES)
void dc_worker_totals_final_kernel(const unsigned long long* __restrict__ partial, uint32_t blocks, uint32_t N,
                                   unsigned long long* __restrict__ result) {
    __shared__ unsigned long long part[DC_FINAL_SLICES][32][3];
    const uint32_t w = threadIdx.x & 31u, slice = threadIdx.x >> 5;
    const uint32_t n = blockIdx.x * 32u + w;
    unsigned long long sum = 0ull;
    unsigned __int128 sq = 0;
    if (n < N) {
        for (uint32_t b0 = slice; b0 < blocks; b0 += DC_FINAL_SLICES * DC_FINAL_BATCH) {
            unsigned long long s[DC_FINAL_BATCH], lo[DC_FINAL_BATCH], hi[DC_FINAL_BATCH];
#pragma unroll
            for (int k = 0; k < DC_FINAL_BATCH; ++k) {
                const uint32_t b = b0 + (uint32_t)k * DC_FINAL_SLICES;
                s[k] = lo[k] = hi[k] = 0ull;
                if (b < blocks) {
                    const unsigned long long* in = partial + (uint64_t)b * 3 * N;
                    s[k] = in[n];
                    lo[k] = in[N + n];
                    hi[k] = in[2 * N + n];
                }
            }
#pragma unroll
            for (int k = 0; k < DC_FINAL_BATCH; ++k) {
                sum += s[k];
                sq += ((unsigned __int128)hi[k] << 64) | lo[k];
            }
        }
    }
    part[slice][w][0] = sum;
    part[slice][w][1] = (unsigned long long)sq;
    part[slice][w][2] = (unsigned long long)(sq >> 64);
    __syncthreads();
    if (slice < 4u) {                                               // 32 -> 4: slices slice, slice + 4, ...
        for (uint32_t q = slice + 4u; q < DC_FINAL_SLICES; q += 4u) {
            sum += part[q][w][0];
            sq += ((unsigned __int128)part[q][w][2] << 64) | part[q][w][1];
        }
        part[slice][w][0] = sum;
        part[slice][w][1] = (unsigned long long)sq;
        part[slice][w][2] = (unsigned long long)(sq >> 64);
    }
    __syncthreads();
    if (slice == 0 && n < N) {
        for (uint32_t q = 1; q < 4u; ++q) {
            sum += part[q][w][0];
            sq += ((unsigned __int128)part[q][w][2] << 64) | part[q][w][1];
        }
        result[n] = sum;
        result[N + n] = (unsigned long long)sq;
        result[2 * N + n] = (unsigned long long)(sq >> 64);
    }
}

__global__ void dc_clear_status_kernel(uint32_t* status) { *status = 0u; }

namespace dc {

template <int L>
static void launch_worker_vec4(const Plan& p, const int32_t* lat, unsigned long long* partial, uint32_t* status,
                               hipStream_t stream, uint32_t rows_override) {
    // a trial of fewer whole loads than a block has waves: every wave takes whole trials (and accumulators) of its own
    const uint32_t rows_per_load = rows_override ? rows_override : 64u / (p.M / 4u);
    const uint32_t by_wave = (p.N % rows_per_load == 0u && p.N / rows_per_load < DC_SCAN_WAVES) ? 1u : 0u;
    hipLaunchKernelGGL(dc_worker_totals_vec4_kernel<L>, dim3(p.grid), dim3(DC_SCAN_THREADS),
                       (size_t)p.N * 24 * (by_wave ? DC_SCAN_WAVES : 1u), stream, lat, p.stride, p.T, p.N, partial, status,
                       p.max_latency, p.M / 4, by_wave, rows_override);
}

// partial: [grid][3][N] u64; result: [3][N] u64 (sum, squares low, squares high per worker)
// before/after: optional events recorded around the streaming kernel
void launch_worker_totals(const Plan& p, const int32_t* lat, unsigned long long* partial,
                          unsigned long long* result, uint32_t* status, hipStream_t stream, hipEvent_t before,
                          hipEvent_t after) {
    hipLaunchKernelGGL(dc_clear_status_kernel, dim3(1), dim3(1), 0, stream, status);
    if (before) (void)hipEventRecord(before, stream);
    if (!p.vec4) {
        if (p.M < 4)
            hipLaunchKernelGGL(dc_worker_totals_flat_kernel<true>, dim3(p.grid), dim3(DC_SCAN_THREADS),
                               (size_t)p.N * 24, stream, lat, p.extent, p.stride, p.T, p.N, p.M, p.per_unit, partial, status,
                               p.max_latency);
        else
            hipLaunchKernelGGL(dc_worker_totals_flat_kernel<false>, dim3(p.grid), dim3(DC_SCAN_THREADS),
                               (size_t)p.N * 24, stream, lat, p.extent, p.stride, p.T, p.N, p.M, p.per_unit, partial, status,
                               p.max_latency);
    } else {
        // A small trial whose worker count is no whole number of full loads is taken as shorter loads (a divisor of N
        // rows each, if that keeps half of the lanes busy or holds the whole trial), so that no wave is left with a
        // partial load per trial: the instantiation for any row length.
        uint32_t rows_override = 0u;
        const uint32_t fit = 64u / (p.M / 4u);
        if (p.N % fit != 0u && p.N < 8u * fit) {
            uint32_t r = fit < p.N ? fit : p.N;
            while (r > 1u && p.N % r) --r;
            if (r * (p.M / 4u) >= 32u || r == p.N) rows_override = r;
        }
        switch (rows_override ? 0u : p.M / 4) {
            case 1:  launch_worker_vec4<1>(p, lat, partial, status, stream, 0u); break;
            case 2:  launch_worker_vec4<2>(p, lat, partial, status, stream, 0u); break;
            case 4:  launch_worker_vec4<4>(p, lat, partial, status, stream, 0u); break;
            case 8:  launch_worker_vec4<8>(p, lat, partial, status, stream, 0u); break;
            case 16: launch_worker_vec4<16>(p, lat, partial, status, stream, 0u); break;
            case 32: launch_worker_vec4<32>(p, lat, partial, status, stream, 0u); break;
            case 64: launch_worker_vec4<64>(p, lat, partial, status, stream, 0u); break;
            default: launch_worker_vec4<0>(p, lat, partial, status, stream, rows_override); break;
        }
    }
    if (after) (void)hipEventRecord(after, stream);
    hipLaunchKernelGGL(dc_worker_totals_final_kernel, dim3((p.N + 31) / 32), dim3(32 * DC_FINAL_SLICES), 0, stream,
                       partial, p.grid, p.N, result);
}

}  // namespace dc
