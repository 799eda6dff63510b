// dc_scan_row_lane_kernel: rows of 17 to 63 elements whose length is no multiple of 4 (where dc_scan_rows_kernel does
// not take them), on 16-byte aligned trials with N*M a multiple of 4.
//
// Neither of the other fast kernels suits such rows: a 16-byte load never holds whole rows, and a lane that keeps
// four whole rows in registers needs a hundred of them and more.  Here a lane owns ONE row and keeps only its running
// total.  A wave copies a chunk of 64 consecutive rows (64 M elements = 16 M vectors, coalesced 16-byte loads, all
// of the next chunk's in flight while this one is worked on) into its own stretch of LDS as it lies in memory, and
// lane l then reads words l M ... l M + M - 1 one by one: for odd M the 64 lanes fall on different banks, for
// M = 2 mod 4 two lanes share one.  The row's total is its last completion time; since completion times do not
// decrease along a row (latencies >= 0) the thresholds are met from the row's end backwards,
// P[M-2-s] = P[M-1-s] - lat[M-1-s] with the latency read from LDS again, and the wave stops at the first step in
// which no lane reaches the smallest threshold: one or two steps with the usual grids.  When most lanes are inside
// the grid, or the walk goes on after two steps, four steps go at once.  About three lane-operations per element instead of the 17 of the kernel for
// arbitrary rows.  NB = 16-byte vectors a lane holds for one chunk (at least M / 4).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dc_device.h"
#include "dc_internal.h"

template <int NB>
__device__ __forceinline__ void row_lane_load(u32x4 (&x)[NB], const u32x4* src, uint32_t nv, uint32_t lane) {
#pragma unroll
    for (int k = 0; k < NB; ++k) {
        const uint32_t i = 64u * k + lane;
        x[k] = u32x4{0u, 0u, 0u, 0u};
        if (i < nv) x[k] = __builtin_nontemporal_load(src + i);
    }
}

template <int NB>
__global__ __launch_bounds__(DC_SCAN_THREADS)
void dc_scan_row_lane_kernel(const int32_t* __restrict__ lat, uint64_t trial_stride, uint32_t N, uint32_t M, uint32_t units,
                             uint32_t units_per_trial, uint32_t run, uint32_t chunks_per_unit,
                             const uint32_t* __restrict__ tau_chunk, uint32_t kc, uint32_t p2,
                             uint32_t* __restrict__ unit_max, uint32_t* __restrict__ hist_part,
                             uint32_t* __restrict__ status, uint32_t max_latency, uint32_t trial_rows) {
    // trial_rows = 0: a unit is a run of chunks inside one trial and unit_max[u] receives its maximum.  Otherwise (few
    // workers per trial, or a worker count that fills its last chunk badly; contiguous tensor): the tensor is one run
    // of N = T * trial_rows rows, units and chunks ignore the trials, and unit_max[t] is trial t's maximum, built with
    // atomic maxima (cleared by the prep kernel).
    extern __shared__ __align__(16) unsigned char smem[];
    const uint32_t stage_words = 64u * M;                                   // per wave; 256 M bytes, a multiple of 16
    const GridView g = stage_grid(reinterpret_cast<uint32_t*>(smem) + DC_SCAN_WAVES * stage_words, tau_chunk, kc, p2);

    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint32_t* stage = reinterpret_cast<uint32_t*>(smem) + wave * stage_words;
    u32x4* stage_v = reinterpret_cast<u32x4*>(stage);
    const uint32_t* row = stage + lane * M;

    WaveState st{0u, 0u, 0u, 0u};
    const UnitRuns ur = unit_runs(units, run, gridDim.x);                                  // as in dc_scan_vec4_kernel
    for (uint32_t r = blockIdx.x; r < ur.padded; r += gridDim.x)                          // block-uniform bounds
    for (uint32_t round = 0; round < ur.rounds; ++round) {
        const uint32_t u = r < ur.runs ? r * run + round * DC_SCAN_WAVES + wave : units;
        if (u < units) {
            const uint32_t t = u / units_per_trial;
            const uint32_t j = u - t * units_per_trial;
            const uint32_t row0 = j * chunks_per_unit * 64u;
            const uint32_t rows_left = row0 < N ? N - row0 : 0u;          // (a unit past the trial's end is empty)
            const uint32_t rows = rows_left < chunks_per_unit * 64u ? rows_left : chunks_per_unit * 64u;
            // row0 is a multiple of 64 and the trial starts on a 16-byte boundary, so every chunk does
            const u32x4* base = reinterpret_cast<const u32x4*>(lat + (uint64_t)t * trial_stride + (uint64_t)row0 * M);
            uint32_t lane_max = 0u;
            u32x4 x[NB];
            {
                const uint32_t first = rows < 64u ? rows : 64u;
                row_lane_load<NB>(x, base, first * M / 4u, lane);
            }
            for (uint32_t c0 = 0; c0 < rows; c0 += 64u) {
                const uint32_t here = rows - c0 < 64u ? rows - c0 : 64u;  // rows of this chunk (wave-uniform)
                const uint32_t nv = here * M / 4u;                          // whole vectors: N*M is a multiple of 4
#pragma unroll
                for (int k = 0; k < NB; ++k) {
                    const uint32_t i = 64u * k + lane;
                    if (i < nv) stage_v[i] = x[k];
                }
                if (c0 + 64u < rows) {                                      // the next chunk's loads fly during this chunk's arithmetic
                    const uint32_t next = rows - c0 - 64u < 64u ? rows - c0 - 64u : 64u;
                    row_lane_load<NB>(x, base + (uint64_t)(c0 + 64u) * M / 4u, next * M / 4u, lane);
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                const bool mine = lane < here;
                uint32_t total = 0u, worst = 0u;
                if (mine) {
                    uint32_t m = 0;
                    for (; m + 8u <= M; m += 8u) {
                        uint32_t e[8];
#pragma unroll
                        for (uint32_t k = 0; k < 8u; ++k) e[k] = row[m + k];
#pragma unroll
                        for (uint32_t k = 0; k < 8u; ++k) { total += e[k]; worst = umax(worst, e[k]); }
                    }
                    for (; m < M; ++m) { const uint32_t e = row[m]; total += e; worst = umax(worst, e); }
                }
                st.check = umax(st.check, worst);
                lane_max = umax(lane_max, total);
                if (trial_rows) {                                           // the lane's row is row0 + c0 + lane of the whole run
                    const uint32_t trial = (row0 + c0 + lane) / trial_rows;
                    add_trial_maxima(total, trial, 0u, mine, lane, trial_rows, unit_max);
                }
                // backwards from the row's end; val = P[M-1-s] (0 in lanes without a row, which count nowhere)
                uint32_t val = total;
                uint32_t s = 0;
                while (s < M) {
                    const uint64_t reach = __ballot(mine && val >= g.tau0);
                    if (reach == 0) break;                                  // wave-uniform
                    // four steps at once when most lanes are inside the grid, and from the third step on in any case: a
                    // walk that goes on after two steps is that of a few rows with long delays, which may go far
                    if (s + 4u <= M && ((uint32_t)__popcll(reach) >= DC_DENSE_LANES || s >= 2u)) {
                        uint32_t x0 = 0u, x1 = 0u, x2 = 0u, x3 = 0u;
                        if (mine) { x0 = row[M - 1u - s]; x1 = row[M - 2u - s]; x2 = row[M - 3u - s]; x3 = row[M - 4u - s]; }
                        uint32_t v[4], b[4];
                        v[0] = val; v[1] = v[0] - x0; v[2] = v[1] - x1; v[3] = v[2] - x2;
                        bins_of<4>(g, v, b);                                 // values below the grid find bin 0
#pragma unroll
                        for (int q = 0; q < 4; ++q) count_bin(g, mine ? b[q] : 0u);
                        val = v[3] - x3;
                        s += 4u;
                    } else {
                        const uint32_t v[1] = {val};
                        uint32_t b[1];
                        bins_of<1>(g, v, b);
                        count_bin(g, mine ? b[0] : 0u);
                        if (mine) val -= row[M - 1u - s];
                        s += 1u;
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");      // read before the next chunk overwrites it
            }
            if (!trial_rows) {
                const uint32_t m = wave_max(lane_max);
                if (lane == 0) unit_max[u] = m;
            }
        }
        __syncthreads();
    }
    report_range(st.check, max_latency, lane, status);

    __syncthreads();
    uint32_t* out = hist_part + (uint64_t)blockIdx.x * p2;
    for (uint32_t i = threadIdx.x; i < p2; i += DC_SCAN_THREADS) out[i] = g.hist[i];
}

namespace dc {

int row_lane_blocks_per_cu(size_t lds) {
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, dc_scan_row_lane_kernel<16>, DC_SCAN_THREADS, lds) != hipSuccess) n = 0;
    return n;
}

void launch_row_lane_scan(const Plan& p, const int32_t* lat, const uint32_t* tau_chunk, uint32_t kc, uint32_t* unit_max,
                          uint32_t* hist_part, uint32_t* status, hipStream_t stream) {
    // over trials of few workers the tensor is one run of T * N rows (one "trial" of that many rows, all units its)
    const uint32_t rows = p.span_rows ? p.T * p.N : p.N;
    const uint32_t units_per_trial = p.span_rows ? p.units : p.units_per_trial;
#define DC_RL(nb) hipLaunchKernelGGL(dc_scan_row_lane_kernel<nb>, dim3(p.grid), dim3(DC_SCAN_THREADS), scan_lds_bytes(p), stream, lat, \
                       p.span_rows ? 0ull : p.stride, rows, p.M, p.units, units_per_trial, p.run, p.per_unit, tau_chunk, kc, p.p2, unit_max, \
                       hist_part, status, p.max_latency, p.span_rows)
    if (p.M <= 32) DC_RL(8); else if (p.M <= 48) DC_RL(12); else DC_RL(16);
#undef DC_RL
}

}  // namespace dc
