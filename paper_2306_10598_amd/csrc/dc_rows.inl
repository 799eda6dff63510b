// The streaming kernel in which every lane holds whole rows, and the launcher of one row length.  Included by the
// translation units that instantiate it (dc_rows.hip: rows of up to 12 elements; dc_rows_long.hip: the longer ones):
// its instantiations are most of the library's build time, so they are spread over two compilations.
#ifndef DC_ROWS_INL
#define DC_ROWS_INL

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dc_device.h"
#include "dc_internal.h"

namespace {

// ---------------------------------------------------------------------------------------------
// dc_scan_rows_kernel: short rows of which a lane can hold several.  M <= 17 or 18, 22, 26, 30, 34 (the lengths of
// dc::lane_rows_length), N a multiple of the rows per lane, every trial on a 16-byte boundary.
// The kernels above spread a row over lanes and pay for it with cross-lane sums and, per 16-byte load, one queue
// slot or one search per element; with rows of a few elements that arithmetic, not HBM, bounds them.  Here a lane
// holds R whole rows in registers (V 16-byte vectors = R*M elements), so completion times are R*M plain additions,
// and because they do not decrease along a row (latencies >= 0) the thresholds are met from the row's end
// backwards: step s bins the (M-1-s)-th completion time of all R rows at once and the wave stops at the first
// step in which no lane reaches the smallest threshold; with the usual grids that is after one or two steps.
// A wave reads a chunk of 64 V consecutive vectors with coalesced loads (lane l takes vectors l, l + 64, ...) and,
// unless a vector holds whole rows anyway (M = 1, 2), passes them through its own stretch of LDS so that lane l ends
// up with vectors l V, ..., l V + V - 1; a lane's stretch is padded to an odd number of vectors, which keeps these
// reads free of bank conflicts for every M.
// ---------------------------------------------------------------------------------------------
template <int M>
struct LaneRows {
    static constexpr bool STAGED = (4 % M) != 0;
    static constexpr int V = !STAGED ? 4 : (M > 16 && (M & 3) == 2) ? M / 2 : M;   // vectors per lane and chunk
    static constexpr int R = 4 * V / M;               // rows per lane and chunk
    static constexpr bool PREFETCH = V <= DC_ROWS_PREFETCH_MAX_V;   // the next chunk's loads are issued before this chunk's arithmetic
    static constexpr int PAIRED_STEPS = M <= 16 ? M : 4;            // backward steps that may take the next one along (code size)
    // A lane's vectors sit SPAN vectors from the next lane's in LDS: an odd number, so that eight lanes reading 16 bytes
    // each fall on different banks (with SPAN = V and V = 8 or 16 every lane of the wave would meet in one bank).
    static constexpr int SPAN = STAGED ? (V | 1) : 0;
    static constexpr uint32_t STAGE_VECTORS = 64u * SPAN;       // per wave
};

template <int M>
__device__ __forceinline__ void rows_load(u32x4 (&x)[LaneRows<M>::V], const u32x4* base, uint32_t first, uint32_t nv,
                                          uint32_t lane) {
    constexpr int V = LaneRows<M>::V;
    if (first + 64u * V <= nv) {                       // wave-uniform: the whole chunk lies inside the unit
#pragma unroll
        for (int j = 0; j < V; ++j) x[j] = __builtin_nontemporal_load(base + first + 64u * j + lane);
    } else {
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const uint32_t i = first + 64u * j + lane;
            u32x4 z = {0u, 0u, 0u, 0u};
            if (i < nv) z = __builtin_nontemporal_load(base + i);
            x[j] = z;
        }
    }
}

// One chunk: `left` = vectors of the unit from the chunk's first one on (the chunk holds min(left, 64 V)).
template <int M, bool FULL>
__device__ __forceinline__ void rows_chunk(WaveState& st, u32x4 (&x)[LaneRows<M>::V], uint32_t left, u32x4* stage,
                                           const GridView& g, uint32_t lane, uint32_t (&total)[LaneRows<M>::R]) {
    using S = LaneRows<M>;
    constexpr int V = S::V, R = S::R;
    if constexpr (S::STAGED) {
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const uint32_t i = 64u * j + lane;                       // vector i of the chunk belongs to lane i / V
            stage[S::SPAN == V ? i : i + i / V] = x[j];
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
        for (int j = 0; j < V; ++j) x[j] = stage[lane * S::SPAN + j];
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");      // read before the next chunk overwrites it
    }
    uint32_t e[4 * V];
#pragma unroll
    for (int j = 0; j < V; ++j) { e[4 * j] = x[j].x; e[4 * j + 1] = x[j].y; e[4 * j + 2] = x[j].z; e[4 * j + 3] = x[j].w; }
    uint32_t worst = st.check;
#pragma unroll
    for (int i = 0; i < 4 * V; ++i) worst = umax(worst, e[i]);
    st.check = worst;
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int m = 1; m < M; ++m) e[r * M + m] += e[r * M + m - 1];
    // which of the lane's rows belong to the unit: all of them in a full chunk; in the last, partial one the lanes
    // (staged) or vectors (not staged) before the unit's end -- N is a multiple of 4, so no vector is split
    bool mine[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        if constexpr (FULL) mine[r] = true;
        else if constexpr (S::STAGED) mine[r] = lane * V < left;
        else mine[r] = 64u * (uint32_t)(r * M / 4) + lane < left;
    }
    uint32_t top = st.lane_max;
#pragma unroll
    for (int r = 0; r < R; ++r) { total[r] = e[r * M + M - 1]; top = umax(top, total[r]); }   // rows outside the unit are all zero
    st.lane_max = top;
    bool taken = false;                                             // wave-uniform: this step went with the one before
#pragma unroll
    for (int s = 0; s < M; ++s) {
        if (taken) { taken = false; continue; }
        uint32_t val[2 * R], b[2 * R];
        uint32_t high = 0u;
#pragma unroll
        for (int r = 0; r < R; ++r) { val[r] = e[r * M + M - 1 - s]; high = umax(high, val[r]); }
        const uint64_t reach = __ballot(high >= g.tau0);
        if (reach == 0) break;                                      // wave-uniform
        if (s + 1 < M && s < S::PAIRED_STEPS && ((uint32_t)__popcll(reach) >= DC_DENSE_LANES || s >= 2)) {
            // most lanes are inside the grid, so the next step would very likely run as well -- or the walk goes on
            // after two steps, which is that of a few rows with long delays and may go far: both steps at once, twice
            // as many independent searches in flight (completion times below the grid find bin 0 and count nowhere)
#pragma unroll
            for (int r = 0; r < R; ++r) val[R + r] = e[r * M + M - 1 - (s + 1 < M ? s + 1 : s)];
            bins_of<2 * R>(g, val, b);
#pragma unroll
            for (int r = 0; r < 2 * R; ++r) count_bin(g, mine[r % R] ? b[r] : 0u);
            taken = true;
        } else {
            uint32_t v1[R], b1[R];
#pragma unroll
            for (int r = 0; r < R; ++r) v1[r] = val[r];
            bins_of<R>(g, v1, b1);
#pragma unroll
            for (int r = 0; r < R; ++r) count_bin(g, mine[r] ? b1[r] : 0u);
        }
    }
}

// SPAN = false: a unit is a run of chunks inside one trial and unit_max[u] receives its maximum.  SPAN = true (few
// workers per trial, contiguous tensor): the tensor is one run of N = T * trial_rows rows, units and chunks ignore
// the trials, and unit_max[t] is trial t's maximum, built with atomic maxima.
template <int M, bool SPAN>
__global__ __launch_bounds__(DC_SCAN_THREADS)
void dc_scan_rows_kernel(const int32_t* __restrict__ lat, uint64_t trial_stride, uint32_t N, uint32_t units, uint32_t units_per_trial,
                         uint32_t run, uint32_t chunks_per_unit, const uint32_t* __restrict__ tau_chunk, uint32_t kc, uint32_t p2,
                         uint32_t* __restrict__ unit_max, uint32_t* __restrict__ hist_part, uint32_t* __restrict__ status,
                         uint32_t max_latency, uint32_t trial_rows) {
    using S = LaneRows<M>;
    constexpr int V = S::V;
    constexpr uint32_t CHUNK_ROWS = 64u * S::R, CHUNK_VECTORS = 64u * V;
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr size_t STAGE_BYTES = (size_t)DC_SCAN_WAVES * S::STAGE_VECTORS * sizeof(u32x4);
    const GridView g = stage_grid(reinterpret_cast<uint32_t*>(smem + STAGE_BYTES), tau_chunk, kc, p2);

    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    u32x4* stage = reinterpret_cast<u32x4*>(smem) + wave * S::STAGE_VECTORS;

    WaveState st{0u, 0u, 0u, 0u};
    const UnitRuns ur = unit_runs(units, run, gridDim.x);                                  // as in dc_scan_vec4_kernel
    for (uint32_t r = blockIdx.x; r < ur.padded; r += gridDim.x)                          // block-uniform bounds
    for (uint32_t round = 0; round < ur.rounds; ++round) {
        const uint32_t u = r < ur.runs ? r * run + round * DC_SCAN_WAVES + wave : units;
        if (u < units) {
            const uint32_t t = u / units_per_trial;
            const uint32_t j = u - t * units_per_trial;
            const uint32_t row0 = j * chunks_per_unit * CHUNK_ROWS;
            const uint32_t rows_left = row0 < N ? N - row0 : 0u;          // (a unit past the trial's end is empty)
            const uint32_t rows = rows_left < chunks_per_unit * CHUNK_ROWS ? rows_left : chunks_per_unit * CHUNK_ROWS;
            const uint32_t nv = rows * (uint32_t)M / 4u;                                  // whole vectors: rows is a multiple of R
            const u32x4* base = reinterpret_cast<const u32x4*>(lat + (uint64_t)t * trial_stride + (uint64_t)row0 * M);
            st.lane_max = 0u;
            uint32_t trial = 0u, within = 0u, trial_recip = 0u;            // SPAN: where the chunk's first row sits
            if constexpr (SPAN) {
                trial = row0 / trial_rows;
                within = row0 - trial * trial_rows;
                trial_recip = trial_rows < 256u ? ((1u << 20) + trial_rows - 1u) / trial_rows : 0u;
            }
            u32x4 x[V];
            rows_load<M>(x, base, 0u, nv, lane);
            for (uint32_t first = 0; first < nv; first += CHUNK_VECTORS) {
                const uint32_t left = nv - first;
                uint32_t total[S::R];
                if constexpr (S::PREFETCH) {
                    u32x4 ahead[V];
#pragma unroll
                    for (int q = 0; q < V; ++q) ahead[q] = x[q];
                    if (left > CHUNK_VECTORS) rows_load<M>(ahead, base, first + CHUNK_VECTORS, nv, lane);
                    if (left >= CHUNK_VECTORS) rows_chunk<M, true>(st, x, left, stage, g, lane, total);
                    else rows_chunk<M, false>(st, x, left, stage, g, lane, total);
#pragma unroll
                    for (int q = 0; q < V; ++q) x[q] = ahead[q];
                } else {
                    if (left >= CHUNK_VECTORS) rows_chunk<M, true>(st, x, left, stage, g, lane, total);
                    else rows_chunk<M, false>(st, x, left, stage, g, lane, total);
                    if (left > CHUNK_VECTORS) rows_load<M>(x, base, first + CHUNK_VECTORS, nv, lane);
                }
                if constexpr (SPAN) {
                    static_assert(!SPAN || (S::STAGED && S::R == 4), "a lane's rows must be consecutive");
                    // the lane's rows are rows ahead .. ahead + 3 counted from the head of trial `trial`; ahead + 3 < 512
                    // and, below 256 rows per trial, the fixed-point quotient is exact; from 256 rows on a chunk holds
                    // at most one boundary
                    const uint32_t ahead = within + 4u * lane;
                    const uint32_t q0 = trial_recip ? (ahead * trial_recip) >> 20 : (ahead >= trial_rows ? 1u : 0u);
                    const uint32_t q3 = trial_recip ? ((ahead + 3u) * trial_recip) >> 20 : (ahead + 3u >= trial_rows ? 1u : 0u);
                    const uint32_t before = q3 != q0 ? q3 * trial_rows - ahead : 0u;   // rows of the lane ahead of the boundary (1..3)
                    uint32_t m_before = 0u, m_after = 0u;
#pragma unroll
                    for (uint32_t q = 0; q < 4u; ++q) {
                        m_before = umax(m_before, q < before ? total[q] : 0u);
                        m_after = umax(m_after, q < before ? 0u : total[q]);
                    }
                    add_trial_maxima(m_after, trial + q3, m_before, row0 + first / (uint32_t)M * 4u + 4u * lane < N, lane,
                                     (trial_rows + 3u) / 4u + 1u, unit_max);
                    trial += CHUNK_ROWS / trial_rows;                       // the next chunk starts 256 rows further on
                    within += CHUNK_ROWS % trial_rows;
                    if (within >= trial_rows) { within -= trial_rows; ++trial; }
                }
            }
            if constexpr (!SPAN) {
                const uint32_t m = wave_max(st.lane_max);
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

}  // namespace

namespace dc {

template <int M>
static void launch_rows(const Plan& p, const int32_t* lat, const uint32_t* tau_chunk, uint32_t kc,
                        uint32_t* unit_max, uint32_t* hist_part, uint32_t* status, hipStream_t stream) {
    if constexpr (LaneRows<M>::STAGED && LaneRows<M>::R == 4 && M <= 16) {
        if (p.span_rows) {                          // the tensor as one run of T * N rows
            hipLaunchKernelGGL((dc_scan_rows_kernel<M, true>), dim3(p.grid), dim3(DC_SCAN_THREADS), scan_lds_bytes(p), stream,
                               lat, 0ull, p.T * p.N, p.units, p.units, p.run, p.per_unit, tau_chunk, kc, p.p2, unit_max,
                               hist_part, status, p.max_latency, p.span_rows);
            return;
        }
    }
    hipLaunchKernelGGL((dc_scan_rows_kernel<M, false>), dim3(p.grid), dim3(DC_SCAN_THREADS), scan_lds_bytes(p), stream, lat,
                       p.stride, p.N, p.units, p.units_per_trial, p.run, p.per_unit, tau_chunk, kc, p.p2, unit_max,
                       hist_part, status, p.max_latency, p.N);
}


}  // namespace dc

#endif
