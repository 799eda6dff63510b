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

#include "dc_internal.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------------------------
// wave-level primitives
// ---------------------------------------------------------------------------------------------

// DPP controls (GCN3+/CDNA encoding)
constexpr int DPP_ROW_SHR = 0x110;      // + n: lane i reads lane i-n of its 16-lane row
constexpr int DPP_ROW_BCAST15 = 0x142;  // lane 15 of each row -> every lane of the next row
constexpr int DPP_ROW_BCAST31 = 0x143;  // lane 31 -> every lane of rows 2 and 3

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_or_zero(uint32_t v) {
    // lanes whose source is outside the row, or that ROW_MASK disables, receive 0
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xf, true);
}

// Inclusive prefix sum over aligned groups of L consecutive lanes (L a power of two, 1..64).
template <int L>
__device__ __forceinline__ uint32_t segmented_inclusive_scan(uint32_t v, uint32_t lane) {
    const uint32_t pos = lane & (L - 1);
    if constexpr (L >= 2) {
        uint32_t t = dpp_or_zero<DPP_ROW_SHR + 1, 0xf>(v);
        if constexpr (L < 16) t = pos >= 1 ? t : 0u;
        v += t;
    }
    if constexpr (L >= 4) {
        uint32_t t = dpp_or_zero<DPP_ROW_SHR + 2, 0xf>(v);
        if constexpr (L < 16) t = pos >= 2 ? t : 0u;
        v += t;
    }
    if constexpr (L >= 8) {
        uint32_t t = dpp_or_zero<DPP_ROW_SHR + 4, 0xf>(v);
        if constexpr (L < 16) t = pos >= 4 ? t : 0u;
        v += t;
    }
    if constexpr (L >= 16) v += dpp_or_zero<DPP_ROW_SHR + 8, 0xf>(v);
    if constexpr (L >= 32) v += dpp_or_zero<DPP_ROW_BCAST15, 0xa>(v);
    if constexpr (L >= 64) v += dpp_or_zero<DPP_ROW_BCAST31, 0xc>(v);
    return v;
}

__device__ __forceinline__ uint32_t umax(uint32_t a, uint32_t b) { return a > b ? a : b; }

// How the rows of lat sit in a wave's 16-byte loads.  The kernels are instantiated for L = 1,2,4,...,64
// lanes per row (M = 4L a power of two: every lane used, rows aligned to the DPP rows) and once more,
// as L = 0, for any other L <= 64 known only at run time: then a load holds floor(64/L) whole rows in
// its first `active` lanes and the remaining lanes stay idle.
struct RowShape {
    uint32_t lanes;      // L: lanes per row
    uint32_t rows;       // whole rows per load
    uint32_t active;     // rows * lanes: lanes that take part (= 16-byte vectors per load)
    uint32_t pos;        // this lane's position inside its row
    uint32_t row;        // which of the load's rows this lane belongs to
    bool ok;             // this lane takes part
};

template <int L>
__device__ __forceinline__ RowShape row_shape(uint32_t lane, uint32_t lanes_per_row) {
    RowShape r;
    r.lanes = L ? (uint32_t)L : lanes_per_row;
    r.rows = 64u / r.lanes;
    r.active = r.rows * r.lanes;
    r.pos = lane % r.lanes;
    r.row = lane / r.lanes;
    r.ok = lane < r.active;
    return r;
}

// Inclusive prefix sum over groups of `lanes` consecutive lanes, any group length: Kogge-Stone steps
// through the LDS crossbar (rows of 3, 5, 6, ... lanes do not line up with the 16-lane DPP rows).
__device__ __forceinline__ uint32_t segmented_inclusive_scan_any(uint32_t v, const RowShape& r) {
    for (uint32_t d = 1; d < r.lanes; d <<= 1) {
        const uint32_t up = (uint32_t)__shfl_up((int)v, d, 64);
        v += r.pos >= d ? up : 0u;
    }
    return v;
}

// Maximum over the 64 lanes, returned in every lane: a running maximum with the scan's DPP
// steps (0 is the identity of an unsigned maximum), then lane 63 holds the result.
__device__ __forceinline__ uint32_t wave_max(uint32_t v) {
    v = umax(v, dpp_or_zero<DPP_ROW_SHR + 1, 0xf>(v));
    v = umax(v, dpp_or_zero<DPP_ROW_SHR + 2, 0xf>(v));
    v = umax(v, dpp_or_zero<DPP_ROW_SHR + 4, 0xf>(v));
    v = umax(v, dpp_or_zero<DPP_ROW_SHR + 8, 0xf>(v));
    v = umax(v, dpp_or_zero<DPP_ROW_BCAST15, 0xa>(v));
    v = umax(v, dpp_or_zero<DPP_ROW_BCAST31, 0xc>(v));
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// b(v) = #{i < n : a[i] <= v} for ascending a[0..p2-2], padded with 0xFFFFFFFF beyond the
// real thresholds; p2 is a power of two.  Result is in [0, p2-1] for every v.
__device__ __forceinline__ uint32_t bin_of(const uint32_t* a, uint32_t p2, uint32_t v) {
    uint32_t b = 0;
    for (uint32_t s = p2 >> 1; s >= 1; s >>= 1)
        if (a[b + s - 1] <= v) b += s;
    return b;
}

// The threshold grid of one pass as the streaming kernel sees it, all in LDS:
//   tau[p2]     ascending thresholds, padded with 0xFFFFFFFF
//   cells[p2]   cells[c].x = #{k : tau_k < tau0 + c*2^shift} (cells[p2-1].x = number of thresholds): p2-1 uniform
//               cells from tau0 on, the last one open-ended, so that a completion time v in cell c has its
//               bin in [cells[c].x, cells[c+1].x] (a short search; one step or none for evenly spaced thresholds);
//               cells[c].y = tau[cells[c].x], the first threshold at or above the cell's lower edge, so that one
//               8-byte read gives both when no cell holds more than one threshold
//   hist[p2]    bin counts of the block
struct GridView {
    const uint32_t* tau;
    const uint2* cells;
    uint32_t* hist;
    uint32_t* sink;      // this lane's word for counts that nobody reads (values below every threshold)
    uint32_t p2;
    uint32_t shift;
    uint32_t tau0;
    bool exact;          // no cell holds more than one threshold: cells[c] and one comparison give the bin
};

// Bins b(v) = #{k : tau_k <= v} of N values at once (the searches interleave their LDS reads).
template <int N>
__device__ __forceinline__ void bins_of(const GridView& g, const uint32_t (&val)[N], uint32_t (&lo)[N]) {
    if (g.exact) {
        // evenly spaced thresholds (the usual case) leave at most one per cell: bin = cells[c].x + (cells[c].y <= v);
        // tau is padded with 0xFFFFFFFF, so a cell without a threshold, or past the last one, adds nothing
        // a value below every threshold lands in cell 0, whose threshold tau0 it does not reach: bin 0
        uint2 cell[N];
#pragma unroll
        for (int i = 0; i < N; ++i) {
            uint32_t c = (umax(val[i], g.tau0) - g.tau0) >> g.shift;
            c = c < g.p2 - 2 ? c : g.p2 - 2;
            cell[i] = g.cells[c];
        }
#pragma unroll
        for (int i = 0; i < N; ++i) lo[i] = cell[i].x + (cell[i].y <= val[i] ? 1u : 0u);
        return;
    }
    uint32_t hi[N];
#pragma unroll
    for (int i = 0; i < N; ++i) {
        uint32_t c = (val[i] - g.tau0) >> g.shift;
        c = c < g.p2 - 2 ? c : g.p2 - 2;
        lo[i] = g.cells[c].x;
        hi[i] = g.cells[c + 1].x;
        if (val[i] < g.tau0) lo[i] = hi[i] = 0u;               // below every threshold
    }
    for (;;) {
        bool open_any = false;
#pragma unroll
        for (int i = 0; i < N; ++i) open_any |= lo[i] < hi[i];
        if (!open_any) break;
        uint32_t t[N], mid[N];
#pragma unroll
        for (int i = 0; i < N; ++i) { mid[i] = (lo[i] + hi[i]) >> 1; t[i] = g.tau[mid[i]]; }   // mid <= p2-1
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const bool open = lo[i] < hi[i], right = t[i] <= val[i];
            lo[i] = open && right ? mid[i] + 1 : lo[i];
            hi[i] = open && !right ? mid[i] : hi[i];
        }
    }
}

__device__ __forceinline__ void bins_of4(const GridView& g, uint4 v, uint32_t (&lo)[4]) {
    const uint32_t val[4] = {v.x, v.y, v.z, v.w};
    bins_of<4>(g, val, lo);
}

// One more completion time in bin b, for the paths that bin straight from registers: bin 0 (below every threshold) is
// never read, and sending it to a word of the lane's own costs one select instead of a branch around the atomic.
__device__ __forceinline__ void count_bin(const GridView& g, uint32_t b) {
    atomicAdd(b ? &g.hist[b] : g.sink, 1u);
}

// Per-wave state of the streaming pass.
struct WaveState {
    uint32_t lane_max;   // running maximum of completion times seen by this lane in the current unit
    uint32_t check;      // running unsigned maximum of raw latencies (negative values show as >= 2^31)
    uint32_t q_head;     // ring-buffer read position (wave-uniform)
    uint32_t q_count;    // items waiting in the ring buffer (wave-uniform)
};

constexpr uint32_t QUEUE_ITEMS = 128;   // per wave; a push adds at most 64, a drain removes 64

// Take up to 64 queued items (one per lane), bin their four completion times, add to the
// block histogram.  Bin 0 (below every threshold) is never needed and is skipped.
__device__ __forceinline__ void drain(WaveState& st, uint4* queue, const GridView& g, uint32_t lane) {
    const uint32_t n = st.q_count < 64u ? st.q_count : 64u;
    if (lane < n) {
        const uint4 item = queue[(st.q_head + lane) & (QUEUE_ITEMS - 1)];
        uint32_t b[4];
        bins_of4(g, item, b);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (b[i]) atomicAdd(&g.hist[b[i]], 1u);
    }
    st.q_head = (st.q_head + n) & (QUEUE_ITEMS - 1);
    st.q_count -= n;
}

// One 16-byte load per lane holds four consecutive latencies of one worker; the lanes of a
// worker are L consecutive lanes, so a wave holds 64/L whole rows.  Completion time of the lane's
// last element:
template <int L>
__device__ __forceinline__ uint32_t lane_completion_time(u32x4 x, uint32_t lane, const RowShape& shape) {
    if constexpr (L == 0) return segmented_inclusive_scan_any(x.x + x.y + x.z + x.w, shape);
    else return segmented_inclusive_scan<L>(x.x + x.y + x.z + x.w, lane);
}

// Lanes whose last completion time reaches the smallest threshold put their four completion
// times into the wave's queue (compaction: the histogram work is done 64 items at a time).
// mask = __ballot(active).
__device__ __forceinline__ void enqueue_active(WaveState& st, u32x4 x, uint32_t incl, bool active, uint64_t mask,
                                               uint4* queue, const GridView& g, uint32_t lane) {
    if (mask) {
        if (active) {
            const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                      __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
            const uint32_t c2 = incl - x.w, c1 = c2 - x.z, c0 = c1 - x.y;
            queue[(st.q_head + st.q_count + rank) & (QUEUE_ITEMS - 1)] = make_uint4(c0, c1, c2, incl);
        }
        st.q_count += (uint32_t)__popcll(mask);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        if (st.q_count >= 64u) drain(st, queue, g, lane);
    }
}

// The other way to count: every lane bins the completion times of G loads straight from its registers, 4 G
// searches interleaved, no queue.  Lanes below the smallest threshold find bin 0 and add nothing.
template <int G>
__device__ __forceinline__ void bin_direct(const u32x4* x, const uint32_t* incl, const GridView& g) {
    uint32_t val[4 * G], b[4 * G];
#pragma unroll
    for (int k = 0; k < G; ++k) {
        val[4 * k + 3] = incl[k];
        val[4 * k + 2] = incl[k] - x[k].w;
        val[4 * k + 1] = val[4 * k + 2] - x[k].z;
        val[4 * k + 0] = val[4 * k + 1] - x[k].y;
    }
    bins_of<4 * G>(g, val, b);
#pragma unroll
    for (int i = 0; i < 4 * G; ++i) count_bin(g, b[i]);
}

// Completion time of each lane's last element for U loads at once (the U scans are independent, so
// their DPP or crossbar steps interleave and no latency adds up).
template <int L, int U>
__device__ __forceinline__ void completion_times(const u32x4 (&x)[U], uint32_t (&incl)[U], uint32_t lane,
                                                 const RowShape& shape) {
    if constexpr (L == 0) {
        // rows of any length: the Kogge-Stone steps of all U scans go through the LDS crossbar together,
        // so their latencies overlap instead of adding up
#pragma unroll
        for (int k = 0; k < U; ++k) incl[k] = x[k].x + x[k].y + x[k].z + x[k].w;
        for (uint32_t d = 1; d < shape.lanes; d <<= 1) {
            const int src = (int)lane - (int)d;
            const int addr = (src < 0 ? (int)lane : src) << 2;
            const bool take = shape.pos >= d;
            uint32_t up[U];
#pragma unroll
            for (int k = 0; k < U; ++k) up[k] = (uint32_t)__builtin_amdgcn_ds_bpermute(addr, (int)incl[k]);
#pragma unroll
            for (int k = 0; k < U; ++k) incl[k] += take ? up[k] : 0u;
        }
    } else {
#pragma unroll
        for (int k = 0; k < U; ++k) incl[k] = lane_completion_time<L>(x[k], lane, shape);   // independent scans interleave
    }
}

template <int L, int U>
__device__ __forceinline__ void process_loads(WaveState& st, const u32x4 (&x)[U], uint4* queue, const GridView& g,
                                              uint32_t lane, const RowShape& shape) {
    uint32_t incl[U];
    completion_times<L, U>(x, incl, lane, shape);
    bool active[U];
    uint64_t mask[U];
    uint32_t busy = 0u;
#pragma unroll
    for (int k = 0; k < U; ++k) {
        st.check = umax(st.check, umax(umax(x[k].x, x[k].y), umax(x[k].z, x[k].w)));
        st.lane_max = umax(st.lane_max, incl[k]);
        active[k] = (L != 0 || shape.ok) && incl[k] >= g.tau0;
        mask[k] = __ballot(active[k]);
        busy += (uint32_t)__popcll(mask[k]);
    }
    // Rows of 128 and 256 elements run with two blocks per compute unit (see the launch shape), too few waves to
    // hide the LDS latencies of the queue when much of the data lies inside the threshold grid.  When at least
    // DC_DENSE_LANES lanes per load are inside it, the lanes bin their registers directly, two loads at a time:
    // measured 3.6 -> 4.6-4.8 TB/s with a grid from 0 to the largest total; below about half of the lanes the
    // queue's compaction wins, and the usual narrow grids never come here.
    if constexpr (U >= 2 && (L == 32 || L == 64)) {
        if (busy >= (uint32_t)U * DC_DENSE_LANES) {
#pragma unroll
            for (int k = 0; k < U; k += 2) bin_direct<2>(&x[k], &incl[k], g);
            return;
        }
    }
#pragma unroll
    for (int k = 0; k < U; ++k) enqueue_active(st, x[k], incl[k], active[k], mask[k], queue, g, lane);
}

}  // namespace

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
// shared pieces of the streaming kernels
// ---------------------------------------------------------------------------------------------

// Stage one pass's thresholds in LDS (tau[p2] | hist[p2] | cells[p2], 16 p2 bytes at `tables`), clear the histogram
// and build the lookup cells.  Every thread of the block must call it (it synchronises the block).
__device__ __forceinline__ GridView stage_grid(uint32_t* tables, const uint32_t* __restrict__ tau_chunk,
                                               uint32_t kc, uint32_t p2) {
    __shared__ uint32_t s_sink[64];
    uint32_t* tau_s = tables;
    uint32_t* hist = tau_s + p2;
    uint2* cells = reinterpret_cast<uint2*>(hist + p2);
    for (uint32_t i = threadIdx.x; i < p2; i += blockDim.x) {
        tau_s[i] = i < kc ? tau_chunk[i] : 0xFFFFFFFFu;
        hist[i] = 0u;
    }
    __syncthreads();
    // Uniform cells of width 2^shift from the smallest threshold.  They cover the thresholds up to tau_s[e];
    // the last cell (p2-2) is open-ended and takes everything above.  e is the last threshold unless the
    // list has a few far outliers at the top (typically one "infinite" threshold that yields the no-drop
    // step time): those would stretch the cells until all other thresholds share two or three of them,
    // so the top is peeled while the upper half of the range is more than 8 times as wide as the lower.
    const uint32_t tau_first = tau_s[0];
    uint32_t e = kc - 1;
    while (e > (kc - 1) / 2 && (uint64_t)(tau_s[e] - tau_first) > 8ull * ((uint64_t)(tau_s[e / 2] - tau_first) + 1ull)) --e;
    const uint32_t tau_last = tau_s[e];
    uint32_t shift = 0;                                        // p2 >= 4, so this stops at shift <= 31
    while (shift < 31 && ((tau_last - tau_first) >> shift) >= p2 - 2) ++shift;
    for (uint32_t c = threadIdx.x; c < p2; c += blockDim.x) {
        const uint64_t edge = (uint64_t)tau_first + ((uint64_t)c << shift);
        uint32_t lo = 0, hi = kc;                              // #{k : tau_k < edge}
        while (lo < hi) {
            const uint32_t mid = (lo + hi) >> 1;
            if ((uint64_t)tau_s[mid] < edge) lo = mid + 1; else hi = mid;
        }
        const uint32_t first = c == p2 - 1 ? kc : lo;          // upper end of the open-ended last cell
        cells[c] = make_uint2(first, tau_s[first]);            // first <= kc <= p2 - 1
    }
    __syncthreads();
    bool single = true;                                        // does every cell hold at most one threshold?
    for (uint32_t c = threadIdx.x; c + 1 < p2; c += blockDim.x) single = single && cells[c + 1].x - cells[c].x <= 1u;
    const bool exact = __syncthreads_and(single) != 0;
    return GridView{tau_s, cells, hist, &s_sink[threadIdx.x & 63u], p2, shift, tau_first, exact};
}

// One wave streams `nfull` consecutive full loads (shape.rows whole rows each, 1 KiB when every lane takes
// part) starting at `base` (already offset by the lane), then, if tail_rows > 0, one partial load holding
// tail_rows rows.
template <int L>
__device__ __forceinline__ u32x4 load_rows(const u32x4* p, const RowShape& shape) {
    if constexpr (L != 0) return __builtin_nontemporal_load(p);
    u32x4 x = {0u, 0u, 0u, 0u};
    if (shape.ok) x = __builtin_nontemporal_load(p);
    return x;
}

template <int L>
__device__ __forceinline__ void stream_rows(WaveState& st, const u32x4* base, uint32_t nfull, uint32_t tail_rows,
                                            uint4* queue, const GridView& g, uint32_t lane, const RowShape& shape) {
    constexpr int U = DC_SCAN_UNROLL;              // loads in flight per lane
    const uint64_t stride = L ? 64u : shape.active;   // 16-byte vectors per load
    uint32_t i = 0;
    for (; i + U <= nfull; i += U) {
        u32x4 x[U];
#pragma unroll
        for (int k = 0; k < U; ++k) x[k] = load_rows<L>(base + (uint64_t)(i + k) * stride, shape);
        process_loads<L, U>(st, x, queue, g, lane, shape);
    }
    for (; i < nfull; ++i) {
        const u32x4 x[1] = {load_rows<L>(base + (uint64_t)i * stride, shape)};
        process_loads<L, 1>(st, x, queue, g, lane, shape);
    }
    if (tail_rows) {                                // rows beyond the trial's last worker belong to the next trial
        const bool valid = lane < tail_rows * shape.lanes;
        u32x4 x = {0u, 0u, 0u, 0u};
        if (valid) x = __builtin_nontemporal_load(base + (uint64_t)nfull * stride);
        const uint32_t incl = lane_completion_time<L>(x, lane, shape);
        st.check = umax(st.check, umax(umax(x.x, x.y), umax(x.z, x.w)));
        st.lane_max = umax(st.lane_max, incl);
        const bool active = valid && incl >= g.tau0;
        enqueue_active(st, x, incl, active, __ballot(active), queue, g, lane);
    }
}

// The kernel for long rows is launched twice when the prep kernel sampled the data: once with the grid that suits
// narrow threshold grids (SHAPE 1) and once with the larger grid for dense ones (SHAPE 2); the launch that the
// sample (status[1]) did not choose returns at once.  SHAPE 0: a single launch, always runs.  The shape is part
// of the kernel's name, so a profile tells the working launch from the idle one.
template <int SHAPE>
__device__ __forceinline__ bool launch_is_chosen(const uint32_t* status) {
    if constexpr (SHAPE == 0) return true;
    const uint32_t dense = (uint32_t)__builtin_amdgcn_readfirstlane((int)status[1]);
    return (dense != 0u) == (SHAPE == 2);
}

// How the units are dealt to the blocks: runs of `run` consecutive units (a multiple of the waves per block),
// round-robin over the blocks.
struct UnitRuns {
    uint32_t runs;       // number of runs (the last one may be short)
    uint32_t padded;     // runs rounded up to a multiple of the grid: every block loops the same number of times
    uint32_t rounds;     // steps of DC_SCAN_WAVES units inside a run
};

__device__ __forceinline__ UnitRuns unit_runs(uint32_t units, uint32_t run, uint32_t blocks) {
    UnitRuns ur;
    ur.runs = (units + run - 1u) / run;
    ur.padded = (ur.runs + blocks - 1u) / blocks * blocks;
    ur.rounds = run / DC_SCAN_WAVES;
    return ur;
}

__device__ __forceinline__ void report_range(uint32_t check, uint32_t max_latency, uint32_t lane, uint32_t* status) {
    const uint32_t worst = wave_max(check);
    if (lane == 0 && worst > max_latency)
        atomicOr(status, worst >= 0x80000000u ? DC_FLAG_NEGATIVE_LATENCY : DC_FLAG_RANGE);
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
                         uint32_t* __restrict__ status, uint32_t max_latency, uint32_t lanes_per_row) {
    extern __shared__ __align__(16) unsigned char smem[];
    if (!launch_is_chosen<SHAPE>(status)) return;
    uint4* queue_all = reinterpret_cast<uint4*>(smem);                                  // [waves][QUEUE_ITEMS]
    const GridView g = stage_grid(reinterpret_cast<uint32_t*>(queue_all + DC_SCAN_WAVES * QUEUE_ITEMS), tau_chunk, kc, p2);

    const uint32_t lane = threadIdx.x & 63u;
    const RowShape shape = row_shape<L>(lane, lanes_per_row);
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
        if (u < units) {
            const uint32_t t = u / units_per_trial;
            const uint32_t j = u - t * units_per_trial;
            const uint32_t row0 = j * loads_per_unit * R;
            const uint32_t rows_left = N - row0;
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
// dc_scan_flat_kernel: any M >= 1, any 4-byte alignment of lat.
// The tensor is read as one flat run of 16-byte vectors from the 16-byte boundary at or below lat
// ("vector space": element e of lat is component (e + off) & 3 of vector (e + off) >> 2, off = the
// number of 4-byte words between that boundary and lat).  A unit is a run of whole rows of one trial;
// its first and last vector may also hold elements of the neighbouring rows, which are masked to zero.
// Row heads fall anywhere in a load, at positions every lane can work out by itself: lane l of load i
// holds unit-relative elements q0 = 256 i + 4 l - k, ..., q0 + 3 (k = components of the unit's first
// vector that precede it), so its first element sits at position pos0 = q0 mod M of its row.
//
// Rows of at least 4 elements (SMALL = false).  A lane then holds at most one row end.  With
//   s_c   the lane's running sums of its four values,   X   the sum of all lanes before it (one DPP scan),
//   ce    = M - pos0: components 0..ce-1 continue the row of the lane's first element, ce.. start the next,
//   E     = X + s_{ce-1}: the load-wide running sum at the lane's row end (meaningful when ce <= 4),
// the completion times are s_c + X - E' for components c < ce, where E' is E of the lane that holds the
// previous row end (one ds_bpermute; when that row end lies before this load, -E' is the wave-uniform
// carry: the open row's sum over the loads before), and s_c - s_{ce-1} for the others.  Sums wrap
// modulo 2^32; the differences are exact because row totals stay below 2^31.
//
// Rows of 1..3 elements (SMALL = true): a completion time is the sum of at most three consecutive
// values, the lane's own and the last two of the lane before.
// ---------------------------------------------------------------------------------------------
struct FlatTensor {
    const int32_t* lat;
    const u32x4* vec;          // 16-byte boundary at or below lat
    uint64_t total;            // elements of lat
    uint64_t total_vectors;    // vectors that hold them
    uint32_t off;              // 4-byte words between vec and lat (0..3)
    bool ragged_end;           // the tensor ends inside its last vector
    uint32_t M;
    uint32_t step;             // 256 mod M: how far a lane's position in its row moves from load to load
    uint32_t row_step;         // 256 div M: how many rows it moves
};

__device__ __forceinline__ FlatTensor flat_tensor(const int32_t* lat, uint64_t total, uint32_t M) {
    FlatTensor f;
    f.lat = lat;
    f.off = (uint32_t)(((uintptr_t)lat & 15u) >> 2);
    f.vec = reinterpret_cast<const u32x4*>(reinterpret_cast<uintptr_t>(lat) & ~(uintptr_t)15u);
    f.total = total;
    f.total_vectors = (total + f.off + 3u) >> 2;
    f.ragged_end = ((total + f.off) & 3u) != 0u;
    f.M = M;
    f.step = 256u % M;
    f.row_step = 256u / M;
    return f;
}

// One lane's vector `v` of vector space.  guard: the load may touch a vector that sticks out of the tensor
// (only the first vector when off != 0 and the last one when the tensor ends inside it): such a vector is
// read one element at a time, so nothing outside [lat, lat + total) is ever addressed.
__device__ __forceinline__ u32x4 flat_load(const FlatTensor& f, uint64_t v, bool in_range, bool guard) {
    u32x4 x = {0u, 0u, 0u, 0u};
    if (!in_range) return x;
    if (guard) {
        const int64_t e = (int64_t)(4u * v) - (int64_t)f.off;                // lat index of component 0
        if (e < 0 || (uint64_t)e + 4u > f.total) {
            if (e + 0 >= 0 && (uint64_t)(e + 0) < f.total) x.x = (uint32_t)f.lat[e + 0];
            if (e + 1 >= 0 && (uint64_t)(e + 1) < f.total) x.y = (uint32_t)f.lat[e + 1];
            if (e + 2 >= 0 && (uint64_t)(e + 2) < f.total) x.z = (uint32_t)f.lat[e + 2];
            if (e + 3 >= 0 && (uint64_t)(e + 3) < f.total) x.w = (uint32_t)f.lat[e + 3];
            return x;
        }
    }
    return __builtin_nontemporal_load(f.vec + v);
}

// Components of a lane's vector that belong to the unit, as a 4-bit mask: component c is element
// 4*lane + c of the load, valid for first <= 4*lane + c < limit.
__device__ __forceinline__ uint32_t flat_valid_mask(uint32_t lane, uint32_t first, uint32_t limit) {
    uint32_t m = 0u;
#pragma unroll
    for (uint32_t c = 0; c < 4; ++c) {
        const uint32_t e = 4u * lane + c;
        m |= (e >= first && e < limit) ? (1u << c) : 0u;
    }
    return m;
}

__device__ __forceinline__ u32x4 flat_masked(u32x4 x, uint32_t vm) {
    x.x = (vm & 1u) ? x.x : 0u;
    x.y = (vm & 2u) ? x.y : 0u;
    x.z = (vm & 4u) ? x.z : 0u;
    x.w = (vm & 8u) ? x.w : 0u;
    return x;
}

// Per-lane, per-unit state of the flat pass.
struct FlatState {
    uint32_t pos0;           // position of the lane's first element inside its row, for the next load
    uint32_t row;            // that row's number within the unit ("negative", wrapped, in the masked run before the unit's head)
    uint32_t pos_last;       // wave-uniform: pos0 of lane 63
    uint32_t carry;          // wave-uniform: sum of the open row over the loads before (rows >= 4)
    uint32_t prev2, prev3;   // wave-uniform: last two values of the load before (rows < 4)
};

__device__ __forceinline__ void flat_advance(FlatState& fs, const FlatTensor& f) {
    fs.pos0 += f.step;
    const bool wrapped = fs.pos0 >= f.M;
    fs.pos0 -= wrapped ? f.M : 0u;
    fs.row += f.row_step + (wrapped ? 1u : 0u);
    fs.pos_last += f.step;
    fs.pos_last -= fs.pos_last >= f.M ? f.M : 0u;
}

// U loads of rows with at least 4 elements.  x is already masked.  emit(p, vm, pos0, row) receives, per load,
// the lane's four completion times (0 for masked components), the validity mask, and where the lane's first
// element sits (position in its row, row number in the unit).
template <int U, typename F>
__device__ __forceinline__ void flat_process(uint32_t& check, FlatState& fs, const FlatTensor& f, const u32x4 (&x)[U],
                                             const uint32_t (&vm)[U], uint32_t lane, F&& emit) {
    uint32_t s0[U], s1[U], s2[U], s3[U], before[U], se[U], prev_end[U], pos[U], row[U];
    bool c1[U], c2[U], c3[U];                               // component 1, 2, 3 continues the row of component 0
    int back[U];                                            // 4 * (lane of the previous row end) + its component; < 0: earlier load
    const int lane4m1 = (int)(4u * lane) - 1;
#pragma unroll
    for (int k = 0; k < U; ++k) {
        s0[k] = x[k].x; s1[k] = s0[k] + x[k].y; s2[k] = s1[k] + x[k].z; s3[k] = s2[k] + x[k].w;
        check = umax(umax(check, x[k].x), x[k].y);
        check = umax(umax(check, x[k].z), x[k].w);
    }
#pragma unroll
    for (int k = 0; k < U; ++k) before[k] = segmented_inclusive_scan<64>(s3[k], lane) - s3[k];
    bool open_end[U];                                       // wave-uniform: the load's last element does not end a row
#pragma unroll
    for (int k = 0; k < U; ++k) {
        pos[k] = fs.pos0;
        row[k] = fs.row;
        const uint32_t ce = f.M - fs.pos0;
        c1[k] = ce > 1u; c2[k] = ce > 2u; c3[k] = ce > 3u;
        se[k] = c3[k] ? s3[k] : c2[k] ? s2[k] : c1[k] ? s1[k] : s0[k];      // s_{ce-1}; unused when ce > 4
        back[k] = lane4m1 - (int)fs.pos0;
        const int from = back[k] < 0 ? 0 : back[k];
        prev_end[k] = (uint32_t)__builtin_amdgcn_ds_bpermute(from & ~3, (int)(before[k] + se[k]));
        open_end[k] = f.M - fs.pos_last != 4u;
        flat_advance(fs, f);
    }
    uint4 p[U];
#pragma unroll
    for (int k = 0; k < U; ++k) {
        const uint32_t a = before[k] - (back[k] >= 0 ? prev_end[k] : 0u - fs.carry);
        const uint32_t b = 0u - se[k];
        p[k].x = s0[k] + a;
        p[k].y = s1[k] + (c1[k] ? a : b);
        p[k].z = s2[k] + (c2[k] ? a : b);
        p[k].w = s3[k] + (c3[k] ? a : b);
        const uint32_t last = (uint32_t)__builtin_amdgcn_readlane((int)p[k].w, 63);
        fs.carry = open_end[k] ? last : 0u;
    }
#pragma unroll
    for (int k = 0; k < U; ++k) emit(p[k], vm[k], pos[k], row[k]);
}

// One load of rows with 1..3 elements.  MS: the row length when the kernel was built for it (then positions wrap by
// a mask or one subtraction, and rows of one element need nothing from the neighbouring lane), else 0.
template <int MS, typename F>
__device__ __forceinline__ void flat_process_small(uint32_t& check, FlatState& fs, const FlatTensor& f, u32x4 x,
                                                   uint32_t vm, uint32_t lane, F&& emit) {
    check = umax(check, umax(umax(x.x, x.y), umax(x.z, x.w)));
    uint32_t out[4];
    if constexpr (MS == 1) {
        out[0] = x.x; out[1] = x.y; out[2] = x.z; out[3] = x.w;          // a completion time is the latency itself
    } else {
        uint32_t y0 = (uint32_t)__shfl_up((int)x.z, 1, 64), y1 = (uint32_t)__shfl_up((int)x.w, 1, 64);
        if (lane == 0) { y0 = fs.prev2; y1 = fs.prev3; }
        const uint32_t y[6] = {y0, y1, x.x, x.y, x.z, x.w};
#pragma unroll
        for (uint32_t c = 0; c < 4; ++c) {
            uint32_t pc = fs.pos0 + c;                                    // <= 5
            if constexpr (MS == 2) pc &= 1u;
            else if constexpr (MS == 3) pc -= pc >= 3u ? 3u : 0u;
            else pc %= f.M;
            out[c] = y[c + 2] + (pc >= 1u ? y[c + 1] : 0u) + (pc >= 2u ? y[c] : 0u);
        }
        fs.prev2 = (uint32_t)__builtin_amdgcn_readlane((int)x.z, 63);
        fs.prev3 = (uint32_t)__builtin_amdgcn_readlane((int)x.w, 63);
    }
    const uint32_t pos = fs.pos0, row = fs.row;
    flat_advance(fs, f);
    emit(make_uint4(out[0], out[1], out[2], out[3]), vm, pos, row);
}

// One wave streams a unit: `len` elements (whole rows) from element `first` of lat.
template <bool SMALL, int U = DC_FLAT_UNROLL, int MS = 0, typename F>
__device__ __forceinline__ void flat_stream_unit(uint32_t& check, const FlatTensor& f, uint64_t first, uint32_t len,
                                                 uint32_t lane, F&& emit) {
    const uint64_t start = first + f.off;                  // vector-space element of the unit's head
    const uint64_t v0 = start >> 2;
    const uint32_t k = (uint32_t)start & 3u;               // components of vector v0 that precede the unit
    const uint32_t nv = (k + len + 3u) >> 2;
    const uint32_t nloads = (nv + 63u) >> 6;
    const bool guard = (f.off != 0u && v0 == 0u) || (f.ragged_end && v0 + nv == f.total_vectors);

    FlatState fs{0u, 0u, 0u, 0u, 0u, 0u};
    {
        const int q0 = (int)(4u * lane) - (int)k;          // unit-relative element of the lane's first component
        fs.pos0 = q0 >= 0 ? (uint32_t)q0 % f.M : (f.M - ((uint32_t)(-q0) % f.M)) % f.M;
        fs.row = q0 >= 0 ? (uint32_t)q0 / f.M : 0u - (((uint32_t)(-q0) + f.M - 1u) / f.M);   // floor(q0 / M)
        fs.pos_last = (252u - k) % f.M;
    }
    // first load: components before the unit's head, and maybe beyond its end, are masked
    {
        const uint32_t limit = len + k < 256u ? len + k : 256u;
        const uint32_t vm[1] = {flat_valid_mask(lane, k, limit)};
        const u32x4 x[1] = {flat_masked(flat_load(f, v0 + lane, lane < nv, guard), vm[0])};
        if constexpr (SMALL) flat_process_small<MS>(check, fs, f, x[0], vm[0], lane, emit);
        else flat_process<1>(check, fs, f, x, vm, lane, emit);
    }
    // middle loads: every component belongs to the unit
    uint32_t i = 1;
    if (nloads > 2u) {
        const u32x4* base = f.vec + v0 + lane;
        if constexpr (!SMALL) {
            uint32_t all[U];
#pragma unroll
            for (int q = 0; q < U; ++q) all[q] = 0xFu;
            for (; i + U <= nloads - 1u; i += U) {
                u32x4 x[U];
#pragma unroll
                for (int q = 0; q < U; ++q) x[q] = __builtin_nontemporal_load(base + (uint64_t)(i + q) * 64u);
                flat_process<U>(check, fs, f, x, all, lane, emit);
            }
        } else {
            for (; i + U <= nloads - 1u; i += U) {              // U loads in flight, then taken in order
                u32x4 x[U];
#pragma unroll
                for (int q = 0; q < U; ++q) x[q] = __builtin_nontemporal_load(base + (uint64_t)(i + q) * 64u);
#pragma unroll
                for (int q = 0; q < U; ++q) flat_process_small<MS>(check, fs, f, x[q], 0xFu, lane, emit);
            }
        }
        const uint32_t all1[1] = {0xFu};
        for (; i < nloads - 1u; ++i) {
            const u32x4 x[1] = {__builtin_nontemporal_load(base + (uint64_t)i * 64u)};
            if constexpr (SMALL) flat_process_small<MS>(check, fs, f, x[0], 0xFu, lane, emit);
            else flat_process<1>(check, fs, f, x, all1, lane, emit);
        }
    }
    // last load (when it is not also the first)
    if (nloads > 1u) {
        i = nloads - 1u;
        const uint32_t limit = len + k - 256u * i;         // 1..256 by the choice of nloads
        const uint32_t vm[1] = {flat_valid_mask(lane, 0u, limit)};
        const u32x4 x[1] = {flat_masked(flat_load(f, v0 + (uint64_t)i * 64u + lane, i * 64u + lane < nv, guard), vm[0])};
        if constexpr (SMALL) flat_process_small<MS>(check, fs, f, x[0], vm[0], lane, emit);
        else flat_process<1>(check, fs, f, x, vm, lane, emit);
    }
}

// Counting consumer: queue the four completion times of every lane that is wholly inside the unit and
// reaches the smallest threshold; a lane that is only partly inside (first and last vector of a unit) bins
// its valid ones itself.
__device__ __forceinline__ void flat_count(WaveState& st, uint4 p, uint32_t vm, uint4* queue, const GridView& g,
                                           uint32_t lane) {
    const uint32_t top = umax(umax(p.x, p.y), umax(p.z, p.w));
    st.lane_max = umax(st.lane_max, top);                    // masked components have completion time 0
    const bool whole = vm == 0xFu;
    const bool active = whole && top >= g.tau0;
    const uint64_t mask = __ballot(active);
    if ((uint32_t)__popcll(mask) >= DC_DENSE_LANES) {
        // Most lanes hold completion times inside the threshold grid (short rows, whose every element is a row end or
        // close to one; grids that cover much of the data): the queue would only copy what is already in registers.
        if (active) {
            uint32_t b[4];
            bins_of4(g, p, b);
#pragma unroll
            for (int i = 0; i < 4; ++i) count_bin(g, b[i]);
        }
    } else if (mask) {
        if (active) {
            const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                      __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
            queue[(st.q_head + st.q_count + rank) & (QUEUE_ITEMS - 1)] = p;
        }
        st.q_count += (uint32_t)__popcll(mask);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        if (st.q_count >= 64u) drain(st, queue, g, lane);
    }
    if (!whole && vm) {
        const uint32_t val[4] = {p.x, p.y, p.z, p.w};
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (((vm >> c) & 1u) && val[c] >= g.tau0) atomicAdd(&g.hist[bin_of(g.tau, g.p2, val[c])], 1u);
    }
}

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
// dc_scan_rows_kernel: short rows that a lane can own.  M <= 16, N a multiple of 4, every trial on a 16-byte
// boundary.
// The kernels above spread a row over lanes and pay for it with cross-lane sums and, per 16-byte load, one queue
// slot or one search per element; with rows of a few elements that arithmetic, not HBM, bounds them.  Here a lane
// holds R whole rows in registers (V 16-byte vectors = R*M elements), so completion times are R*M plain additions,
// and because they do not decrease along a row (latencies >= 0) the thresholds are met from the row's end
// backwards: step s bins the (M-1-s)-th completion time of all R rows at once and the wave stops at the first
// step in which no lane reaches the smallest threshold; with the usual grids that is after one or two steps.
// A wave reads a chunk of 64 V consecutive vectors with coalesced loads (lane l takes vectors l, l + 64, ...) and,
// unless a vector holds whole rows anyway (M = 1, 2), passes them through its own stretch of LDS so that lane l ends
// up with vectors l V, ..., l V + V - 1: for odd M these reads are free of bank conflicts, for even M two-way.
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
        if (s + 1 < M && s < S::PAIRED_STEPS && (uint32_t)__popcll(reach) >= DC_DENSE_LANES) {
            // most lanes are inside the grid, so the next step would very likely run as well: both at once, twice as
            // many independent searches in flight (completion times below the grid find bin 0 and count nowhere)
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

// The lanes' maxima of one chunk, when a chunk may hold rows of several trials (SPAN).  A lane's four consecutive rows
// lie in one trial or, with a trial boundary inside the lane, in two (trials have at least 4 rows).  Key and value
// of a lane are the trial of its last row and the maximum over its rows in that trial; trials are runs of at most
// trial_lanes consecutive lanes, so a running maximum over lanes that restarts where the key changes (steps up to that
// length suffice) leaves every trial's maximum in the last lane with its key, which adds it to the trial's word
// (cleared by the prep kernel) with one atomic maximum.  A lane with a boundary inside adds the maximum of its rows
// before the boundary to the previous trial's word itself.
__device__ __forceinline__ void add_trial_maxima(uint32_t m, uint32_t t, uint32_t m_before, bool valid, uint32_t lane,
                                                 uint32_t trial_lanes, uint32_t* trial_max) {
    const uint32_t key = valid ? t : 0xFFFFFFFFu;
    for (uint32_t d = 1; d < 64u && d < trial_lanes; d <<= 1) {                  // wave-uniform bounds
        const uint32_t om = (uint32_t)__shfl_up((int)m, d, 64);
        const uint32_t ok = (uint32_t)__shfl_up((int)key, d, 64);
        if (lane >= d && ok == key) m = umax(m, om);
    }
    const uint32_t next = (uint32_t)__shfl_down((int)key, 1, 64);
    if (valid && (lane == 63u || next != key)) atomicMax(&trial_max[t], m);
    if (valid && m_before) atomicMax(&trial_max[t - 1u], m_before);              // zero adds nothing to a maximum
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
            const uint32_t rows = (N - row0) < chunks_per_unit * CHUNK_ROWS ? (N - row0) : chunks_per_unit * CHUNK_ROWS;
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

// After every wave has binned its share of trial t: prefix sums over the histogram, S_t per threshold.
__device__ __forceinline__ void finish_trial(const GridView& g, const TrialShared& sh, uint32_t kc, uint32_t t,
                                             const long long* __restrict__ comm_per_trial, long long comm,
                                             double elements_per_trial, uint32_t* status) {
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
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
        sh.acc[b] += (double)((long long)tmax + c) / (double)den * (done / elements_per_trial);
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
        wt.acc[b] += (double)((long long)tmax + c) / (double)den * (done / elements_per_trial);
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
    for (uint32_t t = blockIdx.x * DC_SCAN_WAVES + wave; t < T; t += gridDim.x * DC_SCAN_WAVES) {
        st.lane_max = 0u;
        const u32x4* base = reinterpret_cast<const u32x4*>(lat + (uint64_t)t * N * M) + lane;
        stream_rows<L>(st, base, nfull, tail_rows, queue, g, lane, shape);
        while (st.q_count) drain(st, queue, g, lane);
        finish_wave_trial(g, wt, kc, t, wave_max(st.lane_max), comm_per_trial, comm, elements_per_trial, lane, status);
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
                                  uint32_t max_latency, uint32_t lanes_per_row) {
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned long long* acc = reinterpret_cast<unsigned long long*>(smem);
    for (uint32_t i = threadIdx.x; i < 3 * N; i += DC_SCAN_THREADS) acc[i] = 0ull;
    __syncthreads();

    constexpr int U = DC_SCAN_UNROLL;
    const uint32_t lane = threadIdx.x & 63u;
    const RowShape shape = row_shape<L>(lane, lanes_per_row);
    const uint32_t R = shape.rows, M = 4 * shape.lanes;
    const uint64_t stride = L ? 64u : shape.active;
    const bool row_end = shape.ok && shape.pos == shape.lanes - 1;      // this lane ends a row: it holds the total
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t nfull = N / R, tail_rows = N - nfull * R;
    const uint32_t lo = (uint32_t)((uint64_t)nfull * wave / DC_SCAN_WAVES);
    const uint32_t hi = (uint32_t)((uint64_t)nfull * (wave + 1) / DC_SCAN_WAVES);
    uint32_t check = 0u;
    for (uint32_t t = blockIdx.x; t < T; t += gridDim.x) {
        const u32x4* base = reinterpret_cast<const u32x4*>(lat + (uint64_t)t * trial_stride + (uint64_t)lo * R * M) + lane;
        uint32_t i = 0;
        for (; i + U <= hi - lo; i += U) {
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
        for (; i < hi - lo; ++i) {
            const u32x4 x[1] = {load_rows<L>(base + (uint64_t)i * stride, shape)};
            uint32_t incl[1];
            completion_times<L, 1>(x, incl, lane, shape);
            check = umax(check, umax(umax(x[0].x, x[0].y), umax(x[0].z, x[0].w)));
            if (row_end) add_worker_total(acc, N, (lo + i) * R + shape.row, incl[0]);
        }
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
    for (uint32_t i = threadIdx.x; i < 3 * N; i += DC_SCAN_THREADS) out[i] = acc[i];
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

// result[3][N] = sums over blocks (the 128-bit squares with carry).  A block of 256 threads takes 32 workers; its
// eight groups of 32 threads add every eighth block's partial sums (32 consecutive 8-byte words per read), then the
// eight partial results are added in a fixed order.
__global__ __launch_bounds__(256)
void dc_worker_totals_final_kernel(const unsigned long long* __restrict__ partial, uint32_t blocks, uint32_t N,
                                   unsigned long long* __restrict__ result) {
    __shared__ unsigned long long part[8][32][3];
    const uint32_t w = threadIdx.x & 31u, slice = threadIdx.x >> 5;
    const uint32_t n = blockIdx.x * 32u + w;
    unsigned long long sum = 0ull;
    unsigned __int128 sq = 0;
    if (n < N) {
        for (uint32_t b = slice; b < blocks; b += 8u) {
            const unsigned long long* in = partial + (uint64_t)b * 3 * N;
            sum += in[n];
            sq += ((unsigned __int128)in[2 * N + n] << 64) | in[N + n];
        }
    }
    part[slice][w][0] = sum;
    part[slice][w][1] = (unsigned long long)sq;
    part[slice][w][2] = (unsigned long long)(sq >> 64);
    __syncthreads();
    if (slice == 0 && n < N) {
        for (uint32_t q = 1; q < 8u; ++q) {
            sum += part[q][w][0];
            sq += ((unsigned __int128)part[q][w][2] << 64) | part[q][w][1];
        }
        result[n] = sum;
        result[N + n] = (unsigned long long)sq;
        result[2 * N + n] = (unsigned long long)(sq >> 64);
    }
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
    if (blocks < clearing) blocks = clearing < 64u ? clearing : 64u;
    hipLaunchKernelGGL(dc_prep_kernel, dim3(blocks), dim3(threads), 0, stream, taus, K, tau_sorted, tau_u32, pos,
                       status, bins, bins_words, lat, (unsigned long long)rows_total, N ? N : 1u,
                       (unsigned long long)trial_stride, M, sample_rows, zero_words, zero_count);
}

size_t scan_lds_bytes(const Plan& p) {
    const size_t tables = (size_t)p.p2 * 8;                       // thresholds + histogram
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
    if (p.lane_rows) {
        hipError_t e = hipErrorInvalidValue;
        switch (p.M) {
#define DC_ROWS_CASE(m) case m: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, dc_scan_rows_kernel<m, false>, DC_SCAN_THREADS, lds); break;
            DC_ROWS_CASE(1) DC_ROWS_CASE(2) DC_ROWS_CASE(3) DC_ROWS_CASE(4) DC_ROWS_CASE(5) DC_ROWS_CASE(6) DC_ROWS_CASE(7)
            DC_ROWS_CASE(8) DC_ROWS_CASE(9) DC_ROWS_CASE(10) DC_ROWS_CASE(11) DC_ROWS_CASE(12) DC_ROWS_CASE(13)
            DC_ROWS_CASE(14) DC_ROWS_CASE(15) DC_ROWS_CASE(16)
            DC_ROWS_CASE(17) DC_ROWS_CASE(18) DC_ROWS_CASE(19) DC_ROWS_CASE(21) DC_ROWS_CASE(22) DC_ROWS_CASE(23) DC_ROWS_CASE(25)
            DC_ROWS_CASE(26) DC_ROWS_CASE(30) DC_ROWS_CASE(34)
#undef DC_ROWS_CASE
            default: break;
        }
        return e == hipSuccess ? n : 0;
    }
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
    switch (p.M / 4) {
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
                               hist_part, status, p.max_latency, p.M / 4);
            hipLaunchKernelGGL((dc_scan_vec4_kernel<L, 2>), dim3(p.grid_wide), dim3(DC_SCAN_THREADS), scan_lds_bytes(p),
                               stream, lat, p.stride, p.N, p.units, p.units_per_trial, p.run, p.per_unit, tau_chunk, kc, p.p2,
                               unit_max, hist_part, status, p.max_latency, p.M / 4);
            return;
        }
    }
    hipLaunchKernelGGL((dc_scan_vec4_kernel<L, 0>), dim3(p.grid), dim3(DC_SCAN_THREADS), scan_lds_bytes(p), stream, lat,
                       p.stride, p.N, p.units, p.units_per_trial, p.run, p.per_unit, tau_chunk, kc, p.p2, unit_max, hist_part,
                       status, p.max_latency, p.M / 4);
}

template <int MS>
static void launch_flat(const Plan& p, const int32_t* lat, const uint32_t* tau_chunk, uint32_t kc,
                        uint32_t* unit_max, uint32_t* hist_part, uint32_t* status, hipStream_t stream) {
    hipLaunchKernelGGL(dc_scan_flat_kernel<MS>, dim3(p.grid), dim3(DC_SCAN_THREADS), scan_lds_bytes(p), stream, lat,
                       p.extent, p.stride, p.N, p.M, p.units, p.units_per_trial, p.run, p.per_unit, tau_chunk, kc, p.p2,
                       unit_max, hist_part, status, p.max_latency);
}

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

void launch_scan(const Plan& p, const int32_t* lat, const uint32_t* tau_chunk, uint32_t kc, uint32_t* unit_max,
                 uint32_t* hist_part, uint32_t* status, hipStream_t stream) {
    if (p.lane_rows) {
        switch (p.M) {
#define DC_ROWS_CASE(m) case m: launch_rows<m>(p, lat, tau_chunk, kc, unit_max, hist_part, status, stream); break;
            DC_ROWS_CASE(1) DC_ROWS_CASE(2) DC_ROWS_CASE(3) DC_ROWS_CASE(4) DC_ROWS_CASE(5) DC_ROWS_CASE(6) DC_ROWS_CASE(7)
            DC_ROWS_CASE(8) DC_ROWS_CASE(9) DC_ROWS_CASE(10) DC_ROWS_CASE(11) DC_ROWS_CASE(12) DC_ROWS_CASE(13)
            DC_ROWS_CASE(14) DC_ROWS_CASE(15) DC_ROWS_CASE(16)
            DC_ROWS_CASE(17) DC_ROWS_CASE(18) DC_ROWS_CASE(19) DC_ROWS_CASE(21) DC_ROWS_CASE(22) DC_ROWS_CASE(23) DC_ROWS_CASE(25)
            DC_ROWS_CASE(26) DC_ROWS_CASE(30) DC_ROWS_CASE(34)
#undef DC_ROWS_CASE
            default: break;                         // make_plan sets lane_rows for these row lengths only
        }
        return;
    }
    if (!p.vec4) {
        switch (p.M) {
            case 1:  launch_flat<1>(p, lat, tau_chunk, kc, unit_max, hist_part, status, stream); break;
            case 2:  launch_flat<2>(p, lat, tau_chunk, kc, unit_max, hist_part, status, stream); break;
            case 3:  launch_flat<3>(p, lat, tau_chunk, kc, unit_max, hist_part, status, stream); break;
            default: launch_flat<0>(p, lat, tau_chunk, kc, unit_max, hist_part, status, stream); break;
        }
        return;
    }
    switch (p.M / 4) {
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

__global__ void dc_clear_status_kernel(uint32_t* status) { *status = 0u; }

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

template <int L>
static void launch_worker_vec4(const Plan& p, const int32_t* lat, unsigned long long* partial, uint32_t* status,
                               hipStream_t stream) {
    hipLaunchKernelGGL(dc_worker_totals_vec4_kernel<L>, dim3(p.grid), dim3(DC_SCAN_THREADS), (size_t)p.N * 24, stream,
                       lat, p.stride, p.T, p.N, partial, status, p.max_latency, p.M / 4);
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
        switch (p.M / 4) {
            case 1:  launch_worker_vec4<1>(p, lat, partial, status, stream); break;
            case 2:  launch_worker_vec4<2>(p, lat, partial, status, stream); break;
            case 4:  launch_worker_vec4<4>(p, lat, partial, status, stream); break;
            case 8:  launch_worker_vec4<8>(p, lat, partial, status, stream); break;
            case 16: launch_worker_vec4<16>(p, lat, partial, status, stream); break;
            case 32: launch_worker_vec4<32>(p, lat, partial, status, stream); break;
            case 64: launch_worker_vec4<64>(p, lat, partial, status, stream); break;
            default: launch_worker_vec4<0>(p, lat, partial, status, stream); break;
        }
    }
    if (after) (void)hipEventRecord(after, stream);
    hipLaunchKernelGGL(dc_worker_totals_final_kernel, dim3((p.N + 31) / 32), dim3(256), 0, stream, partial, p.grid,
                       p.N, result);
}

}  // namespace dc
