// Device-side building blocks shared by the kernels of the DropCompute step-time simulator (gfx950: wave64, DPP,
// LDS): wave primitives, the threshold grid in LDS and its lookup, the per-wave queue, the streaming of whole rows
// per load, and the flat pass for rows of any length.  Everything here is inline; every translation unit that
// includes it gets its own copy.
#ifndef DC_DEVICE_H
#define DC_DEVICE_H

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

// rows_per_load (L = 0 only): fewer whole rows per load than fit, 0 = as many as fit
template <int L>
__device__ __forceinline__ RowShape row_shape(uint32_t lane, uint32_t lanes_per_row, uint32_t rows_per_load = 0u) {
    RowShape r;
    r.lanes = L ? (uint32_t)L : lanes_per_row;
    r.rows = (L == 0 && rows_per_load) ? rows_per_load : 64u / r.lanes;
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

// U loads of whole rows: completion times, the lane's running maximum, and the completion times that reach the
// threshold grid on their way into the histogram.  incl[k] returns the completion time of the lane's last element
// in load k.
template <int L, int U>
__device__ __forceinline__ void process_loads(WaveState& st, const u32x4 (&x)[U], uint32_t (&incl)[U], uint4* queue,
                                              const GridView& g, uint32_t lane, const RowShape& shape) {
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

template <int L, int U>
__device__ __forceinline__ void process_loads(WaveState& st, const u32x4 (&x)[U], uint4* queue, const GridView& g,
                                              uint32_t lane, const RowShape& shape) {
    uint32_t incl[U];
    process_loads<L, U>(st, x, incl, queue, g, lane, shape);
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

// Small trials of a contiguous tensor whose worker count is a multiple of the rows per load: a trial is
// loads_per_trial whole loads and the next trial follows at once, so one wave streams `nloads` loads of several
// consecutive trials as one run, eight in flight whatever trial they belong to, and keeps the running maximum per
// trial: after a trial's last load the wave's maximum goes to trial_max[that trial] (counted from the run's first).
template <int L>
__device__ __forceinline__ void stream_small_trials(WaveState& st, const u32x4* base, uint32_t nloads,
                                                    uint32_t loads_per_trial, uint32_t* trial_max, uint4* queue,
                                                    const GridView& g, uint32_t lane, const RowShape& shape) {
    constexpr int U = DC_SCAN_UNROLL;
    const uint64_t stride = L ? 64u : shape.active;   // 16-byte vectors per load
    uint32_t in_trial = 0u, t = 0u;                    // loads of the current trial so far; its number (wave-uniform)
    uint32_t cur = 0u;                                 // the lane's maximum inside the current trial
    uint32_t i = 0;
    for (; i + U <= nloads; i += U) {
        u32x4 x[U];
        uint32_t incl[U];
#pragma unroll
        for (int k = 0; k < U; ++k) x[k] = load_rows<L>(base + (uint64_t)(i + k) * stride, shape);
        process_loads<L, U>(st, x, incl, queue, g, lane, shape);
#pragma unroll
        for (int k = 0; k < U; ++k) {
            cur = umax(cur, incl[k]);
            if (++in_trial == loads_per_trial) {
                const uint32_t m = wave_max(cur);
                if (lane == 0) trial_max[t] = m;
                ++t; in_trial = 0u; cur = 0u;
            }
        }
    }
    for (; i < nloads; ++i) {
        const u32x4 x[1] = {load_rows<L>(base + (uint64_t)i * stride, shape)};
        uint32_t incl[1];
        process_loads<L, 1>(st, x, incl, queue, g, lane, shape);
        cur = umax(cur, incl[0]);
        if (++in_trial == loads_per_trial) {
            const uint32_t m = wave_max(cur);
            if (lane == 0) trial_max[t] = m;
            ++t; in_trial = 0u; cur = 0u;
        }
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

// The lanes' maxima of one chunk, when a chunk may hold rows of several trials (SPAN).  A lane's consecutive rows (four, or one)
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


}  // namespace

#endif
