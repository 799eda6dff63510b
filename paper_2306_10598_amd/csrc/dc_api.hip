// C ABI of the DropCompute step-time simulator (see include/dc.h): argument checks, the plan of a
// call (kernel choice, work units, workspace layout), kernel sequencing, and the host-only
// threshold selection.  No computation on latencies happens on the host.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

#include "dc.h"
#include "dc_internal.h"

namespace {

thread_local char g_error_text[256] = "";

int device_error(hipError_t e, const char* what, int status = DC_ERR_DEVICE) {
    snprintf(g_error_text, sizeof(g_error_text), "%s: %s", what, hipGetErrorString(e));
    return status;
}

#define DC_HIP(call)                                         \
    do {                                                     \
        hipError_t e_ = (call);                              \
        if (e_ != hipSuccess) return device_error(e_, #call); \
    } while (0)

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

uint32_t next_pow2_above(uint32_t n) {   // smallest power of two > n, at least 4 (the lookup cells need p2 - 2 >= 2)
    uint32_t p = 4;
    while (p <= n) p <<= 1;
    return p;
}

// Rows that the kernels with whole rows per load take: 1..32 lanes of 16 bytes, or exactly 64.  Rows of 33..63
// lanes would leave up to half of every load's lanes idle there and stream faster through the flat kernel
// (measured: 6.1 against 3.0 TB/s at M = 132, 6.2 against 4.8 at M = 252).
bool vec4_shape(int64_t M) {
    return M >= 4 && (M & 3) == 0 && (M <= 128 || M == 256);
}

// Rows per unit of the kernels for arbitrary row lengths: a trial is cut into equal runs of whole rows of
// about DC_FLAT_UNIT_ELEMENTS elements (at least one row), so that no short unit is left over at its end.
// share > 1: the units of a trial are dealt to that many waves, so their number is made a multiple of it.
uint64_t flat_rows_per_unit(int64_t N, int64_t M, uint64_t share = 1) {
    const uint64_t per_trial = (uint64_t)N * (uint64_t)M;                   // < 2^62
    uint64_t pieces = (per_trial + DC_FLAT_UNIT_ELEMENTS - 1) / DC_FLAT_UNIT_ELEMENTS;
    pieces = (pieces + share - 1) / share * share;
    if (pieces > (uint64_t)N) pieces = (uint64_t)N;
    return ((uint64_t)N + pieces - 1) / pieces;
}

// The tensor's shape: T trials of N rows of M elements, consecutive trials `stride` elements apart (0: N*M).
// Returns false when it is outside what the library handles; else fills T, N, M, elements, stride, extent.
bool plan_shape(int64_t T, int64_t N, int64_t M, int64_t stride, dc::Plan* p) {
    if (T < 1 || N < 1 || M < 1) return false;
    const int64_t lim = (int64_t)1 << 31;
    if (T >= lim || N >= lim || M >= lim) return false;
    if ((long double)T * (long double)N * (long double)M >= 4.6e18L) return false;   // < 2^62
    const uint64_t row_elements = (uint64_t)N * (uint64_t)M;
    if (stride == 0) stride = (int64_t)row_elements;
    if (stride < 0 || (uint64_t)stride < row_elements) return false;
    if ((long double)(T - 1) * (long double)stride + (long double)row_elements >= 4.6e18L) return false;
    p->T = (uint32_t)T; p->N = (uint32_t)N; p->M = (uint32_t)M;
    p->elements = (uint64_t)T * row_elements;
    p->stride = (uint64_t)stride;
    p->extent = (uint64_t)(T - 1) * (uint64_t)stride + row_elements;
    return true;
}

// Returns false when the sizes are outside what the library handles.  allow_vec4: lat is 16-byte aligned.
bool make_plan(int64_t T, int64_t N, int64_t M, int64_t K, bool allow_vec4, dc::Plan* out, int64_t stride = 0) {
    if (K < 1 || K > DC_MAX_THRESHOLDS) return false;
    dc::Plan p{};
    if (!plan_shape(T, N, M, stride, &p)) return false;
    p.K = (uint32_t)K;
    const bool aligned = allow_vec4 && (p.stride & 3u) == 0;          // every trial starts on a 16-byte boundary
    const bool rows_length = M < 64 && dc::lane_rows_length((uint32_t)M);
    const int64_t rows_per_lane = (M > 16 && (M & 3) == 2) ? 2 : 4;
    p.lane_rows = aligned && rows_length && (N % rows_per_lane) == 0 && N >= (int64_t)DC_LANE_ROWS_MIN_N;
    // other worker counts from 4 on: the same kernel over the tensor as one run of T*N rows (a multiple of 4), when the
    // tensor is contiguous and a lane's four rows are consecutive (rows of 1, 2 and 4 elements are dealt to the lanes
    // vector by vector instead)
    bool span = DC_SPAN_TRIALS != 0 && aligned && !p.lane_rows && M <= 16 && M != 1 && M != 2 && M != 4 && N >= 4 &&
                (((uint64_t)T * (uint64_t)N) & 3u) == 0 && p.stride == (uint64_t)N * (uint64_t)M &&
                (uint64_t)T * (uint64_t)N < ((uint64_t)1 << 31);
    if (span && (M & 3) == 0) {
        // rows of 8, 12 and 16 elements also fit the kernel with whole rows per load, which is the faster one
        // (5.5-5.9 against 4.0-5.4 TB/s on 512 MB with 200 workers) unless the trial's last load is mostly empty
        const int64_t rows_per_load = 64 / (M / 4);
        const int64_t loads = (N + rows_per_load - 1) / rows_per_load;
        span = N * 100 < loads * rows_per_load * 85 && p.elements >= ((uint64_t)1 << 22);   // (below 16 MB either takes 8-9 us)
    }
    if (span) { p.lane_rows = true; p.span_rows = (uint32_t)N; }
    // rows of 17 to 63 elements that are no multiple of 4 and that the kernel above does not take: one row per lane,
    // chunks of 64 rows -- from 25 elements on, and shorter ones with fewer than 256 workers (where the kernel above is
    // not available and the flat pass would take a unit per small trial: 3.5-5.7 against 5.4-6.6 TB/s at 64 and 128
    // workers).  The chunks stay inside the trials when those fill them to 85 % at least (200 workers = 3 chunks and 8
    // rows do not: the flat pass then wins on data with long delays, 4.9 against 4.0 TB/s at 21 elements); trials of
    // fewer than 64 workers on a contiguous tensor are taken as one run of rows as above (8 workers of 45 elements:
    // 2.4 -> 6.3 TB/s).
    const uint64_t row_chunks = ((uint64_t)N + 63) / 64;
    const bool row_lane_ok = aligned && !p.lane_rows && dc::row_lane_length((uint32_t)M) &&
                             (M >= (int64_t)DC_ROW_LANE_MIN_M_MANY || N < (int64_t)DC_LANE_ROWS_MIN_N);
    const bool row_lane_inside = row_lane_ok && (((uint64_t)N * (uint64_t)M) & 3u) == 0 && N >= (int64_t)DC_ROW_LANE_MIN_N &&
                                 (uint64_t)N * 100 >= row_chunks * 64 * 85;
    const bool row_lane_span = DC_SPAN_TRIALS != 0 && row_lane_ok && !row_lane_inside && N >= 4 && N < 64 &&
                               p.stride == (uint64_t)N * (uint64_t)M && (p.elements & 3u) == 0 &&
                               (uint64_t)T * (uint64_t)N < ((uint64_t)1 << 31);
    p.row_lane = row_lane_inside || row_lane_span;
    if (row_lane_span) { span = true; p.span_rows = (uint32_t)N; }
    if (p.row_lane) p.lane_rows = true;
    p.chunk = p.K < DC_CHUNK_THRESHOLDS ? p.K : DC_CHUNK_THRESHOLDS;
    p.p2 = next_pow2_above(p.chunk);
    // These kernels need two blocks per compute unit to hide their LDS round trips (one block: 4.0-4.5 against 5.7-6.2
    // TB/s of the other kernels with 512 thresholds): a plan whose staging areas and threshold tables leave room for
    // one only (rows of 16 or 17 elements with 512 thresholds or more in a pass) goes to the other kernels -- as long as
    // those still run many blocks themselves.  From 2048 table entries on (1024 thresholds in a pass) the tables alone
    // take 32 KiB and more, the kernel for any row length is down to four blocks and fewer, and one block of these
    // kernels is the faster choice again on thin-tailed data by 15-60 %, on heavy-tailed data level.
    if (p.lane_rows && dc::scan_lds_bytes(p) + 1024u > (p.p2 <= 1024u ? DC_LDS_BYTES / 2 : DC_LDS_BYTES)) {   // (+ the kernels' few static words)
        p.lane_rows = p.row_lane = false;
        p.span_rows = 0u;
        span = false;
    }
    p.vec4 = aligned && !p.lane_rows && vec4_shape(M);
    uint64_t upt;
    if (p.lane_rows) {
        // chunks of whole rows; about DC_FLAT_UNIT_ELEMENTS elements per unit, the units of a trial of equal size
        const uint64_t chunk_rows = dc::lane_rows_chunk_rows((uint32_t)M, p.row_lane);
        const uint64_t run_rows = span ? (uint64_t)T * (uint64_t)N : (uint64_t)N;
        const uint64_t chunks = (run_rows + chunk_rows - 1) / chunk_rows;
        uint64_t want = DC_FLAT_UNIT_ELEMENTS / (chunk_rows * (uint64_t)M);
        // a small tensor is cut into more, shorter units, so that every wave of the chip has one
        const uint64_t all_chunks = span ? chunks : chunks * (uint64_t)T;
        if (want > all_chunks / (DC_ROWS_UNITS_PER_WAVE * 4ull * DC_MAX_SCAN_BLOCKS))
            want = all_chunks / (DC_ROWS_UNITS_PER_WAVE * 4ull * DC_MAX_SCAN_BLOCKS);
        if (want < 1) want = 1;
        const uint64_t pieces = (chunks + want - 1) / want;
        p.per_unit = (uint32_t)((chunks + pieces - 1) / pieces);
        upt = (chunks + p.per_unit - 1) / p.per_unit;
    } else if (p.vec4) {
        uint64_t rows_per_load = 64 / (M / 4);
        uint64_t loads_per_trial = ((uint64_t)N + rows_per_load - 1) / rows_per_load;
#ifdef DC_UNIT_LOADS
        p.per_unit = DC_UNIT_LOADS;
#else
        // measured: about 32 rows per unit for long rows (32 loads at M = 256, 16 at M = 128), 64 loads otherwise
        p.per_unit = M >= 128 ? (uint32_t)(32 / rows_per_load < 16 ? 16 : 32 / rows_per_load) : 64u;
#endif
        upt = (loads_per_trial + p.per_unit - 1) / p.per_unit;
        // Small trials (8 workers of 32 accumulations are one load): a unit per trial would leave a wave a load or
        // two at a time and a maximum to reduce after each (2.0-2.8 TB/s on 4.3 GB).  When the trials follow each
        // other without a gap and each is a whole number of loads, a unit is a run of whole trials instead.
        // (As many trials per unit as fill a unit, but no more than leave every wave of the largest grid a unit: 82 MB
        // of 8 KiB trials are over sooner with a unit per trial.)
        // A worker count that is no whole number of loads (8 workers of 20 accumulations: 12 rows fit a load) can still
        // be one of shorter loads: the largest divisor of N below what fits, if it keeps half of the lanes busy or
        // holds the whole trial.
        const bool contiguous = p.stride == (uint64_t)N * (uint64_t)M;
        if (contiguous && M < 128 && (uint64_t)N % rows_per_load != 0) {
            uint64_t r = rows_per_load < (uint64_t)N ? rows_per_load : (uint64_t)N;
            while (r > 1 && (uint64_t)N % r) --r;
            const uint64_t loads = (uint64_t)N / r;
            if ((r * (uint64_t)(M / 4) >= 32 || r == (uint64_t)N) && 2 * loads <= p.per_unit &&
                (uint64_t)T / ((uint64_t)DC_SCAN_WAVES * DC_MAX_SCAN_BLOCKS) >= 2) {
                p.rows_per_load = (uint32_t)r;
                rows_per_load = r;
                loads_per_trial = loads;
                upt = (loads_per_trial + p.per_unit - 1) / p.per_unit;
            }
        }
        if (contiguous && (uint64_t)N % rows_per_load == 0) {
            uint64_t several = p.per_unit / loads_per_trial;
            const uint64_t cap = (uint64_t)T / ((uint64_t)DC_SCAN_WAVES * DC_MAX_SCAN_BLOCKS);
            if (several > cap) several = cap;
            if (several >= 2) {
                p.trials_per_unit = (uint32_t)several;
                upt = 1;
            }
        }
    } else {
        const uint64_t rows = flat_rows_per_unit(N, M);
        p.per_unit = (uint32_t)rows;
        upt = ((uint64_t)N + rows - 1) / rows;
    }
    const uint64_t units = span ? upt
                         : p.trials_per_unit ? ((uint64_t)T + p.trials_per_unit - 1) / p.trials_per_unit
                                             : (uint64_t)T * upt;
    if (units >= ((uint64_t)1 << 31)) return false;
    p.units_per_trial = (uint32_t)upt;
    p.units = (uint32_t)units;
    uint64_t grid = (units + DC_SCAN_WAVES - 1) / DC_SCAN_WAVES;
    p.grid = (uint32_t)(grid < DC_MAX_SCAN_BLOCKS ? grid : DC_MAX_SCAN_BLOCKS);
    p.grid_wide = p.grid;
    p.run = DC_SCAN_WAVES;                                     // both settled in enqueue(), once the device's limits are known
    p.max_latency = (uint32_t)(2147483647ll / M);

    size_t off = 0;
    p.off_status = off;     off += 256;
    p.off_tau_sorted = off; off += align256((size_t)K * 8);
    p.off_tau_u32 = off;    off += align256((size_t)K * 4);
    p.off_pos = off;        off += align256((size_t)K * 4);
    p.off_bins = off;       off += align256((size_t)3 * p.p2 * 8);
    p.off_unit_max = off;   off += align256((size_t)((span || p.trials_per_unit) && p.T > p.units ? p.T : p.units) * 4);   // or one word per trial
    p.off_hist_part = off;  off += align256((size_t)p.grid * p.p2 * 4);
    p.bytes = off;
    *out = p;
    return true;
}

// Plan of the per-iteration speedup pass: one block per trial, float64 sums per block.
bool make_trial_plan(int64_t T, int64_t N, int64_t M, int64_t K, bool allow_vec4, dc::Plan* out, int64_t stride = 0) {
    if (K < 1 || K > DC_MAX_THRESHOLDS) return false;
    dc::Plan p{};
    if (!plan_shape(T, N, M, stride, &p)) return false;
    if (N * M >= ((int64_t)1 << 31)) return false;                            // per-trial counts are 32-bit
    p.K = (uint32_t)K;
    p.vec4 = allow_vec4 && vec4_shape(M) && (p.stride & 3u) == 0;
    p.wave_trials = p.stride == (uint64_t)N * (uint64_t)M && (uint64_t)N * (uint64_t)M <= DC_WAVE_TRIAL_ELEMENTS &&
                    K <= (int64_t)DC_WAVE_TRIAL_THRESHOLDS;
    const int64_t owners = p.wave_trials ? (T + DC_SCAN_WAVES - 1) / DC_SCAN_WAVES : T;     // blocks that can have a trial
    p.grid = (uint32_t)(owners < (int64_t)DC_MAX_TRIAL_BLOCKS ? owners : DC_MAX_TRIAL_BLOCKS);
    p.grid_wide = p.grid;
    if (p.vec4) {
        const uint32_t rows_per_load = 64u / (uint32_t)(M / 4);
        p.per_unit = M >= 128 ? (32u / rows_per_load < 16u ? 16u : 32u / rows_per_load) : 64u;   // as in make_plan
    } else {
        p.per_unit = (uint32_t)flat_rows_per_unit(N, M, DC_SCAN_WAVES);
    }
    p.chunk = p.K < DC_TRIAL_CHUNK_THRESHOLDS ? p.K : DC_TRIAL_CHUNK_THRESHOLDS;
    p.p2 = next_pow2_above(p.chunk);
    p.max_latency = (uint32_t)(2147483647ll / M);
    size_t off = 0;
    p.off_status = off;     off += 256;
    p.off_tau_sorted = off; off += align256((size_t)K * 8);
    p.off_tau_u32 = off;    off += align256((size_t)K * 4);
    p.off_pos = off;        off += align256((size_t)K * 4);
    p.off_partial = off;    off += align256((size_t)p.grid * p.p2 * 8);
    p.bytes = off;
    *out = p;
    return true;
}

// ---- optional timing ---------------------------------------------------------------------------
// Events belong to the workspace that a call runs in, so calls on different streams (each with a workspace of
// its own, as the interface demands) are timed independently.  A fixed table; the slot used longest ago is taken
// over when all are in use.
struct TimingSlot {
    const void* key = nullptr;         // the workspace
    int device = -1;
    bool valid = false, whole = false;
    hipEvent_t begin = nullptr, end = nullptr;
    std::vector<hipEvent_t> scan;      // pairs (before, after) per chunk
    size_t used_pairs = 0;
    uint64_t stamp = 0;
};
constexpr size_t TIMING_SLOTS = 16;
TimingSlot g_slots[TIMING_SLOTS];
uint64_t g_slot_clock = 0;
std::mutex g_timing_mutex;              // guards g_slots' keys, stamps and event creation
std::atomic<int> g_timing_level{0};     // 0 off, 1 streaming kernel, 2 also the whole sequence
thread_local TimingSlot* t_last_slot = nullptr;   // the slot of this thread's last timed call

// The slot of `key` with at least `pairs` event pairs, marked in use by a new call; nullptr on a HIP error (reported
// through *rc).
TimingSlot* acquire_slot(const void* key, size_t pairs, int* rc) {
    std::lock_guard<std::mutex> lock(g_timing_mutex);
    int device = 0;
    (void)hipGetDevice(&device);
    TimingSlot* slot = nullptr;
    for (TimingSlot& s : g_slots)
        if (s.key == key && s.device == device) { slot = &s; break; }
    if (!slot) {
        slot = &g_slots[0];
        for (TimingSlot& s : g_slots)
            if (s.stamp < slot->stamp) slot = &s;
        if (slot->device != device && slot->begin) {           // events belong to the device that created them
            (void)hipEventDestroy(slot->begin); (void)hipEventDestroy(slot->end);
            for (hipEvent_t e : slot->scan) (void)hipEventDestroy(e);
            slot->begin = slot->end = nullptr;
            slot->scan.clear();
        }
        slot->key = key;
        slot->device = device;
    }
    slot->stamp = ++g_slot_clock;
    slot->valid = false;
    slot->whole = g_timing_level.load() >= 2;
    hipError_t e = hipSuccess;
    if (!slot->begin) {
        e = hipEventCreate(&slot->begin);
        if (e == hipSuccess) e = hipEventCreate(&slot->end);
    }
    while (e == hipSuccess && slot->scan.size() < 2 * pairs) {
        hipEvent_t ev;
        e = hipEventCreate(&ev);
        if (e == hipSuccess) slot->scan.push_back(ev);
    }
    if (e != hipSuccess) { *rc = device_error(e, "hipEventCreate"); return nullptr; }
    slot->used_pairs = pairs;
    t_last_slot = slot;
    *rc = DC_OK;
    return slot;
}

int slot_times(TimingSlot* slot, float* scan_ms, float* total_ms) {
    if (!slot || !slot->valid || (total_ms && !slot->whole)) return DC_ERR_INVALID_ARG;
    DC_HIP(hipEventSynchronize(slot->scan[2 * slot->used_pairs - 1]));
    if (total_ms) {
        DC_HIP(hipEventSynchronize(slot->end));
        DC_HIP(hipEventElapsedTime(total_ms, slot->begin, slot->end));
    }
    if (scan_ms) {
        float acc = 0.f;
        for (size_t c = 0; c < slot->used_pairs; ++c) {
            float ms = 0.f;
            DC_HIP(hipEventElapsedTime(&ms, slot->scan[2 * c], slot->scan[2 * c + 1]));
            acc += ms;
        }
        *scan_ms = acc;
    }
    return DC_OK;
}

// ---- grid size of the streaming kernel --------------------------------------------------------------
// The kernel splits the work statically over its waves, so every block must be resident at once (a
// block that waits for a free slot would run alone at the end), and the same number of blocks must
// sit on every compute unit.  Queried once per (device, kernel variant, LDS size).
struct ResidentKey { int device; bool vec4; bool trial; uint32_t M; uint32_t p2; uint32_t wanted; int blocks; int wide_blocks; };
constexpr size_t RESIDENT_SLOTS = 64;         // a fixed table: the enqueue path never touches the host heap
ResidentKey g_resident[RESIDENT_SLOTS];
size_t g_resident_used = 0, g_resident_next = 0;

// Blocks per compute unit that stream best (measured on MI355X with 8 loads in flight per lane): rows that fill
// whole 16-lane groups have few completion times inside a narrow threshold grid and want few, fat waves; short rows
// put a large share of their lanes through the queue and the binning, whose LDS latencies need more waves to hide.
// Rows of 32 and 64 elements on 4.3 GB: 6.8-6.9 TB/s with 2 blocks, 6.4-6.45 with 8; on 512 MB and 82 MB, where the
// kernel is over before few waves have ramped up, 4 blocks are best (6.2 against 5.9-6.0 TB/s and 4.5 against 3.8-4.1).
// `DC_SCAN_BLOCKS_PER_CU` overrides the choice at build time.
// The second launch and the sample behind the choice cost about 15 us per call, so rows of 32 and 64 elements take
// them from 1 GiB on and run tensors below that with one launch of 4 blocks per compute unit.
bool two_launch_shapes(const dc::Plan& p, bool trial) {
    if (!p.vec4 || p.wave_trials) return false;
    if (p.rows_per_load) return false;               // those plans run the instantiation for any row length, built for one shape
    return p.M >= 128 || (!trial && (p.M == 32 || p.M == 64) && p.elements >= ((uint64_t)1 << 28));
}

uint32_t wanted_blocks_per_cu(const dc::Plan& p, bool trial) {
#ifdef DC_SCAN_BLOCKS_PER_CU
    return DC_SCAN_BLOCKS_PER_CU;
#else
    if (p.wave_trials) return 8;
    if (p.vec4 && p.M >= 128) return 2;
    if (two_launch_shapes(p, trial)) return 2;
    if (p.vec4 && !trial && (p.M == 32 || p.M == 64)) return 4;
    return 8;
#endif
}

// ... and for threshold grids that cover much of the data (the second launch shape)
uint32_t dense_blocks_per_cu(const dc::Plan& p) { return p.M >= 128 ? DC_DENSE_BLOCKS_PER_CU : 8; }

// Which instantiation a plan runs, as the M field of the key: the row length for the kernels of whole rows
// per load, else which of the kernels for arbitrary rows (built for rows of 1, 2, 3 elements, or for any longer row).
uint32_t variant_of(const dc::Plan& p) {
    if (p.wave_trials) return 0x20000u + p.M;
    if (p.vec4) return p.rows_per_load ? 0x40000u + p.M : p.M;
    if (p.lane_rows) return 0x10000u + p.M;
    return p.M < 4 ? p.M : 4u;
}

struct Resident {
    uint32_t blocks;        // the grid that streams the usual, narrow threshold grids best
    uint32_t wide_blocks;   // long rows only: the larger grid for threshold grids that cover much of the data (else = blocks)
};

std::mutex g_resident_mutex;             // guards g_resident

Resident resident_blocks(const dc::Plan& p, bool trial = false) {
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) return {DC_MAX_SCAN_BLOCKS, DC_MAX_SCAN_BLOCKS};
    std::lock_guard<std::mutex> lock(g_resident_mutex);
    for (size_t i = 0; i < g_resident_used; ++i) {
        const ResidentKey& k = g_resident[i];
        if (k.device == device && k.vec4 == p.vec4 && k.trial == trial && k.M == variant_of(p) && k.p2 == p.p2 &&
            k.wanted == wanted_blocks_per_cu(p, trial))
            return {(uint32_t)k.blocks, (uint32_t)k.wide_blocks};
    }
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || cus < 1) cus = 256;
    int fit = trial ? dc::trial_scan_blocks_per_cu(p) : dc::scan_blocks_per_cu(p);      // what fits
    if (fit < 1) fit = 1;
    const int wanted = (int)wanted_blocks_per_cu(p, trial);                             // what streams best
    const int per_cu = fit > wanted ? wanted : fit;
    int wide_per_cu = per_cu;
    const int dense = (int)dense_blocks_per_cu(p);
    if (two_launch_shapes(p, trial) && per_cu < dense) wide_per_cu = fit > dense ? dense : fit;
    g_resident[g_resident_next] = {device, p.vec4, trial, variant_of(p), p.p2, (uint32_t)wanted, cus * per_cu, cus * wide_per_cu};
    g_resident_next = (g_resident_next + 1) % RESIDENT_SLOTS;          // when full, the oldest entry is replaced
    if (g_resident_used < RESIDENT_SLOTS) ++g_resident_used;
    return {(uint32_t)(cus * per_cu), (uint32_t)(cus * wide_per_cu)};
}

// An error that an earlier, unrelated HIP call of this thread left behind must not be blamed on this call.
void drop_stale_hip_error() { (void)hipGetLastError(); }

// The status of the launches made since drop_stale_hip_error.
int launches_ok(const char* what) {
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? DC_OK : device_error(e, what);
}

// ---- the enqueued sequence ---------------------------------------------------------------------
// timed: bracket the kernels with the events of the workspace's timing slot.  Takes no lock while it enqueues:
// calls with different workspaces may run on different threads and streams at the same time.
int enqueue(const dc::Plan& plan, const int32_t* lat, const int64_t* taus_dev, int64_t comm, int64_t* out_step_dev,
            int64_t* out_done_dev, unsigned char* ws, hipStream_t stream, bool timed) {
    dc::Plan p = plan;
    const Resident resident = resident_blocks(p);
    // Long rows stream narrow threshold grids best with two blocks per compute unit and grids that cover much of
    // the data with three (+25-30 % there, -4.5 % on narrow ones), so the kernel is launched once with either grid
    // and a sample taken by the prep kernel decides on the device which launch works; the other returns at once.
    const uint32_t planned = p.grid;                            // the workspace was sized for this many blocks
    p.grid_wide = planned < resident.wide_blocks ? planned : resident.wide_blocks;
    if (p.grid > resident.blocks) p.grid = resident.blocks;
    if (p.grid_wide < p.grid) p.grid_wide = p.grid;
    // Long runs of consecutive units per block stream best in the kernels with whole rows per load (+2-3.5 %), as
    // long as every block still gets several runs; the flat kernel, with its larger units, is 6-11 % faster when
    // every block jumps ahead by the whole grid after each round of four units.
    p.run = DC_SCAN_WAVES;
    if (p.vec4) {
        p.run = DC_UNIT_RUN;
        while (p.run > DC_SCAN_WAVES && (uint64_t)p.units < 4ull * p.run * p.grid) p.run >>= 1;
    }
    const uint32_t sample_rows = p.grid_wide > p.grid ? DC_SAMPLE_ROWS : 0u;
    uint32_t* status = reinterpret_cast<uint32_t*>(ws + p.off_status);
    int64_t* tau_sorted = reinterpret_cast<int64_t*>(ws + p.off_tau_sorted);
    uint32_t* tau_u32 = reinterpret_cast<uint32_t*>(ws + p.off_tau_u32);
    uint32_t* pos = reinterpret_cast<uint32_t*>(ws + p.off_pos);
    unsigned long long* hist_total = reinterpret_cast<unsigned long long*>(ws + p.off_bins);
    unsigned long long* trial_cnt = hist_total + p.p2;
    unsigned long long* trial_sum = trial_cnt + p.p2;
    uint32_t* unit_max = reinterpret_cast<uint32_t*>(ws + p.off_unit_max);
    uint32_t* hist_part = reinterpret_cast<uint32_t*>(ws + p.off_hist_part);

    const uint32_t chunks = (p.K + p.chunk - 1) / p.chunk;
    TimingSlot* slot = nullptr;
    if (timed) {
        int rc = DC_OK;
        slot = acquire_slot(ws, chunks, &rc);
        if (!slot) return rc;
        if (slot->whole) DC_HIP(hipEventRecord(slot->begin, stream));
    }
    drop_stale_hip_error();
    dc::launch_prep(taus_dev, p.K, tau_sorted, tau_u32, pos, status, hist_total, 3 * p.p2, lat,
                    (uint64_t)p.T * p.N, p.N, p.stride, p.M, sample_rows, p.span_rows ? unit_max : nullptr,
                    p.span_rows ? p.T : 0u, stream);
    for (uint32_t c = 0; c < chunks; ++c) {
        const uint32_t chunk0 = c * p.chunk;
        const uint32_t kc = p.K - chunk0 < p.chunk ? p.K - chunk0 : p.chunk;
        if (slot) DC_HIP(hipEventRecord(slot->scan[2 * c], stream));
        dc::launch_scan(p, lat, tau_u32 + chunk0, kc, unit_max, hist_part, status, stream);
        if (slot) DC_HIP(hipEventRecord(slot->scan[2 * c + 1], stream));
        dc::launch_reduce(p, hist_part, hist_total, unit_max, tau_u32 + chunk0, kc, trial_cnt, trial_sum, status, chunk0,
                          tau_sorted, pos, comm, out_step_dev, out_done_dev, stream);
    }
    if (slot) {
        if (slot->whole) DC_HIP(hipEventRecord(slot->end, stream));
        slot->valid = true;
    }
    return launches_ok("launch of the ranking, streaming or reduction kernel");
}

int compute_units() {
    int device = 0, cus = 0;
    if (hipGetDevice(&device) != hipSuccess) return 256;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || cus < 1) return 256;
    return cus;
}

int enqueue_speedup(const dc::Plan& plan, const int32_t* lat, const int64_t* taus_dev, int64_t comm,
                    const int64_t* comm_per_trial_dev, double* out_seff_dev, unsigned char* ws, hipStream_t stream,
                    bool timed) {
    dc::Plan p = plan;
    const Resident resident = resident_blocks(p, true);
    const uint32_t planned = p.grid;                            // the workspace was sized for this many blocks
    p.grid_wide = planned < resident.wide_blocks ? planned : resident.wide_blocks;   // two launch shapes, as in enqueue()
    if (p.grid > resident.blocks) p.grid = resident.blocks;
    if (p.grid_wide < p.grid) p.grid_wide = p.grid;
    const uint32_t sample_rows = p.grid_wide > p.grid ? DC_SAMPLE_ROWS : 0u;
    uint32_t* status = reinterpret_cast<uint32_t*>(ws + p.off_status);
    int64_t* tau_sorted = reinterpret_cast<int64_t*>(ws + p.off_tau_sorted);
    uint32_t* tau_u32 = reinterpret_cast<uint32_t*>(ws + p.off_tau_u32);
    uint32_t* pos = reinterpret_cast<uint32_t*>(ws + p.off_pos);
    double* partial = reinterpret_cast<double*>(ws + p.off_partial);
    const uint32_t chunks = (p.K + p.chunk - 1) / p.chunk;
    TimingSlot* slot = nullptr;
    if (timed) {
        int rc = DC_OK;
        slot = acquire_slot(ws, chunks, &rc);
        if (!slot) return rc;
        if (slot->whole) DC_HIP(hipEventRecord(slot->begin, stream));
    }
    drop_stale_hip_error();
    dc::launch_prep(taus_dev, p.K, tau_sorted, tau_u32, pos, status, nullptr, 0, lat, (uint64_t)p.T * p.N, p.N, p.stride,
                    p.M, sample_rows, nullptr, 0u, stream);
    for (uint32_t c = 0; c < chunks; ++c) {
        const uint32_t chunk0 = c * p.chunk;
        const uint32_t kc = p.K - chunk0 < p.chunk ? p.K - chunk0 : p.chunk;
        if (slot) DC_HIP(hipEventRecord(slot->scan[2 * c], stream));
        dc::launch_trial_scan(p, lat, tau_u32 + chunk0, kc, comm_per_trial_dev, comm, partial, status, stream);
        if (slot) DC_HIP(hipEventRecord(slot->scan[2 * c + 1], stream));
        dc::launch_speedup_finalize(p, partial, kc, chunk0, pos, status, tau_sorted, out_seff_dev, stream);
    }
    if (slot) {
        if (slot->whole) DC_HIP(hipEventRecord(slot->end, stream));
        slot->valid = true;
    }
    return launches_ok("launch of the ranking, per-iteration or finishing kernel");
}

int flags_to_status(uint32_t flags) {
    if (flags & (DC_FLAG_NEGATIVE_TAU | DC_FLAG_ZERO_STEP)) return DC_ERR_INVALID_ARG;
    if (flags & DC_FLAG_NEGATIVE_LATENCY) return DC_ERR_NEGATIVE_LATENCY;
    if (flags & DC_FLAG_RANGE) return DC_ERR_RANGE;
    return DC_OK;
}

bool sizes_ok(int64_t T, int64_t N, int64_t M, int64_t K, int64_t comm) {
    return T >= 1 && N >= 1 && M >= 1 && K >= 0 && K <= DC_MAX_THRESHOLDS && comm >= 0;
}

// cached allocation of the synchronous entry points
std::mutex g_cache_mutex;               // guards the cache and the staging buffer: the synchronous calls are serialised
unsigned char* g_cache = nullptr;
size_t g_cache_bytes = 0;
int g_cache_device = -1;
std::vector<unsigned char> g_staging;   // host side of the synchronous entry point's result copy

// Grow (never shrink) the cached device allocation of the synchronous entry points.  Caller holds g_cache_mutex.
int ensure_cache(size_t need) {
    int device = 0;
    DC_HIP(hipGetDevice(&device));
    if (device == g_cache_device && need <= g_cache_bytes) return DC_OK;
    if (g_cache) { (void)hipFree(g_cache); g_cache = nullptr; g_cache_bytes = 0; }
    void* mem = nullptr;
    hipError_t e = hipMalloc(&mem, need);
    if (e != hipSuccess) return device_error(e, "hipMalloc(workspace)", DC_ERR_NOMEM);
    g_cache = static_cast<unsigned char*>(mem);
    g_cache_bytes = need;
    g_cache_device = device;
    return DC_OK;
}

// ---- device memory for the entry point that allocates nothing ---------------------------------------
// One array per GPU, part of the loaded code object and held until the process ends.  In host code the
// array's name is only a handle for hipGetSymbolAddress; the address it returns (looked up once per device,
// with that device current) is what kernels and copies are given.
static __device__ __align__(256) unsigned char scratch[DC_STATIC_SCRATCH_BYTES];
constexpr int SCRATCH_DEVICES = 64;
unsigned char* g_scratch_ptr[SCRATCH_DEVICES] = {};
std::mutex g_scratch_mutex;             // guards g_scratch_ptr

int scratch_pointer(unsigned char** out) {
    int device = 0;
    DC_HIP(hipGetDevice(&device));
    if (device < 0 || device >= SCRATCH_DEVICES) return DC_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return device_error(e, "hipGetSymbolAddress(scratch)");
        if (!ptr || ((uintptr_t)ptr & 255u)) {
            snprintf(g_error_text, sizeof(g_error_text), "hipGetSymbolAddress(scratch): unusable address %p", ptr);
            return DC_ERR_DEVICE;
        }
        g_scratch_ptr[device] = static_cast<unsigned char*>(ptr);
    }
    *out = g_scratch_ptr[device];
    return DC_OK;
}

bool timing_on() { return g_timing_level.load() != 0; }

}  // namespace

extern "C" {

// The largest of the plans that a call with these sizes can end up with: a contiguous 16-byte aligned tensor, an aligned
// worker range of a larger tensor (trials further apart than they are long), and a tensor that is not 16-byte aligned.
size_t dc_workspace_bytes(int64_t T, int64_t N, int64_t M, int64_t K) {
    dc::Plan a{}, b{}, c{};
    if (!make_plan(T, N, M, K, true, &a)) return 0;
    if (!make_plan(T, N, M, K, false, &b)) return 0;
    size_t bytes = a.bytes > b.bytes ? a.bytes : b.bytes;
    if (make_plan(T, N, M, K, true, &c, N * M + 4) && c.bytes > bytes) bytes = c.bytes;
    return bytes;
}

int dc_simulate_strided_async(const int32_t* lat, int64_t T, int64_t N, int64_t M, int64_t trial_stride,
                              const int64_t* taus_dev, int64_t K, int64_t comm, int64_t* out_step_dev,
                              int64_t* out_done_dev, void* workspace_dev, size_t workspace_bytes, void* stream) {
    if (!sizes_ok(T, N, M, K, comm) || !lat || trial_stride < N * M) return DC_ERR_INVALID_ARG;
    if (K == 0) return DC_OK;
    if (!taus_dev || !out_step_dev || !out_done_dev || !workspace_dev) return DC_ERR_INVALID_ARG;
    if (((uintptr_t)lat & 3u) || ((uintptr_t)workspace_dev & 255u)) return DC_ERR_INVALID_ARG;
    dc::Plan p{};
    const bool aligned = ((uintptr_t)lat & 15u) == 0;
    if (!make_plan(T, N, M, K, aligned, &p, trial_stride)) return DC_ERR_INVALID_ARG;
    if (workspace_bytes < p.bytes) return DC_ERR_INVALID_ARG;
    return enqueue(p, lat, taus_dev, comm, out_step_dev, out_done_dev, static_cast<unsigned char*>(workspace_dev),
                   static_cast<hipStream_t>(stream), timing_on());
}

int dc_simulate_async(const int32_t* lat, int64_t T, int64_t N, int64_t M, const int64_t* taus_dev, int64_t K,
                      int64_t comm, int64_t* out_step_dev, int64_t* out_done_dev, void* workspace_dev,
                      size_t workspace_bytes, void* stream) {
    if (T < 1 || N < 1 || M < 1 || N >= ((int64_t)1 << 31) || M >= ((int64_t)1 << 31)) return DC_ERR_INVALID_ARG;
    return dc_simulate_strided_async(lat, T, N, M, N * M, taus_dev, K, comm, out_step_dev, out_done_dev, workspace_dev,
                                     workspace_bytes, stream);
}

int dc_simulate_static(const int32_t* lat, int64_t T, int64_t N, int64_t M, const int64_t* taus_dev, int64_t K,
                       int64_t comm, int64_t* out_step_dev, int64_t* out_done_dev, int32_t* out_status_dev,
                       void* stream) {
    if (!sizes_ok(T, N, M, K, comm) || !lat) return DC_ERR_INVALID_ARG;
    if (K == 0) return DC_OK;
    if (!taus_dev || !out_step_dev || !out_done_dev || ((uintptr_t)lat & 3u)) return DC_ERR_INVALID_ARG;
    dc::Plan p{};
    if (!make_plan(T, N, M, K, ((uintptr_t)lat & 15u) == 0, &p)) return DC_ERR_INVALID_ARG;
    if (p.bytes > (size_t)DC_STATIC_SCRATCH_BYTES) {
        snprintf(g_error_text, sizeof(g_error_text), "dc_simulate_static: these sizes need %zu bytes of scratch, the limit is %u",
                 p.bytes, (unsigned)DC_STATIC_SCRATCH_BYTES);
        return DC_ERR_INVALID_ARG;
    }
    unsigned char* ws = nullptr;
    int rc = scratch_pointer(&ws);
    if (rc) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    rc = enqueue(p, lat, taus_dev, comm, out_step_dev, out_done_dev, ws, s, false);
    if (rc) return rc;
    if (out_status_dev) {
        dc::launch_export_status(reinterpret_cast<const uint32_t*>(ws + p.off_status), out_status_dev, s);
        return launches_ok("launch of the status kernel");
    }
    return DC_OK;
}

int dc_workspace_status(const void* workspace_dev, void* stream) {
    if (!workspace_dev) return DC_ERR_INVALID_ARG;
    DC_HIP(hipStreamSynchronize(static_cast<hipStream_t>(stream)));
    uint32_t flags = 0;
    DC_HIP(hipMemcpy(&flags, workspace_dev, sizeof(flags), hipMemcpyDeviceToHost));
    return flags_to_status(flags);
}

int dc_simulate_strided(const int32_t* lat, int64_t T, int64_t N, int64_t M, int64_t trial_stride, const int64_t* taus,
                        int64_t K, int64_t comm, int64_t* out_step, int64_t* out_done) {
    if (!sizes_ok(T, N, M, K, comm) || !lat || trial_stride < N * M) return DC_ERR_INVALID_ARG;
    if (K == 0) return DC_OK;
    if (!taus || !out_step || !out_done || ((uintptr_t)lat & 3u)) return DC_ERR_INVALID_ARG;
    for (int64_t k = 0; k < K; ++k)
        if (taus[k] < 0) return DC_ERR_INVALID_ARG;
    dc::Plan p{};
    const bool aligned = ((uintptr_t)lat & 15u) == 0;
    if (!make_plan(T, N, M, K, aligned, &p, trial_stride)) return DC_ERR_INVALID_ARG;

    std::lock_guard<std::mutex> lock(g_cache_mutex);
    // cached allocation: thresholds | step | done | workspace (whose first word is the status): the two result
    // arrays are adjacent, so one copy brings both back
    const size_t io_bytes = align256((size_t)K * 8);
    {
        int rc = ensure_cache(3 * io_bytes + p.bytes);
        if (rc) return rc;
    }
    int64_t* taus_dev = reinterpret_cast<int64_t*>(g_cache);
    int64_t* step_dev = reinterpret_cast<int64_t*>(g_cache + io_bytes);
    int64_t* done_dev = reinterpret_cast<int64_t*>(g_cache + 2 * io_bytes);
    unsigned char* ws = g_cache + 3 * io_bytes;

    hipStream_t stream = nullptr;
    DC_HIP(hipMemcpy(taus_dev, taus, (size_t)K * 8, hipMemcpyHostToDevice));
    int rc = enqueue(p, lat, taus_dev, comm, step_dev, done_dev, ws, stream, timing_on());
    if (rc) return rc;
    // results and status word in one device-to-host copy (it also waits for the kernels)
    g_staging.resize(2 * io_bytes + 256);
    DC_HIP(hipMemcpy(g_staging.data(), step_dev, 2 * io_bytes + 256, hipMemcpyDeviceToHost));
    uint32_t flags = 0;
    memcpy(&flags, g_staging.data() + 2 * io_bytes + p.off_status, sizeof(flags));
    rc = flags_to_status(flags);
    if (rc) return rc;
    memcpy(out_step, g_staging.data(), (size_t)K * 8);
    memcpy(out_done, g_staging.data() + io_bytes, (size_t)K * 8);
    return DC_OK;
}

int dc_simulate(const int32_t* lat, int64_t T, int64_t N, int64_t M, const int64_t* taus, int64_t K, int64_t comm,
                int64_t* out_step, int64_t* out_done) {
    if (T < 1 || N < 1 || M < 1 || N >= ((int64_t)1 << 31) || M >= ((int64_t)1 << 31)) return DC_ERR_INVALID_ARG;
    return dc_simulate_strided(lat, T, N, M, N * M, taus, K, comm, out_step, out_done);
}

size_t dc_speedup_workspace_bytes(int64_t T, int64_t N, int64_t M, int64_t K) {
    dc::Plan p{};
    return make_trial_plan(T, N, M, K, true, &p) ? p.bytes : 0;
}

int dc_speedup_per_step_async(const int32_t* lat, int64_t T, int64_t N, int64_t M, const int64_t* taus_dev, int64_t K,
                              int64_t comm, const int64_t* comm_per_trial_dev, double* out_seff_dev,
                              void* workspace_dev, size_t workspace_bytes, void* stream) {
    if (!sizes_ok(T, N, M, K, comm) || !lat) return DC_ERR_INVALID_ARG;
    if (K == 0) return DC_OK;
    if (!taus_dev || !out_seff_dev || !workspace_dev) return DC_ERR_INVALID_ARG;
    if (((uintptr_t)lat & 3u) || ((uintptr_t)workspace_dev & 255u)) return DC_ERR_INVALID_ARG;
    dc::Plan p{};
    if (!make_trial_plan(T, N, M, K, ((uintptr_t)lat & 15u) == 0, &p)) return DC_ERR_INVALID_ARG;
    if (workspace_bytes < p.bytes) return DC_ERR_INVALID_ARG;
    return enqueue_speedup(p, lat, taus_dev, comm, comm_per_trial_dev, out_seff_dev,
                           static_cast<unsigned char*>(workspace_dev), static_cast<hipStream_t>(stream), timing_on());
}

int dc_speedup_per_step(const int32_t* lat, int64_t T, int64_t N, int64_t M, const int64_t* taus, int64_t K,
                        int64_t comm, const int64_t* comm_per_trial, double* out_seff) {
    if (!sizes_ok(T, N, M, K, comm) || !lat) return DC_ERR_INVALID_ARG;
    if (K == 0) return DC_OK;
    if (!taus || !out_seff || ((uintptr_t)lat & 3u)) return DC_ERR_INVALID_ARG;
    for (int64_t k = 0; k < K; ++k)
        if (taus[k] < 0) return DC_ERR_INVALID_ARG;
    if (comm_per_trial)
        for (int64_t t = 0; t < T; ++t)
            if (comm_per_trial[t] < 0) return DC_ERR_INVALID_ARG;
    dc::Plan p{};
    if (!make_trial_plan(T, N, M, K, ((uintptr_t)lat & 15u) == 0, &p)) return DC_ERR_INVALID_ARG;

    std::lock_guard<std::mutex> lock(g_cache_mutex);
    const size_t tau_bytes = align256((size_t)K * 8), comm_bytes = comm_per_trial ? align256((size_t)T * 8) : 0;
    int rc = ensure_cache(2 * tau_bytes + comm_bytes + p.bytes);
    if (rc) return rc;
    int64_t* taus_dev = reinterpret_cast<int64_t*>(g_cache);
    double* seff_dev = reinterpret_cast<double*>(g_cache + tau_bytes);
    int64_t* comm_dev = comm_per_trial ? reinterpret_cast<int64_t*>(g_cache + 2 * tau_bytes) : nullptr;
    unsigned char* ws = g_cache + 2 * tau_bytes + comm_bytes;
    hipStream_t stream = nullptr;
    DC_HIP(hipMemcpy(taus_dev, taus, (size_t)K * 8, hipMemcpyHostToDevice));
    if (comm_dev) DC_HIP(hipMemcpy(comm_dev, comm_per_trial, (size_t)T * 8, hipMemcpyHostToDevice));
    rc = enqueue_speedup(p, lat, taus_dev, comm, comm_dev, seff_dev, ws, stream, timing_on());
    if (rc) return rc;
    DC_HIP(hipStreamSynchronize(stream));
    uint32_t flags = 0;
    DC_HIP(hipMemcpy(&flags, ws + p.off_status, sizeof(flags), hipMemcpyDeviceToHost));
    rc = flags_to_status(flags);
    if (rc) return rc;
    DC_HIP(hipMemcpy(out_seff, seff_dev, (size_t)K * 8, hipMemcpyDeviceToHost));
    return DC_OK;
}

int dc_moments(const int32_t* lat, int64_t T, int64_t N, int64_t M, int64_t* out_sum, uint64_t* out_sumsq,
               double* out_mean, double* out_variance) {
    if (!lat || T < 1 || N < 1 || M < 1 || ((uintptr_t)lat & 3u)) return DC_ERR_INVALID_ARG;
    if ((long double)T * (long double)N * (long double)M >= 4.6e18L) return DC_ERR_INVALID_ARG;
    const uint64_t n = (uint64_t)T * (uint64_t)N * (uint64_t)M;
    std::lock_guard<std::mutex> lock(g_cache_mutex);
    const uint32_t grid = (uint32_t)compute_units() * 2u;        // 8 waves per compute unit saturate a plain read
    const size_t partial_bytes = align256((size_t)grid * 4 * 8);
    int rc = ensure_cache(256 + 256 + partial_bytes);
    if (rc) return rc;
    uint32_t* status = reinterpret_cast<uint32_t*>(g_cache);
    unsigned long long* result = reinterpret_cast<unsigned long long*>(g_cache + 256);
    unsigned long long* partial = reinterpret_cast<unsigned long long*>(g_cache + 512);
    hipStream_t stream = nullptr;
    TimingSlot* slot = nullptr;
    if (timing_on()) {
        slot = acquire_slot(g_cache, 1, &rc);
        if (!slot) return rc;
        if (slot->whole) DC_HIP(hipEventRecord(slot->begin, stream));
        DC_HIP(hipEventRecord(slot->scan[0], stream));
    }
    drop_stale_hip_error();
    dc::launch_moments(lat, n, grid, partial, result, status, stream);
    if (slot) {
        DC_HIP(hipEventRecord(slot->scan[1], stream));
        if (slot->whole) DC_HIP(hipEventRecord(slot->end, stream));
        slot->valid = true;
    }
    rc = launches_ok("launch of the moments kernels");
    if (rc) return rc;
    unsigned long long host[4] = {0, 0, 0, 0};
    DC_HIP(hipMemcpy(host, result, sizeof(host), hipMemcpyDeviceToHost));
    if (host[3] & 0x80000000ull) return DC_ERR_NEGATIVE_LATENCY;
    // The sum is kept in 64 bits.  host[3] is the OR of all latencies, hence at least the largest one: when
    // n * host[3] stays below 2^63 the sum cannot have wrapped; otherwise that cannot be told and the call refuses.
    if ((unsigned __int128)n * (unsigned __int128)host[3] >= ((unsigned __int128)1 << 63)) return DC_ERR_RANGE;
    if (out_sum) *out_sum = (int64_t)host[0];
    if (out_sumsq) { out_sumsq[0] = host[1]; out_sumsq[1] = host[2]; }
    const unsigned __int128 sq = ((unsigned __int128)host[2] << 64) | host[1];
    if (out_mean) *out_mean = (double)host[0] / (double)n;
    if (out_variance) {
        // (sumsq*n - sum^2) / n^2 with the numerator exact in 128 bits when it fits, else in long double
        const long double nl = (long double)n;
        if (sq <= ((unsigned __int128)1 << 126) / n) {
            const unsigned __int128 num = sq * n - (unsigned __int128)host[0] * host[0];
            *out_variance = (double)((long double)num / (nl * nl));
        } else {
            const long double m = (long double)host[0] / nl;
            *out_variance = (double)((long double)sq / nl - m * m);
        }
    }
    return DC_OK;
}

int dc_worker_moments_strided(const int32_t* lat, int64_t T, int64_t N, int64_t M, int64_t trial_stride,
                              int64_t* out_sum, uint64_t* out_sumsq, double* out_mean, double* out_variance) {
    if (!lat || ((uintptr_t)lat & 3u) || N < 1 || M < 1 || trial_stride < N * M) return DC_ERR_INVALID_ARG;
    {
        dc::Plan whole{};
        if (!make_trial_plan(T, N, M, 1, false, &whole, trial_stride)) return DC_ERR_INVALID_ARG;
    }
    std::lock_guard<std::mutex> lock(g_cache_mutex);
    const long double tl = (long double)T;
    hipStream_t stream = nullptr;
    bool first_pass = true;
    // The accumulators of all workers of a pass live in LDS, so more than DC_MAX_STAT_WORKERS workers are taken in
    // several passes over lat, each over a range of workers of every trial (a pass reads only its workers' rows).
    for (int64_t n0 = 0; n0 < N; n0 += (int64_t)DC_MAX_STAT_WORKERS) {
        const int64_t nc = N - n0 < (int64_t)DC_MAX_STAT_WORKERS ? N - n0 : (int64_t)DC_MAX_STAT_WORKERS;
        const int32_t* base = lat + n0 * M;
        dc::Plan p{};
        if (!make_trial_plan(T, nc, M, 1, ((uintptr_t)base & 15u) == 0, &p, trial_stride)) return DC_ERR_INVALID_ARG;
        const uint32_t want = (uint32_t)compute_units() * 2u;             // 2 x 60 KiB of LDS always fit
        if (p.grid > want) p.grid = want;
        const size_t row_bytes = (size_t)nc * 3 * 8;
        int rc = ensure_cache(256 + align256(row_bytes) + align256((size_t)p.grid * row_bytes));
        if (rc) return rc;
        uint32_t* status = reinterpret_cast<uint32_t*>(g_cache);
        unsigned long long* result = reinterpret_cast<unsigned long long*>(g_cache + 256);
        unsigned long long* partial = reinterpret_cast<unsigned long long*>(g_cache + 256 + align256(row_bytes));
        TimingSlot* slot = nullptr;
        if (timing_on() && first_pass) {                                   // the first pass is the one that is timed
            slot = acquire_slot(g_cache, 1, &rc);
            if (!slot) return rc;
            if (slot->whole) DC_HIP(hipEventRecord(slot->begin, stream));
        }
        first_pass = false;
        drop_stale_hip_error();
        dc::launch_worker_totals(p, base, partial, result, status, stream, slot ? slot->scan[0] : nullptr,
                                 slot ? slot->scan[1] : nullptr);
        if (slot) {
            if (slot->whole) DC_HIP(hipEventRecord(slot->end, stream));
            slot->valid = true;
        }
        rc = launches_ok("launch of the per-worker kernels");
        if (rc) return rc;
        uint32_t flags = 0;
        DC_HIP(hipMemcpy(&flags, status, sizeof(flags), hipMemcpyDeviceToHost));
        rc = flags_to_status(flags);
        if (rc) return rc;
        std::vector<unsigned long long> host((size_t)nc * 3);
        DC_HIP(hipMemcpy(host.data(), result, row_bytes, hipMemcpyDeviceToHost));
        for (int64_t i = 0; i < nc; ++i) {
            const int64_t n = n0 + i;
            const unsigned long long sum = host[i], lo = host[nc + i], hi = host[2 * nc + i];
            if (out_sum) out_sum[n] = (int64_t)sum;
            if (out_sumsq) { out_sumsq[2 * n] = lo; out_sumsq[2 * n + 1] = hi; }
            if (out_mean) out_mean[n] = (double)((long double)sum / tl);
            if (out_variance) {
                // (sumsq*T - sum^2) / T^2: sumsq < 2^93 and T < 2^31, so the numerator is exact in 128 bits
                const unsigned __int128 sq = ((unsigned __int128)hi << 64) | lo;
                const unsigned __int128 num = sq * (unsigned __int128)T - (unsigned __int128)sum * sum;
                out_variance[n] = (double)((long double)num / (tl * tl));
            }
        }
    }
    return DC_OK;
}

int dc_worker_moments(const int32_t* lat, int64_t T, int64_t N, int64_t M, int64_t* out_sum, uint64_t* out_sumsq,
                      double* out_mean, double* out_variance) {
    if (N < 1 || M < 1 || N >= ((int64_t)1 << 31) || M >= ((int64_t)1 << 31)) return DC_ERR_INVALID_ARG;
    return dc_worker_moments_strided(lat, T, N, M, N * M, out_sum, out_sumsq, out_mean, out_variance);
}

namespace {

// Standard normal quantile: a textbook starting value (rational approximation in t = sqrt(-2 ln q)),
// then Newton steps on the upper tail 0.5*erfc(x/sqrt 2) = q, which converge to double precision.
double normal_quantile(double p) {
    if (!(p > 0.0 && p < 1.0)) return p <= 0.0 ? -INFINITY : INFINITY;
    const bool upper = p > 0.5;
    const double q = upper ? 1.0 - p : p;                    // tail mass, <= 0.5
    if (q == 0.5) return 0.0;
    const double t = std::sqrt(-2.0 * std::log(q));
    double x = t - (2.30753 + 0.27061 * t) / (1.0 + 0.99229 * t + 0.04481 * t * t);
    for (int it = 0; it < 8; ++it) {
        const double tail = 0.5 * std::erfc(x * 0.70710678118654752440);
        const double pdf = 0.39894228040143267794 * std::exp(-0.5 * x * x);
        const double step = (tail - q) / pdf;               // d(tail)/dx = -pdf
        x += step;
        if (std::fabs(step) <= 1e-16 * std::fabs(x)) break;
    }
    return upper ? x : -x;
}

}  // namespace

int dc_analytic_curves(double mu, double sigma2, int64_t N, int64_t M, const int64_t* taus, int64_t K, int64_t comm,
                       double mean_tmax, double* out_edone, double* out_seff, double* out_et, int64_t* out_best_k) {
    if (!(mu >= 0.0) || !(sigma2 >= 0.0) || !std::isfinite(mu) || !std::isfinite(sigma2)) return DC_ERR_INVALID_ARG;
    if (N < 2 || M < 1 || M >= ((int64_t)1 << 31) || K < 0 || K > DC_MAX_THRESHOLDS || comm < 0) return DC_ERR_INVALID_ARG;
    const double gamma = 0.57721566490153286061;
    const double z = (1.0 - gamma) * normal_quantile(1.0 - 1.0 / (double)N) +
                     gamma * normal_quantile(1.0 - 1.0 / (std::exp(1.0) * (double)N));
    const double et_model = std::sqrt((double)M * sigma2) * z + (double)M * mu;
    if (out_et) *out_et = et_model;
    if (K == 0) return DC_OK;
    if (!taus || !out_edone) return DC_ERR_INVALID_ARG;
    for (int64_t k = 0; k < K; ++k)
        if (taus[k] < 0) return DC_ERR_INVALID_ARG;

    std::lock_guard<std::mutex> lock(g_cache_mutex);
    const size_t io = align256((size_t)K * 8);
    int rc = ensure_cache(2 * io);
    if (rc) return rc;
    int64_t* taus_dev = reinterpret_cast<int64_t*>(g_cache);
    double* edone_dev = reinterpret_cast<double*>(g_cache + io);
    hipStream_t stream = nullptr;
    DC_HIP(hipMemcpy(taus_dev, taus, (size_t)K * 8, hipMemcpyHostToDevice));
    drop_stale_hip_error();
    dc::launch_expected_done(taus_dev, (uint32_t)K, (uint32_t)M, mu, sigma2, edone_dev, stream);
    rc = launches_ok("launch of the expected-completions kernel");
    if (rc) return rc;
    DC_HIP(hipMemcpy(out_edone, edone_dev, (size_t)K * 8, hipMemcpyDeviceToHost));

    const double et = mean_tmax >= 0.0 ? mean_tmax : et_model;
    int64_t best = 0;
    double best_score = -1.0;
    for (int64_t k = 0; k < K; ++k) {
        const double tau = (double)taus[k];
        if (out_seff) out_seff[k] = out_edone[k] / (double)M * (et + (double)comm) / ((tau < et ? tau : et) + (double)comm);
        const double score = out_edone[k] / (tau + (double)comm);     // Appendix C.2, "Finding tau*"
        if (k == 0 || score > best_score || (score == best_score && taus[k] > taus[best])) { best = k; best_score = score; }
    }
    if (out_best_k) *out_best_k = best;
    return DC_OK;
}

int dc_select_tau(const int64_t* step_sum, const int64_t* done_sum, const int64_t* taus, int64_t K, int64_t T,
                  int64_t N, int64_t M, int64_t base_step_sum, double* out_thr, double* out_seff,
                  int64_t* out_best_k) {
    if (!step_sum || !done_sum || !taus || !out_best_k || K < 1 || T < 1 || N < 1 || M < 1 || base_step_sum < 0)
        return DC_ERR_INVALID_ARG;
    for (int64_t k = 0; k < K; ++k)
        if (step_sum[k] <= 0 || done_sum[k] < 0) return DC_ERR_INVALID_ARG;
    const double full = (double)T * (double)N * (double)M;
    int64_t best = 0;
    for (int64_t k = 0; k < K; ++k) {
        const double thr = (double)done_sum[k] / (double)step_sum[k];
        if (out_thr) out_thr[k] = thr;
        if (out_seff) out_seff[k] = base_step_sum > 0 ? thr * (double)base_step_sum / full : NAN;
        if (k == 0) continue;
        // done[k]/step[k] > done[best]/step[best]  <=>  done[k]*step[best] > done[best]*step[k]
        const unsigned __int128 lhs = (unsigned __int128)(uint64_t)done_sum[k] * (uint64_t)step_sum[best];
        const unsigned __int128 rhs = (unsigned __int128)(uint64_t)done_sum[best] * (uint64_t)step_sum[k];
        if (lhs > rhs || (lhs == rhs && taus[k] > taus[best])) best = k;
    }
    *out_best_k = best;
    return DC_OK;
}

int dc_select_tau_per_step(const double* seff, const int64_t* taus, int64_t K, int64_t* out_best_k) {
    if (!seff || !taus || !out_best_k || K < 1) return DC_ERR_INVALID_ARG;
    for (int64_t k = 0; k < K; ++k)
        if (std::isnan(seff[k]) || taus[k] < 0) return DC_ERR_INVALID_ARG;
    int64_t best = 0;
    for (int64_t k = 1; k < K; ++k)
        if (seff[k] > seff[best] || (seff[k] == seff[best] && taus[k] > taus[best])) best = k;
    *out_best_k = best;
    return DC_OK;
}

int dc_set_kernel_timing(int enable) {
    g_timing_level.store(enable <= 0 ? 0 : (enable >= 2 ? 2 : 1));
    t_last_slot = nullptr;
    return DC_OK;
}

int dc_last_kernel_ms(float* scan_ms, float* total_ms) {
    if (!timing_on()) return DC_ERR_INVALID_ARG;
    return slot_times(t_last_slot, scan_ms, total_ms);
}

int dc_workspace_kernel_ms(const void* workspace_dev, float* scan_ms, float* total_ms) {
    if (!workspace_dev || !timing_on()) return DC_ERR_INVALID_ARG;
    TimingSlot* slot = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_timing_mutex);
        int device = 0;
        (void)hipGetDevice(&device);
        for (TimingSlot& s : g_slots)
            if (s.key == workspace_dev && s.device == device) slot = &s;
    }
    return slot_times(slot, scan_ms, total_ms);
}

const char* dc_status_string(int status) {
    switch (status) {
        case DC_OK: return "ok";
        case DC_ERR_INVALID_ARG: return "invalid argument";
        case DC_ERR_NEGATIVE_LATENCY: return "negative latency";
        case DC_ERR_RANGE: return "latency too large for 31-bit worker totals";
        case DC_ERR_DEVICE: return "HIP error";
        case DC_ERR_NOMEM: return "out of memory";
        default: return "unknown status";
    }
}

const char* dc_last_device_error(void) { return g_error_text; }

int dc_device_info(int32_t* compute_units, int32_t* memory_clock_khz, int32_t* memory_bus_bits, int32_t* l2_bytes) {
    int device = 0, v = 0;
    DC_HIP(hipGetDevice(&device));
    if (compute_units) { DC_HIP(hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, device)); *compute_units = v; }
    if (memory_clock_khz) { DC_HIP(hipDeviceGetAttribute(&v, hipDeviceAttributeMemoryClockRate, device)); *memory_clock_khz = v; }
    if (memory_bus_bits) { DC_HIP(hipDeviceGetAttribute(&v, hipDeviceAttributeMemoryBusWidth, device)); *memory_bus_bits = v; }
    if (l2_bytes) { DC_HIP(hipDeviceGetAttribute(&v, hipDeviceAttributeL2CacheSize, device)); *l2_bytes = v; }
    return DC_OK;
}

void dc_shutdown(void) {
    {
        std::lock_guard<std::mutex> lock(g_cache_mutex);
        if (g_cache) { (void)hipFree(g_cache); g_cache = nullptr; g_cache_bytes = 0; g_cache_device = -1; }
    }
    std::lock_guard<std::mutex> lock(g_timing_mutex);
    for (TimingSlot& s : g_slots) {
        if (s.begin) { (void)hipEventDestroy(s.begin); s.begin = nullptr; }
        if (s.end) { (void)hipEventDestroy(s.end); s.end = nullptr; }
        for (hipEvent_t e : s.scan) (void)hipEventDestroy(e);
        s.scan.clear();
        s.key = nullptr;
        s.valid = false;
        s.stamp = 0;
    }
    t_last_slot = nullptr;
}

}  // extern "C"
