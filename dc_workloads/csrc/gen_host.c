/* CPU implementation of the synthetic latency generator defined in dc_workloads/spec.py.
 * Integer arithmetic only; must produce exactly the integers of the NumPy reference
 * (dc_workloads/host.py) and of the device generator (gen_device.hip).
 * Input preparation only: nothing of the simulated method is computed here. */
#include <stdint.h>
#include <stddef.h>

#define DCGEN_GOLDEN 0x9E3779B97F4A7C15ull

static inline uint64_t mix64(uint64_t z) {
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

static inline uint64_t draw_q8(uint64_t h, const int64_t* main_t, const int64_t* lo_t, const int64_t* hi_t) {
    uint32_t cell = (uint32_t)(h >> 48);
    uint64_t f = (h >> 16) & 0xFFFFFFFFull;
    if (cell >= 16u && cell < 65520u) {
        uint64_t a = (uint64_t)main_t[cell], b = (uint64_t)main_t[cell + 1];
        return a + (((b - a) * f) >> 32);
    }
    const int64_t* tab = cell < 16u ? lo_t : hi_t;
    uint32_t c = cell < 16u ? cell : cell - 65520u;
    uint32_t j = c * 256u + (uint32_t)(f >> 24);
    uint64_t g = f & 0xFFFFFFull;
    uint64_t a = (uint64_t)tab[j], b = (uint64_t)tab[j + 1];
    return a + (((b - a) * g) >> 24);
}

/* Fill out[0..count) with elements idx0..idx0+count of the workload. */
void dcgen_fill_host(int32_t* out, uint64_t idx0, uint64_t count,
                     uint64_t key_value, uint64_t key_spike,
                     int64_t N, int64_t M,
                     const int64_t* main_t, const int64_t* lo_t, const int64_t* hi_t,
                     const uint32_t* scale_q16, const int64_t* worker_add,
                     int64_t add, int64_t clip_min,
                     uint32_t spike_thresh, uint32_t spike_mul, int64_t spike_add, int64_t spike_workers) {
    for (uint64_t e = 0; e < count; ++e) {
        uint64_t i = idx0 + e;
        uint64_t q = draw_q8(mix64(key_value + DCGEN_GOLDEN * (i + 1)), main_t, lo_t, hi_t);
        uint64_t s = 65536u;
        const uint64_t worker = (i / (uint64_t)M) % (uint64_t)N;
        if (scale_q16) s = scale_q16[worker];
        int spike = 0;
        if (spike_thresh && (spike_workers <= 0 || worker < (uint64_t)spike_workers))
            spike = (uint32_t)(mix64(key_spike + DCGEN_GOLDEN * (i + 1)) >> 32) < spike_thresh;
        uint64_t mul = spike ? spike_mul : 1u;
        int64_t v = (int64_t)((q * s * mul + (1ull << 23)) >> 24);
        if (worker_add) v += worker_add[worker];
        if (v < clip_min) v = clip_min;
        v += add + (spike ? spike_add : 0);
        out[e] = (int32_t)v;
    }
}

/* q8 draws for a list of counters (used for the per-worker slowdown table). */
void dcgen_draw_host(uint64_t* out_q8, const uint64_t* counters, uint64_t count, uint64_t key,
                     const int64_t* main_t, const int64_t* lo_t, const int64_t* hi_t) {
    for (uint64_t e = 0; e < count; ++e)
        out_q8[e] = draw_q8(mix64(key + DCGEN_GOLDEN * (counters[e] + 1)), main_t, lo_t, hi_t);
}
