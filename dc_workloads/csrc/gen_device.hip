// GPU implementation of the synthetic latency generator defined in dc_workloads/spec.py.
// Integer arithmetic only: it must write exactly the integers of the CPU implementations
// (gen_host.c and the NumPy reference).  Input preparation only; it is not part of the
// simulator library and shares no code with it.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

constexpr uint64_t GOLDEN = 0x9E3779B97F4A7C15ull;

__device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

__device__ __forceinline__ uint64_t draw_q8(uint64_t h, const int64_t* __restrict__ main_t,
                                            const int64_t* __restrict__ lo_t, const int64_t* __restrict__ hi_t) {
    const uint32_t cell = (uint32_t)(h >> 48);
    const uint64_t f = (h >> 16) & 0xFFFFFFFFull;
    if (cell >= 16u && cell < 65520u) {
        const uint64_t a = (uint64_t)main_t[cell], b = (uint64_t)main_t[cell + 1];
        return a + (((b - a) * f) >> 32);
    }
    const int64_t* tab = cell < 16u ? lo_t : hi_t;
    const uint32_t c = cell < 16u ? cell : cell - 65520u;
    const uint32_t j = c * 256u + (uint32_t)(f >> 24);
    const uint64_t g = f & 0xFFFFFFull;
    const uint64_t a = (uint64_t)tab[j], b = (uint64_t)tab[j + 1];
    return a + (((b - a) * g) >> 24);
}

__global__ __launch_bounds__(256)
void dcgen_fill_kernel(int32_t* __restrict__ out, uint64_t idx0, uint64_t count, uint64_t key_value,
                       uint64_t key_spike, uint64_t N, uint64_t M, const int64_t* __restrict__ main_t,
                       const int64_t* __restrict__ lo_t, const int64_t* __restrict__ hi_t,
                       const uint32_t* __restrict__ scale_q16, const int64_t* __restrict__ worker_add, int64_t add,
                       int64_t clip_min,
                       uint32_t spike_thresh, uint32_t spike_mul, int64_t spike_add, int64_t spike_workers) {
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t e = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; e < count; e += stride) {
        const uint64_t i = idx0 + e;
        const uint64_t q = draw_q8(mix64(key_value + GOLDEN * (i + 1)), main_t, lo_t, hi_t);
        uint64_t s = 65536u;
        const uint64_t worker = (i / M) % N;
        if (scale_q16) s = scale_q16[worker];
        bool spike = false;
        if (spike_thresh && (spike_workers <= 0 || worker < (uint64_t)spike_workers))
            spike = (uint32_t)(mix64(key_spike + GOLDEN * (i + 1)) >> 32) < spike_thresh;
        const uint64_t mul = spike ? spike_mul : 1u;
        int64_t v = (int64_t)((q * s * mul + (1ull << 23)) >> 24);
        if (worker_add) v += worker_add[worker];
        if (v < clip_min) v = clip_min;
        v += add + (spike ? spike_add : 0);
        out[e] = (int32_t)v;
    }
}

}  // namespace

// out, tables, scale_q16 and worker_add are DEVICE pointers; scale_q16 and worker_add may be NULL.  Enqueues on `stream`
// (hipStream_t as void*) and returns the hipError_t of the launch.
extern "C" int dcgen_fill_device(int32_t* out, uint64_t idx0, uint64_t count, uint64_t key_value, uint64_t key_spike,
                                 int64_t N, int64_t M, const int64_t* main_t, const int64_t* lo_t,
                                 const int64_t* hi_t, const uint32_t* scale_q16, const int64_t* worker_add, int64_t add,
                                 int64_t clip_min,
                                 uint32_t spike_thresh, uint32_t spike_mul, int64_t spike_add, int64_t spike_workers,
                                 void* stream) {
    if (count == 0) return 0;
    uint64_t blocks = (count + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(dcgen_fill_kernel, dim3((uint32_t)blocks), dim3(256), 0, static_cast<hipStream_t>(stream), out,
                       idx0, count, key_value, key_spike, (uint64_t)N, (uint64_t)M, main_t, lo_t, hi_t, scale_q16, worker_add, add,
                       clip_min, spike_thresh, spike_mul, spike_add, spike_workers);
    return (int)hipGetLastError();
}
