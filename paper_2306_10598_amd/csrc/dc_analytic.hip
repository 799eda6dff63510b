// Kernels behind the analytical side of the library (Sections 4.2-4.4, Appendix C.2):
//   dc_moments_kernel / dc_moments_final_kernel   exact sum and sum of squares of all latencies (one pass over lat)
//   dc_expected_done_kernel                       sum_{m=1..M} Phi((tau - m mu)/sqrt(m sigma^2)) for every threshold
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dc_internal.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned __int128 u128;

struct Acc {
    unsigned long long sum;
    u128 sq;
    uint32_t bits;      // OR of all values: bit 31 set <=> some latency was negative
};

__device__ __forceinline__ void take(Acc& a, uint32_t x) {
    a.sum += x;
    a.sq += (unsigned long long)x * x;
    a.bits |= x;
}

// Block-wide sums by a fixed tree in LDS; thread 0 ends up with the totals.
__device__ __forceinline__ void block_reduce(Acc& a, unsigned long long (*lds)[3], uint32_t* lds_bits) {
    const uint32_t tid = threadIdx.x;
    lds[tid][0] = a.sum;
    lds[tid][1] = (unsigned long long)a.sq;
    lds[tid][2] = (unsigned long long)(a.sq >> 64);
    lds_bits[tid] = a.bits;
    __syncthreads();
    for (uint32_t d = blockDim.x >> 1; d >= 1; d >>= 1) {
        if (tid < d) {
            lds[tid][0] += lds[tid + d][0];
            const u128 mine = ((u128)lds[tid][2] << 64) | lds[tid][1];
            const u128 other = ((u128)lds[tid + d][2] << 64) | lds[tid + d][1];
            const u128 both = mine + other;
            lds[tid][1] = (unsigned long long)both;
            lds[tid][2] = (unsigned long long)(both >> 64);
            lds_bits[tid] |= lds_bits[tid + d];
        }
        __syncthreads();
    }
    a.sum = lds[0][0];
    a.sq = ((u128)lds[0][2] << 64) | lds[0][1];
    a.bits = lds_bits[0];
}

}  // namespace

// partial[block] = {sum, squares low word, squares high word, OR of values}.  `vec_units` units of 32 KiB
// (16-byte loads, a wave per unit) cover the elements [head, head + vec_units*8192), where head (0..3) is the
// number of elements before the first 16-byte boundary; the elements before and after, [0, head) and
// [scalar_from, n), are read one by one.  The units are dealt as in the threshold pass: a block takes runs of
// `run` consecutive units (a multiple of 4) and its four waves walk a run four adjacent units at a time, in step.
__global__ __launch_bounds__(256)
void dc_moments_kernel(const int32_t* __restrict__ lat, unsigned long long n, uint32_t head, uint32_t vec_units, uint32_t run,
                       unsigned long long scalar_from, unsigned long long* __restrict__ partial) {
    __shared__ unsigned long long lds[256][3];
    __shared__ uint32_t lds_bits[256];
    Acc a{0ull, 0, 0u};
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t runs = (vec_units + run - 1u) / run;
    const uint32_t padded = (runs + gridDim.x - 1u) / gridDim.x * gridDim.x;     // block-uniform loop bounds
    for (uint32_t r = blockIdx.x; r < padded; r += gridDim.x)
    for (uint32_t round = 0; round < run / 4u; ++round) {
        const uint32_t u = r < runs ? r * run + round * 4u + wave : vec_units;
        if (u < vec_units) {
            const u32x4* base = reinterpret_cast<const u32x4*>(lat + head) + (uint64_t)u * 2048 + lane;
            for (uint32_t i = 0; i < 32; i += 8) {
                u32x4 x[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) x[k] = __builtin_nontemporal_load(base + (uint64_t)(i + k) * 64);
#pragma unroll
                for (int k = 0; k < 8; ++k) { take(a, x[k].x); take(a, x[k].y); take(a, x[k].z); take(a, x[k].w); }
            }
        }
        __syncthreads();
    }
    const unsigned long long stride = (unsigned long long)gridDim.x * blockDim.x;
    for (unsigned long long i = scalar_from + (unsigned long long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
        take(a, (uint32_t)lat[i]);
    if (blockIdx.x == 0 && threadIdx.x < head && threadIdx.x < n) take(a, (uint32_t)lat[threadIdx.x]);
    block_reduce(a, lds, lds_bits);
    if (threadIdx.x == 0) {
        unsigned long long* out = partial + (uint64_t)blockIdx.x * 4;
        out[0] = a.sum;
        out[1] = (unsigned long long)a.sq;
        out[2] = (unsigned long long)(a.sq >> 64);
        out[3] = a.bits;
    }
}

// result = {sum, squares low, squares high, flags} over all blocks; sets the negative-latency flag.
__global__ __launch_bounds__(256)
void dc_moments_final_kernel(const unsigned long long* __restrict__ partial, uint32_t blocks,
                             unsigned long long* __restrict__ result, uint32_t* __restrict__ status) {
    __shared__ unsigned long long lds[256][3];
    __shared__ uint32_t lds_bits[256];
    Acc a{0ull, 0, 0u};
    for (uint32_t b = threadIdx.x; b < blocks; b += blockDim.x) {
        const unsigned long long* in = partial + (uint64_t)b * 4;
        a.sum += in[0];
        a.sq += ((u128)in[2] << 64) | in[1];
        a.bits |= (uint32_t)in[3];
    }
    block_reduce(a, lds, lds_bits);
    if (threadIdx.x == 0) {
        result[0] = a.sum;
        result[1] = (unsigned long long)a.sq;
        result[2] = (unsigned long long)(a.sq >> 64);
        result[3] = a.bits;
        *status = (a.bits & 0x80000000u) ? DC_FLAG_NEGATIVE_LATENCY : 0u;
    }
}

// out[k] = sum_{m=1..M} Phi((tau_k - m mu) / sqrt(m sigma2)), the CLT estimate of the completed micro-batches
// per worker (Section 4.3).  sigma2 = 0: the step function #{m : m mu < tau_k}.  One block per threshold,
// terms added in a fixed order.
__global__ __launch_bounds__(256)
void dc_expected_done_kernel(const long long* __restrict__ taus, uint32_t K, uint32_t M, double mu, double sigma2,
                             double* __restrict__ out) {
    __shared__ double lds[256];
    for (uint32_t k = blockIdx.x; k < K; k += gridDim.x) {
        const double tau = (double)taus[k];
        double acc = 0.0;
        for (uint32_t m = threadIdx.x + 1; m <= M; m += blockDim.x) {
            const double mean = (double)m * mu;
            if (sigma2 > 0.0) {
                const double z = (tau - mean) / sqrt((double)m * sigma2);
                acc += 0.5 * erfc(-z * 0.70710678118654752440);
            } else {
                acc += mean < tau ? 1.0 : 0.0;
            }
        }
        lds[threadIdx.x] = acc;
        __syncthreads();
        for (uint32_t d = 128; d >= 1; d >>= 1) {
            if (threadIdx.x < d) lds[threadIdx.x] += lds[threadIdx.x + d];
            __syncthreads();
        }
        if (threadIdx.x == 0) out[k] = lds[0];
        __syncthreads();
    }
}

namespace dc {

void launch_moments(const int32_t* lat, uint64_t n, uint32_t grid, unsigned long long* partial,
                    unsigned long long* result, uint32_t* status, hipStream_t stream) {
    uint64_t head = (4u - (uint32_t)(((uintptr_t)lat >> 2) & 3u)) & 3u;     // elements before the first 16-byte boundary
    if (head > n) head = n;
    const uint64_t units = (n - head) / 8192;
    const uint32_t vec_units = (uint32_t)(units < 0x7FFFFFFFull ? units : 0x7FFFFFFFull);
    uint32_t run = DC_UNIT_RUN;                          // long runs only while every block still gets several of them
    while (run > 4u && (uint64_t)vec_units < 4ull * run * grid) run >>= 1;
    hipLaunchKernelGGL(dc_moments_kernel, dim3(grid), dim3(256), 0, stream, lat, (unsigned long long)n, (uint32_t)head,
                       vec_units, run, (unsigned long long)(head + (uint64_t)vec_units * 8192ull), partial);
    hipLaunchKernelGGL(dc_moments_final_kernel, dim3(1), dim3(256), 0, stream, partial, grid, result, status);
}

void launch_expected_done(const int64_t* taus, uint32_t K, uint32_t M, double mu, double sigma2, double* out,
                          hipStream_t stream) {
    const uint32_t grid = K < 1024 ? K : 1024;
    hipLaunchKernelGGL(dc_expected_done_kernel, dim3(grid), dim3(256), 0, stream, (const long long*)taus, K, M, mu,
                       sigma2, out);
}

}  // namespace dc
