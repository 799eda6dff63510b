/* A plain C caller of the library's C ABI (include/dc.h): no Python, no torch.
 *
 * Reads one problem from standard input as text,
 *     T N M K comm
 *     T*N*M latencies (int32 microseconds, m fastest)
 *     K thresholds    (int64 microseconds)
 * copies the latencies to the GPU, calls dc_simulate and dc_select_tau, and prints
 *     step <K sums>
 *     done <K sums>
 *     best <index of the selected threshold>
 * Exit status 0 on success, 1 on bad input, 2 when the library or the GPU reports an error.
 *
 * Build (see __graft_entry__.build):
 *     gcc -std=c11 -D__HIP_PLATFORM_AMD__ -I/opt/rocm/include -Iinclude paper_2306_10598_amd/examples/dc_from_c.c \
 *         -Lpaper_2306_10598_amd -ldc -L/opt/rocm/lib -lamdhip64 -Wl,-rpath,$PWD/paper_2306_10598_amd -o paper_2306_10598_amd/examples/dc_from_c
 */
#include <hip/hip_runtime_api.h>
#include <inttypes.h>
#include <stdio.h>
#include <stdlib.h>

#include "dc.h"

int main(void) {
    long long T, N, M, K, comm;
    if (scanf("%lld %lld %lld %lld %lld", &T, &N, &M, &K, &comm) != 5 || T < 1 || N < 1 || M < 1 || K < 1) return 1;
    const size_t elements = (size_t)T * (size_t)N * (size_t)M;
    int32_t* lat = (int32_t*)malloc(elements * sizeof(int32_t));
    int64_t* taus = (int64_t*)malloc((size_t)K * sizeof(int64_t));
    int64_t* step = (int64_t*)malloc((size_t)K * sizeof(int64_t));
    int64_t* done = (int64_t*)malloc((size_t)K * sizeof(int64_t));
    if (!lat || !taus || !step || !done) return 1;
    for (size_t i = 0; i < elements; ++i) {
        long long v;
        if (scanf("%lld", &v) != 1) return 1;
        lat[i] = (int32_t)v;
    }
    for (long long k = 0; k < K; ++k) {
        long long v;
        if (scanf("%lld", &v) != 1) return 1;
        taus[k] = (int64_t)v;
    }

    void* lat_dev = NULL;
    if (hipMalloc(&lat_dev, elements * sizeof(int32_t)) != hipSuccess ||
        hipMemcpy(lat_dev, lat, elements * sizeof(int32_t), hipMemcpyHostToDevice) != hipSuccess) {
        fprintf(stderr, "no device memory\n");
        return 2;
    }
    int rc = dc_simulate((const int32_t*)lat_dev, T, N, M, taus, K, comm, step, done);
    if (rc != DC_OK) {
        fprintf(stderr, "dc_simulate: %s (%s)\n", dc_status_string(rc), dc_last_device_error());
        return 2;
    }
    int64_t best = -1;
    rc = dc_select_tau(step, done, taus, K, T, N, M, 0, NULL, NULL, &best);
    if (rc != DC_OK) {
        fprintf(stderr, "dc_select_tau: %s\n", dc_status_string(rc));
        return 2;
    }
    printf("step");
    for (long long k = 0; k < K; ++k) printf(" %" PRId64, step[k]);
    printf("\ndone");
    for (long long k = 0; k < K; ++k) printf(" %" PRId64, done[k]);
    printf("\nbest %" PRId64 "\n", best);
    (void)hipFree(lat_dev);
    dc_shutdown();
    free(lat); free(taus); free(step); free(done);
    return 0;
}
