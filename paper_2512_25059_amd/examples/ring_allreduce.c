/* The C ABI from plain C: an fp32 ring all-reduce over four simulated ranks with a NIC channel that
 * fails half-way, checked against the sum computed on the host.
 *
 *   hipcc --offload-arch=gfx950 -I include paper_2512_25059_amd/examples/ring_allreduce.c \
 *         -L paper_2512_25059_amd -lr2ccl -Wl,-rpath,$PWD/paper_2512_25059_amd -o ring_allreduce
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

#include "r2ccl.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 2; } } while (0)
#define CHECK_R2(x) do { int r_ = (x); if (r_ != R2_OK) { fprintf(stderr, "%s: %s\n", #x, r2_strerror(r_)); return 3; } } while (0)

int main(void)
{
    enum { R = 4, C = 4 };
    const uint64_t n = 1u << 20; /* elements per rank */
    const uint32_t weights[C] = {50000, 50000, 25000, 25000};
    const r2_epoch epochs[2] = {{0, 0, weights}, {3, 1u << 1, weights}}; /* channel 1 fails at transmission 3 */
    const r2_sim_desc desc = {R, 1, C, 256, n, R2_F32, R2_PHASE_RS | R2_PHASE_AG, 0, R2_SCHED_AUTO, 0};

    /* the partition of one ring chunk under the second state, through the host convenience call */
    uint64_t off[C + 1];
    CHECK_R2(r2_partition(weights, 1u << 1, C, n / R * 4, 256, off));
    printf("chunk of %llu bytes over channels:", (unsigned long long)(n / R * 4));
    for (int c = 0; c < C; ++c) printf(" %llu", (unsigned long long)(off[c + 1] - off[c]));
    printf("\n");

    float *host[R], *expect = (float *)calloc(n, sizeof(float));
    void *dev[R], *ws;
    for (int r = 0; r < R; ++r) {
        host[r] = (float *)malloc(n * sizeof(float));
        for (uint64_t i = 0; i < n; ++i) {
            host[r][i] = (float)((i * 2654435761u + r * 40503u) % 2001) - 1000.0f; /* small integers: exact sums */
            expect[i] += host[r][i];
        }
        CHECK_HIP(hipMalloc(&dev[r], n * sizeof(float)));
        CHECK_HIP(hipMemcpy(dev[r], host[r], n * sizeof(float), hipMemcpyHostToDevice));
    }
    const uint64_t ws_bytes = r2_sim_workspace_bytes(&desc);
    if (ws_bytes == 0) { fprintf(stderr, "bad descriptor\n"); return 3; }
    CHECK_HIP(hipMalloc(&ws, ws_bytes));

    CHECK_R2(r2_ring_allreduce_sim(&desc, dev, epochs, 2, ws, ws_bytes, NULL, NULL));
    CHECK_HIP(hipDeviceSynchronize());

    for (int r = 0; r < R; ++r) {
        CHECK_HIP(hipMemcpy(host[r], dev[r], n * sizeof(float), hipMemcpyDeviceToHost));
        for (uint64_t i = 0; i < n; ++i)
            if (host[r][i] != expect[i]) {
                fprintf(stderr, "rank %d element %llu: %g, expected %g\n", r, (unsigned long long)i, host[r][i], expect[i]);
                return 1;
            }
    }
    printf("all-reduce of %d ranks x %llu fp32 elements: every rank holds the exact sum\n", R, (unsigned long long)n);
    return 0;
}
