/* Plain C user of the C ABI: no Python, no torch.  Allocates P rank buffers and the scratch with
 * hipMalloc, runs rar_allreduce in every mode and rar_allreduce_chain (two calls in one launch,
 * against the oracle applied twice) and compares the bytes with the CPU oracle
 * (nvrar_oracle_allreduce, linked from oracle/).
 * Exit status 0 = bit-exact everywhere.
 * usage: c_abi_parity P G n dtype(0 bf16 | 1 f32) */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "rar.h"

int nvrar_oracle_allreduce(const void *const *in, void *const *out, int G, int N, size_t n, int dtype, int threads);

#define HIP_OK(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { \
    fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_)); return 2; } } while (0)
#define RAR_CHECK(call) do { int s_ = (call); if (s_ != RAR_OK) { \
    fprintf(stderr, "%s failed: %s\n", #call, rar_strerror(s_)); return 3; } } while (0)

/* xorshift values in a sane range, stored in the message type (bf16 by truncation of a float:
 * inputs only have to be valid bit patterns, the same ones on both sides) */
static uint32_t rng_state = 2463534242u;
static uint32_t rng(void) { rng_state ^= rng_state << 13; rng_state ^= rng_state >> 17; rng_state ^= rng_state << 5; return rng_state; }
static float rnd_float(void) { return ((float)(rng() & 0xffffff) / 8388608.0f - 1.0f) * 3.0f; }

int main(int argc, char **argv) {
    if (argc != 5) { fprintf(stderr, "usage: %s P G n dtype\n", argv[0]); return 1; }
    const int P = atoi(argv[1]), G = atoi(argv[2]), dtype = atoi(argv[4]);
    const size_t n = (size_t)strtoull(argv[3], NULL, 10);
    const size_t es = dtype == RAR_BF16 ? 2 : 4, bytes = n * es;

    rar_plan_t *plan = NULL;
    RAR_CHECK(rar_plan(P, G, n, dtype, &plan));
    void **host_in = calloc((size_t)P, sizeof *host_in), **host_want = calloc((size_t)P, sizeof *host_want);
    void **dev = calloc((size_t)P, sizeof *dev);
    void *host_got = malloc(bytes);
    for (int p = 0; p < P; ++p) {
        host_in[p] = malloc(bytes);
        host_want[p] = malloc(bytes);
        for (size_t i = 0; i < n; ++i) {
            float f = rnd_float();
            uint32_t u; memcpy(&u, &f, 4);
            if (dtype == RAR_BF16) ((uint16_t *)host_in[p])[i] = (uint16_t)(u >> 16);
            else ((float *)host_in[p])[i] = f;
        }
        HIP_OK(hipMalloc(&dev[p], bytes));
    }
    if (nvrar_oracle_allreduce((const void *const *)host_in, host_want, G, P / G, n, dtype, 4) != 0) return 4;

    void *scratch = NULL;
    const size_t sbytes = rar_plan_scratch_bytes(plan);
    HIP_OK(hipMalloc(&scratch, sbytes));
    RAR_CHECK(rar_plan_set_scratch(plan, scratch, sbytes));

    int failures = 0;
    for (int mode = RAR_MODE_STEPWISE; mode <= RAR_MODE_AUTO; ++mode) {
        int rc = rar_plan_set_mode(plan, mode);
        if (rc == RAR_ERR_LIMIT && mode == RAR_MODE_FUSED_PACKED) { printf("mode %d: not offered for this size\n", mode); continue; }
        RAR_CHECK(rc);
        for (int p = 0; p < P; ++p) HIP_OK(hipMemcpy(dev[p], host_in[p], bytes, hipMemcpyHostToDevice));
        printf("mode %d: launching P=%d G=%d n=%zu dtype=%d\n", mode, P, G, n, dtype); fflush(stdout);
        RAR_CHECK(rar_allreduce(dev, plan, NULL));
        RAR_CHECK(rar_plan_status(plan, NULL));
        for (int p = 0; p < P; ++p) {
            HIP_OK(hipMemcpy(host_got, dev[p], bytes, hipMemcpyDeviceToHost));
            if (memcmp(host_got, host_want[p], bytes) != 0) { ++failures; fprintf(stderr, "mode %d rank %d differs\n", mode, p); break; }
        }
    }
    /* two chained calls in one launch = the oracle applied to its own result */
    void **host_twice = calloc((size_t)P, sizeof *host_twice);
    for (int p = 0; p < P; ++p) host_twice[p] = malloc(bytes);
    if (nvrar_oracle_allreduce((const void *const *)host_want, host_twice, G, P / G, n, dtype, 4) != 0) return 4;
    for (int mode = RAR_MODE_FUSED; mode <= RAR_MODE_FUSED_PACKED; ++mode) {
        if (rar_plan_set_mode(plan, mode) != RAR_OK) continue;
        for (int p = 0; p < P; ++p) HIP_OK(hipMemcpy(dev[p], host_in[p], bytes, hipMemcpyHostToDevice));
        printf("mode %d: chain of 2\n", mode); fflush(stdout);
        RAR_CHECK(rar_allreduce_chain(dev, plan, 2, NULL));
        RAR_CHECK(rar_plan_status(plan, NULL));
        for (int p = 0; p < P; ++p) {
            HIP_OK(hipMemcpy(host_got, dev[p], bytes, hipMemcpyDeviceToHost));
            if (memcmp(host_got, host_twice[p], bytes) != 0) { ++failures; fprintf(stderr, "chain, mode %d rank %d differs\n", mode, p); break; }
        }
    }
    for (int p = 0; p < P; ++p) free(host_twice[p]);
    free(host_twice);
    for (int p = 0; p < P; ++p) { (void)hipFree(dev[p]); free(host_in[p]); free(host_want[p]); }
    (void)hipFree(scratch);
    RAR_CHECK(rar_plan_free(plan));
    free(host_in); free(host_want); free(dev); free(host_got);
    printf(failures ? "FAILED\n" : "c abi parity ok\n");
    return failures ? 5 : 0;
}
