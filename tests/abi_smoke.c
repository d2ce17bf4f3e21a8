/*
 * abi_smoke.c -- calls libgbmuf through its C ABI from plain C (no Python, no torch): makes a
 * plan, runs three syncs of a small ragged model on device buffers obtained from the HIP
 * runtime, and compares every value with the CPU oracle (test infrastructure, linked in).
 * Built by __graft_entry__.build(); run by tests/test_gpu_parity.py on a GPU machine.
 * Exit status 0 and a line starting with "abi_smoke ok" mean success.
 */
#include <hip/hip_runtime_api.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../include/gbmuf.h"

int gbmuf_oracle_sync_f32(const int64_t *off, int32_t m, int32_t K, int32_t p, int32_t q, uint64_t seed,
                          uint64_t round, const uint8_t *active, float *theta, float *omega, float *delta,
                          int64_t stride, float eta, float zeta, int32_t mode);
int gbmuf_oracle_neighbour_table(int32_t m, int32_t K, int32_t p, int32_t q, uint64_t seed, uint64_t round,
                                 int32_t *nbr);

#define CHECK(x) do { int rc_ = (x); if (rc_ != 0) { fprintf(stderr, "%s failed: %d (%s) [%s]\n", #x, rc_, gbmuf_strerror(rc_), gbmuf_last_error_detail()); return 1; } } while (0)
#define HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_)); return 1; } } while (0)

int main(void)
{
    enum { K = 8, Q = 2, M = 4 };
    const int64_t off[M + 1] = {0, 1000, 1003, 1003, 50001};
    const int64_t P = off[M], stride = 50176;
    const uint64_t seed = 0x5eedULL;
    const float eta = 0.9f, zeta = 1.0f;
    const size_t n = (size_t)K * (size_t)stride, bytes = n * sizeof(float);

    float *h[3], *ref[3], *d[3];
    unsigned s = 12345u;
    for (int a = 0; a < 3; ++a) {
        h[a] = (float *)malloc(bytes); ref[a] = (float *)malloc(bytes);
        if (!h[a] || !ref[a]) return 1;
        for (size_t i = 0; i < n; ++i) {
            s = s * 1664525u + 1013904223u;                              /* any deterministic filler */
            h[a][i] = ((float)(s >> 8) / 16777216.0f - 0.5f) * (a == 2 ? 0.001f : 0.1f);
        }
        memcpy(ref[a], h[a], bytes);
        HIP(hipMalloc((void **)&d[a], bytes));
        HIP(hipMemcpy(d[a], h[a], bytes, hipMemcpyHostToDevice));
    }

    gbmuf_plan_t *plan = NULL;
    gbmuf_info_t info;
    CHECK(gbmuf_plan(&plan, off, M, K, Q, 0, seed));
    CHECK(gbmuf_plan_info(plan, &info));
    if (!info.has_device) { fprintf(stderr, "no device\n"); return 1; }

    int32_t *tab_host = (int32_t *)malloc(sizeof(int32_t) * M * K * Q), *tab_ref = (int32_t *)malloc(sizeof(int32_t) * M * K * Q);
    int32_t *tab_dev = NULL;
    HIP(hipMalloc((void **)&tab_dev, sizeof(int32_t) * M * K * Q));
    hipStream_t stream;
    HIP(hipStreamCreate(&stream));
    for (uint64_t round = 0; round < 3; ++round) {
        CHECK(gbmuf_sync(plan, d[0], d[1], d[2], stride, eta, zeta, GBMUF_MODE_PAPER, round, stream));
        CHECK(gbmuf_oracle_sync_f32(off, M, K, info.p, Q, seed, round, NULL, ref[0], ref[1], ref[2], stride, eta, zeta, 1));
        CHECK(gbmuf_neighbours_device(plan, round, tab_dev, stream));
        HIP(hipStreamSynchronize(stream));
        HIP(hipMemcpy(tab_host, tab_dev, sizeof(int32_t) * M * K * Q, hipMemcpyDeviceToHost));
        CHECK(gbmuf_oracle_neighbour_table(M, K, info.p, Q, seed, round, tab_ref));
        if (memcmp(tab_host, tab_ref, sizeof(int32_t) * M * K * Q) != 0) { fprintf(stderr, "neighbour table differs in round %d\n", (int)round); return 1; }
    }
    size_t differ = 0;
    for (int a = 0; a < 3; ++a) {
        HIP(hipMemcpy(h[a], d[a], bytes, hipMemcpyDeviceToHost));
        differ += memcmp(h[a], ref[a], bytes) != 0;
    }
    if (differ) { fprintf(stderr, "%zu of 3 state arrays differ from the oracle\n", differ); return 1; }

    /* The same state moved into the library's blocked arena (gbmuf_recommend_layout,
     * gbmuf_state_copy), two more syncs there (gbmuf_sync_state), and back to rows. */
    gbmuf_layout_t lay;
    CHECK(gbmuf_recommend_layout(plan, P, K, GBMUF_LAYOUT_BLOCKED, &lay));
    float *arena = NULL;
    HIP(hipMalloc((void **)&arena, sizeof(float) * (size_t)lay.arena_floats));
    gbmuf_state_t rows = {d[0], d[1], d[2], stride, 0, 0};
    gbmuf_state_t blocked = {arena, arena + lay.omega_offset, arena + lay.delta_offset,
                             lay.worker_stride, lay.block_floats, lay.block_stride};
    CHECK(gbmuf_state_copy(plan, &blocked, &rows, 7, stream));
    for (uint64_t round = 3; round < 5; ++round) {
        CHECK(gbmuf_sync_state(plan, &blocked, eta, zeta, GBMUF_MODE_PAPER, round, stream));
        CHECK(gbmuf_oracle_sync_f32(off, M, K, info.p, Q, seed, round, NULL, ref[0], ref[1], ref[2], stride, eta, zeta, 1));
    }
    CHECK(gbmuf_state_copy(plan, &rows, &blocked, 7, stream));
    HIP(hipStreamSynchronize(stream));
    for (int a = 0; a < 3; ++a) {
        HIP(hipMemcpy(h[a], d[a], bytes, hipMemcpyDeviceToHost));
        differ += memcmp(h[a], ref[a], bytes) != 0;
    }
    if (differ) { fprintf(stderr, "%zu of 3 state arrays differ from the oracle after the blocked syncs\n", differ); return 1; }
    CHECK(gbmuf_plan_destroy(plan));
    printf("abi_smoke ok: K=%d P=%lld, 3 syncs in rows and 2 in the blocked arena: 3 state arrays and 3 neighbour tables "
           "bit-identical to the oracle (padding included)\n", K, (long long)P);
    return 0;
}
