/*
 * Timing client of the C ABI written in plain C: what a caller without Python or PyTorch gets from the update pass
 * when it places its arrays (a) with ordinary hipMalloc and (b) through the library's region-sorted arena.
 * One local server over one tensor of `n` floats (default 2^28 = 1 GiB per array), bf16 or fp32 delta, the update
 * pass with the model handed back to the worker (4 arrays read, 4 written), always accumulating.
 * Prints GB/s (algorithmic bytes / time between HIP events) for both placements; exit status 0 unless a call failed.
 *     arena_client [n_floats] [reps]
 */
#include <hip/hip_runtime_api.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../include/halos.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s (%s:%d)\n", hipGetErrorString(e_), __FILE__, __LINE__); return 2; } } while (0)
#define CHECK_HALOS(x) do { halos_status s_ = (x); if (s_ != HALOS_OK) { printf("halos status %d: %s (%s:%d)\n", (int)s_, halos_last_error(), __FILE__, __LINE__); return 3; } } while (0)

/* roles: 0 m, 1 third buffer, 2 theta, 3 delta, 4 GPS momentum, 5 worker model, 6 GPS model */
enum { R_M, R_ACC, R_THETA, R_DELTA, R_GM, R_WM, R_GTHETA, N_ROLES };
static const int class_of_role[N_ROLES] = {0, 0, 1, 1, 1, 2, 2};

static int time_update(void *buf[N_ROLES], int64_t n, int reps, double *gbps) {
    const int64_t numel[1] = {n};
    halos_layout layout = {1, numel};
    halos_hparams hp;
    memset(&hp, 0, sizeof hp);
    hp.local.eta = 0.2f; hp.local.beta = 0.9f; hp.local.cg = 1.0f - 0.9f;
    hp.global.eta = 0.15f; hp.global.beta = 0.5f; hp.global.cg = 0.5f;
    hp.alpha = 0.25f; hp.K = 1 << 30;
    CHECK_HIP(hipMemset(buf[R_GTHETA], 0, (size_t)n * 4));
    CHECK_HIP(hipMemset(buf[R_DELTA], 0, (size_t)n * 4));
    halos_gps *gps = NULL;
    halos_lps *lps = NULL;
    void *pT[1] = {buf[R_GTHETA]}, *pM[1] = {buf[R_GM]}, *th[1] = {buf[R_THETA]}, *m[1] = {buf[R_M]}, *acc[1] = {buf[R_ACC]};
    void *wm[1] = {buf[R_WM]};
    const void *g[1] = {buf[R_DELTA]};
    CHECK_HALOS(halos_gps_create(&layout, &hp, pT, pM, NULL, &gps));
    CHECK_HALOS(halos_lps_create(gps, 0, 1, th, m, acc, NULL, &lps));
    CHECK_HALOS(halos_lps_set_worker_model(lps, 0, wm, NULL));
    hipEvent_t e0, e1;
    CHECK_HIP(hipEventCreate(&e0));
    CHECK_HIP(hipEventCreate(&e1));
    for (int r = 0; r < reps + 2; ++r) {
        if (r == 2) CHECK_HIP(hipEventRecord(e0, NULL));
        CHECK_HALOS(halos_lps_push_update(lps, 0, g, HALOS_F32, 0));
        CHECK_HALOS(halos_lps_step_pull(lps, NULL, NULL));
    }
    CHECK_HIP(hipEventRecord(e1, NULL));
    CHECK_HIP(hipEventSynchronize(e1));
    float ms = 0.f;
    CHECK_HIP(hipEventElapsedTime(&ms, e0, e1));
    *gbps = (double)n * 32.0 * reps / ((double)ms * 1e-3) / 1e9;      /* fp32 delta: 16 bytes read, 16 written */
    halos_lps_destroy(lps);
    halos_gps_destroy(gps);
    CHECK_HIP(hipEventDestroy(e0));
    CHECK_HIP(hipEventDestroy(e1));
    return 0;
}

int main(int argc, char **argv) {
    const int64_t n = argc > 1 ? atoll(argv[1]) : (1ll << 28);
    const int reps = argc > 2 ? atoi(argv[2]) : 10;
    if (n < 4096 || reps < 1) { printf("usage: arena_client [n_floats >= 4096] [reps >= 1]\n"); return 1; }
    const size_t bytes = (size_t)n * 4;
    void *buf[N_ROLES];
    double plain = 0.0, placed = 0.0;

    for (int r = 0; r < N_ROLES; ++r) CHECK_HIP(hipMalloc(&buf[r], bytes));
    int rc = time_update(buf, n, reps, &plain);
    for (int r = 0; r < N_ROLES; ++r) CHECK_HIP(hipFree(buf[r]));
    if (rc) return rc;

    uint64_t need[3] = {0, 0, 0};
    for (int r = 0; r < N_ROLES; ++r) need[class_of_role[r]] += bytes;
    halos_arena *arena = NULL;
    CHECK_HALOS(halos_arena_create(3, need, 0, &arena));
    int32_t n_regions = 0, region_of_class[3];
    uint64_t walked = 0;
    CHECK_HALOS(halos_arena_info(arena, &n_regions, &walked, NULL, region_of_class, NULL));
    for (int r = 0; r < N_ROLES; ++r) CHECK_HALOS(halos_arena_alloc(arena, class_of_role[r], bytes, &buf[r]));
    rc = time_update(buf, n, reps, &placed);
    halos_arena_destroy(arena);
    if (rc) return rc;

    printf("arena_client: n=%lld floats per array, %d timed updates (fp32 delta, fused pull, 32 B/parameter)\n", (long long)n, reps);
    printf("arena_client: plain hipMalloc       %8.0f GB/s  (%.1f %% of 8 TB/s)\n", plain, plain / 80.0);
    printf("arena_client: region-sorted arena   %8.0f GB/s  (%.1f %% of 8 TB/s)  regions found %d, classes in regions %d %d %d, walked %llu GiB\n",
           placed, placed / 80.0, n_regions, region_of_class[0], region_of_class[1], region_of_class[2],
           (unsigned long long)(walked >> 30));
    printf("RESULT plain_gbps=%.1f arena_gbps=%.1f regions=%d\n", plain, placed, n_regions);
    return 0;
}
