/*
 * A client of the C ABI written in plain C: no Python, no PyTorch, device memory from hipMalloc.
 * It replays the integer example that tests/golden/alg1_worked_example.json derives by hand from
 * Algorithm 1 of the HALoS paper (beta = 0, eta = 1, alpha = 1/2, K = 2, two local servers) and checks
 * every intermediate and final value.  Exit status 0 = all values as derived.
 */
#include <hip/hip_runtime_api.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../include/halos.h"

#define N 4
#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s (%s:%d)\n", hipGetErrorString(e_), __FILE__, __LINE__); return 2; } } while (0)
#define CHECK_HALOS(x) do { halos_status s_ = (x); if (s_ != HALOS_OK) { printf("halos status %d: %s (%s:%d)\n", (int)s_, halos_last_error(), __FILE__, __LINE__); return 3; } } while (0)

static float *dev_vec(const float *host) {
    float *d = NULL;
    if (hipMalloc((void **)&d, N * sizeof(float)) != hipSuccess) return NULL;
    if (host && hipMemcpy(d, host, N * sizeof(float), hipMemcpyHostToDevice) != hipSuccess) return NULL;
    return d;
}

static int expect(const char *what, const float *dev, const float *want) {
    float got[N];
    if (hipDeviceSynchronize() != hipSuccess) return 1;
    if (hipMemcpy(got, dev, sizeof got, hipMemcpyDeviceToHost) != hipSuccess) return 1;
    for (int i = 0; i < N; ++i)
        if (got[i] != want[i]) {
            printf("MISMATCH %s[%d]: got %g, derived %g\n", what, i, got[i], want[i]);
            return 1;
        }
    return 0;
}

static int expect_step(const char *what, const halos_step_info *s, int kind, long long t, long long t_last, int ready) {
    if (s->kind != kind || s->t != t || s->t_last != t_last || s->delta_ready != ready) {
        printf("MISMATCH %s: kind %d t %lld t_last %lld ready %d\n", what, s->kind, (long long)s->t, (long long)s->t_last,
               s->delta_ready);
        return 1;
    }
    return 0;
}

int main(void) {
    const float theta0[N] = {8, -4, 0, 16};
    const float g1[N] = {1, 2, 3, 4}, g2[N] = {2, 0, -2, 4}, g3[N] = {4, 4, 4, 4}, g4[N] = {1, 1, 1, 1};
    const float g5[N] = {0, 2, 0, 2}, g6[N] = {2, 2, 2, 2}, g7[N] = {1, 0, 1, 0};
    const int64_t numel[1] = {N};
    halos_layout layout = {1, numel};
    halos_hparams hp;
    memset(&hp, 0, sizeof hp);
    hp.local.eta = 1.f; hp.local.beta = 0.f; hp.local.cg = 1.f;
    hp.global.eta = 1.f; hp.global.beta = 0.f; hp.global.cg = 1.f;
    hp.alpha = 0.5f; hp.K = 2; hp.flags = 0;

    float *Theta = dev_vec(theta0), *M = dev_vec(NULL);
    float *th[2] = {dev_vec(NULL), dev_vec(NULL)}, *m[2] = {dev_vec(NULL), dev_vec(NULL)}, *acc[2] = {dev_vec(NULL), dev_vec(NULL)};
    float *d1 = dev_vec(g1), *d2 = dev_vec(g2), *d3 = dev_vec(g3), *d4 = dev_vec(g4), *d5 = dev_vec(g5), *d6 = dev_vec(g6), *d7 = dev_vec(g7);
    float *pulled = dev_vec(NULL);
    if (!Theta || !M || !th[0] || !th[1] || !m[0] || !m[1] || !acc[0] || !acc[1] || !d1 || !d2 || !d3 || !d4 || !d5 || !d6 || !d7 || !pulled) {
        printf("device allocation failed\n");
        return 2;
    }
    halos_gps *gps = NULL;
    halos_lps *lps[2] = {NULL, NULL};
    void *pT[1] = {Theta}, *pM[1] = {M};
    CHECK_HALOS(halos_gps_create(&layout, &hp, pT, pM, NULL, &gps));
    for (int l = 0; l < 2; ++l) {
        void *a[1] = {th[l]}, *b[1] = {m[l]}, *c[1] = {acc[l]};
        CHECK_HALOS(halos_lps_create(gps, l, 2, a, b, c, NULL, &lps[l]));
    }
    int bad = 0;
    halos_step_info s;
#define PUSH(l, w, d) do { const void *p_[1] = {d}; CHECK_HALOS(halos_lps_push_update(lps[l], w, p_, HALOS_F32, 0)); } while (0)
    PUSH(0, 0, d1); CHECK_HALOS(halos_lps_step(lps[0], NULL, &s)); bad += expect_step("A step 1", &s, 1, 1, 0, 0);
    PUSH(0, 1, d2); CHECK_HALOS(halos_lps_step(lps[0], NULL, &s)); bad += expect_step("A step 2", &s, 1, 2, 0, 1);
    PUSH(1, 0, d3); CHECK_HALOS(halos_lps_step(lps[1], NULL, &s)); bad += expect_step("B step 1", &s, 1, 1, 0, 0);
    PUSH(0, 0, d4); CHECK_HALOS(halos_lps_step(lps[0], NULL, &s)); bad += expect_step("A step 3 (in flight)", &s, 1, 3, 0, 0);
    CHECK_HALOS(halos_gps_merge(gps, lps[0], NULL));
    { const float want[N] = {5, -6, -1, 8}; bad += expect("Theta after A's update", Theta, want); }
    PUSH(1, 1, d5); CHECK_HALOS(halos_lps_step(lps[1], NULL, &s)); bad += expect_step("B step 2", &s, 1, 2, 0, 1);
    CHECK_HALOS(halos_gps_merge(gps, lps[1], NULL));
    { const float want[N] = {1, -12, -5, 2}; bad += expect("Theta after B's update", Theta, want); }
    CHECK_HALOS(halos_lps_push_global(lps[0]));
    CHECK_HALOS(halos_lps_step(lps[0], NULL, &s)); bad += expect_step("A merge", &s, 2, 3, 3, 0);
    { const float want[N] = {4.5f, -6.5f, -1.5f, 7.5f}; bad += expect("theta_A after merging Theta_1", th[0], want); }
    PUSH(0, 1, d6); CHECK_HALOS(halos_lps_step(lps[0], NULL, &s)); bad += expect_step("A step 4", &s, 1, 4, 3, 0);
    PUSH(0, 0, d7); CHECK_HALOS(halos_lps_step(lps[0], NULL, &s)); bad += expect_step("A step 5", &s, 1, 5, 3, 1);
    CHECK_HALOS(halos_gps_merge(gps, lps[0], NULL));
    { const float want[N] = {-2, -14, -8, 0}; bad += expect("Theta after A's second update", Theta, want); }
    CHECK_HALOS(halos_lps_push_global(lps[1]));
    CHECK_HALOS(halos_lps_step(lps[1], NULL, &s)); bad += expect_step("B merge", &s, 2, 2, 2, 0);
    { const float want[N] = {2.5f, -11, -4.5f, 6}; bad += expect("theta_B after merging Theta_2", th[1], want); }
    { const float want[N] = {1.5f, -8.5f, -4.5f, 5.5f}; bad += expect("theta_A at the end", th[0], want); }
    { const float want[N] = {-2, -14, -8, 0}; bad += expect("A's third buffer (returned model in flight)", acc[0], want); }
    { const float want[N] = {0, 0, 0, 0}; bad += expect("B's third buffer (restarted accumulation)", acc[1], want); }
    { void *dst[1] = {pulled}; CHECK_HALOS(halos_pull_model(lps[0], 0, dst, NULL));
      const float want[N] = {1.5f, -8.5f, -4.5f, 5.5f}; bad += expect("pulled model of A", pulled, want); }
    /* a protocol violation must be reported, not executed */
    if (halos_gps_merge(gps, lps[1], NULL) != HALOS_ESTATE) { printf("MISMATCH: merge with nothing in flight was accepted\n"); ++bad; }
    int64_t updates = 0;
    CHECK_HALOS(halos_gps_get_counters(gps, &updates));
    if (updates != 3) { printf("MISMATCH: %lld GPS updates, derived 3\n", (long long)updates); ++bad; }
    halos_lps_destroy(lps[0]); halos_lps_destroy(lps[1]); halos_gps_destroy(gps);
    printf(bad ? "abi_client: %d mismatches\n" : "abi_client: all values as derived from Algorithm 1\n", bad);
    return bad ? 1 : 0;
}
