/* The C ABI on the GPU from plain C (no Python, no tensor library): device memory from the HIP runtime,
 * pure gossip events (synthetic gradients of standard deviation 0) on unequal initial models.
 * Checks what Algorithm 1's averaging step fixes: column sums (the mean model) are preserved, the
 * consensus distance shrinks, nothing becomes non-finite. */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

#include <hip/hip_runtime_api.h>

#include "adpsgd.h"

#define CHECK(cond, code) do { if (!(cond)) { fprintf(stderr, "check failed: %s (line %d): %s\n", #cond, __LINE__, h ? adpsgd_last_error(h) : adpsgd_last_error(NULL)); return code; } } while (0)

/* caller-supplied gradient: g_k = xhat (the gradient of |x|^2 / 2), copied on the handle's stream */
static int n_requested = 0;
static int copy_gradient(void* user, int32_t n_requests, const adpsgd_grad_request_t* rq, void* stream) {
    const size_t bytes = *(const size_t*)user;
    for (int32_t t = 0; t < n_requests; ++t) {
        if (hipMemcpyAsync(rq[t].g, rq[t].xhat, bytes, hipMemcpyDeviceToDevice, (hipStream_t)stream) != hipSuccess) return 1;
        ++n_requested;
    }
    return 0;
}

int main(void) {
    enum { N = 6, D = 1000, LD = 1024, K = 400 };
    adpsgd_t* h = NULL;
    int32_t rowptr[N + 1], col[2 * N];
    for (int i = 0; i < N; ++i) { rowptr[i] = 2 * i; col[2 * i] = (i + N - 1) % N; col[2 * i + 1] = (i + 1) % N; }
    rowptr[N] = 2 * N;
    adpsgd_graph_t g = {N, rowptr, col};
    float* X = NULL;
    CHECK(hipMalloc((void**)&X, sizeof(float) * N * LD) == hipSuccess, 1);
    adpsgd_opts_t o = {0};
    o.model = ADPSGD_MODEL_SYNTH;
    o.gamma = 0.1f;
    o.T_max = 2;
    o.synth_std = 0.0f;
    o.X = X;
    o.ldx = LD;
    o.flags = ADPSGD_FLAG_VERIFY_PLAN;
    CHECK(adpsgd_create(&h, &g, D, &o) == ADPSGD_OK, 2);
    float* x0 = malloc(sizeof(float) * N * D);
    double colsum0[D];
    for (int e = 0; e < D; ++e) colsum0[e] = 0.0;
    for (int i = 0; i < N; ++i)
        for (int e = 0; e < D; ++e) {
            x0[i * D + e] = (float)((i * 37 + e * 11) % 101) / 50.0f - 1.0f;
            colsum0[e] += x0[i * D + e];
        }
    CHECK(adpsgd_set_models(h, x0, D, 0) == ADPSGD_OK, 3);
    double c0 = 0.0, c1 = 0.0;
    CHECK(adpsgd_consensus_distance(h, &c0) == ADPSGD_OK, 4);
    adpsgd_sched_params_t sp = {{N, rowptr, col}, NULL, 0, 2, NULL, NULL, 0, NULL, 0};
    int32_t *worker = malloc(sizeof(int32_t) * K), *nbr = malloc(sizeof(int32_t) * K), *tau = malloc(sizeof(int32_t) * K);
    CHECK(adpsgd_make_schedule(&sp, 3, 0, K, worker, nbr, tau, NULL) == ADPSGD_OK, 5);
    adpsgd_schedule_t s = {0};
    s.K = K;
    s.worker = worker;
    s.neighbour = nbr;
    s.tau = tau;
    CHECK(adpsgd_run_events(h, &s, NULL) == ADPSGD_OK, 6);
    CHECK(adpsgd_consensus_distance(h, &c1) == ADPSGD_OK, 7);
    float* x1 = malloc(sizeof(float) * N * D);
    CHECK(adpsgd_get_models(h, x1, D, 0) == ADPSGD_OK, 8);
    for (int e = 0; e < D; ++e) {
        double sum = 0.0;
        for (int i = 0; i < N; ++i) sum += x1[i * D + e];
        CHECK(fabs(sum - colsum0[e]) <= 1e-5 * N, 9);            /* averaging preserves the sum over the workers */
    }
    int64_t bad = -1;
    uint64_t count = 0;
    CHECK(adpsgd_count_nonfinite(h, &bad) == ADPSGD_OK && bad == 0, 10);
    CHECK(adpsgd_get_event_count(h, &count) == ADPSGD_OK && count == K, 11);
    CHECK(c1 < 1e-3 * c0 && c0 > 0.1, 12);                        /* 400 gossip events on a ring of 6 reach consensus */
    /* a neighbour that is not adjacent is refused and changes nothing */
    nbr[0] = (worker[0] + 3) % N;
    CHECK(adpsgd_run_events(h, &s, NULL) == ADPSGD_ERR_SCHEDULE, 13);
    CHECK(adpsgd_get_event_count(h, &count) == ADPSGD_OK && count == K, 14);
    adpsgd_destroy(h);
    h = NULL;
    /* the same events with the gradient step supplied by this program: f_i(x) = |x|^2 / 2, so every event
     * shrinks the sum over the workers by the factor (1 - gamma) of the stale row: all models go to zero */
    float* slots = NULL;
    CHECK(hipMalloc((void**)&slots, sizeof(float) * 4 * LD) == hipSuccess, 15);
    o.model = ADPSGD_MODEL_EXTERNAL;
    o.workspace = slots;
    o.workspace_bytes = (int64_t)sizeof(float) * 4 * LD;
    CHECK(adpsgd_create(&h, &g, D, &o) == ADPSGD_OK, 16);
    CHECK(adpsgd_set_models(h, x0, D, 0) == ADPSGD_OK, 17);
    size_t row_bytes = sizeof(float) * D;
    nbr[0] = (worker[0] + 1) % N;
    CHECK(adpsgd_run_events(h, &s, NULL) == ADPSGD_ERR_STATE, 18);
    CHECK(adpsgd_run_events_with(h, &s, copy_gradient, &row_bytes) == ADPSGD_OK, 19);
    CHECK(adpsgd_get_models(h, x1, D, 0) == ADPSGD_OK, 20);
    CHECK(n_requested == K, 21);
    double biggest = 0.0;
    for (int t = 0; t < N * D; ++t) biggest = fmax(biggest, fabs(x1[t]));
    CHECK(biggest < 0.05, 22);                                    /* from entries of size 1 */
    printf("c abi gpu ok: consensus distance %.3e -> %.3e; own gradients: largest entry %.3e\n", c0, c1, biggest);
    adpsgd_destroy(h);
    (void)hipFree(slots);
    (void)hipFree(X);
    free(x0); free(x1); free(worker); free(nbr); free(tau);
    return 0;
}
