/* The C ABI used from plain C (no Python, no GPU): schedule generator, round planner, plan check and
 * Metropolis weights.  Compiled with -std=c11 -Wall -Werror by tests/test_host_logic.py. */
#include <stdio.h>
#include <stdlib.h>

#include "adpsgd.h"

int main(void) {
    enum { N = 8, K = 500, T = 3, M = 4 };
    int32_t rowptr[N + 1], col[2 * N], rows[N];
    for (int i = 0; i < N; ++i) {
        rowptr[i] = 2 * i;
        col[2 * i] = (i + N - 1) % N;
        col[2 * i + 1] = (i + 1) % N;
        rows[i] = 32;
    }
    rowptr[N] = 2 * N;
    adpsgd_sched_params_t sp = {{N, rowptr, col}, NULL, 0, T, NULL, NULL, M, rows, 0};
    int32_t *worker = malloc(sizeof(int32_t) * K), *nbr = malloc(sizeof(int32_t) * K), *tau = malloc(sizeof(int32_t) * K);
    int32_t* batch = malloc(sizeof(int32_t) * K * M);
    if (adpsgd_make_schedule(&sp, 7, 0, K, worker, nbr, tau, batch) != ADPSGD_OK) return 1;
    for (int k = 0; k < K; ++k) {
        if (worker[k] < 0 || worker[k] >= N || tau[k] > T || tau[k] > k) return 2;
        if (nbr[k] != (worker[k] + 1) % N && nbr[k] != (worker[k] + N - 1) % N) return 3;
        for (int m = 0; m < M; ++m)
            if (batch[k * M + m] < 0 || batch[k * M + m] >= 32) return 4;
    }
    int32_t *r = malloc(sizeof(int32_t) * K), *u = malloc(sizeof(int32_t) * K), *slot = malloc(sizeof(int32_t) * K), n_rounds = 0;
    if (adpsgd_plan_rounds(N, K, worker, nbr, tau, T + 2, 1, r, u, slot, &n_rounds, NULL, NULL, NULL, 0, NULL, -1, NULL) != ADPSGD_OK) return 5;
    if (n_rounds < K / (N / 2) || n_rounds > K) return 6;
    if (adpsgd_verify_plan(N, K, worker, nbr, tau, T + 2, 1, r, u, slot, n_rounds, NULL, NULL, NULL, NULL, -1, NULL) != ADPSGD_OK) return 7;
    /* damage the plan: an update moved into the round of its predecessor on the same row must be caught */
    int damaged = 0;
    for (int k = 1; k < K && !damaged; ++k)
        if (u[k] > 0) { u[k] -= 1; damaged = adpsgd_verify_plan(N, K, worker, nbr, tau, T + 2, 1, r, u, slot, n_rounds, NULL, NULL, NULL, NULL, -1, NULL) == ADPSGD_ERR_STATE; u[k] += 1; }
    if (!damaged) return 8;
    float w_self[N], w_edge[2 * N];
    adpsgd_graph_t g = {N, rowptr, col};
    if (adpsgd_metropolis_weights(&g, w_self, w_edge) != ADPSGD_OK) return 9;
    for (int i = 0; i < N; ++i)
        if (w_self[i] < 0.333f || w_self[i] > 0.334f || w_edge[2 * i] != w_edge[2 * i + 1]) return 10;
    /* a null handle is an argument error, not a crash */
    if (adpsgd_run_events(NULL, NULL, NULL) != ADPSGD_ERR_ARG) return 11;
    printf("c abi ok: %d events in %d rounds\n", K, (int)n_rounds);
    free(worker); free(nbr); free(tau); free(batch); free(r); free(u); free(slot);
    return 0;
}
