// Host-side random choices of Algorithm 1 (worker i_k, neighbour j_k, staleness
// tau_k, minibatch xi_k) and graph validation.  Integer-only, so that the draws
// are reproducible bit for bit by any other implementation of the same recipe.
//
// Generator: Philox4x32 with 10 rounds (Salmon et al., SC'11), addressed as
//   counter = (lane_lo, lane_hi, k_lo, (k_hi & 0xFFFFFF) | stream << 24), key = seed
// with stream 0 = event header (lane 0: words 0..2 -> worker, neighbour, tau),
// stream 1 = minibatch (lane m/4, word m%4), stream 2 = synthetic gradient.
// A word u is mapped to {0..m-1} by the high half of the 64-bit product u*m.
#include <algorithm>

#include "internal.hpp"

namespace adpsgd_impl {

void philox4x32_10_host(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t x[4] = {ctr[0], ctr[1], ctr[2], ctr[3]};
    uint32_t ka = key[0], kb = key[1];
    for (int r = 0; r < 10; ++r, ka += 0x9E3779B9u, kb += 0xBB67AE85u) {
        const uint64_t p0 = 0xD2511F53ull * x[0];
        const uint64_t p1 = 0xCD9E8D57ull * x[2];
        const uint32_t y0 = static_cast<uint32_t>(p1 >> 32) ^ x[1] ^ ka;
        const uint32_t y2 = static_cast<uint32_t>(p0 >> 32) ^ x[3] ^ kb;
        x[0] = y0;
        x[1] = static_cast<uint32_t>(p1);
        x[2] = y2;
        x[3] = static_cast<uint32_t>(p0);
    }
    for (int t = 0; t < 4; ++t) out[t] = x[t];
}

namespace {

struct Stream {
    uint32_t key[2];
    uint32_t tag;
    Stream(uint64_t seed, uint32_t stream_tag) : tag(stream_tag << 24) {
        key[0] = static_cast<uint32_t>(seed);
        key[1] = static_cast<uint32_t>(seed >> 32);
    }
    void words(uint64_t k, uint64_t lane, uint32_t out[4]) const {
        const uint32_t ctr[4] = {static_cast<uint32_t>(lane), static_cast<uint32_t>(lane >> 32),
                                 static_cast<uint32_t>(k),
                                 (static_cast<uint32_t>(k >> 32) & 0x00FFFFFFu) | tag};
        philox4x32_10_host(ctr, key, out);
    }
};

inline uint32_t below(uint32_t u, uint32_t m) {
    return static_cast<uint32_t>((static_cast<uint64_t>(u) * m) >> 32);
}

}  // namespace

bool graph_ok(const adpsgd_graph_t* g, std::string& err) {
    if (!g || g->n < 1 || !g->rowptr || (g->rowptr[g->n] > 0 && !g->col)) {
        err = "graph: null pointer or n < 1";
        return false;
    }
    const int32_t n = g->n;
    if (g->rowptr[0] != 0) { err = "graph: rowptr[0] != 0"; return false; }
    for (int32_t v = 0; v < n; ++v)
        if (g->rowptr[v + 1] < g->rowptr[v]) { err = "graph: rowptr not monotone"; return false; }
    std::vector<int32_t> mark(n, -1);
    for (int32_t v = 0; v < n; ++v) {
        for (int32_t e = g->rowptr[v]; e < g->rowptr[v + 1]; ++e) {
            const int32_t u = g->col[e];
            if (u < 0 || u >= n) { err = "graph: neighbour out of range"; return false; }
            if (u == v) { err = "graph: self loop"; return false; }
            if (mark[u] == v) { err = "graph: duplicate edge"; return false; }
            mark[u] = v;
            bool back = false;
            for (int32_t f = g->rowptr[u]; f < g->rowptr[u + 1] && !back; ++f) back = g->col[f] == v;
            if (!back) { err = "graph: not symmetric"; return false; }
        }
    }
    // connected: the problem statement needs information to reach every worker
    std::vector<char> seen(n, 0);
    std::vector<int32_t> stack{0};
    seen[0] = 1;
    int32_t reached = 1;
    while (!stack.empty()) {
        const int32_t v = stack.back();
        stack.pop_back();
        for (int32_t e = g->rowptr[v]; e < g->rowptr[v + 1]; ++e)
            if (!seen[g->col[e]]) { seen[g->col[e]] = 1; ++reached; stack.push_back(g->col[e]); }
    }
    if (reached != n) { err = "graph: not connected"; return false; }
    return true;
}

}  // namespace adpsgd_impl

using namespace adpsgd_impl;

extern "C" int adpsgd_make_schedule(const adpsgd_sched_params_t* p, uint64_t seed, uint64_t k_begin,
                                    int64_t K, int32_t* worker, int32_t* neighbour, int32_t* tau,
                                    int32_t* batch_idx) {
    if (!p || K < 0 || !worker || !neighbour || !tau) return ADPSGD_ERR_ARG;
    std::string graph_err;
    if (!graph_ok(&p->graph, graph_err)) return ADPSGD_ERR_GRAPH;   // the arrays are indexed below
    const int32_t n = p->graph.n;
    if (p->T_max < 0 || p->M < 0) return ADPSGD_ERR_ARG;
    if (p->M > 0 && (!p->rows || !batch_idx)) return ADPSGD_ERR_ARG;
    if (p->tau_mode != 0 && p->tau_mode != 1) return ADPSGD_ERR_ARG;
    if (p->tau_mode == 1 && (!p->tau_num || !p->tau_den)) return ADPSGD_ERR_ARG;

    // cumulative integer weights for the categorical draw of i_k
    std::vector<uint64_t> cum;
    if (p->weight) {
        cum.resize(n);
        uint64_t run = 0;
        for (int32_t v = 0; v < n; ++v) {
            if (p->weight[v] < 0) return ADPSGD_ERR_ARG;
            run += static_cast<uint64_t>(p->weight[v]);
            cum[v] = run;
        }
        if (run == 0 || run >= (1ull << 31)) return ADPSGD_ERR_ARG;
    }
    // geometric staleness: thresholds 2^32 * q^t by an integer recurrence, per worker class
    std::vector<std::vector<uint64_t>> thr;
    if (p->tau_mode == 1) {
        thr.resize(n);
        for (int32_t v = 0; v < n; ++v) {
            if (p->tau_den[v] <= 0 || p->tau_num[v] < 0 || p->tau_num[v] > p->tau_den[v]) return ADPSGD_ERR_ARG;
            thr[v].resize(static_cast<size_t>(p->T_max) + 1);
            uint64_t cur = 1ull << 32;
            thr[v][0] = cur;
            for (int32_t t = 1; t <= p->T_max; ++t) {
                cur = cur * static_cast<uint64_t>(p->tau_num[v]) / static_cast<uint64_t>(p->tau_den[v]);
                thr[v][t] = cur;
            }
        }
    }
    if (p->M > 0)
        for (int32_t v = 0; v < n; ++v)
            if (p->rows[v] < 1) return ADPSGD_ERR_ARG;

    const Stream header(seed, 0), batch(seed, 1);
    for (int64_t q = 0; q < K; ++q) {
        const uint64_t k = k_begin + static_cast<uint64_t>(q);
        uint32_t w[4];
        header.words(k, 0, w);

        int32_t i;
        if (cum.empty()) {
            i = static_cast<int32_t>(below(w[0], static_cast<uint32_t>(n)));
        } else {
            const uint64_t r = below(w[0], static_cast<uint32_t>(cum.back()));
            i = static_cast<int32_t>(std::upper_bound(cum.begin(), cum.end(), r) - cum.begin());
        }
        worker[q] = i;

        const int32_t first = p->graph.rowptr[i], deg = p->graph.rowptr[i + 1] - first;
        neighbour[q] = deg > 0 ? p->graph.col[first + static_cast<int32_t>(below(w[1], static_cast<uint32_t>(deg)))] : i;

        int64_t t = 0;
        if (p->tau_mode == 0) {
            t = below(w[2], static_cast<uint32_t>(p->T_max) + 1u);
        } else {
            const std::vector<uint64_t>& th = thr[i];   // non-increasing in t
            while (t < p->T_max && static_cast<uint64_t>(w[2]) < th[t + 1]) ++t;
        }
        // staleness cannot reach behind event 0: of this call, or of the whole run when the call is a piece of it
        const uint64_t behind = p->piece_of_run ? k : static_cast<uint64_t>(q);
        tau[q] = static_cast<int32_t>(static_cast<uint64_t>(t) < behind ? static_cast<uint64_t>(t) : behind);

        if (p->M > 0) {
            int32_t* dst = batch_idx + q * static_cast<int64_t>(p->M);
            const uint32_t cnt = static_cast<uint32_t>(p->rows[i]);
            for (int32_t m0 = 0; m0 < p->M; m0 += 4) {
                uint32_t b[4];
                batch.words(k, static_cast<uint64_t>(m0 / 4), b);
                for (int32_t t4 = 0; t4 < 4 && m0 + t4 < p->M; ++t4) dst[m0 + t4] = static_cast<int32_t>(below(b[t4], cnt));
            }
        }
    }
    return ADPSGD_OK;
}
