// C-ABI entry points of libadpsgd, part 2: the synchronous comparison schedule.
#include <cmath>
#include <cstring>

#include "handle.hpp"

using namespace adpsgd_impl;

namespace {

int run_sync_steps_impl(adpsgd_t* h, const adpsgd_sync_schedule_t* s, float* loss, adpsgd_gradient_fn fn, void* user) {
    if (!s || s->S < 0) return fail(h, ADPSGD_ERR_ARG, "run_sync_steps: schedule is NULL or S < 0");
    const int64_t S = s->S;
    if (S == 0) return ADPSGD_OK;
    const int32_t n = h->n;
    const bool external = h->o.model == ADPSGD_MODEL_EXTERNAL;
    const bool with_grad = h->o.model != ADPSGD_MODEL_SYNTH;
    const bool with_data = with_grad && !external;
    const int32_t M = with_data ? h->o.M : 0;
    if (S * n > 0x7FFFFFF0) return fail(h, ADPSGD_ERR_ARG, "run_sync_steps: S * n must stay below 2^31 - 16");
    if (sync_tile_cols(n) == 0) return fail(h, ADPSGD_ERR_ARG, "run_sync_steps: at most 1024 workers");
    if (!h->pending.empty())
        return fail(h, ADPSGD_ERR_STATE, "run_sync_steps: the last run_events call looked ahead; finish it with a call without lookahead first");
    if (with_data && !s->batch_idx) return fail(h, ADPSGD_ERR_ARG, "run_sync_steps: batch_idx is NULL");
    if (with_grad && h->n_slots < n)
        return fail(h, ADPSGD_ERR_STATE, "run_sync_steps: the workspace must hold one gradient slot per worker");
    if ((s->w_self == nullptr) != (s->w_edge == nullptr) && h->rowptr[n] > 0)
        return fail(h, ADPSGD_ERR_ARG, "run_sync_steps: give both w_self and w_edge, or neither");

    // ---- validation: nothing is launched and no state changes on failure ----
    const int32_t nnz = h->rowptr[n];
    std::vector<float> w_self(n), w_edge(std::max(nnz, 1));
    if (s->w_self) {
        std::copy(s->w_self, s->w_self + n, w_self.begin());
        if (nnz > 0) std::copy(s->w_edge, s->w_edge + nnz, w_edge.begin());
        for (int32_t i = 0; i < n; ++i) {
            double row = w_self[i];
            if (!(w_self[i] >= 0.0f) || !std::isfinite(w_self[i]))
                return fail(h, ADPSGD_ERR_SCHEDULE, "run_sync_steps: weight negative or not finite");
            for (int32_t e = h->rowptr[i]; e < h->rowptr[i + 1]; ++e) {
                if (!(w_edge[e] >= 0.0f) || !std::isfinite(w_edge[e]))
                    return fail(h, ADPSGD_ERR_SCHEDULE, "run_sync_steps: weight negative or not finite");
                row += w_edge[e];
                const int32_t j = h->col[e];
                bool sym = false;
                for (int32_t f = h->rowptr[j]; f < h->rowptr[j + 1] && !sym; ++f) sym = h->col[f] == i && w_edge[f] == w_edge[e];
                if (!sym) return fail(h, ADPSGD_ERR_SCHEDULE, "run_sync_steps: weights are not symmetric");
            }
            if (std::fabs(row - 1.0) > 1e-5)
                return fail(h, ADPSGD_ERR_SCHEDULE, "run_sync_steps: weights of worker " + std::to_string(i) + " do not sum to 1");
        }
    } else {
        metropolis(h->rowptr, h->col, w_self.data(), w_edge.data());
    }
    for (int64_t t = 0; t < S; ++t)
        if (s->gamma && !std::isfinite(s->gamma[t])) return fail(h, ADPSGD_ERR_SCHEDULE, "run_sync_steps: gamma not finite");
    if (with_data) {
        for (int32_t i = 0; i < n; ++i)
            if (!h->data[i].features) return fail(h, ADPSGD_ERR_STATE, "run_sync_steps: no data loaded for worker " + std::to_string(i));
        for (int64_t t = 0; t < S; ++t)
            for (int32_t i = 0; i < n; ++i) {
                const int32_t* b = s->batch_idx + (t * n + i) * static_cast<int64_t>(M);
                for (int32_t m = 0; m < M; ++m)
                    if (b[m] < 0 || b[m] >= h->data[i].rows)
                        return fail(h, ADPSGD_ERR_SCHEDULE, "run_sync_steps: batch index out of range at iteration " + std::to_string(t));
            }
    }

    // ---- tables: [GradOp x S n][batch_idx S n M][w_self n][w_edge nnz][rowptr n + 1][col nnz] ----
    const size_t bytes_r = with_data ? static_cast<size_t>(S) * n * sizeof(GradOp) : 0;
    const size_t bytes_b = with_data ? static_cast<size_t>(S) * n * M * sizeof(int32_t) : 0;
    const size_t off_b = bytes_r, off_ws = (off_b + bytes_b + 15) & ~size_t(15);
    const size_t off_we = off_ws + static_cast<size_t>(n) * 4, off_rp = off_we + static_cast<size_t>(std::max(nnz, 1)) * 4;
    const size_t off_col = off_rp + static_cast<size_t>(n + 1) * 4, total = off_col + static_cast<size_t>(std::max(nnz, 1)) * 4;
    TableSet& T = h->tables[h->next_table];
    h->next_table ^= 1;
    if (T.in_flight) {
        HIP_TRY(h, hipEventSynchronize(T.done));
        T.in_flight = false;
    }
    HIP_TRY(h, T.stage.reserve(total));
    HIP_TRY(h, T.dev.reserve(total));
    char* stage = static_cast<char*>(T.stage.p);
    if (with_data) {
        GradOp* rops = reinterpret_cast<GradOp*>(stage);
        for (int64_t t = 0; t < S; ++t)
            for (int32_t i = 0; i < n; ++i)
                rops[t * n + i] = GradOp{i, i, static_cast<int32_t>(t * n + i), -1, 0.0f, 0,
                                         h->data[i].features, h->data[i].targets, h->data[i].ld, nullptr};
        std::memcpy(stage + off_b, s->batch_idx, bytes_b);
    }
    std::memcpy(stage + off_ws, w_self.data(), static_cast<size_t>(n) * 4);
    std::memcpy(stage + off_we, w_edge.data(), static_cast<size_t>(std::max(nnz, 1)) * 4);
    std::memcpy(stage + off_rp, h->rowptr.data(), static_cast<size_t>(n + 1) * 4);
    if (nnz > 0) std::memcpy(stage + off_col, h->col.data(), static_cast<size_t>(nnz) * 4);
    HIP_TRY(h, hipMemcpyAsync(T.dev.p, T.stage.p, total, hipMemcpyHostToDevice, h->stream));
    const char* dev = static_cast<const char*>(T.dev.p);
    const GradOp* d_rops = reinterpret_cast<const GradOp*>(dev);
    const int32_t* d_batch = reinterpret_cast<const int32_t*>(dev + off_b);

    int32_t group = 1;
    size_t off_coef = 0;
    if (with_data) {
        if (h->o.model == ADPSGD_MODEL_MLP) {
            group = std::min<int32_t>(n, 64);
            HIP_TRY(h, h->grad_scratch.reserve(mlp_scratch_bytes(group, M, h->o.mlp_in, h->o.mlp_hidden, h->o.mlp_out)));
        } else {
            group = n;
            const size_t partial_bytes = static_cast<size_t>(group) * (M + 1) * linear_grad_chunks(h->d) * 4;
            off_coef = (partial_bytes + 255) & ~size_t(255);
            HIP_TRY(h, h->grad_scratch.reserve(off_coef + static_cast<size_t>(group) * M * 4));
        }
    }
    const bool profile = (h->o.flags & ADPSGD_FLAG_PROFILE) != 0;
    // a ring in canonical order: row i mixes with rows i - 1 and i + 1 only, listed in that order
    bool ring = n >= 3 && nnz == 2 * n;
    for (int32_t i = 0; ring && i < n; ++i)
        ring = h->rowptr[i] == 2 * i && h->col[2 * i] == (i + n - 1) % n && h->col[2 * i + 1] == (i + 1) % n;
    // Iterations that come in pairs write the new models to a second matrix and back (blocks in row order: faster
    // than mixing in place, on a ring and on any other graph); an odd iteration runs in place first, so the models
    // end where the caller keeps them.  Without memory for the second matrix every iteration runs in place.
    float* other = nullptr;
    if (S >= 2 && !(h->o.flags & ADPSGD_FLAG_SYNC_IN_PLACE) && !h->sync_other_refused && sync_out_of_place_ok(n, h->d)) {
        if (h->sync_other.reserve(static_cast<size_t>(n) * static_cast<size_t>(h->o.ldx) * sizeof(float)) == hipSuccess) {
            other = static_cast<float*>(h->sync_other.p);
        } else {
            (void)hipGetLastError();
            h->sync_other_refused = true;
        }
    }
    float* cur = h->o.X;
    float* slots = static_cast<float*>(h->o.workspace);
    const float gscale = h->o.grad_sum ? 1.0f : 1.0f / static_cast<float>(std::max(M, 1));
    std::vector<adpsgd_grad_request_t> requests(external ? n : 0);
    for (int64_t t = 0; t < S; ++t) {
        if (external) {       // every worker's gradient at the model the iteration starts from, into slot i
            for (int32_t i = 0; i < n; ++i)
                requests[i] = adpsgd_grad_request_t{i, 0, t * n + i, cur + static_cast<int64_t>(i) * h->o.ldx,
                                                    slots + static_cast<int64_t>(i) * h->o.ldx};
            if (fn(user, n, requests.data(), h->stream) != 0) {
                if (cur != h->o.X)     // the models of the iterations done so far go back where the caller keeps them
                    (void)hipMemcpyAsync(h->o.X, cur, static_cast<size_t>(n) * static_cast<size_t>(h->o.ldx) * sizeof(float),
                                         hipMemcpyDeviceToDevice, h->stream);
                (void)hipStreamSynchronize(h->stream);
                return fail(h, ADPSGD_ERR_CALLBACK, "run_sync_steps_with: the gradient function failed in iteration " + std::to_string(t));
            }
            ++h->stats.grad_launches;
        }
        for (int32_t g0 = 0; with_data && g0 < n; g0 += group) {
            const int32_t cnt = std::min<int32_t>(group, n - g0);
            int launches = 0;
            if (h->o.model == ADPSGD_MODEL_MLP) {
                MlpGradArgs a{cur, h->o.Xbf16, h->o.ldx, h->o.mlp_in, h->o.mlp_hidden, h->o.mlp_out, d_rops + t * n + g0, cnt, M,
                              d_batch + (t * n + g0) * static_cast<int64_t>(M), slots, gscale, loss,
                              h->grad_scratch.p, false, false};
                HIP_TRY(h, launch_mlp_gradient(a, h->stream, &launches));
            } else {
                LinearGradArgs a{h->o.model, cur, h->o.ldx, h->d, d_rops + t * n + g0, cnt, M, d_batch,
                                 slots, gscale, h->o.lambda,
                                 static_cast<float*>(h->grad_scratch.p),
                                 reinterpret_cast<float*>(static_cast<char*>(h->grad_scratch.p) + off_coef), loss, false};
                HIP_TRY(h, launch_linear_gradient(a, h->stream, &launches));
            }
            h->stats.grad_launches += launches;
        }
        hipEvent_t e0 = nullptr, e1 = nullptr;
        if (profile) {
            e0 = take_event(h);
            e1 = take_event(h);
            if (!e0 || !e1) return fail(h, ADPSGD_ERR_HIP, "run_sync_steps: hipEventCreate failed");
            HIP_TRY(h, hipEventRecord(e0, h->stream));
        }
        // in place while an odd number of iterations is left with the models at home, else into the other matrix
        float* dst = other && !(cur == h->o.X && ((S - t) & 1)) ? (cur == h->o.X ? other : h->o.X) : nullptr;
        SyncArgs a{cur, h->o.ldx, h->d, n,
                   reinterpret_cast<const int32_t*>(dev + off_rp), reinterpret_cast<const int32_t*>(dev + off_col),
                   reinterpret_cast<const float*>(dev + off_ws), reinterpret_cast<const float*>(dev + off_we),
                   with_grad ? slots : nullptr, h->o.model == ADPSGD_MODEL_MLP ? h->o.Xbf16 : nullptr,
                   s->gamma ? s->gamma[t] : h->o.gamma, h->o.synth_std, h->o.synth_seed,
                   h->events_done + static_cast<uint64_t>(t) * static_cast<uint64_t>(n), !with_grad,
                   h->o.V, h->o.momentum, h->o.weight_decay, ring, dst};
        HIP_TRY(h, launch_sync_mix_apply(a, h->stream));
        if (dst) cur = dst;
        ++h->stats.fused_launches;
        if (profile) {
            HIP_TRY(h, hipEventRecord(e1, h->stream));
            h->ev_fused.push_back({e0, e1});
        }
    }
    HIP_TRY(h, hipEventRecord(T.done, h->stream));
    T.in_flight = true;
    h->events_done += static_cast<uint64_t>(S) * static_cast<uint64_t>(n);
    h->stats.events += S * n;
    h->stats.rounds += S;
    return ADPSGD_OK;
}

}  // namespace

extern "C" int adpsgd_run_sync_steps(adpsgd_t* h, const adpsgd_sync_schedule_t* s, float* loss) {
    if (!h) return ADPSGD_ERR_ARG;
    if (h->o.model == ADPSGD_MODEL_EXTERNAL)
        return fail(h, ADPSGD_ERR_STATE, "run_sync_steps: caller-supplied gradients need adpsgd_run_sync_steps_with");
    return run_sync_steps_impl(h, s, loss, nullptr, nullptr);
}

extern "C" int adpsgd_run_sync_steps_with(adpsgd_t* h, const adpsgd_sync_schedule_t* s, adpsgd_gradient_fn fn, void* user) {
    if (!h) return ADPSGD_ERR_ARG;
    if (h->o.model != ADPSGD_MODEL_EXTERNAL)
        return fail(h, ADPSGD_ERR_STATE, "run_sync_steps_with: the handle was not created with ADPSGD_MODEL_EXTERNAL");
    if (!fn) return fail(h, ADPSGD_ERR_ARG, "run_sync_steps_with: fn is NULL");
    return run_sync_steps_impl(h, s, nullptr, fn, user);
}

extern "C" int adpsgd_metropolis_weights(const adpsgd_graph_t* graph, float* w_self, float* w_edge) {
    std::string err;
    if (!graph || !w_self || !graph_ok(graph, err)) return ADPSGD_ERR_GRAPH;
    if (graph->rowptr[graph->n] > 0 && !w_edge) return ADPSGD_ERR_ARG;
    std::vector<int32_t> rowptr(graph->rowptr, graph->rowptr + graph->n + 1), col(graph->col, graph->col + graph->rowptr[graph->n]);
    metropolis(rowptr, col, w_self, w_edge);
    return ADPSGD_OK;
}
