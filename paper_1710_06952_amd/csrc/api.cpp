// C-ABI entry points of libadpsgd, part 1: handle life cycle, validation, per-call planning and
// the per-round launch loop of adpsgd_run_events.  See include/adpsgd.h for the contract.
#include <cmath>
#include <cstring>
#include <memory>

#include "handle.hpp"

namespace adpsgd_impl {

hipError_t DevBuf::reserve(size_t bytes) {
    if (bytes <= cap) return hipSuccess;
    if (p) {
        // kernels enqueued earlier may still read the old buffer
        hipError_t e = hipDeviceSynchronize();
        if (e == hipSuccess) e = hipFree(p);
        p = nullptr;
        cap = 0;
        if (e != hipSuccess) return e;
    }
    size_t want = std::max<size_t>(bytes, 256);
    hipError_t e = hipMalloc(&p, want);
    if (e != hipSuccess) { p = nullptr; return e; }
    cap = want;
    return hipSuccess;
}
void DevBuf::release() {
    if (p) (void)hipFree(p);
    p = nullptr;
    cap = 0;
}

namespace {
thread_local std::string g_create_error;
}  // namespace

const std::string& create_error() { return g_create_error; }

int fail(adpsgd_t* h, int code, const std::string& msg) {
    if (h) h->err = msg;
    else g_create_error = msg;
    return code;
}
int hip_fail(adpsgd_t* h, hipError_t e, const char* what) {
    return fail(h, ADPSGD_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

bool is_neighbour(const adpsgd_t* h, int32_t i, int32_t j) {
    if (j == i) return true;     // W_k = I: a gradient step without averaging
    const int32_t b = h->rowptr[i], e = h->rowptr[i + 1];
    for (int32_t t = b; t < e; ++t)
        if (h->col[t] == j) return true;
    return false;
}

void metropolis(const std::vector<int32_t>& rowptr, const std::vector<int32_t>& col, float* w_self, float* w_edge) {
    const int32_t n = static_cast<int32_t>(rowptr.size()) - 1;
    for (int32_t i = 0; i < n; ++i) {
        const int32_t di = rowptr[i + 1] - rowptr[i];
        double self = 1.0;
        for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            const int32_t j = col[e], dj = rowptr[j + 1] - rowptr[j];
            const double w = 1.0 / (1.0 + static_cast<double>(std::max(di, dj)));
            w_edge[e] = static_cast<float>(w);
            self -= w;
        }
        w_self[i] = static_cast<float>(self);
    }
}

hipEvent_t take_event(adpsgd_t* h) {
    if (!h->ev_pool.empty()) {
        hipEvent_t e = h->ev_pool.back();
        h->ev_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

// Fold the timings of finished launches into the statistics (synchronises the stream).
int drain_profile(adpsgd_t* h) {
    if (h->ev_fused.empty() && h->ev_grad.empty()) return ADPSGD_OK;
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    for (int which = 0; which < 2; ++which) {
        auto& list = which == 0 ? h->ev_fused : h->ev_grad;
        double& total = which == 0 ? h->stats.fused_ms : h->stats.grad_ms;
        for (auto& pr : list) {
            float ms = 0.0f;
            HIP_TRY(h, hipEventElapsedTime(&ms, pr.first, pr.second));
            total += ms;
            h->ev_pool.push_back(pr.first);
            h->ev_pool.push_back(pr.second);
        }
        list.clear();
    }
    return ADPSGD_OK;
}

}  // namespace adpsgd_impl

using namespace adpsgd_impl;

extern "C" const char* adpsgd_last_error(const adpsgd_t* h) { return h ? h->err.c_str() : create_error().c_str(); }

extern "C" int adpsgd_create(adpsgd_t** out, const adpsgd_graph_t* graph, int64_t d, const adpsgd_opts_t* opts) {
    if (!out) return fail(nullptr, ADPSGD_ERR_ARG, "create: out is NULL");
    *out = nullptr;
    if (!graph || !opts) return fail(nullptr, ADPSGD_ERR_ARG, "create: graph or opts is NULL");
    std::string msg;
    if (!graph_ok(graph, msg)) return fail(nullptr, ADPSGD_ERR_GRAPH, msg);
    const int32_t n = graph->n;
    if (n > 65535) return fail(nullptr, ADPSGD_ERR_ARG, "create: at most 65535 workers");
    if (d < 1) return fail(nullptr, ADPSGD_ERR_ARG, "create: d < 1");
    const adpsgd_opts_t& o = *opts;
    if (o.model < ADPSGD_MODEL_LSQ || o.model > ADPSGD_MODEL_EXTERNAL) return fail(nullptr, ADPSGD_ERR_ARG, "create: unknown model");
    const bool external = o.model == ADPSGD_MODEL_EXTERNAL;
    if (!o.X || !aligned16(o.X)) return fail(nullptr, ADPSGD_ERR_ARG, "create: X is NULL or not 16-byte aligned");
    if (o.ldx < d || (o.ldx & 3)) return fail(nullptr, ADPSGD_ERR_ARG, "create: ldx must be >= d and a multiple of 4");
    if (o.T_max < 0) return fail(nullptr, ADPSGD_ERR_ARG, "create: T_max < 0");
    if (!std::isfinite(o.gamma)) return fail(nullptr, ADPSGD_ERR_ARG, "create: gamma not finite");
    int32_t n_slots = 0;
    if (o.model != ADPSGD_MODEL_SYNTH) {
        if (!external && (o.M < 1 || o.M > 65536)) return fail(nullptr, ADPSGD_ERR_ARG, "create: minibatch size M outside [1, 65536]");
        if (!o.workspace || !aligned16(o.workspace)) return fail(nullptr, ADPSGD_ERR_ARG, "create: workspace is NULL or misaligned");
        const int64_t slot_bytes = o.ldx * 4;
        const int64_t have = o.workspace_bytes / slot_bytes;
        if (have < static_cast<int64_t>(o.T_max) + 1)
            return fail(nullptr, ADPSGD_ERR_ARG, "create: workspace smaller than (T_max + 1) gradient slots");
        n_slots = static_cast<int32_t>(std::min<int64_t>(have, kMaxSlots));
    }
    if (o.model == ADPSGD_MODEL_MLP) {
        if (o.mlp_in < 1 || o.mlp_hidden < 1 || o.mlp_out < 1 ||
            d != static_cast<int64_t>(o.mlp_in) * o.mlp_hidden + o.mlp_hidden +
                     static_cast<int64_t>(o.mlp_hidden) * o.mlp_out + o.mlp_out)
            return fail(nullptr, ADPSGD_ERR_ARG, "create: d does not match the MLP layer sizes");
        if (!o.Xbf16 || !aligned16(o.Xbf16)) return fail(nullptr, ADPSGD_ERR_ARG, "create: Xbf16 is NULL or misaligned");
        if (o.ldx & 7) return fail(nullptr, ADPSGD_ERR_ARG, "create: ldx must be a multiple of 8 for the MLP");
        if (mlp_scratch_bytes(1, o.M, o.mlp_in, o.mlp_hidden, o.mlp_out) == 0)
            return fail(nullptr, ADPSGD_ERR_ARG, "create: MLP shape not supported by the gradient kernel");
    }
    if (!std::isfinite(o.momentum) || !std::isfinite(o.weight_decay))
        return fail(nullptr, ADPSGD_ERR_ARG, "create: momentum or weight_decay not finite");
    if ((o.momentum != 0.0f || o.weight_decay != 0.0f) && (!o.V || !aligned16(o.V)))
        return fail(nullptr, ADPSGD_ERR_ARG, "create: momentum / weight decay need the buffer V (16-byte aligned)");
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || count < 1)
        return fail(nullptr, ADPSGD_ERR_HIP, "create: no HIP device available");

    std::unique_ptr<adpsgd> h(new (std::nothrow) adpsgd);
    if (!h) return fail(nullptr, ADPSGD_ERR_ARG, "create: out of host memory");
    h->n = n;
    h->d = d;
    h->o = o;
    h->rowptr.assign(graph->rowptr, graph->rowptr + n + 1);
    h->col.assign(graph->col, graph->col + graph->rowptr[n]);
    h->data.resize(n);
    h->n_slots = n_slots;
    h->stream = static_cast<hipStream_t>(o.stream);
    h->streaming = static_cast<int64_t>(n) * o.ldx * 4 > kStreamingThreshold;
    h->stats.slots = n_slots;
    for (auto& t : h->tables) {
        hipError_t e = hipEventCreateWithFlags(&t.done, hipEventDisableTiming);
        if (e != hipSuccess) {
            for (auto& u : h->tables)
                if (u.done) (void)hipEventDestroy(u.done);
            return hip_fail(nullptr, e, "create: hipEventCreate");
        }
    }
    *out = h.release();
    return ADPSGD_OK;
}

extern "C" void adpsgd_destroy(adpsgd_t* h) {
    if (!h) return;
    (void)hipStreamSynchronize(h->stream);
    for (auto& t : h->tables) {
        t.stage.release();
        t.dev.release();
        if (t.done) (void)hipEventDestroy(t.done);
    }
    for (auto& pr : h->ev_fused) { (void)hipEventDestroy(pr.first); (void)hipEventDestroy(pr.second); }
    for (auto& pr : h->ev_grad) { (void)hipEventDestroy(pr.first); (void)hipEventDestroy(pr.second); }
    for (auto e : h->ev_pool) (void)hipEventDestroy(e);
    h->grad_scratch.release();
    h->comp_rows.release();
    h->diag.release();
    h->sync_other.release();
    delete h;
}

extern "C" int adpsgd_load_data(adpsgd_t* h, int32_t worker, const void* features, int64_t rows, int64_t ld,
                                const void* targets) {
    if (!h) return ADPSGD_ERR_ARG;
    if (h->o.model == ADPSGD_MODEL_SYNTH || h->o.model == ADPSGD_MODEL_EXTERNAL)
        return fail(h, ADPSGD_ERR_STATE, "load_data: this model takes no data");
    if (worker < 0 || worker >= h->n) return fail(h, ADPSGD_ERR_ARG, "load_data: worker out of range");
    if (!features || !targets || rows < 1 || rows > 0x7FFFFFFF) return fail(h, ADPSGD_ERR_ARG, "load_data: null data or bad row count");
    if (!aligned16(features)) return fail(h, ADPSGD_ERR_ARG, "load_data: features not 16-byte aligned");
    if (h->o.model == ADPSGD_MODEL_MLP) {
        if (ld < h->o.mlp_in || (ld & 7)) return fail(h, ADPSGD_ERR_ARG, "load_data: ld must be >= mlp_in and a multiple of 8");
    } else {
        if (ld < h->d || (ld & 3)) return fail(h, ADPSGD_ERR_ARG, "load_data: ld must be >= d and a multiple of 4");
    }
    WorkerData& w = h->data[worker];
    w.features = features;
    w.targets = targets;
    w.rows = rows;
    w.ld = ld;
    return ADPSGD_OK;
}

extern "C" int adpsgd_set_models(adpsgd_t* h, const float* x, int64_t ld_in, int32_t on_device) {
    if (!h || !x) return h ? fail(h, ADPSGD_ERR_ARG, "set_models: x is NULL") : ADPSGD_ERR_ARG;
    if (ld_in != 0 && ld_in < h->d) return fail(h, ADPSGD_ERR_ARG, "set_models: ld_in < d");
    h->pending.clear();      // gradients evaluated at the old models are dropped
    h->pending_batch.clear();
    const hipMemcpyKind kind = on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
    if (ld_in == 0) {
        const float* src = x;
        if (!on_device) {
            HIP_TRY(h, hipStreamSynchronize(h->stream));
            HIP_TRY(h, h->diag.reserve(static_cast<size_t>(h->d) * 4));
            HIP_TRY(h, hipMemcpy(h->diag.p, x, static_cast<size_t>(h->d) * 4, hipMemcpyHostToDevice));
            src = static_cast<const float*>(h->diag.p);
        }
        HIP_TRY(h, launch_broadcast_rows(h->o.X, h->o.ldx, h->d, h->n, src, h->stream));
    } else {
        HIP_TRY(h, hipMemsetAsync(h->o.X, 0, static_cast<size_t>(h->n) * h->o.ldx * 4, h->stream));
        HIP_TRY(h, hipMemcpy2DAsync(h->o.X, static_cast<size_t>(h->o.ldx) * 4, x, static_cast<size_t>(ld_in) * 4,
                                    static_cast<size_t>(h->d) * 4, h->n, kind, h->stream));
    }
    if (h->o.model == ADPSGD_MODEL_MLP)
        HIP_TRY(h, launch_refresh_bf16(h->o.X, h->o.Xbf16, h->o.ldx, h->n, h->stream));
    if (h->o.V) HIP_TRY(h, hipMemsetAsync(h->o.V, 0, static_cast<size_t>(h->n) * h->o.ldx * 4, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return ADPSGD_OK;
}

namespace {

// Checks a schedule against the documented constraints; nothing is launched and no state changes
// when it fails.
int validate_schedule(adpsgd_t* h, const adpsgd_schedule_t* s, bool with_data, int32_t M, int64_t n_extra) {
    const int64_t K = s->K;
    const int64_t n_pending = static_cast<int64_t>(h->pending.size());
    if (s->lookahead < 0 || s->lookahead > K) return fail(h, ADPSGD_ERR_ARG, "run_events: lookahead outside [0, K]");
    if (s->lookahead > 0 && h->o.model == ADPSGD_MODEL_SYNTH)
        return fail(h, ADPSGD_ERR_ARG, "run_events: the synthetic-gradient model has no stale reads to look ahead to");
    if (K < n_pending)
        return fail(h, ADPSGD_ERR_SCHEDULE, "run_events: the call must start with the " + std::to_string(n_pending) +
                                                " events the previous call looked ahead to");
    for (int64_t k = 0; k < n_pending; ++k) {
        const PendingEvent& e = h->pending[k];
        bool same = s->worker[k] == e.worker && s->tau[k] == e.tau;
        for (int32_t m = 0; same && m < M; ++m) same = s->batch_idx[k * static_cast<int64_t>(M) + m] == h->pending_batch[k * static_cast<int64_t>(M) + m];
        if (!same)
            return fail(h, ADPSGD_ERR_SCHEDULE, "run_events: event " + std::to_string(k) + " differs from the event the previous call looked ahead to");
    }
    if (s->extra_ptr) {
        if (s->extra_ptr[0] != 0 || n_extra < 0 || (n_extra > 0 && (!s->extra_a || !s->extra_b)))
            return fail(h, ADPSGD_ERR_ARG, "run_events: malformed extra-pair arrays");
        std::vector<int64_t> stamp(h->n, -1);
        for (int64_t k = 0; k < K; ++k) {
            if (s->extra_ptr[k + 1] < s->extra_ptr[k] || s->extra_ptr[k + 1] > n_extra)
                return fail(h, ADPSGD_ERR_SCHEDULE, "run_events: extra_ptr not monotone at event " + std::to_string(k));
            if (s->worker[k] >= 0 && s->worker[k] < h->n) stamp[s->worker[k]] = k;
            if (s->neighbour[k] >= 0 && s->neighbour[k] < h->n) stamp[s->neighbour[k]] = k;
            for (int64_t q = s->extra_ptr[k]; q < s->extra_ptr[k + 1]; ++q) {
                const int32_t a = s->extra_a[q], b = s->extra_b[q];
                if (a < 0 || a >= h->n || b < 0 || b >= h->n || a == b || !is_neighbour(h, a, b))
                    return fail(h, ADPSGD_ERR_SCHEDULE, "run_events: extra pair is not an edge of the graph at event " + std::to_string(k));
                if (stamp[a] == k || stamp[b] == k)
                    return fail(h, ADPSGD_ERR_SCHEDULE, "run_events: the pairs of one event must be disjoint (event " + std::to_string(k) + ")");
                stamp[a] = stamp[b] = k;
            }
        }
    }
    for (int64_t k = 0; k < K; ++k) {
        const int32_t i = s->worker[k], j = s->neighbour[k];
        if (i < 0 || i >= h->n || j < 0 || j >= h->n)
            return fail(h, ADPSGD_ERR_SCHEDULE, "run_events: worker or neighbour out of range at event " + std::to_string(k));
        if (!is_neighbour(h, i, j))
            return fail(h, ADPSGD_ERR_SCHEDULE, "run_events: neighbour is not adjacent to worker at event " + std::to_string(k));
        const bool carried = k < n_pending && h->pending[k].slot >= 0;      // read before this call began
        if (s->tau[k] < 0 || s->tau[k] > h->o.T_max || (carried ? s->tau[k] <= k : s->tau[k] > k))
            return fail(h, ADPSGD_ERR_SCHEDULE, "run_events: tau outside [0, min(k, T_max)] at event " + std::to_string(k));
        if (s->gamma && !std::isfinite(s->gamma[k]))
            return fail(h, ADPSGD_ERR_SCHEDULE, "run_events: gamma not finite at event " + std::to_string(k));
        if (with_data) {
            const WorkerData& w = h->data[i];
            if (!w.features) return fail(h, ADPSGD_ERR_STATE, "run_events: no data loaded for worker " + std::to_string(i));
            const int32_t* b = s->batch_idx + k * static_cast<int64_t>(M);
            for (int32_t m = 0; m < M; ++m)
                if (b[m] < 0 || b[m] >= w.rows)
                    return fail(h, ADPSGD_ERR_SCHEDULE, "run_events: batch index out of range at event " + std::to_string(k));
        }
    }
    return ADPSGD_OK;
}

// What one call of run_events works with: the paths taken, the plan sorted by round, the tables.
struct EventCall {
    const adpsgd_schedule_t* s = nullptr;
    int64_t K = 0;              // events in the arrays
    int64_t A = 0;              // of which this call applies the first A (the others are looked ahead to)
    int64_t n_extra = 0;        // extra averaging pairs of the applied events
    int32_t M = 0;
    bool external = false;      // gradients from the caller's function
    bool with_grad = false;     // the events carry gradients held in pending slots (every model but SYNTH)
    bool mlp_comp = false;      // perceptron, wait-free variant: compensated bf16 rows
    bool ext_comp = false;      // caller's function, wait-free variant: compensated fp32 rows
    bool factored = false;      // perceptron: dW1 stays in factored form until the update kernel
    bool lin_factored = false;  // least squares on long models: the gradient stays M coefficients
    Plan plan;
    std::vector<int64_t> u_off, r_off;      // first update / gradient operation of every round
    int32_t group = 1;                      // gradients of a round are launched in groups of this many operations
    TableSet* T = nullptr;
    PairOp* uops = nullptr;                 // pinned staging, sorted by round
    GradOp* rops = nullptr;
    const PairOp* d_uops = nullptr;         // the device copy
    const GradOp* d_rops = nullptr;
    const int32_t* d_batch = nullptr;
    int32_t* batch_r = nullptr;             // perceptron: the minibatch indices again, in the order of rops ...
    int32_t* batch_u = nullptr;             // ... and of uops (pinned staging)
    const int32_t* d_batch_r = nullptr;
    const int32_t* d_batch_u = nullptr;
    size_t off_coef = 0;                    // linear models: offset of the coefficients in the gradient scratch
};

// Validation, choice of paths, plan of rounds, counting sort of the operations by round.
int prepare_call(adpsgd_t* h, const adpsgd_schedule_t* s, EventCall& c) {
    c.s = s;
    c.K = s->K;
    if (c.K > 0x7FFFFFF0) return fail(h, ADPSGD_ERR_ARG, "run_events: at most 2^31 - 16 events per call");
    if (!s->worker || !s->neighbour || !s->tau) return fail(h, ADPSGD_ERR_ARG, "run_events: null schedule array");
    c.external = h->o.model == ADPSGD_MODEL_EXTERNAL;
    c.with_grad = h->o.model != ADPSGD_MODEL_SYNTH;
    const bool with_data = c.with_grad && !c.external;
    c.M = with_data ? h->o.M : 0;
    if (with_data && !s->batch_idx) return fail(h, ADPSGD_ERR_ARG, "run_events: batch_idx is NULL");
    const int rc_valid = validate_schedule(h, s, with_data, c.M, s->extra_ptr ? s->extra_ptr[c.K] : 0);
    if (rc_valid != ADPSGD_OK) return rc_valid;
    c.A = c.K - s->lookahead;
    c.n_extra = s->extra_ptr ? s->extra_ptr[c.A] : 0;
    std::vector<int32_t> carried_slot;
    if (!h->pending.empty()) {
        carried_slot.assign(static_cast<size_t>(c.K), -1);
        for (size_t k = 0; k < h->pending.size(); ++k) carried_slot[k] = h->pending[k].slot;
    }
    const int32_t* carried = carried_slot.empty() ? nullptr : carried_slot.data();

    // the wait-free variant reads the pending gradient as a dense vector, so it keeps the dense form
    const bool comp = h->o.local_compensation != 0, dense = (h->o.flags & ADPSGD_FLAG_DENSE_GRADIENT) != 0;
    c.mlp_comp = h->o.model == ADPSGD_MODEL_MLP && comp;
    c.ext_comp = c.external && comp;
    c.factored = h->o.model == ADPSGD_MODEL_MLP && !dense && !comp && mlp_can_factor(h->o.mlp_in, h->o.mlp_hidden, c.M);
    c.lin_factored = with_data && !dense && !comp && linear_can_factor(h->o.model, h->d, c.M, h->o.ldx);

    std::string perr;
    const int rc = plan_rounds(h->n, c.K, s->worker, s->neighbour, s->tau, h->n_slots, c.with_grad, c.plan, perr,
                               s->extra_ptr, s->extra_a, s->extra_b, comp, c.A, carried);
    if (rc != ADPSGD_OK) return fail(h, rc, perr);
    if ((h->o.flags & ADPSGD_FLAG_VERIFY_PLAN) &&
        !verify_plan(h->n, c.K, s->worker, s->neighbour, s->tau, h->n_slots, c.with_grad, c.plan, perr, s->extra_ptr, s->extra_a,
                     s->extra_b, c.A, carried))
        return fail(h, ADPSGD_ERR_STATE, perr);

    const int32_t R = c.plan.n_rounds;
    c.u_off.assign(static_cast<size_t>(R) + 1, 0);
    c.r_off.assign(static_cast<size_t>(R) + 1, 0);
    for (int64_t k = 0; k < c.K; ++k) {
        if (k < c.A) c.u_off[c.plan.u_round[k] + 1] += 1 + (s->extra_ptr ? s->extra_ptr[k + 1] - s->extra_ptr[k] : 0);
        if (c.with_grad && c.plan.r_round[k] >= 0) ++c.r_off[c.plan.r_round[k] + 1];      // not carried, not left to the next call
    }
    int64_t max_r = 0;
    for (int32_t r = 0; r < R; ++r) {
        max_r = std::max(max_r, c.r_off[r + 1]);
        c.u_off[r + 1] += c.u_off[r];
        c.r_off[r + 1] += c.r_off[r];
    }
    if (c.with_grad)
        c.group = static_cast<int32_t>(std::min<int64_t>(std::max<int64_t>(max_r, 1), h->o.model == ADPSGD_MODEL_MLP ? 64 : 65535));
    return ADPSGD_OK;
}

// The update operations of event k (its own pair and the extra pairs of its W_k), appended to the event's round.
void fill_update(adpsgd_t* h, EventCall& c, int64_t k, std::vector<int64_t>& u_fill) {
    const adpsgd_schedule_t* s = c.s;
    const uint64_t gk = h->events_done + static_cast<uint64_t>(k);
    const int32_t ur = c.plan.u_round[k];
    const bool factors = c.factored || c.lin_factored;
    if (c.batch_u) std::memcpy(c.batch_u + u_fill[ur] * c.M, s->batch_idx + k * static_cast<int64_t>(c.M), static_cast<size_t>(c.M) * 4);
    PairOp& u = c.uops[u_fill[ur]++];
    u.i = s->worker[k];
    u.j = s->neighbour[k];
    u.k_lo = static_cast<uint32_t>(gk);
    u.k_hi = static_cast<uint32_t>(gk >> 32);
    u.gamma = s->gamma ? s->gamma[k] : h->o.gamma;
    u.slot = c.with_grad ? c.plan.slot[k] : 0;
    u.flags = 0;
    u.event = static_cast<int32_t>(k);
    u.features = factors ? h->data[u.i].features : nullptr;
    u.feat_ld = factors ? h->data[u.i].ld : 0;
    if (s->extra_ptr)
        for (int64_t q = s->extra_ptr[k]; q < s->extra_ptr[k + 1]; ++q)
            c.uops[u_fill[ur]++] = PairOp{s->extra_a[q], s->extra_b[q], 0u, 0u, 0.0f, 0, 1, 0, nullptr, 0};
}

// The stale read and gradient of event k, appended to its round.
void fill_gradient(adpsgd_t* h, EventCall& c, int64_t k, std::vector<int64_t>& r_fill) {
    const adpsgd_schedule_t* s = c.s;
    const int32_t rr = c.plan.r_round[k];
    const int64_t at = r_fill[rr]++;
    if (c.batch_r) std::memcpy(c.batch_r + at * c.M, s->batch_idx + k * static_cast<int64_t>(c.M), static_cast<size_t>(c.M) * 4);
    GradOp& g = c.rops[at];
    g.worker = s->worker[k];
    g.slot = c.plan.slot[k];
    g.event = static_cast<int32_t>(k);
    const int64_t kp = c.plan.prev[k];
    g.comp_slot = kp >= 0 ? c.plan.slot[kp] : -1;
    g.comp_gamma = kp >= 0 ? (s->gamma ? s->gamma[kp] : h->o.gamma) : 0.0f;
    g.count = 0;
    const WorkerData& w = h->data[g.worker];
    g.features = w.features;
    g.targets = w.targets;
    g.ld = w.ld;
    g.xrow_bf16 = nullptr;
    if (c.mlp_comp && kp >= 0)      // one compensated row per operation of a launch group
        g.xrow_bf16 = static_cast<uint16_t*>(h->comp_rows.p) + ((at - c.r_off[rr]) % c.group) * h->o.ldx;
}

// Tables [PairOp x (K + extra pairs)][GradOp x K][batch_idx K x M], filled in pinned memory in round
// order and uploaded with one copy; scratch memory of the gradient kernels.
int upload_tables(adpsgd_t* h, EventCall& c) {
    const adpsgd_schedule_t* s = c.s;
    const int64_t K = c.K;
    const int32_t M = c.M;
    if (c.mlp_comp) HIP_TRY(h, h->comp_rows.reserve(static_cast<size_t>(c.group) * h->o.ldx * sizeof(uint16_t)));
    if (c.ext_comp) HIP_TRY(h, h->comp_rows.reserve(static_cast<size_t>(c.group) * h->o.ldx * sizeof(float)));
    const size_t bytes_u = static_cast<size_t>(c.A + c.n_extra) * sizeof(PairOp);
    const size_t bytes_r = c.with_grad ? static_cast<size_t>(K) * sizeof(GradOp) : 0;
    const size_t bytes_b = static_cast<size_t>(K) * M * sizeof(int32_t);
    const size_t off_r = bytes_u, off_b = (off_r + bytes_r + 15) & ~size_t(15);
    // the perceptron's kernels read the indices by operation instead of by event: one copy in the order of the
    // gradient operations, one in the order of the update operations (rows of averaging-only pairs stay zero)
    const bool by_op = h->o.model == ADPSGD_MODEL_MLP;
    const size_t bytes_br = by_op ? bytes_b : 0, bytes_bu = by_op ? static_cast<size_t>(c.A + c.n_extra) * M * sizeof(int32_t) : 0;
    const size_t off_br = off_b + (by_op ? 0 : bytes_b), off_bu = off_br + bytes_br;
    const size_t total = off_bu + bytes_bu;

    TableSet& T = h->tables[h->next_table];
    h->next_table ^= 1;
    if (T.in_flight) {
        HIP_TRY(h, hipEventSynchronize(T.done));
        T.in_flight = false;
    }
    HIP_TRY(h, T.stage.reserve(total));
    HIP_TRY(h, T.dev.reserve(total));
    c.T = &T;
    char* stage = static_cast<char*>(T.stage.p);
    c.uops = reinterpret_cast<PairOp*>(stage);
    c.rops = reinterpret_cast<GradOp*>(stage + off_r);
    if (by_op) {
        c.batch_r = reinterpret_cast<int32_t*>(stage + off_br);
        c.batch_u = reinterpret_cast<int32_t*>(stage + off_bu);
        std::memset(stage + off_br, 0, bytes_br + bytes_bu);
    }
    std::vector<int64_t> u_fill(c.u_off.begin(), c.u_off.end() - 1), r_fill(c.r_off.begin(), c.r_off.end() - 1);
    for (int64_t k = 0; k < K; ++k) {
        if (k < c.A) fill_update(h, c, k, u_fill);
        if (c.with_grad && c.plan.r_round[k] >= 0) fill_gradient(h, c, k, r_fill);
    }
    if (bytes_b > 0 && !by_op) std::memcpy(stage + off_b, s->batch_idx, bytes_b);
    HIP_TRY(h, hipMemcpyAsync(T.dev.p, T.stage.p, total, hipMemcpyHostToDevice, h->stream));
    const char* dev = static_cast<const char*>(T.dev.p);
    c.d_uops = reinterpret_cast<const PairOp*>(dev);
    c.d_rops = reinterpret_cast<const GradOp*>(dev + off_r);
    c.d_batch = reinterpret_cast<const int32_t*>(dev + off_b);
    c.d_batch_r = reinterpret_cast<const int32_t*>(dev + off_br);
    c.d_batch_u = reinterpret_cast<const int32_t*>(dev + off_bu);

    if (c.with_grad && !c.external) {
        if (h->o.model == ADPSGD_MODEL_MLP) {
            HIP_TRY(h, h->grad_scratch.reserve(mlp_scratch_bytes(c.group, M, h->o.mlp_in, h->o.mlp_hidden, h->o.mlp_out)));
        } else {
            // all gradients of a round go into one set of launches (measured: splitting a round so
            // that the gathered rows stay within the memory-side cache only adds launches)
            const size_t partial_bytes = static_cast<size_t>(c.group) * (M + 1) * linear_grad_chunks(h->d) * 4;
            c.off_coef = (partial_bytes + 255) & ~size_t(255);
            HIP_TRY(h, h->grad_scratch.reserve(c.off_coef + static_cast<size_t>(c.group) * M * 4));
        }
    }
    return ADPSGD_OK;
}

// A pair of HIP events around a launch when per-launch timing is on (nullptr otherwise).
int begin_timing(adpsgd_t* h, hipEvent_t& e0, hipEvent_t& e1) {
    e0 = e1 = nullptr;
    if (!(h->o.flags & ADPSGD_FLAG_PROFILE)) return ADPSGD_OK;
    e0 = take_event(h);
    e1 = take_event(h);
    if (!e0 || !e1) return fail(h, ADPSGD_ERR_HIP, "run_events: hipEventCreate failed");
    HIP_TRY(h, hipEventRecord(e0, h->stream));
    return ADPSGD_OK;
}
int end_timing(adpsgd_t* h, hipEvent_t e0, hipEvent_t e1, std::vector<std::pair<hipEvent_t, hipEvent_t>>& into) {
    if (!e0) return ADPSGD_OK;
    HIP_TRY(h, hipEventRecord(e1, h->stream));
    into.push_back({e0, e1});
    return ADPSGD_OK;
}

// The stale gradients of round r: the library's kernels, or the caller's function.
int launch_gradients(adpsgd_t* h, const EventCall& c, int32_t r, float* loss, adpsgd_gradient_fn fn, void* user,
                     std::vector<adpsgd_grad_request_t>& requests) {
    float* slots = static_cast<float*>(h->o.workspace);
    const float gscale = h->o.grad_sum ? 1.0f : 1.0f / static_cast<float>(std::max(c.M, 1));
    for (int64_t g0 = c.r_off[r]; g0 < c.r_off[r + 1]; g0 += c.group) {
        const int32_t cnt = static_cast<int32_t>(std::min<int64_t>(c.group, c.r_off[r + 1] - g0));
        hipEvent_t e0, e1;
        int rc = begin_timing(h, e0, e1);
        if (rc != ADPSGD_OK) return rc;
        int launches = 0;
        if (c.external) {
            requests.resize(static_cast<size_t>(cnt));
            bool any_comp = false;
            for (int32_t t = 0; t < cnt; ++t) {
                const GradOp& g = c.rops[g0 + t];
                const bool comp = c.ext_comp && g.comp_slot >= 0;
                any_comp |= comp;
                requests[t] = adpsgd_grad_request_t{
                    g.worker, 0, g.event,
                    comp ? static_cast<const float*>(h->comp_rows.p) + static_cast<int64_t>(t) * h->o.ldx
                         : h->o.X + static_cast<int64_t>(g.worker) * h->o.ldx,
                    slots + static_cast<int64_t>(g.slot) * h->o.ldx};
            }
            if (any_comp)
                HIP_TRY(h, launch_compensated_rows(h->o.X, h->o.ldx, c.d_rops + g0, cnt, slots, static_cast<float*>(h->comp_rows.p),
                                                   h->stream));
            if (fn(user, cnt, requests.data(), h->stream) != 0) {
                (void)hipStreamSynchronize(h->stream);      // the table upload and the rounds enqueued so far
                return fail(h, ADPSGD_ERR_CALLBACK, "run_events_with: the gradient function failed in round " + std::to_string(r));
            }
            launches = 1;
        } else if (h->o.model == ADPSGD_MODEL_MLP) {
            MlpGradArgs a{h->o.X, h->o.Xbf16, h->o.ldx, h->o.mlp_in, h->o.mlp_hidden, h->o.mlp_out, c.d_rops + g0, cnt, c.M,
                          c.d_batch_r + g0 * c.M, slots, gscale, loss, h->grad_scratch.p, c.factored, c.mlp_comp};
            HIP_TRY(h, launch_mlp_gradient(a, h->stream, &launches));
        } else {
            LinearGradArgs a{h->o.model, h->o.X, h->o.ldx, h->d, c.d_rops + g0, cnt, c.M, c.d_batch, slots, gscale, h->o.lambda,
                             static_cast<float*>(h->grad_scratch.p),
                             reinterpret_cast<float*>(static_cast<char*>(h->grad_scratch.p) + c.off_coef), loss, c.lin_factored};
            HIP_TRY(h, launch_linear_gradient(a, h->stream, &launches));
        }
        h->stats.grad_launches += launches;
        rc = end_timing(h, e0, e1, h->ev_grad);
        if (rc != ADPSGD_OK) return rc;
    }
    return ADPSGD_OK;
}

// The averaging and update operations of round r: one launch.
int launch_updates(adpsgd_t* h, const EventCall& c, int32_t r) {
    const int64_t nu = c.u_off[r + 1] - c.u_off[r];
    if (nu <= 0) return ADPSGD_OK;
    float* slots = static_cast<float*>(h->o.workspace);
    const PairOp* d_ops = c.d_uops + c.u_off[r];
    hipEvent_t e0, e1;
    int rc = begin_timing(h, e0, e1);
    if (rc != ADPSGD_OK) return rc;
    if (c.lin_factored) {
        LinearApplyArgs a{h->o.X, h->o.ldx, h->d, d_ops, static_cast<int32_t>(nu), slots, c.d_batch, c.M,
                          h->streaming, h->o.V, h->o.momentum, h->o.weight_decay};
        HIP_TRY(h, launch_linear_apply_factored(a, h->stream));
    } else if (c.factored) {
        MlpApplyArgs a{h->o.X, h->o.ldx, h->d, h->o.mlp_in, h->o.mlp_hidden, c.M, d_ops, static_cast<int32_t>(nu), slots, h->o.Xbf16,
                       c.d_batch_u + c.u_off[r] * c.M, h->o.V, h->o.momentum, h->o.weight_decay};
        HIP_TRY(h, launch_mlp_apply_factored(a, h->stream));
    } else {
        bool has_solo = false;
        for (int64_t t = c.u_off[r]; t < c.u_off[r + 1] && !has_solo; ++t) has_solo = c.uops[t].i == c.uops[t].j;
        FusedArgs a{h->o.X, h->o.ldx, h->d, d_ops, static_cast<int32_t>(nu), slots,
                    h->o.model == ADPSGD_MODEL_MLP ? h->o.Xbf16 : nullptr, h->o.synth_std, h->o.synth_seed,
                    !c.with_grad, h->streaming, has_solo, h->o.V, h->o.momentum, h->o.weight_decay};
        HIP_TRY(h, launch_fused_gossip_apply(a, h->stream));
    }
    ++h->stats.fused_launches;
    h->stats.max_round_pairs = std::max<int64_t>(h->stats.max_round_pairs, nu);
    return end_timing(h, e0, e1, h->ev_fused);
}

// The events of one call: plan, tables, then per round the gradients and one update launch.
int run_events_impl(adpsgd_t* h, const adpsgd_schedule_t* s, float* loss, adpsgd_gradient_fn fn, void* user) {
    if (!s || s->K < 0) return fail(h, ADPSGD_ERR_ARG, "run_events: schedule is NULL or K < 0");
    if (s->K == 0) return ADPSGD_OK;
    EventCall c;
    int rc = prepare_call(h, s, c);
    if (rc != ADPSGD_OK) return rc;
    rc = upload_tables(h, c);
    if (rc != ADPSGD_OK) return rc;
    std::vector<adpsgd_grad_request_t> requests;
    for (int32_t r = 0; r < c.plan.n_rounds; ++r) {
        rc = launch_gradients(h, c, r, loss, fn, user, requests);
        if (rc != ADPSGD_OK) return rc;
        rc = launch_updates(h, c, r);
        if (rc != ADPSGD_OK) return rc;
    }
    HIP_TRY(h, hipEventRecord(c.T->done, h->stream));
    c.T->in_flight = true;
    h->events_done += static_cast<uint64_t>(c.A);
    h->stats.events += c.A;
    h->stats.rounds += c.plan.n_rounds;
    // the events looked ahead to: the next call must start with them; some have their gradient pending already
    h->pending.clear();
    h->pending_batch.clear();
    for (int64_t k = c.A; k < c.K; ++k) h->pending.push_back(PendingEvent{s->worker[k], s->tau[k], c.with_grad ? c.plan.slot[k] : -1});
    if (c.M > 0 && c.A < c.K)
        h->pending_batch.assign(s->batch_idx + c.A * static_cast<int64_t>(c.M), s->batch_idx + c.K * static_cast<int64_t>(c.M));
    return ADPSGD_OK;
}

}  // namespace

extern "C" int adpsgd_run_events(adpsgd_t* h, const adpsgd_schedule_t* s, float* loss) {
    if (!h) return ADPSGD_ERR_ARG;
    if (h->o.model == ADPSGD_MODEL_EXTERNAL)
        return fail(h, ADPSGD_ERR_STATE, "run_events: caller-supplied gradients need adpsgd_run_events_with");
    return run_events_impl(h, s, loss, nullptr, nullptr);
}

extern "C" int adpsgd_run_events_with(adpsgd_t* h, const adpsgd_schedule_t* s, adpsgd_gradient_fn fn, void* user) {
    if (!h) return ADPSGD_ERR_ARG;
    if (h->o.model != ADPSGD_MODEL_EXTERNAL)
        return fail(h, ADPSGD_ERR_STATE, "run_events_with: the handle was not created with ADPSGD_MODEL_EXTERNAL");
    if (!fn) return fail(h, ADPSGD_ERR_ARG, "run_events_with: fn is NULL");
    return run_events_impl(h, s, nullptr, fn, user);
}

extern "C" int adpsgd_get_stats(adpsgd_t* h, adpsgd_stats_t* out) {
    if (!h) return ADPSGD_ERR_ARG;
    if (!out) return fail(h, ADPSGD_ERR_ARG, "get_stats: out is NULL");
    const int rc = drain_profile(h);
    if (rc != ADPSGD_OK) return rc;
    *out = h->stats;
    return ADPSGD_OK;
}

extern "C" int adpsgd_get_event_count(adpsgd_t* h, uint64_t* out) {
    if (!h) return ADPSGD_ERR_ARG;
    if (!out) return fail(h, ADPSGD_ERR_ARG, "get_event_count: out is NULL");
    *out = h->events_done;
    return ADPSGD_OK;
}

extern "C" int adpsgd_set_event_count(adpsgd_t* h, uint64_t events) {
    if (!h) return ADPSGD_ERR_ARG;
    h->events_done = events;
    h->pending.clear();
    h->pending_batch.clear();
    return ADPSGD_OK;
}

extern "C" int adpsgd_synth_gradient(uint64_t seed, uint64_t k, float std, int64_t d, float* out_device, void* stream) {
    if (!out_device || d < 0) return ADPSGD_ERR_ARG;
    const hipError_t e = launch_synth_gradient(seed, k, std, d, out_device, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? ADPSGD_OK : ADPSGD_ERR_HIP;
}
