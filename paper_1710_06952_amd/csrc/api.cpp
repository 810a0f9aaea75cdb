// C-ABI entry points of libadpsgd: handle life cycle, validation, per-call
// planning and the per-round launch loop.  See include/adpsgd.h for the contract.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <memory>

#include "internal.hpp"

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

// Pinned host staging buffer (grow-only).
struct HostBuf {
    void* p = nullptr;
    size_t cap = 0;
    hipError_t reserve(size_t bytes) {
        if (bytes <= cap) return hipSuccess;
        if (p) (void)hipHostFree(p);
        p = nullptr;
        cap = 0;
        size_t want = std::max<size_t>(bytes, 4096);
        hipError_t e = hipHostMalloc(&p, want, hipHostMallocDefault);
        if (e != hipSuccess) { p = nullptr; return e; }
        cap = want;
        return hipSuccess;
    }
    void release() {
        if (p) (void)hipHostFree(p);
        p = nullptr;
        cap = 0;
    }
};

// The tables of one adpsgd_run_events call; two sets alternate so that planning
// call c+1 can overlap the kernels of call c.
struct TableSet {
    HostBuf stage;
    DevBuf dev;
    hipEvent_t done = nullptr;   // recorded after the last kernel that reads the tables
    bool in_flight = false;
};

constexpr int64_t kStreamingThreshold = 256ll << 20;
constexpr int32_t kMaxSlots = 4096;

thread_local std::string g_create_error;

}  // namespace
}  // namespace adpsgd_impl

using namespace adpsgd_impl;

struct adpsgd {
    int32_t n = 0;
    int64_t d = 0;
    adpsgd_opts_t o{};
    std::vector<int32_t> rowptr, col;
    std::vector<WorkerData> data;
    int32_t n_slots = 0;
    hipStream_t stream = nullptr;
    bool streaming = false;
    uint64_t events_done = 0;
    TableSet tables[2];
    int next_table = 0;
    DevBuf grad_scratch;     // dots partials + coefficients / MLP activations
    DevBuf comp_rows;        // perceptron, wait-free variant: compensated bf16 copies of the rows a group of gradients reads
    DevBuf diag;             // consensus partials, result, mean / broadcast staging
    adpsgd_stats_t stats{};
    std::vector<hipEvent_t> ev_pool;                       // profiling events
    std::vector<std::pair<hipEvent_t, hipEvent_t>> ev_fused, ev_grad;
    std::string err;
};

namespace {

int fail(adpsgd_t* h, int code, const std::string& msg) {
    if (h) h->err = msg;
    else g_create_error = msg;
    return code;
}
int hip_fail(adpsgd_t* h, hipError_t e, const char* what) {
    return fail(h, ADPSGD_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}
#define HIP_TRY(h, expr)                                           \
    do {                                                           \
        hipError_t e__ = (expr);                                   \
        if (e__ != hipSuccess) return hip_fail((h), e__, #expr);   \
    } while (0)

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool is_neighbour(const adpsgd_t* h, int32_t i, int32_t j) {
    const int32_t b = h->rowptr[i], e = h->rowptr[i + 1];
    if (b == e) return j == i;
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

}  // namespace

extern "C" const char* adpsgd_last_error(const adpsgd_t* h) { return h ? h->err.c_str() : g_create_error.c_str(); }

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
    if (o.model < ADPSGD_MODEL_LSQ || o.model > ADPSGD_MODEL_MLP) return fail(nullptr, ADPSGD_ERR_ARG, "create: unknown model");
    if (!o.X || !aligned16(o.X)) return fail(nullptr, ADPSGD_ERR_ARG, "create: X is NULL or not 16-byte aligned");
    if (o.ldx < d || (o.ldx & 3)) return fail(nullptr, ADPSGD_ERR_ARG, "create: ldx must be >= d and a multiple of 4");
    if (o.T_max < 0) return fail(nullptr, ADPSGD_ERR_ARG, "create: T_max < 0");
    if (!std::isfinite(o.gamma)) return fail(nullptr, ADPSGD_ERR_ARG, "create: gamma not finite");
    int32_t n_slots = 0;
    if (o.model != ADPSGD_MODEL_SYNTH) {
        if (o.M < 1 || o.M > 65536) return fail(nullptr, ADPSGD_ERR_ARG, "create: minibatch size M outside [1, 65536]");
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
    if (o.local_compensation) {
        if (o.momentum != 0.0f || o.weight_decay != 0.0f)
            return fail(nullptr, ADPSGD_ERR_ARG, "create: local_compensation cannot be combined with momentum or weight decay");
    }
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
    delete h;
}

extern "C" int adpsgd_load_data(adpsgd_t* h, int32_t worker, const void* features, int64_t rows, int64_t ld,
                                const void* targets) {
    if (!h) return ADPSGD_ERR_ARG;
    if (h->o.model == ADPSGD_MODEL_SYNTH) return fail(h, ADPSGD_ERR_STATE, "load_data: the synthetic-gradient model takes no data");
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

extern "C" int adpsgd_run_events(adpsgd_t* h, const adpsgd_schedule_t* s, float* loss) {
    if (!h) return ADPSGD_ERR_ARG;
    if (!s || s->K < 0) return fail(h, ADPSGD_ERR_ARG, "run_events: schedule is NULL or K < 0");
    const int64_t K = s->K;
    if (K == 0) return ADPSGD_OK;
    if (K > 0x7FFFFFF0) return fail(h, ADPSGD_ERR_ARG, "run_events: at most 2^31 - 16 events per call");
    if (!s->worker || !s->neighbour || !s->tau) return fail(h, ADPSGD_ERR_ARG, "run_events: null schedule array");
    const bool with_grad = h->o.model != ADPSGD_MODEL_SYNTH;
    const int32_t M = with_grad ? h->o.M : 0;
    if (with_grad && !s->batch_idx) return fail(h, ADPSGD_ERR_ARG, "run_events: batch_idx is NULL");

    // ---- validation: nothing is launched and no state changes on failure ----
    const int64_t n_extra = s->extra_ptr ? s->extra_ptr[K] : 0;
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
        if (s->tau[k] < 0 || s->tau[k] > k || s->tau[k] > h->o.T_max)
            return fail(h, ADPSGD_ERR_SCHEDULE, "run_events: tau outside [0, min(k, T_max)] at event " + std::to_string(k));
        if (s->gamma && !std::isfinite(s->gamma[k]))
            return fail(h, ADPSGD_ERR_SCHEDULE, "run_events: gamma not finite at event " + std::to_string(k));
        if (with_grad) {
            const WorkerData& w = h->data[i];
            if (!w.features) return fail(h, ADPSGD_ERR_STATE, "run_events: no data loaded for worker " + std::to_string(i));
            const int32_t* b = s->batch_idx + k * static_cast<int64_t>(M);
            for (int32_t m = 0; m < M; ++m)
                if (b[m] < 0 || b[m] >= w.rows)
                    return fail(h, ADPSGD_ERR_SCHEDULE, "run_events: batch index out of range at event " + std::to_string(k));
        }
    }

    // perceptron without momentum: dW1 stays in factored form until the update kernel
    // (the wait-free variant reads the pending gradient as a dense vector, so it keeps the dense form)
    const bool mlp_comp = h->o.model == ADPSGD_MODEL_MLP && h->o.local_compensation != 0;
    const bool factored = h->o.model == ADPSGD_MODEL_MLP && !h->o.V && !(h->o.flags & ADPSGD_FLAG_DENSE_GRADIENT) &&
                          !mlp_comp && mlp_can_factor(h->o.mlp_in, h->o.mlp_hidden, M);

    // least squares on long models: the gradient stays M coefficients until the update kernel applies it
    const bool lin_factored = !h->o.V && !h->o.local_compensation && !(h->o.flags & ADPSGD_FLAG_DENSE_GRADIENT) &&
                              with_grad && linear_can_factor(h->o.model, h->d, M, h->o.ldx);

    // ---- plan ----
    Plan plan;
    std::string perr;
    int rc = plan_rounds(h->n, K, s->worker, s->neighbour, s->tau, h->n_slots, with_grad, plan, perr,
                         s->extra_ptr, s->extra_a, s->extra_b, h->o.local_compensation != 0);
    if (rc != ADPSGD_OK) return fail(h, rc, perr);
    if ((h->o.flags & ADPSGD_FLAG_VERIFY_PLAN) &&
        !verify_plan(h->n, K, s->worker, s->neighbour, s->tau, h->n_slots, with_grad, plan, perr, s->extra_ptr, s->extra_a, s->extra_b))
        return fail(h, ADPSGD_ERR_STATE, perr);
    const int32_t R = plan.n_rounds;

    // counting sort of the operations by round
    std::vector<int64_t> u_off(static_cast<size_t>(R) + 1, 0), r_off(static_cast<size_t>(R) + 1, 0);
    for (int64_t k = 0; k < K; ++k) {
        u_off[plan.u_round[k] + 1] += 1 + (s->extra_ptr ? s->extra_ptr[k + 1] - s->extra_ptr[k] : 0);
        if (with_grad) ++r_off[plan.r_round[k] + 1];
    }
    for (int32_t r = 0; r < R; ++r) { u_off[r + 1] += u_off[r]; r_off[r + 1] += r_off[r]; }

    // gradients of a round are launched in groups of this many operations
    int32_t group = 1;
    if (with_grad) {
        int64_t max_r = 0;
        for (int32_t r = 0; r < R; ++r) max_r = std::max(max_r, r_off[r + 1] - r_off[r]);
        group = static_cast<int32_t>(std::min<int64_t>(std::max<int64_t>(max_r, 1), h->o.model == ADPSGD_MODEL_MLP ? 64 : 65535));
    }
    if (mlp_comp) HIP_TRY(h, h->comp_rows.reserve(static_cast<size_t>(group) * h->o.ldx * sizeof(uint16_t)));

    // ---- tables: [PairOp x K][GradOp x K][batch_idx K x M] ----
    const size_t bytes_u = static_cast<size_t>(K + n_extra) * sizeof(PairOp);
    const size_t bytes_r = with_grad ? static_cast<size_t>(K) * sizeof(GradOp) : 0;
    const size_t bytes_b = with_grad ? static_cast<size_t>(K) * M * sizeof(int32_t) : 0;
    const size_t off_r = bytes_u, off_b = (off_r + bytes_r + 15) & ~size_t(15);
    const size_t total = off_b + bytes_b;

    TableSet& T = h->tables[h->next_table];
    h->next_table ^= 1;
    if (T.in_flight) {
        HIP_TRY(h, hipEventSynchronize(T.done));
        T.in_flight = false;
    }
    HIP_TRY(h, T.stage.reserve(total));
    HIP_TRY(h, T.dev.reserve(total));
    char* stage = static_cast<char*>(T.stage.p);
    PairOp* uops = reinterpret_cast<PairOp*>(stage);
    GradOp* rops = reinterpret_cast<GradOp*>(stage + off_r);
    {
        std::vector<int64_t> u_fill(u_off.begin(), u_off.end() - 1), r_fill(r_off.begin(), r_off.end() - 1);
        for (int64_t k = 0; k < K; ++k) {
            const uint64_t gk = h->events_done + static_cast<uint64_t>(k);
            PairOp& u = uops[u_fill[plan.u_round[k]]++];
            u.i = s->worker[k];
            u.j = s->neighbour[k];
            u.k_lo = static_cast<uint32_t>(gk);
            u.k_hi = static_cast<uint32_t>(gk >> 32);
            u.gamma = s->gamma ? s->gamma[k] : h->o.gamma;
            u.slot = with_grad ? plan.slot[k] : 0;
            u.flags = 0;
            u.event = static_cast<int32_t>(k);
            u.features = (factored || lin_factored) ? h->data[u.i].features : nullptr;
            u.feat_ld = (factored || lin_factored) ? h->data[u.i].ld : 0;
            if (s->extra_ptr) {
                for (int64_t q = s->extra_ptr[k]; q < s->extra_ptr[k + 1]; ++q) {
                    PairOp& x = uops[u_fill[plan.u_round[k]]++];
                    x = PairOp{s->extra_a[q], s->extra_b[q], 0u, 0u, 0.0f, 0, 1, 0, nullptr, 0};
                }
            }
            if (with_grad) {
                const int64_t at = r_fill[plan.r_round[k]]++;
                GradOp& g = rops[at];
                g.worker = s->worker[k];
                g.slot = plan.slot[k];
                g.event = static_cast<int32_t>(k);
                const int64_t kp = plan.prev[k];
                g.comp_slot = kp >= 0 ? plan.slot[kp] : -1;
                g.comp_gamma = kp >= 0 ? (s->gamma ? s->gamma[kp] : h->o.gamma) : 0.0f;
                g.count = 0;
                const WorkerData& w = h->data[g.worker];
                g.features = w.features;
                g.targets = w.targets;
                g.ld = w.ld;
                g.xrow_bf16 = nullptr;
                if (mlp_comp && kp >= 0)      // one compensated row per operation of a launch group
                    g.xrow_bf16 = static_cast<uint16_t*>(h->comp_rows.p) + ((at - r_off[plan.r_round[k]]) % group) * h->o.ldx;
            }
        }
    }
    if (with_grad) std::memcpy(stage + off_b, s->batch_idx, bytes_b);
    HIP_TRY(h, hipMemcpyAsync(T.dev.p, T.stage.p, total, hipMemcpyHostToDevice, h->stream));
    const char* dev = static_cast<const char*>(T.dev.p);
    const PairOp* d_uops = reinterpret_cast<const PairOp*>(dev);
    const GradOp* d_rops = reinterpret_cast<const GradOp*>(dev + off_r);
    const int32_t* d_batch = reinterpret_cast<const int32_t*>(dev + off_b);


    // ---- gradient scratch ----
    size_t off_coef = 0;
    if (with_grad) {
        if (h->o.model == ADPSGD_MODEL_MLP) {
            HIP_TRY(h, h->grad_scratch.reserve(mlp_scratch_bytes(group, M, h->o.mlp_in, h->o.mlp_hidden, h->o.mlp_out)));
        } else {
            // all gradients of a round go into one set of launches (measured: splitting a round so
            // that the gathered rows stay within the memory-side cache only adds launches)
            const size_t partial_bytes = static_cast<size_t>(group) * (M + 1) * linear_grad_chunks(h->d) * 4;
            off_coef = (partial_bytes + 255) & ~size_t(255);
            HIP_TRY(h, h->grad_scratch.reserve(off_coef + static_cast<size_t>(group) * M * 4));
        }
    }

    // ---- rounds ----
    const bool profile = (h->o.flags & ADPSGD_FLAG_PROFILE) != 0;
    float* slots = static_cast<float*>(h->o.workspace);
    const float gscale = h->o.grad_sum ? 1.0f : 1.0f / static_cast<float>(std::max(M, 1));
    for (int32_t r = 0; r < R; ++r) {
        for (int64_t g0 = r_off[r]; g0 < r_off[r + 1]; g0 += group) {
            const int32_t cnt = static_cast<int32_t>(std::min<int64_t>(group, r_off[r + 1] - g0));
            hipEvent_t e0 = nullptr, e1 = nullptr;
            if (profile) {
                e0 = take_event(h);
                e1 = take_event(h);
                if (!e0 || !e1) return fail(h, ADPSGD_ERR_HIP, "run_events: hipEventCreate failed");
                HIP_TRY(h, hipEventRecord(e0, h->stream));
            }
            int launches = 0;
            if (h->o.model == ADPSGD_MODEL_MLP) {
                MlpGradArgs a{h->o.X, h->o.Xbf16, h->o.ldx, h->o.mlp_in, h->o.mlp_hidden, h->o.mlp_out, d_rops + g0, cnt, M,
                              d_batch, slots, gscale, loss,
                              h->grad_scratch.p, factored, mlp_comp};
                HIP_TRY(h, launch_mlp_gradient(a, h->stream, &launches));
            } else {
                LinearGradArgs a{h->o.model, h->o.X, h->o.ldx, h->d, d_rops + g0, cnt, M, d_batch,
                                 slots, gscale, h->o.lambda,
                                 static_cast<float*>(h->grad_scratch.p),
                                 reinterpret_cast<float*>(static_cast<char*>(h->grad_scratch.p) + off_coef), loss, lin_factored};
                HIP_TRY(h, launch_linear_gradient(a, h->stream, &launches));
            }
            h->stats.grad_launches += launches;
            if (profile) {
                HIP_TRY(h, hipEventRecord(e1, h->stream));
                h->ev_grad.push_back({e0, e1});
            }
        }
        const int64_t nu = u_off[r + 1] - u_off[r];
        if (nu > 0) {
            hipEvent_t e0 = nullptr, e1 = nullptr;
            if (profile) {
                e0 = take_event(h);
                e1 = take_event(h);
                if (!e0 || !e1) return fail(h, ADPSGD_ERR_HIP, "run_events: hipEventCreate failed");
                HIP_TRY(h, hipEventRecord(e0, h->stream));
            }
            bool has_solo = false;
            for (int64_t t = u_off[r]; t < u_off[r + 1] && !has_solo; ++t) has_solo = uops[t].i == uops[t].j;
            if (lin_factored) {
                LinearApplyArgs a{h->o.X, h->o.ldx, h->d, d_uops + u_off[r], static_cast<int32_t>(nu), slots, d_batch, M,
                                  h->streaming};
                HIP_TRY(h, launch_linear_apply_factored(a, h->stream));
            } else if (factored) {
                MlpApplyArgs a{h->o.X, h->o.ldx, h->d, h->o.mlp_in, h->o.mlp_hidden, M, d_uops + u_off[r],
                               static_cast<int32_t>(nu), slots, h->o.Xbf16, d_batch};
                HIP_TRY(h, launch_mlp_apply_factored(a, h->stream));
            } else {
                FusedArgs a{h->o.X, h->o.ldx, h->d, d_uops + u_off[r], static_cast<int32_t>(nu), slots,
                            h->o.model == ADPSGD_MODEL_MLP ? h->o.Xbf16 : nullptr, h->o.synth_std, h->o.synth_seed,
                            !with_grad, h->streaming, has_solo, h->o.V, h->o.momentum, h->o.weight_decay};
                HIP_TRY(h, launch_fused_gossip_apply(a, h->stream));
            }
            ++h->stats.fused_launches;
            h->stats.max_round_pairs = std::max<int64_t>(h->stats.max_round_pairs, nu);
            if (profile) {
                HIP_TRY(h, hipEventRecord(e1, h->stream));
                h->ev_fused.push_back({e0, e1});
            }
        }
    }
    HIP_TRY(h, hipEventRecord(T.done, h->stream));
    T.in_flight = true;
    h->events_done += static_cast<uint64_t>(K);
    h->stats.events += K;
    h->stats.rounds += R;
    return ADPSGD_OK;
}

extern "C" int adpsgd_run_sync_steps(adpsgd_t* h, const adpsgd_sync_schedule_t* s, float* loss) {
    if (!h) return ADPSGD_ERR_ARG;
    if (!s || s->S < 0) return fail(h, ADPSGD_ERR_ARG, "run_sync_steps: schedule is NULL or S < 0");
    const int64_t S = s->S;
    if (S == 0) return ADPSGD_OK;
    const int32_t n = h->n;
    const bool with_grad = h->o.model != ADPSGD_MODEL_SYNTH;
    const int32_t M = with_grad ? h->o.M : 0;
    if (S * n > 0x7FFFFFF0) return fail(h, ADPSGD_ERR_ARG, "run_sync_steps: S * n must stay below 2^31 - 16");
    if (h->o.V) return fail(h, ADPSGD_ERR_STATE, "run_sync_steps: not available with momentum / weight decay");
    if (sync_tile_cols(n) == 0) return fail(h, ADPSGD_ERR_ARG, "run_sync_steps: at most 1024 workers");
    if (with_grad && !s->batch_idx) return fail(h, ADPSGD_ERR_ARG, "run_sync_steps: batch_idx is NULL");
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
    if (with_grad) {
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
    const size_t bytes_r = with_grad ? static_cast<size_t>(S) * n * sizeof(GradOp) : 0;
    const size_t bytes_b = with_grad ? static_cast<size_t>(S) * n * M * sizeof(int32_t) : 0;
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
    if (with_grad) {
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
    if (with_grad) {
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
    float* slots = static_cast<float*>(h->o.workspace);
    const float gscale = h->o.grad_sum ? 1.0f : 1.0f / static_cast<float>(std::max(M, 1));
    for (int64_t t = 0; t < S; ++t) {
        for (int32_t g0 = 0; with_grad && g0 < n; g0 += group) {
            const int32_t cnt = std::min<int32_t>(group, n - g0);
            int launches = 0;
            if (h->o.model == ADPSGD_MODEL_MLP) {
                MlpGradArgs a{h->o.X, h->o.Xbf16, h->o.ldx, h->o.mlp_in, h->o.mlp_hidden, h->o.mlp_out, d_rops + t * n + g0, cnt, M,
                              d_batch, slots, gscale, loss,
                              h->grad_scratch.p, false, false};
                HIP_TRY(h, launch_mlp_gradient(a, h->stream, &launches));
            } else {
                LinearGradArgs a{h->o.model, h->o.X, h->o.ldx, h->d, d_rops + t * n + g0, cnt, M, d_batch,
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
        SyncArgs a{h->o.X, h->o.ldx, h->d, n,
                   reinterpret_cast<const int32_t*>(dev + off_rp), reinterpret_cast<const int32_t*>(dev + off_col),
                   reinterpret_cast<const float*>(dev + off_ws), reinterpret_cast<const float*>(dev + off_we),
                   with_grad ? slots : nullptr, h->o.model == ADPSGD_MODEL_MLP ? h->o.Xbf16 : nullptr,
                   s->gamma ? s->gamma[t] : h->o.gamma, h->o.synth_std, h->o.synth_seed,
                   h->events_done + static_cast<uint64_t>(t) * static_cast<uint64_t>(n), !with_grad};
        HIP_TRY(h, launch_sync_mix_apply(a, h->stream));
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

extern "C" int adpsgd_metropolis_weights(const adpsgd_graph_t* graph, float* w_self, float* w_edge) {
    std::string err;
    if (!graph || !w_self || !graph_ok(graph, err)) return ADPSGD_ERR_GRAPH;
    if (graph->rowptr[graph->n] > 0 && !w_edge) return ADPSGD_ERR_ARG;
    std::vector<int32_t> rowptr(graph->rowptr, graph->rowptr + graph->n + 1), col(graph->col, graph->col + graph->rowptr[graph->n]);
    metropolis(rowptr, col, w_self, w_edge);
    return ADPSGD_OK;
}

extern "C" int adpsgd_get_models(adpsgd_t* h, float* out, int64_t ld_out, int32_t on_device) {
    if (!h) return ADPSGD_ERR_ARG;
    if (!out || ld_out < h->d) return fail(h, ADPSGD_ERR_ARG, "get_models: out is NULL or ld_out < d");
    HIP_TRY(h, hipMemcpy2DAsync(out, static_cast<size_t>(ld_out) * 4, h->o.X, static_cast<size_t>(h->o.ldx) * 4,
                                static_cast<size_t>(h->d) * 4, h->n,
                                on_device ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return ADPSGD_OK;
}

extern "C" int adpsgd_get_momentum(adpsgd_t* h, float* out, int64_t ld_out, int32_t on_device) {
    if (!h) return ADPSGD_ERR_ARG;
    if (!h->o.V) return fail(h, ADPSGD_ERR_STATE, "get_momentum: the engine was created without momentum buffers");
    if (!out || ld_out < h->d) return fail(h, ADPSGD_ERR_ARG, "get_momentum: out is NULL or ld_out < d");
    HIP_TRY(h, hipMemcpy2DAsync(out, static_cast<size_t>(ld_out) * 4, h->o.V, static_cast<size_t>(h->o.ldx) * 4,
                                static_cast<size_t>(h->d) * 4, h->n,
                                on_device ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return ADPSGD_OK;
}

extern "C" int adpsgd_get_bf16_models(adpsgd_t* h, uint16_t* out, int64_t ld_out, int32_t on_device) {
    if (!h) return ADPSGD_ERR_ARG;
    if (h->o.model != ADPSGD_MODEL_MLP) return fail(h, ADPSGD_ERR_STATE, "get_bf16_models: only the MLP model keeps a bf16 shadow");
    if (!out || ld_out < h->d) return fail(h, ADPSGD_ERR_ARG, "get_bf16_models: out is NULL or ld_out < d");
    HIP_TRY(h, hipMemcpy2DAsync(out, static_cast<size_t>(ld_out) * 2, h->o.Xbf16, static_cast<size_t>(h->o.ldx) * 2,
                                static_cast<size_t>(h->d) * 2, h->n,
                                on_device ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return ADPSGD_OK;
}

extern "C" int adpsgd_get_mean_model(adpsgd_t* h, float* out, int32_t on_device) {
    if (!h) return ADPSGD_ERR_ARG;
    if (!out) return fail(h, ADPSGD_ERR_ARG, "get_mean_model: out is NULL");
    float* dst = out;
    if (!on_device) {
        HIP_TRY(h, hipStreamSynchronize(h->stream));
        HIP_TRY(h, h->diag.reserve(static_cast<size_t>(h->d) * 4));
        dst = static_cast<float*>(h->diag.p);
    }
    HIP_TRY(h, launch_mean_model(h->o.X, h->o.ldx, h->d, h->n, dst, h->stream));
    if (!on_device)
        HIP_TRY(h, hipMemcpyAsync(out, dst, static_cast<size_t>(h->d) * 4, hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return ADPSGD_OK;
}

extern "C" int adpsgd_consensus_distance(adpsgd_t* h, double* out) {
    if (!h) return ADPSGD_ERR_ARG;
    if (!out) return fail(h, ADPSGD_ERR_ARG, "consensus_distance: out is NULL");
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    const int32_t blocks = consensus_blocks(h->d);
    HIP_TRY(h, h->diag.reserve(static_cast<size_t>(blocks + 1) * sizeof(double)));
    double* partial = static_cast<double*>(h->diag.p);
    HIP_TRY(h, launch_consensus(h->o.X, h->o.ldx, h->d, h->n, partial, partial + blocks, h->stream));
    HIP_TRY(h, hipMemcpyAsync(out, partial + blocks, sizeof(double), hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return ADPSGD_OK;
}

extern "C" int adpsgd_count_nonfinite(adpsgd_t* h, int64_t* out) {
    if (!h) return ADPSGD_ERR_ARG;
    if (!out) return fail(h, ADPSGD_ERR_ARG, "count_nonfinite: out is NULL");
    const int32_t blocks = 2048;
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    HIP_TRY(h, h->diag.reserve(static_cast<size_t>(blocks) * sizeof(unsigned long long)));
    HIP_TRY(h, launch_count_nonfinite(h->o.X, h->o.ldx, h->d, h->n, static_cast<unsigned long long*>(h->diag.p), blocks, h->stream));
    std::vector<unsigned long long> part(blocks);
    HIP_TRY(h, hipMemcpyAsync(part.data(), h->diag.p, part.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    unsigned long long total = 0;
    for (unsigned long long v : part) total += v;
    *out = static_cast<int64_t>(total);
    return ADPSGD_OK;
}

namespace {

// The perceptron's objective: forward pass and cross-entropy over all local samples, in chunks of
// M samples (the last chunk of a worker is padded with its last sample and counts only its own).
int mlp_objective(adpsgd_t* h, const float* x, double* out) {
    const int32_t n = h->n, M = h->o.M;
    std::vector<int64_t> first(n + 1, 0);          // first operation of every worker
    for (int32_t i = 0; i < n; ++i) {
        if (!h->data[i].features) return fail(h, ADPSGD_ERR_STATE, "objective: no data loaded for worker " + std::to_string(i));
        first[i + 1] = first[i] + (h->data[i].rows + M - 1) / M;
    }
    const int64_t n_ops = first[n];
    if (n_ops > 0x7FFFFFF0) return fail(h, ADPSGD_ERR_ARG, "objective: too many samples");
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    const int32_t group = static_cast<int32_t>(std::min<int64_t>(n_ops, 64));
    HIP_TRY(h, h->grad_scratch.reserve(mlp_scratch_bytes(group, M, h->o.mlp_in, h->o.mlp_hidden, h->o.mlp_out)));
    // diag buffer: [point fp32 ld][point bf16 ld][GradOp x n_ops][batch_idx n_ops x M][loss sums]
    const size_t ld = static_cast<size_t>(h->o.ldx);
    const size_t off_b16 = (ld * 4 + 255) & ~size_t(255);
    const size_t off_ops = (off_b16 + ld * 2 + 255) & ~size_t(255);
    const size_t off_idx = (off_ops + static_cast<size_t>(n_ops) * sizeof(GradOp) + 255) & ~size_t(255);
    const size_t off_sum = (off_idx + static_cast<size_t>(n_ops) * M * 4 + 255) & ~size_t(255);
    HIP_TRY(h, h->diag.reserve(off_sum + static_cast<size_t>(n_ops) * sizeof(double)));
    char* base = static_cast<char*>(h->diag.p);
    float* point = reinterpret_cast<float*>(base);
    uint16_t* point_b16 = reinterpret_cast<uint16_t*>(base + off_b16);
    HIP_TRY(h, hipMemsetAsync(point, 0, ld * 4, h->stream));
    if (x) HIP_TRY(h, hipMemcpyAsync(point, x, static_cast<size_t>(h->d) * 4, hipMemcpyDeviceToDevice, h->stream));
    else HIP_TRY(h, launch_mean_model(h->o.X, h->o.ldx, h->d, n, point, h->stream));
    HIP_TRY(h, launch_refresh_bf16(point, point_b16, h->o.ldx, 1, h->stream));
    std::vector<GradOp> ops(static_cast<size_t>(n_ops));
    std::vector<int32_t> idx(static_cast<size_t>(n_ops) * M);
    for (int32_t i = 0; i < n; ++i)
        for (int64_t c = 0; c < first[i + 1] - first[i]; ++c) {
            const int64_t o = first[i] + c, r0 = c * M;
            const int64_t have = std::min<int64_t>(M, h->data[i].rows - r0);
            ops[o] = GradOp{i, 0, static_cast<int32_t>(o), -1, 0.0f, static_cast<int32_t>(have),
                            h->data[i].features, h->data[i].targets, h->data[i].ld, point_b16};
            for (int32_t m = 0; m < M; ++m) idx[o * M + m] = static_cast<int32_t>(r0 + std::min<int64_t>(m, have - 1));
        }
    HIP_TRY(h, hipMemcpyAsync(base + off_ops, ops.data(), ops.size() * sizeof(GradOp), hipMemcpyHostToDevice, h->stream));
    HIP_TRY(h, hipMemcpyAsync(base + off_idx, idx.data(), idx.size() * 4, hipMemcpyHostToDevice, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));      // the host vectors may go out of scope after this point
    double* d_sum = reinterpret_cast<double*>(base + off_sum);
    for (int64_t g0 = 0; g0 < n_ops; g0 += group) {
        const int32_t cnt = static_cast<int32_t>(std::min<int64_t>(group, n_ops - g0));
        MlpGradArgs a{nullptr, point_b16, h->o.ldx, h->o.mlp_in, h->o.mlp_hidden, h->o.mlp_out,
                      reinterpret_cast<const GradOp*>(base + off_ops) + g0, cnt, M,
                      reinterpret_cast<const int32_t*>(base + off_idx), nullptr, 1.0f, nullptr, h->grad_scratch.p, false, false};
        HIP_TRY(h, launch_mlp_loss(a, d_sum + g0, h->stream));
    }
    std::vector<double> sums(static_cast<size_t>(n_ops));
    HIP_TRY(h, hipMemcpyAsync(sums.data(), d_sum, sums.size() * sizeof(double), hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    double total = 0.0;
    for (int32_t i = 0; i < n; ++i) {
        double s = 0.0;
        for (int64_t o = first[i]; o < first[i + 1]; ++o) s += sums[o];
        total += s / static_cast<double>(h->data[i].rows);
    }
    *out = total / n;
    return ADPSGD_OK;
}

}  // namespace

extern "C" int adpsgd_objective(adpsgd_t* h, const float* x, double* out) {
    if (!h) return ADPSGD_ERR_ARG;
    if (!out) return fail(h, ADPSGD_ERR_ARG, "objective: out is NULL");
    if (h->o.model == ADPSGD_MODEL_SYNTH)
        return fail(h, ADPSGD_ERR_STATE, "objective: the synthetic-gradient model has no objective");
    if (x && !aligned16(x)) return fail(h, ADPSGD_ERR_ARG, "objective: x is not 16-byte aligned");
    if (h->o.model == ADPSGD_MODEL_MLP) return mlp_objective(h, x, out);
    std::vector<ObjectiveWorker> tab(h->n);
    int64_t max_rows = 0;
    for (int32_t i = 0; i < h->n; ++i) {
        if (!h->data[i].features) return fail(h, ADPSGD_ERR_STATE, "objective: no data loaded for worker " + std::to_string(i));
        tab[i] = {h->data[i].features, h->data[i].targets, h->data[i].rows, h->data[i].ld};
        max_rows = std::max(max_rows, h->data[i].rows);
    }
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    // diag buffer: [mean model d floats, 256-byte padded][worker table][partials][result]
    const int64_t groups = objective_row_groups(max_rows);
    const size_t off_tab = (static_cast<size_t>(h->d) * 4 + 255) & ~size_t(255);
    const size_t off_part = (off_tab + tab.size() * sizeof(ObjectiveWorker) + 255) & ~size_t(255);
    const size_t off_res = off_part + static_cast<size_t>(groups) * h->n * sizeof(double);
    HIP_TRY(h, h->diag.reserve(off_res + sizeof(double)));
    char* base = static_cast<char*>(h->diag.p);
    const float* point = x;
    if (!x) {
        HIP_TRY(h, launch_mean_model(h->o.X, h->o.ldx, h->d, h->n, reinterpret_cast<float*>(base), h->stream));
        point = reinterpret_cast<const float*>(base);
    }
    HIP_TRY(h, hipMemcpyAsync(base + off_tab, tab.data(), tab.size() * sizeof(ObjectiveWorker), hipMemcpyHostToDevice, h->stream));
    HIP_TRY(h, launch_objective(h->o.model, point, h->d, h->n, reinterpret_cast<const ObjectiveWorker*>(base + off_tab), max_rows,
                                h->o.lambda, reinterpret_cast<double*>(base + off_part), reinterpret_cast<double*>(base + off_res),
                                h->stream));
    HIP_TRY(h, hipMemcpyAsync(out, base + off_res, sizeof(double), hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return ADPSGD_OK;
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
    return ADPSGD_OK;
}

extern "C" int adpsgd_synth_gradient(uint64_t seed, uint64_t k, float std, int64_t d, float* out_device, void* stream) {
    if (!out_device || d < 0) return ADPSGD_ERR_ARG;
    const hipError_t e = launch_synth_gradient(seed, k, std, d, out_device, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? ADPSGD_OK : ADPSGD_ERR_HIP;
}
