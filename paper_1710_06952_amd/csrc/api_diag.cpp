// C-ABI entry points of libadpsgd, part 3: reading the state back and the diagnostics
// (models, momentum, mean model, consensus distance, divergence check, objective).
#include <cmath>
#include <cstring>

#include "handle.hpp"

using namespace adpsgd_impl;

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
    if (on_device) return ADPSGD_OK;      // ready in stream order: the caller goes on working on the stream
    HIP_TRY(h, hipMemcpyAsync(out, dst, static_cast<size_t>(h->d) * 4, hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return ADPSGD_OK;
}

namespace {

int consensus(adpsgd_t* h, const double* p, double* out) {
    if (!out) return fail(h, ADPSGD_ERR_ARG, "consensus_distance: out is NULL");
    double psum = 0.0;
    if (p) {
        for (int32_t i = 0; i < h->n; ++i) {
            if (!(p[i] >= 0.0) || !std::isfinite(p[i])) return fail(h, ADPSGD_ERR_ARG, "consensus_distance: weight negative or not finite");
            psum += p[i];
        }
        if (std::fabs(psum - 1.0) > 1e-9) return fail(h, ADPSGD_ERR_ARG, "consensus_distance: the weights do not sum to 1");
    }
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    const int32_t blocks = consensus_blocks(h->d);
    // diag buffer: [partials][result][weights]
    HIP_TRY(h, h->diag.reserve(static_cast<size_t>(blocks + 1 + (p ? h->n : 0)) * sizeof(double)));
    double* partial = static_cast<double*>(h->diag.p);
    double* d_p = nullptr;
    if (p) {
        d_p = partial + blocks + 1;
        HIP_TRY(h, hipMemcpyAsync(d_p, p, static_cast<size_t>(h->n) * sizeof(double), hipMemcpyHostToDevice, h->stream));
    }
    HIP_TRY(h, launch_consensus(h->o.X, h->o.ldx, h->d, h->n, partial, partial + blocks, d_p, psum, h->stream));
    HIP_TRY(h, hipMemcpyAsync(out, partial + blocks, sizeof(double), hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return ADPSGD_OK;
}

}  // namespace

extern "C" int adpsgd_consensus_distance(adpsgd_t* h, double* out) {
    if (!h) return ADPSGD_ERR_ARG;
    return consensus(h, nullptr, out);
}

extern "C" int adpsgd_consensus_distance_weighted(adpsgd_t* h, const double* p, double* out) {
    if (!h) return ADPSGD_ERR_ARG;
    if (!p) return fail(h, ADPSGD_ERR_ARG, "consensus_distance_weighted: p is NULL");
    return consensus(h, p, out);
}

extern "C" int adpsgd_consensus_distance_static(adpsgd_t* h, const double* p, double* out_device) {
    if (!h) return ADPSGD_ERR_ARG;
    if (!out_device) return fail(h, ADPSGD_ERR_ARG, "consensus_distance_static: out_device is NULL");
    const int32_t blocks = consensus_blocks(h->d);
    if (blocks > kStaticPartials)
        return fail(h, ADPSGD_ERR_ARG, "consensus_distance_static: d needs more block partials than the fixed array holds");
    double psum = 0.0;
    if (p) {
        if (h->n > kStaticWeights)
            return fail(h, ADPSGD_ERR_ARG, "consensus_distance_static: more than " + std::to_string(kStaticWeights) +
                                               " workers: the weights do not fit the fixed array (pass p = NULL, or use "
                                               "adpsgd_consensus_distance_weighted)");
        for (int32_t i = 0; i < h->n; ++i) {
            if (!(p[i] >= 0.0) || !std::isfinite(p[i])) return fail(h, ADPSGD_ERR_ARG, "consensus_distance_static: weight negative or not finite");
            psum += p[i];
        }
        if (std::fabs(psum - 1.0) > 1e-9) return fail(h, ADPSGD_ERR_ARG, "consensus_distance_static: the weights do not sum to 1");
    }
    double* base = nullptr;                       // the fixed array's address on this GPU
    HIP_TRY(h, static_scratch(&base));
    double* d_p = nullptr;
    if (p) {
        d_p = base + kStaticPartials + 8;
        HIP_TRY(h, hipMemcpyAsync(d_p, p, static_cast<size_t>(h->n) * sizeof(double), hipMemcpyHostToDevice, h->stream));
    }
    // every partial the final kernel reads is written by this launch: nothing has to start at zero
    HIP_TRY(h, launch_consensus(h->o.X, h->o.ldx, h->d, h->n, base, out_device, d_p, psum, h->stream));
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
int mlp_objective(adpsgd_t* h, const float* x, double* out, bool count_errors, const double* p) {
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
                      reinterpret_cast<const int32_t*>(base + off_idx) + g0 * static_cast<int64_t>(M), nullptr, 1.0f, nullptr, h->grad_scratch.p, false, false};
        HIP_TRY(h, launch_mlp_loss(a, d_sum + g0, count_errors, h->stream));
    }
    std::vector<double> sums(static_cast<size_t>(n_ops));
    HIP_TRY(h, hipMemcpyAsync(sums.data(), d_sum, sums.size() * sizeof(double), hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    double total = 0.0;
    for (int32_t i = 0; i < n; ++i) {
        double s = 0.0;
        for (int64_t o = first[i]; o < first[i + 1]; ++o) s += sums[o];
        total += (p ? p[i] : 1.0 / n) * (s / static_cast<double>(h->data[i].rows));
    }
    *out = total;
    return ADPSGD_OK;
}

// mean over the workers of the mean over their rows of the loss (or of the 0/1 classification error) at x
int evaluate(adpsgd_t* h, const float* x, double* out, bool count_errors, const double* p = nullptr) {
    if (x && !aligned16(x)) return fail(h, ADPSGD_ERR_ARG, "objective: x is not 16-byte aligned");
    if (p) {
        double psum = 0.0;
        for (int32_t i = 0; i < h->n; ++i) {
            if (!(p[i] >= 0.0) || !std::isfinite(p[i])) return fail(h, ADPSGD_ERR_ARG, "objective: weight negative or not finite");
            psum += p[i];
        }
        if (std::fabs(psum - 1.0) > 1e-9) return fail(h, ADPSGD_ERR_ARG, "objective: the weights do not sum to 1");
    }
    if (h->o.model == ADPSGD_MODEL_MLP) return mlp_objective(h, x, out, count_errors, p);
    std::vector<ObjectiveWorker> tab(h->n);
    int64_t max_rows = 0;
    for (int32_t i = 0; i < h->n; ++i) {
        if (!h->data[i].features) return fail(h, ADPSGD_ERR_STATE, "objective: no data loaded for worker " + std::to_string(i));
        tab[i] = {h->data[i].features, h->data[i].targets, h->data[i].rows, h->data[i].ld};
        max_rows = std::max(max_rows, h->data[i].rows);
    }
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    // diag buffer: [mean model d floats, 256-byte padded][worker table][partials][result][weights]
    const int64_t groups = objective_row_groups(max_rows);
    const size_t off_tab = (static_cast<size_t>(h->d) * 4 + 255) & ~size_t(255);
    const size_t off_part = (off_tab + tab.size() * sizeof(ObjectiveWorker) + 255) & ~size_t(255);
    const size_t off_res = off_part + static_cast<size_t>(groups) * h->n * sizeof(double);
    const size_t off_w = off_res + sizeof(double);
    HIP_TRY(h, h->diag.reserve(off_w + (p ? static_cast<size_t>(h->n) * sizeof(double) : 0)));
    char* base = static_cast<char*>(h->diag.p);
    if (p) HIP_TRY(h, hipMemcpyAsync(base + off_w, p, static_cast<size_t>(h->n) * sizeof(double), hipMemcpyHostToDevice, h->stream));
    const float* point = x;
    if (!x) {
        HIP_TRY(h, launch_mean_model(h->o.X, h->o.ldx, h->d, h->n, reinterpret_cast<float*>(base), h->stream));
        point = reinterpret_cast<const float*>(base);
    }
    HIP_TRY(h, hipMemcpyAsync(base + off_tab, tab.data(), tab.size() * sizeof(ObjectiveWorker), hipMemcpyHostToDevice, h->stream));
    HIP_TRY(h, launch_objective(h->o.model, point, h->d, h->n, reinterpret_cast<const ObjectiveWorker*>(base + off_tab), max_rows,
                                h->o.lambda, reinterpret_cast<double*>(base + off_part), reinterpret_cast<double*>(base + off_res),
                                count_errors, p ? reinterpret_cast<const double*>(base + off_w) : nullptr, h->stream));
    HIP_TRY(h, hipMemcpyAsync(out, base + off_res, sizeof(double), hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return ADPSGD_OK;
}

}  // namespace

extern "C" int adpsgd_objective(adpsgd_t* h, const float* x, double* out) {
    if (!h) return ADPSGD_ERR_ARG;
    if (!out) return fail(h, ADPSGD_ERR_ARG, "objective: out is NULL");
    if (h->o.model == ADPSGD_MODEL_SYNTH)
        return fail(h, ADPSGD_ERR_STATE, "objective: the synthetic-gradient model has no objective");
    return evaluate(h, x, out, false);
}

extern "C" int adpsgd_objective_weighted(adpsgd_t* h, const float* x, const double* p, double* out) {
    if (!h) return ADPSGD_ERR_ARG;
    if (!out || !p) return fail(h, ADPSGD_ERR_ARG, "objective_weighted: p or out is NULL");
    if (h->o.model == ADPSGD_MODEL_SYNTH)
        return fail(h, ADPSGD_ERR_STATE, "objective: the synthetic-gradient model has no objective");
    return evaluate(h, x, out, false, p);
}

extern "C" int adpsgd_classification_error(adpsgd_t* h, const float* x, double* out) {
    if (!h) return ADPSGD_ERR_ARG;
    if (!out) return fail(h, ADPSGD_ERR_ARG, "classification_error: out is NULL");
    if (h->o.model != ADPSGD_MODEL_LOGREG && h->o.model != ADPSGD_MODEL_MLP)
        return fail(h, ADPSGD_ERR_STATE, "classification_error: the model has no labels");
    return evaluate(h, x, out, true);
}
