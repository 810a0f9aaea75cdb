// Internal declarations shared by the host-side translation units of libadpsgd.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <string>
#include <vector>

#include "adpsgd.h"

namespace adpsgd_impl {

// One update event as the fused gossip-average + apply kernel sees it.
struct alignas(32) PairOp {
    int32_t i;        // worker i_k (takes the gradient step)
    int32_t j;        // neighbour j_k (i == j: no partner, plain SGD step)
    uint32_t k_lo;    // global event number (addresses the synthetic-gradient generator)
    uint32_t k_hi;
    float gamma;
    int32_t slot;     // pending-gradient slot holding g_k (data models)
    int32_t flags;    // bit 0: average only (an extra pair of a general W_k): no gradient, no step
    int32_t event;    // index into the call's batch_idx array (perceptron, factored gradient)
    const void* features;   // worker i's inputs (perceptron, factored gradient), else nullptr
    int64_t feat_ld;
};

// One stale read / gradient evaluation as the gradient kernels see it.
struct GradOp {
    int32_t worker;   // row read, and owner of the local data
    int32_t slot;     // where g_k goes
    int32_t event;    // index into the call's batch_idx / loss arrays
    int32_t comp_slot;   // wait-free variant: slot of the worker's own pending gradient g_k', or -1
    float comp_gamma;    // its step size: the read is x^ = row - comp_gamma * g_k'
    int32_t count;    // loss evaluation only: samples of the operation that count (the rest is padding)
    const void* features;   // the worker's local data (device), copied here so that a kernel reaches
    const void* targets;    //   it with one load instead of a second table look-up
    int64_t ld;             // leading dimension of features, in elements
    const void* xrow_bf16;  // perceptron, wait-free variant: bf16 row the gradient reads instead of the worker's
                            //   shadow (the compensated copy x - gamma_k' g_k'), or nullptr
};

struct WorkerData {
    const void* features = nullptr;
    const void* targets = nullptr;
    int64_t rows = 0;
    int64_t ld = 0;
};

struct Plan {
    std::vector<int32_t> r_round, u_round, slot;
    std::vector<int64_t> prev;   // wait-free variant: event whose pending gradient compensates the read, or -1
    int32_t n_rounds = 0;
};

// Grow-only device buffer owned by the library (small tables only).
struct DevBuf {
    void* p = nullptr;
    size_t cap = 0;
    hipError_t reserve(size_t bytes);
    void release();
};

// ---- host logic ------------------------------------------------------------
void philox4x32_10_host(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
int plan_rounds(int32_t n, int64_t K, const int32_t* worker, const int32_t* neighbour,
                const int32_t* tau, int32_t n_slots, bool with_gradients, Plan& plan,
                std::string& err, const int64_t* extra_ptr = nullptr, const int32_t* extra_a = nullptr,
                const int32_t* extra_b = nullptr, bool local_compensation = false,
                int64_t n_apply = -1, const int32_t* carried_slot = nullptr);
bool verify_plan(int32_t n, int64_t K, const int32_t* worker, const int32_t* neighbour, const int32_t* tau,
                 int32_t n_slots, bool with_gradients, const Plan& plan, std::string& err,
                 const int64_t* extra_ptr = nullptr, const int32_t* extra_a = nullptr, const int32_t* extra_b = nullptr,
                 int64_t n_apply = -1, const int32_t* carried_slot = nullptr);
bool graph_ok(const adpsgd_graph_t* g, std::string& err);

// ---- kernel launchers (each returns the hipError_t of the launch) ------------
struct FusedArgs {
    float* X;
    int64_t ld;
    int64_t d;
    const PairOp* ops;   // device
    int32_t n_ops;
    const float* slots;  // device, slot s at slots + s * ld (data models)
    uint16_t* Xbf16;     // device bf16 shadow or nullptr
    float synth_std;
    uint64_t synth_seed;
    bool synth;
    bool streaming;      // rows do not fit the caches: bypass them
    bool has_solo;       // some event of the round has i == j (worker without a neighbour)
    float* V;            // device momentum buffers (n x ld) or nullptr: plain event
    float momentum;
    float weight_decay;
};
hipError_t launch_fused_gossip_apply(const FusedArgs& a, hipStream_t st);

struct LinearGradArgs {
    int model;              // LSQ or LOGREG
    const float* X;
    int64_t ld;
    int64_t d;
    const GradOp* ops;      // device, this group's ops
    int32_t n_ops;
    int32_t M;
    const int32_t* batch_idx;  // device, K x M
    float* slots;
    float gscale;           // 1/M or 1
    float lambda;
    float* partial;         // device scratch: n_ops x (M + 1) x n_chunks
    float* coef;            // device scratch: n_ops x M
    float* loss;            // device, indexed by event, or nullptr
    bool factored;          // least squares: leave g as its M coefficients (start of the slot), no combine launch
};
int64_t linear_grad_chunks(int64_t d);
bool linear_can_factor(int model, int64_t d, int32_t M, int64_t ld);

// The update of a round with the least-squares gradients still in factored form (see the kernel).
struct LinearApplyArgs {
    float* X;
    int64_t ld;
    int64_t d;
    const PairOp* ops;      // device; features / feat_ld / event / slot name the factors
    int32_t n_ops;
    const float* slots;
    const int32_t* batch_idx;
    int32_t M;
    bool streaming;         // X does not fit the caches
    float* V;               // momentum buffers or nullptr
    float momentum, weight_decay;
};
hipError_t launch_linear_apply_factored(const LinearApplyArgs& a, hipStream_t st);
hipError_t launch_linear_gradient(const LinearGradArgs& a, hipStream_t st, int* n_launches);

struct MlpGradArgs {
    const float* X;         // device fp32 master, n x ld (read by the wait-free variant only)
    const uint16_t* Xbf16;  // device bf16 shadow, n x ld
    int64_t ld;
    int32_t in, hid, out;
    const GradOp* ops;
    int32_t n_ops;
    int32_t M;
    const int32_t* batch_by_op;   // device, n_ops x M: row t holds the minibatch indices of ops[t] (a kernel finds them
                                  //   from its block index, without waiting for the operation's descriptor)
    float* slots;
    float gscale;
    float* loss;
    void* scratch;          // device scratch, mlp_scratch_bytes(n_ops, ...)
    bool factored;          // leave dW1 as its factors: dH goes to the start of the slot, no dW1 launch
    bool compensate;        // wait-free variant: first build the compensated bf16 rows the operations name
};
size_t mlp_scratch_bytes(int32_t n_ops, int32_t M, int32_t in, int32_t hid, int32_t out);
// forward pass and cross-entropy only: loss_sum[op] = sum over the first `count` samples of the operation (fp64);
// count_errors: the number of those samples whose largest logit (lowest class on ties) is not their label instead
hipError_t launch_mlp_loss(const MlpGradArgs& a, double* loss_sum, bool count_errors, hipStream_t st);
bool mlp_can_factor(int32_t in, int32_t hid, int32_t M);

// The perceptron's model update with the first-layer gradient still in factored form
// (dW1 = Xb^T dH, rank <= M): the product is formed tile by tile on the matrix cores inside
// the update kernel instead of being written to and read back from the pending slot.
struct MlpApplyArgs {
    float* X;
    int64_t ld;
    int64_t d;
    int32_t in, hid, M;
    const PairOp* ops;      // device
    int32_t n_ops;
    const float* slots;
    uint16_t* Xbf16;
    const int32_t* batch_by_op; // device, n_ops x M: row t holds the minibatch indices of the event of ops[t]
    float* V;                   // momentum buffers or nullptr
    float momentum, weight_decay;
};
hipError_t launch_mlp_apply_factored(const MlpApplyArgs& a, hipStream_t st);
hipError_t launch_mlp_gradient(const MlpGradArgs& a, hipStream_t st, int* n_launches);

struct SyncArgs {
    float* X;
    int64_t ld;
    int64_t d;
    int32_t n;
    const int32_t* rowptr;   // device
    const int32_t* col;      // device
    const float* w_self;     // device
    const float* w_edge;     // device
    const float* slots;      // gradient of worker i in slot i, or nullptr with synth
    uint16_t* Xbf16;         // bf16 shadow to refresh, or nullptr
    float gamma;
    float synth_std;
    uint64_t synth_seed;
    uint64_t event0;         // synthetic gradients: worker i draws event event0 + i
    bool synth;
    float* V;                // momentum buffers or nullptr
    float momentum, weight_decay;
    bool ring;               // the graph is a ring with neighbour lists (i - 1, i + 1) mod n, n >= 3: no LDS staging needed
    float* Xdst = nullptr;   // write the new models to this matrix (same ld, not X) instead of in place
};
int32_t sync_tile_cols(int32_t n);   // 0: n too large for the in-place mixing kernel
bool sync_out_of_place_ok(int32_t n, int64_t d);   // the launch geometry of the out-of-place kernels exists
hipError_t launch_sync_mix_apply(const SyncArgs& a, hipStream_t st);

hipError_t launch_broadcast_rows(float* X, int64_t ld, int64_t d, int32_t n, const float* x0, hipStream_t st);
hipError_t launch_refresh_bf16(const float* X, uint16_t* Xb, int64_t ld, int32_t n, hipStream_t st);
hipError_t launch_mean_model(const float* X, int64_t ld, int64_t d, int32_t n, float* out, hipStream_t st);
int32_t consensus_blocks(int64_t d);
// adpsgd_consensus_distance_static: capacity of the library's fixed device array (block partials, worker
// probabilities) and its address on the current GPU (resolved on the first call per device)
constexpr int kStaticPartials = 2048;
constexpr int kStaticWeights = 4096;
hipError_t static_scratch(double** out);
// p: device, n doubles (the workers' update probabilities, psum their sum), or nullptr for the uniform weights 1 / n
hipError_t launch_consensus(const float* X, int64_t ld, int64_t d, int32_t n, double* partial,
                            double* result, const double* p, double psum, hipStream_t st);
hipError_t launch_count_nonfinite(const float* X, int64_t ld, int64_t d, int32_t n, unsigned long long* partial,
                                  int32_t blocks, hipStream_t st);
// one worker's local data as the objective kernel sees it
struct ObjectiveWorker {
    const void* features;
    const void* targets;
    int64_t rows;
    int64_t ld;
};
int64_t objective_row_groups(int64_t max_rows);
hipError_t launch_objective(int model, const float* x, int64_t d, int32_t n, const ObjectiveWorker* workers, int64_t max_rows,
                            float lambda, double* partial, double* result, bool count_errors, const double* weights,
                            hipStream_t st);   // weights: device, n probabilities, or nullptr for 1 / n
// out[t] (ld floats each) = X[ops[t].worker] - comp_gamma * slot[comp_slot] for the compensated operations of a group
hipError_t launch_compensated_rows(const float* X, int64_t ld, const GradOp* ops, int32_t n_ops, const float* slots, float* out,
                                   hipStream_t st);
hipError_t launch_synth_gradient(uint64_t seed, uint64_t k, float std, int64_t d, float* out, hipStream_t st);

}  // namespace adpsgd_impl
