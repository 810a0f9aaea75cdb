// The handle behind adpsgd_t and the small helpers shared by the translation units that
// implement the C ABI (api.cpp, api_sync.cpp, api_diag.cpp).
#pragma once

#include <algorithm>
#include <string>
#include <utility>
#include <vector>

#include "internal.hpp"

namespace adpsgd_impl {

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

// An event the previous call has looked ahead to: the next call must start with these events.
struct PendingEvent {
    int32_t worker;
    int32_t tau;
    int32_t slot;      // pending-gradient slot that holds its gradient, or -1 when it is still to be evaluated
};

constexpr int64_t kStreamingThreshold = 256ll << 20;
constexpr int32_t kMaxSlots = 4096;

}  // namespace adpsgd_impl

struct adpsgd {
    int32_t n = 0;
    int64_t d = 0;
    adpsgd_opts_t o{};
    std::vector<int32_t> rowptr, col;
    std::vector<adpsgd_impl::WorkerData> data;
    int32_t n_slots = 0;
    hipStream_t stream = nullptr;
    bool streaming = false;
    uint64_t events_done = 0;
    std::vector<adpsgd_impl::PendingEvent> pending;   // events looked ahead to by the last call, in order
    std::vector<int32_t> pending_batch;               // their minibatch indices, M each
    adpsgd_impl::TableSet tables[2];
    int next_table = 0;
    adpsgd_impl::DevBuf grad_scratch;     // dots partials + coefficients / MLP activations
    adpsgd_impl::DevBuf comp_rows;        // perceptron, wait-free variant: compensated bf16 copies of the rows a group of gradients reads
    adpsgd_impl::DevBuf diag;             // consensus partials, result, mean / broadcast staging
    adpsgd_impl::DevBuf sync_other;       // synchronous schedule: the second model matrix of the out-of-place iterations
    bool sync_other_refused = false;      // ... its allocation failed once: the iterations run in place from then on
    adpsgd_stats_t stats{};
    std::vector<hipEvent_t> ev_pool;                       // profiling events
    std::vector<std::pair<hipEvent_t, hipEvent_t>> ev_fused, ev_grad;
    std::string err;
};

namespace adpsgd_impl {

// record a message for adpsgd_last_error and return the code (h == nullptr: message of a failed create)
int fail(adpsgd_t* h, int code, const std::string& msg);
int hip_fail(adpsgd_t* h, hipError_t e, const char* what);
const std::string& create_error();
#define HIP_TRY(h, expr)                                           \
    do {                                                           \
        hipError_t e__ = (expr);                                   \
        if (e__ != hipSuccess) return hip_fail((h), e__, #expr);   \
    } while (0)

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool is_neighbour(const adpsgd_t* h, int32_t i, int32_t j);
void metropolis(const std::vector<int32_t>& rowptr, const std::vector<int32_t>& col, float* w_self, float* w_edge);
hipEvent_t take_event(adpsgd_t* h);
// Fold the timings of finished launches into the statistics (synchronises the stream).
int drain_profile(adpsgd_t* h);

}  // namespace adpsgd_impl
