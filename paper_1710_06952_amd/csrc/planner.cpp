// Round planner: turns the serial event order of Algorithm 1 into rounds of
// operations that touch disjoint model rows.
//
// Event k contributes two operations:
//   R_k  reads row i_k as it was before event s_k = k - tau_k (the stale model
//        x^_k = column i_k of X_{k - tau_k}) and evaluates g_k into a slot;
//   U_k  averages rows i_k, j_k and applies -gamma g_k to row i_k.
// A round executes all its R operations first, then all its U operations.
// Per row the plan keeps: the U operations in event order; R_k after every U_m
// with m < s_k on row i_k and not after any U_m with m >= s_k on that row
// (the same round is allowed, because reads precede updates inside a round);
// a slot is reused only in a later round than the update that consumed it.
// Disjoint pairwise averages commute, so executing the rounds in order gives
// exactly the serial result.
//
// A call may look ahead: of the K events in the arrays only the first n_apply are applied; the others
// are the first events of the next call, named now so that those of their stale reads that fall before
// event n_apply are evaluated while the models they need still exist.  Such a gradient stays in its
// slot after the call ("carried"); the next call names it through carried_slot and plans no read for it.
#include <algorithm>
#include <queue>

#include "internal.hpp"

namespace adpsgd_impl {

int plan_rounds(int32_t n, int64_t K, const int32_t* worker, const int32_t* neighbour,
                const int32_t* tau, int32_t n_slots, bool with_gradients, Plan& plan,
                std::string& err, const int64_t* extra_ptr, const int32_t* extra_a, const int32_t* extra_b,
                bool local_compensation, int64_t n_apply, const int32_t* carried_slot) {
    if (n_apply < 0 || n_apply > K) n_apply = K;
    if (!with_gradients) carried_slot = nullptr;
    auto carried = [&](int64_t k) { return carried_slot && carried_slot[k] >= 0; };
    plan.r_round.assign(static_cast<size_t>(K), -1);
    plan.u_round.assign(static_cast<size_t>(K), -1);
    plan.slot.assign(static_cast<size_t>(K), -1);
    plan.prev.assign(static_cast<size_t>(K), -1);
    plan.n_rounds = 0;

    // rounds are numbered from 1 while planning (0 = "never touched"), shifted to 0 at the end
    std::vector<int32_t> last_write(n, 0);  // round of the last U on the row
    std::vector<int32_t> last_read(n, 0);   // latest round of an R on the row

    // events grouped by the logical time of their read, s_k = k - tau_k
    std::vector<int64_t> head(static_cast<size_t>(K) + 1, -1), next(static_cast<size_t>(K), -1);
    int32_t tau_max = 0;
    std::vector<char> slot_taken(with_gradients ? static_cast<size_t>(std::max(n_slots, 0)) : 0, 0);
    if (with_gradients) {
        for (int64_t k = K - 1; k >= 0; --k) {
            if (tau[k] < 0) { err = "plan: tau[k] < 0"; return ADPSGD_ERR_SCHEDULE; }
            tau_max = std::max(tau_max, tau[k]);
            if (carried(k)) {        // evaluated by an earlier call: no read here, the slot is in use from the start
                const int32_t sl = carried_slot[k];
                if (tau[k] <= k) { err = "plan: a carried gradient has its read time before this call"; return ADPSGD_ERR_SCHEDULE; }
                if (sl >= n_slots || slot_taken[sl]) { err = "plan: carried slot out of range or named twice"; return ADPSGD_ERR_SCHEDULE; }
                slot_taken[sl] = 1;
                plan.slot[k] = sl;
                plan.r_round[k] = 0;
                continue;
            }
            if (tau[k] > k) { err = "plan: tau[k] outside [0, k]"; return ADPSGD_ERR_SCHEDULE; }
            const int64_t s = k - tau[k];
            if (s >= n_apply) continue;      // a read of the next call
            next[k] = head[s];
            head[s] = k;
        }
        if (n_slots <= tau_max) {
            err = "plan: need more pending-gradient slots than the largest staleness";
            return ADPSGD_ERR_SCHEDULE;
        }
    }
    // Wait-free variant: R_k also reads the pending gradient of the worker's previous event k' when
    // that gradient exists at the time of the read and is not applied yet (s_k' <= s_k <= k').
    // R_k then runs after R_k'; it cannot run after U_k' (it reads row i_k before that update), and
    // the slot of k' is rewritten only in a later round than U_k', so the slot is still intact.
    if (with_gradients && local_compensation) {
        std::vector<int64_t> last_of(n, -1);
        for (int64_t k = 0; k < K; ++k) {
            const int64_t kp = last_of[worker[k]], s = k - tau[k];
            if (kp >= 0 && !carried(k) && s < n_apply && kp - tau[kp] <= s && s <= kp) plan.prev[k] = kp;
            last_of[worker[k]] = k;
        }
    }
    // free slots ordered by the round after which they may be rewritten
    using Free = std::pair<int32_t, int32_t>;  // (round of the consuming update, slot)
    std::priority_queue<Free, std::vector<Free>, std::greater<Free>> free_slots;
    if (with_gradients)
        for (int32_t s = 0; s < n_slots; ++s)
            if (!slot_taken[s]) free_slots.push({0, s});

    int32_t rounds = 0;
    for (int64_t t = 0; t < n_apply; ++t) {
        if (with_gradients) {
            for (int64_t k = head[t]; k >= 0; k = next[k]) {
                const int32_t i = worker[k];
                if (free_slots.empty()) { err = "plan: internal error, no free slot"; return ADPSGD_ERR_STATE; }
                const Free f = free_slots.top();
                free_slots.pop();
                int32_t r = std::max(last_write[i], f.first) + 1;
                if (plan.prev[k] >= 0) r = std::max(r, plan.r_round[plan.prev[k]] + 1);
                plan.r_round[k] = r;
                plan.slot[k] = f.second;
                last_read[i] = std::max(last_read[i], r);
                rounds = std::max(rounds, r);      // a looked-ahead read may come after the last update
            }
        }
        const int32_t i = worker[t], j = neighbour[t];
        int32_t u = std::max(last_write[i], last_write[j]) + 1;
        u = std::max(u, std::max(last_read[i], last_read[j]));
        if (with_gradients) u = std::max(u, plan.r_round[t]);
        if (extra_ptr) {      // every pair of W_t runs in the event's round
            for (int64_t q = extra_ptr[t]; q < extra_ptr[t + 1]; ++q) {
                const int32_t a = extra_a[q], b = extra_b[q];
                u = std::max(u, std::max(last_write[a], last_write[b]) + 1);
                u = std::max(u, std::max(last_read[a], last_read[b]));
            }
            for (int64_t q = extra_ptr[t]; q < extra_ptr[t + 1]; ++q) last_write[extra_a[q]] = last_write[extra_b[q]] = u;
        }
        plan.u_round[t] = u;
        last_write[i] = last_write[j] = u;
        rounds = std::max(rounds, u);
        if (with_gradients) free_slots.push({u, plan.slot[t]});
    }
    for (int64_t k = 0; k < K; ++k) {      // to 0-based rounds; -1: no such operation in this call
        plan.u_round[k] = k < n_apply ? plan.u_round[k] - 1 : -1;
        if (with_gradients && plan.r_round[k] >= 0) plan.r_round[k] -= 1;
    }
    plan.n_rounds = rounds;
    return ADPSGD_OK;
}

// Independent check of a plan against the serial semantics (the library's race detector):
//   1. the updates of a round touch pairwise distinct rows;
//   2. per row the updates keep their event order, in strictly increasing rounds;
//   3. the read of event k sees exactly the updates of its row with index < s_k = k - tau_k: the last
//      such update lies in an earlier round, the first update with index >= s_k in the same or a later one;
//   4. a gradient is computed no later than the round that applies it, and a slot is rewritten only in
//      a later round than the update that consumed it;
//   5. wait-free variant: a compensated read runs after the gradient it uses and no later than the round
//      that applies that gradient;
//   6. looking ahead: only the first n_apply events are updated; an event beyond them has a read in this
//      call exactly when its read time lies before event n_apply, and its slot is not given away; a
//      carried gradient keeps its slot and has no read.
bool verify_plan(int32_t n, int64_t K, const int32_t* worker, const int32_t* neighbour, const int32_t* tau,
                 int32_t n_slots, bool with_gradients, const Plan& plan, std::string& err,
                 const int64_t* extra_ptr, const int32_t* extra_a, const int32_t* extra_b,
                 int64_t n_apply, const int32_t* carried_slot) {
    if (n_apply < 0 || n_apply > K) n_apply = K;
    if (!with_gradients) carried_slot = nullptr;
    auto carried = [&](int64_t k) { return carried_slot && carried_slot[k] >= 0; };
    auto bad = [&](const std::string& what, int64_t k) {
        err = "plan check: " + what + " at event " + std::to_string(k);
        return false;
    };
    if (static_cast<int64_t>(plan.u_round.size()) != K) return bad("wrong size", 0);
    // rows of every event, and per row the events that update it (in event order)
    std::vector<std::vector<int64_t>> touches(n);
    std::vector<int64_t> stamp_round(n, -1), stamp_event(n, -1);
    auto rows_of = [&](int64_t k, std::vector<int32_t>& rows) {
        rows.clear();
        rows.push_back(worker[k]);
        if (neighbour[k] != worker[k]) rows.push_back(neighbour[k]);
        if (extra_ptr)
            for (int64_t q = extra_ptr[k]; q < extra_ptr[k + 1]; ++q) {
                rows.push_back(extra_a[q]);
                rows.push_back(extra_b[q]);
            }
    };
    std::vector<int32_t> rows;
    for (int64_t k = n_apply; k < K; ++k)
        if (plan.u_round[k] != -1) return bad("update planned for an event that is only looked ahead to", k);        // 6
    for (int64_t k = 0; k < n_apply; ++k) {
        const int32_t u = plan.u_round[k];
        if (u < 0 || u >= plan.n_rounds) return bad("update round out of range", k);
        rows_of(k, rows);
        for (int32_t r : rows) {
            if (!touches[r].empty()) {
                const int64_t m = touches[r].back();
                if (m == k) return bad("an event names a row twice", k);
                if (plan.u_round[m] >= u) return bad("updates of a row out of order or sharing a round", k);   // 1 and 2
            }
            touches[r].push_back(k);
        }
    }
    if (!with_gradients) return true;
    std::vector<int64_t> slot_last(n_slots, -1);      // event that last used the slot, in order of the rounds
    std::vector<int64_t> order;
    for (int64_t k = 0; k < K; ++k) {
        const int32_t sl = plan.slot[k];
        if (carried(k)) {                                                                                      // 6
            if (sl != carried_slot[k] || plan.r_round[k] != -1) return bad("carried gradient moved or read again", k);
            if (sl >= n_slots || slot_last[sl] >= 0) return bad("carried slot out of range or named twice", k);
            if (tau[k] <= k) return bad("carried gradient with a read time inside this call", k);
            slot_last[sl] = k;
        } else if (k - tau[k] >= n_apply) {
            if (sl != -1 || plan.r_round[k] != -1) return bad("read planned for an event of the next call", k);
        } else {
            order.push_back(k);
        }
    }
    // an event that is not applied in this call never gives its slot away
    auto applied_before = [&](int64_t m, int32_t r) { return m < n_apply && plan.u_round[m] < r; };
    std::stable_sort(order.begin(), order.end(), [&](int64_t a, int64_t b) { return plan.r_round[a] < plan.r_round[b]; });
    for (int64_t k : order) {
        const int32_t r = plan.r_round[k], i = worker[k];
        if (r < 0 || r >= plan.n_rounds || (k < n_apply && r > plan.u_round[k])) return bad("gradient later than its update", k);   // 4
        const int64_t s = k - tau[k];
        const auto& tv = touches[i];
        const auto it = std::lower_bound(tv.begin(), tv.end(), s);      // first update of the row with index >= s
        if (it != tv.begin() && plan.u_round[*(it - 1)] >= r) return bad("stale read misses an earlier update", k);   // 3
        if (it != tv.end() && plan.u_round[*it] < r) return bad("stale read sees a later update", k);                // 3
        const int32_t sl = plan.slot[k];
        if (sl < 0 || sl >= n_slots) return bad("slot out of range", k);
        if (slot_last[sl] >= 0 && !applied_before(slot_last[sl], r)) return bad("slot rewritten before its gradient was applied", k);   // 4
        slot_last[sl] = k;
        const int64_t kp = plan.prev[k];
        if (kp >= 0 && !(plan.r_round[kp] < r && plan.slot[kp] >= 0 && (kp >= n_apply || r <= plan.u_round[kp])))
            return bad("compensated read outside the life of its gradient", k);   // 5
    }
    return true;
}

}  // namespace adpsgd_impl

using namespace adpsgd_impl;

extern "C" int adpsgd_verify_plan(int32_t n, int64_t K, const int32_t* worker, const int32_t* neighbour,
                                  const int32_t* tau, int32_t n_slots, int32_t with_gradients,
                                  const int32_t* r_round, const int32_t* u_round, const int32_t* slot, int32_t n_rounds,
                                  const int64_t* extra_ptr, const int32_t* extra_a, const int32_t* extra_b,
                                  const int64_t* prev, int64_t n_apply, const int32_t* carried_slot) {
    if (n < 1 || K < 0 || !worker || !neighbour || !tau || !r_round || !u_round || !slot) return ADPSGD_ERR_ARG;
    for (int64_t k = 0; k < K; ++k)
        if (worker[k] < 0 || worker[k] >= n || neighbour[k] < 0 || neighbour[k] >= n || tau[k] < 0 ||
            (tau[k] > k && !(carried_slot && carried_slot[k] >= 0)))
            return ADPSGD_ERR_SCHEDULE;
    Plan plan;
    plan.r_round.assign(r_round, r_round + K);
    plan.u_round.assign(u_round, u_round + K);
    plan.slot.assign(slot, slot + K);
    if (prev) plan.prev.assign(prev, prev + K);
    else plan.prev.assign(static_cast<size_t>(K), -1);
    plan.n_rounds = n_rounds;
    std::string err;
    return verify_plan(n, K, worker, neighbour, tau, n_slots, with_gradients != 0, plan, err, extra_ptr, extra_a, extra_b,
                       n_apply, carried_slot)
               ? ADPSGD_OK : ADPSGD_ERR_STATE;
}

extern "C" int adpsgd_plan_rounds(int32_t n, int64_t K, const int32_t* worker, const int32_t* neighbour,
                                  const int32_t* tau, int32_t n_slots, int32_t with_gradients,
                                  int32_t* r_round, int32_t* u_round, int32_t* slot, int32_t* n_rounds,
                                  const int64_t* extra_ptr, const int32_t* extra_a, const int32_t* extra_b,
                                  int32_t local_compensation, int64_t* prev, int64_t n_apply, const int32_t* carried_slot) {
    if (n < 1 || K < 0 || !worker || !neighbour || !tau || !r_round || !u_round || !slot || !n_rounds)
        return ADPSGD_ERR_ARG;
    for (int64_t k = 0; k < K; ++k)
        if (worker[k] < 0 || worker[k] >= n || neighbour[k] < 0 || neighbour[k] >= n) return ADPSGD_ERR_SCHEDULE;
    if (extra_ptr) {
        if (!extra_a || !extra_b || extra_ptr[0] != 0) return ADPSGD_ERR_ARG;
        for (int64_t k = 0; k < K; ++k)
            if (extra_ptr[k + 1] < extra_ptr[k]) return ADPSGD_ERR_SCHEDULE;
        for (int64_t q = 0; q < extra_ptr[K]; ++q)
            if (extra_a[q] < 0 || extra_a[q] >= n || extra_b[q] < 0 || extra_b[q] >= n) return ADPSGD_ERR_SCHEDULE;
    }
    Plan plan;
    std::string err;
    const int rc = plan_rounds(n, K, worker, neighbour, tau, n_slots, with_gradients != 0, plan, err, extra_ptr, extra_a, extra_b,
                               local_compensation != 0, n_apply, carried_slot);
    if (rc != ADPSGD_OK) return rc;
    std::copy(plan.r_round.begin(), plan.r_round.end(), r_round);
    std::copy(plan.u_round.begin(), plan.u_round.end(), u_round);
    std::copy(plan.slot.begin(), plan.slot.end(), slot);
    if (prev) std::copy(plan.prev.begin(), plan.prev.end(), prev);
    *n_rounds = plan.n_rounds;
    return ADPSGD_OK;
}
