/*
 * adpsgd.h -- C ABI of the MI355X-native AD-PSGD worker-update engine.
 *
 * The library simulates the n worker replicas of asynchronous decentralized
 * parallel SGD as an n x d fp32 matrix X in one GPU's memory (row i = worker
 * i's model x^i; the paper stores the replicas as the columns of an N x n
 * matrix) and executes a seeded schedule of update events.  One event k is the
 * loop body of Algorithm 1 ("AD-PSGD, logical view"), in the matrix form given
 * at the start of the theory section:
 *
 *     X_{k+1} = X_k W_k - gamma * dg(X^_k; xi_k, i_k),   X^_k = X_{k - tau_k}
 *
 *   - worker i_k computes a minibatch gradient g_k at a stale read x^ of its
 *     own model (row i_k as it was before event k - tau_k);
 *   - W_k averages worker i_k with one graph neighbour j_k: both rows become
 *     (x^i + x^j)/2  (Sec. 3.2 "Averaging"; W_k = I - (e_i-e_j)(e_i-e_j)^T/2 is
 *     symmetric and doubly stochastic, assumption 2 of the theory section);
 *   - row i_k then takes the step  x^i <- x^i - gamma * g_k.
 *
 * Events whose rows are disjoint commute, so the library reorders the schedule
 * into rounds of row-disjoint operations; the result is identical, bit for
 * bit, to executing the events one after another.
 *
 * General conventions
 *   - Every function returns ADPSGD_OK (0) or a negative ADPSGD_ERR_* code and
 *     never throws.  adpsgd_last_error() gives a message for the last failure
 *     on a handle.  A call that fails validation changes no state.
 *   - "host" / "device" is stated for every pointer.  The library never frees
 *     caller memory.  Device pointers handed to the library stay BORROWED for
 *     the life of the handle (the caller, e.g. a tensor library, owns them).
 *   - A handle is not thread safe.  All GPU work of a handle is enqueued on the
 *     stream given at creation; calls are asynchronous unless stated.
 *   - All floating-point state is fp32; gradients accumulate in fp32.
 */
#ifndef ADPSGD_H
#define ADPSGD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct adpsgd adpsgd_t;

enum {
    ADPSGD_OK = 0,
    ADPSGD_ERR_ARG = -1,      /* null pointer, bad size, misaligned buffer      */
    ADPSGD_ERR_GRAPH = -2,    /* graph not symmetric / simple / connected       */
    ADPSGD_ERR_SCHEDULE = -3, /* schedule violates a documented constraint      */
    ADPSGD_ERR_STATE = -4,    /* call not valid in the handle's current state   */
    ADPSGD_ERR_HIP = -5,      /* a HIP runtime call failed                      */
    ADPSGD_ERR_CALLBACK = -6  /* the caller's gradient function reported an error */
};

/* Local loss F_i(x; xi) of the problem statement  min_x sum_i p_i E_xi F_i(x; xi)
 * (Sec. 3.1).  The paper leaves F abstract; these are the workloads built in. */
enum {
    ADPSGD_MODEL_LSQ = 0,    /* F = (a.x - b)^2 / 2                               */
    ADPSGD_MODEL_LOGREG = 1, /* F = log(1 + exp(-y a.x)) + lambda |x|^2 / 2        */
    ADPSGD_MODEL_SYNTH = 2,  /* no data: g_k[e] = synth_std * N(0,1)(seed, k, e)   */
    ADPSGD_MODEL_MLP = 3,    /* in -> hidden (ReLU) -> out, softmax cross-entropy, */
                             /* bf16 weights/inputs, fp32 master and accumulation  */
    ADPSGD_MODEL_EXTERNAL = 4 /* F is the caller's: the gradient step of Algorithm 1 is a function the caller
                                 passes to adpsgd_run_events_with; sampling, stale reads, averaging and the
                                 update stay the library's.  No data is loaded; M, lambda, grad_sum unused */
};

enum {
    ADPSGD_FLAG_PROFILE = 1, /* time every kernel launch with HIP events (see adpsgd_get_stats) */
    ADPSGD_FLAG_VERIFY_PLAN = 4, /* check every plan of rounds against the serial semantics before anything is
                                    launched (no two updates of a round share a row, every stale read sees exactly
                                    the updates before its logical time, slots live long enough); a violation is a
                                    library bug and returns ADPSGD_ERR_STATE.  O(K log K) host work per call */
    ADPSGD_FLAG_SYNC_IN_PLACE = 8,  /* adpsgd_run_sync_steps: never allocate the second model matrix that the iterations
                                       otherwise alternate with; every iteration then mixes in place (same
                                       results, 12 - 30 % slower at n = 128, d = 25.6 M depending on the graph) */
    ADPSGD_FLAG_DENSE_GRADIENT = 2  /* always write gradients out as dense vectors.  By default (without the
                                       wait-free variant) low-rank gradients stay in factored form until the
                                       update kernel applies them: the MLP's first layer as dH and the minibatch
                                       inputs, least squares on long models as its M coefficients.  The values
                                       are the same; the dense form costs one more launch and a write and
                                       read-back of the gradient per event */
};

/* Undirected communication graph (V, E) of Sec. 3.1 as CSR adjacency lists.
 * host memory, copied by adpsgd_create.  Must be symmetric, without self loops
 * or duplicate edges, and connected. */
typedef struct {
    int32_t n;             /* number of workers                                  */
    const int32_t* rowptr; /* host, n + 1 entries, rowptr[0] = 0                  */
    const int32_t* col;    /* host, rowptr[n] entries: neighbours of each worker  */
} adpsgd_graph_t;

typedef struct {
    int32_t model;       /* ADPSGD_MODEL_*                                        */
    int32_t M;           /* minibatch size (ignored for SYNTH)                    */
    float gamma;         /* step size, used when a schedule carries no per-event gamma */
    float lambda;        /* L2 coefficient (LOGREG)                               */
    int32_t grad_sum;    /* 0: g = (1/M) sum_m grad F  (mean);  1: the paper's literal sum */
    int32_t T_max;       /* bound T on the staleness tau_k (assumption 7)         */
    float synth_std;     /* SYNTH: standard deviation of every gradient entry     */
    uint64_t synth_seed; /* SYNTH: seed of the counter-based generator            */
    int32_t mlp_in, mlp_hidden, mlp_out; /* MLP layer sizes; d must equal
                            in*hidden + hidden + hidden*out + out, parameters flattened as
                            [W1 (in x hidden, row-major), b1, W2 (hidden x out), b2] */
    float* X;            /* device, n x ldx fp32, 16-byte aligned, caller-owned    */
    int64_t ldx;         /* leading dimension in floats, >= d, multiple of 4; entries
                            [d, ldx) of every row must be zero and stay zero        */
    uint16_t* Xbf16;     /* device, n x ldx bf16 shadow of X (MLP only, else NULL)  */
    void* workspace;     /* device, 16-byte aligned: pending-gradient slots, each
                            ldx floats.  NULL allowed for SYNTH                    */
    int64_t workspace_bytes; /* >= (T_max + 1) * ldx * 4 for the data models; more
                            slots let more events run per round                    */
    void* stream;        /* hipStream_t on the current device; NULL = default stream */
    int32_t flags;       /* ADPSGD_FLAG_*                                         */
    /* Optimizer of the paper's experiments (Sec. 5.2: momentum 0.9, weight decay 1e-4); Algorithm 1
     * itself has neither (both 0: the plain event).  Each worker keeps its own momentum buffer v^i
     * (local state, never averaged); both act on the model being updated, the averaged x_{k+1/2}^i:
     *     u = g_k + weight_decay * x_{k+1/2}^i;  v^i <- momentum * v^i + u;  x^i <- x_{k+1/2}^i - gamma * v^i */
    float momentum;
    float weight_decay;
    float* V;            /* device, n x ldx fp32 momentum buffers, caller-owned; required when momentum or
                            weight_decay is non-zero, else NULL.  adpsgd_set_models zeroes it */
    /* Wait-free variant (appendix "Wait-free (continuous) training and communication", the
     * computation thread): a worker applies its own gradient that is computed but not yet applied
     * to the copy it reads, and evaluates the next gradient there:
     *     x^_k = X_{k - tau_k}[i_k] - gamma_k' g_k'
     * where k' is the latest earlier event of worker i_k in the same call, taken when
     * k' - tau_k' <= k - tau_k <= k' (else no compensation).  Ignored by SYNTH, whose gradients do
     * not depend on the model; the MLP reads bf16(x^_k) and keeps its pending gradients dense for
     * it.  With momentum or weight decay the compensation stays this line (the computation thread
     * holds the buffered gradient and the step size, nothing of the optimizer); only the update
     * follows the optimizer's rule. */
    int32_t local_compensation;
} adpsgd_opts_t;

/* A batch of K events, all arrays in host memory, read during the call only.
 * Constraints (else ADPSGD_ERR_SCHEDULE, with no state change):
 *   0 <= worker[k] < n;  neighbour[k] is a graph neighbour of worker[k], or
 *   equals worker[k]: W_k = I, the worker applies the gradient without
 *   averaging.  That is the step of a worker that has no neighbour, and it
 *   expresses the gradient queue the wait-free appendix mentions (computation
 *   thread): q gradients queued before one communication step are that step's
 *   event followed by q - 1 such events of the same worker, each with the
 *   staleness its gradient had;
 *   0 <= tau[k] <= min(k, T_max): staleness does not reach behind the first event of the
 *   call, except for the events an earlier call has looked ahead to (see lookahead);
 *   0 <= batch_idx[k*M + m] < rows loaded for worker[k]. */
typedef struct {
    int64_t K;
    const int32_t* worker;    /* i_k                                             */
    const int32_t* neighbour; /* j_k: fixes W_k                                  */
    const int32_t* tau;       /* tau_k                                           */
    const int32_t* batch_idx; /* K x M sample indices xi_k (NULL for SYNTH)      */
    const float* gamma;       /* K per-event step sizes, or NULL                 */
    /* General averaging matrix (Sec. 3.2: W may be any doubly stochastic matrix): event k may
     * average further pairs of neighbours (extra_a[q], extra_b[q]), extra_ptr[k] <= q < extra_ptr[k+1],
     * in the same W_k.  All rows of one event (worker, neighbour, extras) must be distinct and every
     * extra pair must be an edge of the graph; W_k is then the product of disjoint pairwise
     * averagings (symmetric, doubly stochastic).  Extra pairs carry no gradient.  NULL = none. */
    const int64_t* extra_ptr; /* K + 1 entries, extra_ptr[0] = 0                  */
    const int32_t* extra_a;
    const int32_t* extra_b;
    /* A long run split into calls keeps Algorithm 1's staleness across the call boundaries when every
     * call looks ahead: of the K events in the arrays the last `lookahead` are NOT applied by this call;
     * they are the first events of the next call, named now so that those of their stale reads that fall
     * before the end of this call (k - tau[k] < K - lookahead) are evaluated while the models they need
     * exist.  Such a gradient stays pending in its slot.  The next call must then start with exactly these
     * events (same worker, tau and batch indices, else ADPSGD_ERR_SCHEDULE); for them tau[k] > k is what
     * is expected, up to T_max.  0 = none: the call is self-contained.  A loss array has K entries; the
     * entry of an event is written by the call that evaluates its gradient.  adpsgd_set_models and
     * adpsgd_set_event_count drop what is pending. */
    int64_t lookahead;
} adpsgd_schedule_t;

/* Parameters of the built-in schedule generator (all host memory). */
typedef struct {
    adpsgd_graph_t graph;
    const int32_t* weight;  /* n integer update frequencies (p_i = weight_i / sum), NULL = uniform */
    int32_t tau_mode;       /* 0: tau ~ Uniform{0..T_max};  1: geometric P(tau >= t) = (num_i/den_i)^t, capped at T_max */
    int32_t T_max;
    const int32_t* tau_num; /* n entries (tau_mode 1) */
    const int32_t* tau_den; /* n entries (tau_mode 1) */
    int32_t M;              /* minibatch size, 0 = no batch indices */
    const int32_t* rows;    /* n local sample counts (M > 0) */
    int32_t piece_of_run;   /* 0: the K events stand alone, tau_k <= k - k_begin;  1: they are events k_begin .. of one
                               long schedule, tau_k <= k: exactly the slice of the schedule generated in one go (for
                               calls that look ahead, see adpsgd_schedule_t) */
} adpsgd_sched_params_t;

typedef struct {
    int64_t events;          /* events executed since creation                    */
    int64_t rounds;          /* conflict-free rounds they were packed into        */
    int64_t fused_launches;  /* launches of the gossip-average + apply kernel     */
    int64_t grad_launches;   /* launches of gradient kernels                      */
    int64_t max_round_pairs; /* most update events in one round                   */
    int64_t slots;           /* pending-gradient slots available                  */
    double fused_ms;         /* summed kernel time, only with ADPSGD_FLAG_PROFILE */
    double grad_ms;
} adpsgd_stats_t;

/* Create an engine for n = graph->n workers and d parameters.
 * Algorithm 1 requires equal initial models: call adpsgd_set_models before the
 * first event.  Validates the graph (ADPSGD_ERR_GRAPH) and the buffers
 * (ADPSGD_ERR_ARG).  *out is NULL on failure. */
int adpsgd_create(adpsgd_t** out, const adpsgd_graph_t* graph, int64_t d, const adpsgd_opts_t* opts);

void adpsgd_destroy(adpsgd_t* h);

/* Message for the last error on h (h may be NULL: message of the last failed create). */
const char* adpsgd_last_error(const adpsgd_t* h);

/* Local data of one worker: D_i is the uniform distribution over its rows
 * (Strategy-2 of the remark in Sec. 3.1).
 *   features: device, rows x ld elements, 16-byte aligned, ld a multiple of 4 (fp32)
 *             or of 8 (bf16); fp32 for LSQ/LOGREG (ld >= d), bf16 for MLP (ld >= mlp_in);
 *   targets:  device, rows entries: fp32 b (LSQ), fp32 y in {-1,+1} (LOGREG), int32 class (MLP).
 * Both borrowed until adpsgd_destroy. */
int adpsgd_load_data(adpsgd_t* h, int32_t worker, const void* features, int64_t rows, int64_t ld,
                     const void* targets);

/* Set the models.  ld_in = 0: x holds d floats, broadcast to every worker (the
 * equal initialisation of Algorithm 1); otherwise x is n x ld_in.  x is host
 * (on_device = 0) or device (1) memory.  Synchronous. */
int adpsgd_set_models(adpsgd_t* h, const float* x, int64_t ld_in, int32_t on_device);

/* Execute the events of s in order semantics (Algorithm 1, one loop iteration
 * per event).  loss (device, K floats, or NULL) receives the minibatch loss at
 * x^_k of every event (data models only).  Asynchronous on the stream, but the
 * schedule arrays may be reused as soon as the call returns. */
int adpsgd_run_events(adpsgd_t* h, const adpsgd_schedule_t* s, float* loss);

/* Synchronous comparison schedule: S iterations of decentralized parallel SGD as the paper's
 * related-work section describes it (every worker computes a stochastic gradient at its current
 * model while the models are averaged with the neighbours; then the gradients are applied):
 *     X_{t+1}[i] = w_self[i] X_t[i] + sum_{j in N(i)} w_edge[i,j] X_t[j] - gamma_t g_i(X_t[i]; xi_{t,i})
 * One iteration counts as n worker updates; the synthetic gradient of worker i in iteration t is
 * that of event number (events executed so far on the handle) + t n + i.  All arrays are host
 * memory, read during the call only. */
typedef struct {
    int64_t S;                 /* iterations */
    const int32_t* batch_idx;  /* S * n * M minibatch indices, [t][i][m]; NULL for SYNTH */
    const float* gamma;        /* S step sizes, or NULL: the handle's gamma */
    const float* w_self;       /* n diagonal weights, or NULL: Metropolis weights (see below) */
    const float* w_edge;       /* one weight per entry of the graph's col array; NULL with w_self.
                                  Must be non-negative, symmetric, rows summing to 1 (|err| <= 1e-5) */
} adpsgd_sync_schedule_t;

/* One gradient the library asks the caller for (ADPSGD_MODEL_EXTERNAL): evaluate the stochastic
 * gradient of worker `worker` for event `event` of the call's schedule at the model xhat and write it to g. */
typedef struct {
    int32_t worker;     /* i_k: whose local data the gradient samples                              */
    int32_t reserved;
    int64_t event;      /* k, the index into the arrays of the schedule of this call               */
    const float* xhat;  /* device, d floats, read only: row i_k of X as of logical time k - tau_k
                           (the wait-free variant: a copy of it with the worker's pending gradient applied) */
    float* g;           /* device, d floats: receives g_k (a pending-gradient slot of the workspace) */
} adpsgd_grad_request_t;

/* Called on the calling thread, once per group of gradients that may be evaluated together (the
 * requests of one call are independent of each other).  It must enqueue all its GPU work on `stream`
 * (the handle's stream), or finish it before returning; it must not call into the same handle.
 * requests is host memory, valid during the call.  Return 0, or non-zero to abort the run. */
typedef int (*adpsgd_gradient_fn)(void* user, int32_t n_requests, const adpsgd_grad_request_t* requests, void* stream);

/* adpsgd_run_events for ADPSGD_MODEL_EXTERNAL (else ADPSGD_ERR_STATE): the same events, rounds and update
 * kernel, with every stale gradient obtained from fn (batch_idx of the schedule is not read: the caller
 * draws its own minibatches, e.g. from the event number).  If fn returns non-zero the call waits for the
 * stream and returns ADPSGD_ERR_CALLBACK; the updates of the rounds already enqueued have happened, which
 * is in general not a prefix of the serial order: restore the models before going on. */
int adpsgd_run_events_with(adpsgd_t* h, const adpsgd_schedule_t* s, adpsgd_gradient_fn fn, void* user);

/* Runs the iterations on the handle's stream (asynchronous, arrays reusable on return).  loss
 * (device, S * n floats, [t][i], or NULL) receives the minibatch losses.  Needs at least n
 * pending-gradient slots in the workspace (data models) and n <= 1024.  With momentum / weight
 * decay the optimizer rule of adpsgd_opts_t acts on the mixed model in place of x_{k+1/2}^i.
 * Memory: a call with S >= 2 lets the handle
 * allocate (once, kept until adpsgd_destroy) a second matrix of n * ldx floats: iterations then alternate
 * between X and that matrix, which is faster than mixing in place, and the models are back in X when the
 * call's work is done.  If that allocation fails, or with ADPSGD_FLAG_SYNC_IN_PLACE, the iterations run in
 * place, with the same results.
 * Errors as adpsgd_run_events, with no state change. */
int adpsgd_run_sync_steps(adpsgd_t* h, const adpsgd_sync_schedule_t* s, float* loss);

/* The same iterations for ADPSGD_MODEL_EXTERNAL (else ADPSGD_ERR_STATE): in iteration t the function is
 * asked for the gradients of all n workers at once (request i: worker i, event t * n + i, xhat = row i
 * of the models as the iteration starts, which may lie in the handle's second matrix and not in X: read it
 * through the request; g = slot i), then the mixing kernel runs.  batch_idx is not read.
 * Failure of fn as in adpsgd_run_events_with; X then holds the models of the iterations done so far. */
int adpsgd_run_sync_steps_with(adpsgd_t* h, const adpsgd_sync_schedule_t* s, adpsgd_gradient_fn fn, void* user);

/* Host-only: Metropolis mixing weights of a graph, w_edge[e] = 1 / (1 + max(deg i, deg j)) for the
 * entry e = (i, j) of the CSR arrays, w_self[i] = 1 - sum of its edge weights (fp64, rounded once);
 * on a regular graph of degree q every weight is 1 / (q + 1).  Outputs: n and rowptr[n] floats. */
int adpsgd_metropolis_weights(const adpsgd_graph_t* graph, float* w_self, float* w_edge);

/* Copy the n x d models to out (host or device, leading dimension ld_out >= d).
 * Synchronises the stream. */
int adpsgd_get_models(adpsgd_t* h, float* out, int64_t ld_out, int32_t on_device);

/* Algorithm 1's output: the average of all workers' models (d floats), column sums in row order accumulated in
 * fp64.  out on the host (on_device == 0): the call waits for the stream and copies the result.  out on the device:
 * the kernel is enqueued on the handle's stream and the call returns; the result is ready in stream order and out
 * must stay valid until then. */
int adpsgd_get_mean_model(adpsgd_t* h, float* out, int32_t on_device);

/* Consensus distance (1/n) sum_i |mean - x^i|^2: the quantity M_k of the proofs
 * appendix with uniform p.  *out is host memory.  Synchronous. */
int adpsgd_consensus_distance(adpsgd_t* h, double* out);

/* The same with the workers' update probabilities as weights, sum_i p_i |mean - x^i|^2 (mean = the
 * plain average): M_k as the proofs appendix defines it when the workers are not equally fast.
 * p: host, n non-negative values that sum to 1 (|err| <= 1e-9), else ADPSGD_ERR_ARG. */
int adpsgd_consensus_distance_weighted(adpsgd_t* h, const double* p, double* out);

/* The objective of the problem statement (Sec. 3.1, uniform p) at one point:
 *     f(x) = (1/n) sum_i (1/rows_i) sum_{rows of worker i} F(x; row)
 * over ALL local data, F as in ADPSGD_MODEL_* (the logistic loss includes lambda |x|^2 / 2).
 * x: device, d floats, or NULL for the mean of the workers' models (Algorithm 1's output).
 * *out is host memory.  Every data model (the MLP evaluates at the bf16 rounding of x, as its gradient
 * does); ADPSGD_ERR_STATE for SYNTH or when a worker has no data.  Synchronous; reads every local
 * row once. */
int adpsgd_objective(adpsgd_t* h, const float* x, double* out);

/* The same with the workers' probabilities, f(x) = sum_i p_i f_i(x): the objective of Sec. 3.1 when the
 * workers are not equally fast.  p: host, n non-negative values that sum to 1, else ADPSGD_ERR_ARG. */
int adpsgd_objective_weighted(adpsgd_t* h, const float* x, const double* p, double* out);

/* Classification error at one point, 1 - accuracy (the quantity of the accuracy tables of the
 * experiments section, here over the loaded local data):
 *     (1/n) sum_i (1/rows_i) #{rows of worker i whose predicted label differs from the target}
 * LOGREG predicts +1 when a.x >= 0 and -1 otherwise; the MLP predicts the class of its largest
 * logit (the lowest class on ties), from the same forward pass as its gradient.  x, *out, cost and
 * errors as for adpsgd_objective; ADPSGD_ERR_STATE for SYNTH and LSQ, which have no labels.
 * For held-out data, create a second handle on the same X (models are borrowed, not owned) and load
 * that data into it: its objective and classification error are the test loss and test error. */
int adpsgd_classification_error(adpsgd_t* h, const float* x, double* out);

/* For callers that cannot allocate device memory: code under HIP graph capture, tight serving loops that
 * watch the consensus distance between events, harnesses that forbid hipMalloc.  The same quantity and the
 * same kernels as adpsgd_consensus_distance (p = NULL) / adpsgd_consensus_distance_weighted (p: host, n
 * probabilities), but the block partials and the weights live in a fixed device array inside the library
 * (49 KB per GPU, held until the process ends) instead of a buffer the library allocates, and the result goes
 * to out_device (DEVICE memory, one double, written asynchronously on the handle's stream; the call does
 * not wait for it).  The call allocates and frees nothing.  Limits: the partials of any d fit (the grid is
 * capped at the array's 2048 partials); with p the handle may have at most 4096 workers, more gives
 * ADPSGD_ERR_ARG (as do invalid weights).  With p the weights are copied from host memory on the stream,
 * which is not something a graph capture can record: capture the p = NULL form.  All calls on one GPU share
 * the array and the last call's contents stay in it: calls that overlap on one GPU (two streams, two
 * threads) race, calls on one stream do not. */
int adpsgd_consensus_distance_static(adpsgd_t* h, const double* p, double* out_device);

/* Divergence check: the number of entries of the models that are NaN or infinite (0 for a healthy
 * run; a step size beyond the stability limit shows up here long before anything else fails).
 * *out is host memory.  Synchronous; reads X once. */
int adpsgd_count_nonfinite(adpsgd_t* h, int64_t* out);

/* Copy the n x d momentum buffers (only when opts.V was given). Synchronises the stream. */
int adpsgd_get_momentum(adpsgd_t* h, float* out, int64_t ld_out, int32_t on_device);

/* MLP only: copy the n x d bf16 shadow weights (bit patterns). Synchronous. */
int adpsgd_get_bf16_models(adpsgd_t* h, uint16_t* out, int64_t ld_out, int32_t on_device);

int adpsgd_get_stats(adpsgd_t* h, adpsgd_stats_t* out);

/* Checkpoint and resume.  The state of a run is the models (adpsgd_get_models / adpsgd_set_models
 * with ld_in > 0), the caller-owned momentum buffers, and the number of events executed so far,
 * which addresses the synthetic-gradient generator (event k of the handle's life draws stream k).
 * A new handle restored with these three continues bit for bit.  The count includes the n worker
 * updates of every synchronous iteration. */
int adpsgd_get_event_count(adpsgd_t* h, uint64_t* out);
int adpsgd_set_event_count(adpsgd_t* h, uint64_t events);

/* Host-only helpers (no GPU needed) ------------------------------------------ */

/* The random choices of Algorithm 1 for events k_begin .. k_begin + K - 1 of the
 * stream identified by seed: worker i_k ~ p, neighbour j_k uniform over the
 * neighbours of i_k, staleness tau_k (clipped to the events available in this
 * window: tau_k <= k - k_begin), and M minibatch indices drawn with replacement.
 * Integer arithmetic on a counter-based generator (Philox4x32-10) only; outputs
 * are caller-allocated host arrays (batch_idx: K*M, may be NULL when M = 0).
 * The graph is validated as by adpsgd_create (ADPSGD_ERR_GRAPH), the other parameters give ADPSGD_ERR_ARG. */
int adpsgd_make_schedule(const adpsgd_sched_params_t* p, uint64_t seed, uint64_t k_begin, int64_t K,
                         int32_t* worker, int32_t* neighbour, int32_t* tau, int32_t* batch_idx);

/* The round planner on its own: assigns every event a round for its stale read /
 * gradient (r_round, -1 when with_gradients = 0), a round for its update
 * (u_round) and a pending-gradient slot, such that within a round no model row
 * is written twice or read and written in the wrong order, and executing the
 * rounds in order (reads of a round before its updates) equals executing the
 * events one by one.  Outputs are host arrays of K entries; *n_rounds receives
 * the number of rounds.  extra_* as in adpsgd_schedule_t (NULL = none): the extra pairs of
 * event k run in round u_round[k].  local_compensation != 0 plans the wait-free variant
 * (see adpsgd_opts_t): the gradient of event k then also waits for the gradient of the
 * event k' it compensates with, and prev (K entries, may be NULL) receives k' or -1.
 * Looking ahead (see adpsgd_schedule_t): only the first n_apply events are applied (n_apply < 0 or
 * > K means K); an event beyond them gets a read round and a slot when k - tau[k] < n_apply, else
 * r_round = slot = -1, and u_round = -1 in both cases.  carried_slot (K entries or NULL) names, for the
 * events whose gradient an earlier call has evaluated, the slot that holds it (else -1): such an event
 * gets r_round = -1 and keeps that slot; it needs tau[k] > k.
 * Returns ADPSGD_ERR_SCHEDULE for tau[k] > k on an event that is not carried, or n_slots <= max tau. */
int adpsgd_plan_rounds(int32_t n, int64_t K, const int32_t* worker, const int32_t* neighbour,
                       const int32_t* tau, int32_t n_slots, int32_t with_gradients,
                       int32_t* r_round, int32_t* u_round, int32_t* slot, int32_t* n_rounds,
                       const int64_t* extra_ptr, const int32_t* extra_a, const int32_t* extra_b,
                       int32_t local_compensation, int64_t* prev, int64_t n_apply, const int32_t* carried_slot);

/* The check behind ADPSGD_FLAG_VERIFY_PLAN on its own (host only): ADPSGD_OK when the plan
 * (arrays as produced by adpsgd_plan_rounds; prev may be NULL) keeps the serial semantics of the
 * events, ADPSGD_ERR_STATE when it does not. */
int adpsgd_verify_plan(int32_t n, int64_t K, const int32_t* worker, const int32_t* neighbour,
                       const int32_t* tau, int32_t n_slots, int32_t with_gradients,
                       const int32_t* r_round, const int32_t* u_round, const int32_t* slot, int32_t n_rounds,
                       const int64_t* extra_ptr, const int32_t* extra_a, const int32_t* extra_b,
                       const int64_t* prev, int64_t n_apply, const int32_t* carried_slot);

/* Fill a device buffer with the synthetic gradient g_k[0..d) of global event k
 * (ADPSGD_MODEL_SYNTH's generator), on `stream`.  For tests of the generator. */
int adpsgd_synth_gradient(uint64_t seed, uint64_t k, float std, int64_t d, float* out_device,
                          void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ADPSGD_H */
