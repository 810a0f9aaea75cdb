/*
 * AD-PSGD serial CPU oracle  --  TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, single-threaded implementation of the per-event worker update
 * of AD-PSGD, written from the paper (Algorithm 1 "AD-PSGD (logical view)" and
 * the matrix form X_{k+1} = X_k W_k - gamma * dg(X^_k; xi_k, i_k) at the start
 * of the "Theoretical analysis" section).  It shares no code with the HIP
 * library; only tests, the smoke check and the benchmark's cpu_baseline leg
 * may call it.
 *
 * Conventions
 *   X is n x ldx fp32, row i = worker i's replica x^i (the paper stores the
 *   replicas as the columns of an N x n matrix; the transposed layout is the
 *   same object).  Dot products and gradient sums are accumulated in fp64 and
 *   rounded once to fp32; the three elementwise operations of an event
 *   (average, gamma*g, subtract) are done in fp32 with separate roundings
 *   (compile with -ffp-contract=off).
 *
 * Readings of the paper taken here (each is listed again in the design notes):
 *   - order inside an event: average first, then apply the gradient to the
 *     averaged model of worker i_k (Algorithm 1, the two steps after the
 *     gradient; the prose of Sec. 3.2 lists them in the other order);
 *   - x^_k = row i_k of X_{k - tau_k}; tau_k = 0 reads the row BEFORE event
 *     k's own average (X^_k = X_{k-tau_k}, end of the matrix-form paragraph);
 *   - W_k for a pairwise average of workers i, j is I - (e_i - e_j)(e_i - e_j)^T / 2;
 *   - the minibatch gradient is the paper's sum over the M samples times
 *     `gscale` (1/M gives the mean; 1 gives the paper's literal sum).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------- */
/* Counter-based generator: Philox4x32 with 10 rounds (Salmon, Moraes, Dror,  */
/* Shaw, "Parallel random numbers: as easy as 1, 2, 3", SC'11, Sec. 3.3 and   */
/* the constants of its Table 2 / reference description).                     */
/* ------------------------------------------------------------------------- */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint64_t mul_a = 0xD2511F53u, mul_b = 0xCD9E8D57u;   /* round multipliers   */
    const uint32_t weyl_a = 0x9E3779B9u, weyl_b = 0xBB67AE85u; /* key increments      */
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t pa = mul_a * (uint64_t)c0;
        uint64_t pb = mul_b * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(pb >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)pb;
        uint32_t n2 = (uint32_t)(pa >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)pa;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += weyl_a; k1 += weyl_b;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Stream tags: the generator is addressed as (seed, stream, event k, lane). */
enum { STREAM_EVENT = 0, STREAM_BATCH = 1, STREAM_GRAD = 2 };

static void draw4(uint64_t seed, int stream, uint64_t k, uint64_t lane, uint32_t out[4])
{
    uint32_t ctr[4], key[2];
    ctr[0] = (uint32_t)lane;
    ctr[1] = (uint32_t)(lane >> 32);
    ctr[2] = (uint32_t)k;
    ctr[3] = ((uint32_t)(k >> 32) & 0x00FFFFFFu) | ((uint32_t)stream << 24);
    key[0] = (uint32_t)seed;
    key[1] = (uint32_t)(seed >> 32);
    oracle_philox4x32_10(ctr, key, out);
}

/* uniform integer in [0, m): high word of the 64-bit product */
static uint32_t scale_to_range(uint32_t u, uint32_t m)
{
    return (uint32_t)(((uint64_t)u * (uint64_t)m) >> 32);
}

/* ------------------------------------------------------------------------- */
/* Schedule: the random choices of Algorithm 1 for events k_begin .. +K-1.    */
/*   i_k   ~ p  (uniform, or proportional to integer weights)                 */
/*   j_k   uniform over the graph neighbours of i_k (this fixes W_k)          */
/*   tau_k uniform on {0..T_max}, or geometric P(tau>=t) = (num_i/den_i)^t    */
/*         capped at T_max; always clipped to the events available (k local)  */
/*   batch M independent uniform row indices into worker i_k's local data     */
/* Integer arithmetic only, so that a second implementation can agree bit for */
/* bit.  Returns 0, or -1 on a bad argument.                                  */
/* ------------------------------------------------------------------------- */
int oracle_make_schedule(int32_t n, const int32_t* rowptr, const int32_t* col,
                         const int32_t* weight, int32_t tau_mode, int32_t T_max,
                         const int32_t* tau_num, const int32_t* tau_den, int32_t M,
                         const int32_t* rows, uint64_t seed, uint64_t k_begin, int64_t K,
                         int32_t* worker, int32_t* neighbour, int32_t* tau, int32_t* batch_idx,
                         int32_t piece_of_run)
{
    if (n < 1 || K < 0 || T_max < 0 || M < 0) return -1;
    if (tau_mode != 0 && (!tau_num || !tau_den)) return -1;
    if (M > 0 && !rows) return -1;
    uint64_t wtotal = 0;
    if (weight) {
        for (int32_t i = 0; i < n; ++i) {
            if (weight[i] < 0) return -1;
            wtotal += (uint64_t)weight[i];
        }
        if (wtotal == 0 || wtotal >= (1ull << 31)) return -1;
    }
    for (int64_t kk = 0; kk < K; ++kk) {
        uint64_t k = k_begin + (uint64_t)kk;
        uint32_t w[4];
        draw4(seed, STREAM_EVENT, k, 0, w);

        /* worker i_k */
        int32_t i;
        if (!weight) {
            i = (int32_t)scale_to_range(w[0], (uint32_t)n);
        } else {
            uint64_t r = scale_to_range(w[0], (uint32_t)wtotal), cum = 0;
            i = 0;
            for (int32_t c = 0; c < n; ++c) {
                cum += (uint64_t)weight[c];
                if (r < cum) { i = c; break; }
            }
        }
        worker[kk] = i;

        /* neighbour j_k (n = 1 or an isolated vertex: no partner, j = i) */
        int32_t deg = rowptr[i + 1] - rowptr[i];
        neighbour[kk] = deg > 0 ? col[rowptr[i] + (int32_t)scale_to_range(w[1], (uint32_t)deg)] : i;

        /* staleness tau_k */
        int64_t t;
        if (tau_mode == 0) {
            t = scale_to_range(w[2], (uint32_t)T_max + 1u);
        } else {
            uint64_t thr = 1ull << 32;
            t = 0;
            for (int32_t s = 1; s <= T_max; ++s) {
                thr = thr * (uint64_t)tau_num[i] / (uint64_t)tau_den[i];
                if ((uint64_t)w[2] < thr) t = s; else break;
            }
        }
        /* the read cannot lie before event 0 -- of these K events, or of the whole run when they are a piece of it */
        if (piece_of_run) { if ((uint64_t)t > k) t = (int64_t)k; }
        else if (t > kk) t = kk;
        tau[kk] = (int32_t)t;

        /* minibatch xi_k: M draws with replacement from the local rows */
        for (int32_t m = 0; m < M; ++m) {
            uint32_t b[4];
            draw4(seed, STREAM_BATCH, k, (uint64_t)(m / 4), b);
            batch_idx[kk * (int64_t)M + m] = (int32_t)scale_to_range(b[m % 4], (uint32_t)rows[i]);
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Synthetic gradient (the ResNet-50-sized workload has no data):             */
/*   g_k[e] = std * z(seed, k, e),  z ~ N(0,1) by the Box-Muller transform.   */
/* One generator call (lane q = e/4) gives four words; (w0,w1) -> elements    */
/* 4q, 4q+1 (cos, sin branch) and (w2,w3) -> 4q+2, 4q+3.  The uniforms are    */
/* u1 = ((w>>9) + 1/2) 2^-23 in (0,1) and u2 = (w>>8) 2^-24 in [0,1), both    */
/* exact in fp32, so only the transcendental functions can differ between     */
/* two implementations.                                                       */
/* ------------------------------------------------------------------------- */
static void synth_normals4(uint64_t seed, uint64_t k, uint64_t q, double z[4])
{
    const double two_pi = 6.283185307179586476925286766559;
    uint32_t w[4];
    draw4(seed, STREAM_GRAD, k, q, w);
    for (int h = 0; h < 2; ++h) {
        double u1 = ((double)(w[2 * h] >> 9) + 0.5) * (1.0 / 8388608.0);
        double u2 = (double)(w[2 * h + 1] >> 8) * (1.0 / 16777216.0);
        double r = sqrt(-2.0 * log(u1));
        z[2 * h]     = r * cos(two_pi * u2);
        z[2 * h + 1] = r * sin(two_pi * u2);
    }
}

void oracle_synth_grad(uint64_t seed, uint64_t k, double std, int64_t ncoords,
                       const int64_t* coords, float* g)
{
    for (int64_t c = 0; c < ncoords; ++c) {
        int64_t e = coords ? coords[c] : c;
        double z[4];
        synth_normals4(seed, k, (uint64_t)(e / 4), z);
        g[c] = (float)(std * z[e % 4]);
    }
}

/* ------------------------------------------------------------------------- */
/* bf16 helpers for the mixed-precision MLP workload (round to nearest even)  */
/* ------------------------------------------------------------------------- */
static uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u); /* NaN */
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    return (uint16_t)(u >> 16);
}
static float bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}
static float round_bf16(float f) { return bf16_to_f32(f32_to_bf16_rne(f)); }

void oracle_round_bf16(int64_t count, const float* in, float* out)
{
    for (int64_t t = 0; t < count; ++t) out[t] = round_bf16(in[t]);
}

/* ------------------------------------------------------------------------- */
/* Per-sample losses F(x; xi) and the minibatch gradient                      */
/*   g = gscale * sum_{m=1..M} grad F(x^; xi_m)     (Algorithm 1, gradient    */
/*   step; Sec. 3.2 "Compute gradients")                                      */
/* ------------------------------------------------------------------------- */
enum { MODEL_LSQ = 0, MODEL_LOGREG = 1, MODEL_SYNTH = 2, MODEL_MLP = 3 };

typedef struct {
    int model;
    int64_t d;
    int M;
    double gscale;     /* 1/M (mean) or 1 (the paper's sum) */
    double lambda;     /* L2 coefficient of the logistic model */
    int mlp_in, mlp_hid, mlp_out;
} grad_spec;

/* least squares: F(x; (a,b)) = (a.x - b)^2 / 2,  grad = a (a.x - b) */
static double grad_lsq(const grad_spec* s, const float* xhat, const float* A, int64_t lda,
                       const float* b, const int32_t* idx, double* gacc)
{
    double loss = 0.0;
    for (int m = 0; m < s->M; ++m) {
        const float* a = A + (int64_t)idx[m] * lda;
        double z = 0.0;
        for (int64_t e = 0; e < s->d; ++e) z += (double)a[e] * (double)xhat[e];
        double r = z - (double)b[idx[m]];
        loss += 0.5 * r * r;
        for (int64_t e = 0; e < s->d; ++e) gacc[e] += r * (double)a[e];
    }
    for (int64_t e = 0; e < s->d; ++e) gacc[e] *= s->gscale;
    return loss * s->gscale;
}

/* logistic: F(x; (a,y)) = log(1 + exp(-y a.x)) + lambda |x|^2 / 2,
 * grad = -y sigmoid(-y a.x) a + lambda x */
static double grad_logreg(const grad_spec* s, const float* xhat, const float* A, int64_t lda,
                          const float* y, const int32_t* idx, double* gacc)
{
    double loss = 0.0, xnorm2 = 0.0;
    for (int64_t e = 0; e < s->d; ++e) xnorm2 += (double)xhat[e] * (double)xhat[e];
    for (int m = 0; m < s->M; ++m) {
        const float* a = A + (int64_t)idx[m] * lda;
        double z = 0.0;
        for (int64_t e = 0; e < s->d; ++e) z += (double)a[e] * (double)xhat[e];
        double t = -(double)y[idx[m]] * z;               /* F = log(1 + e^t) + reg */
        loss += (t > 0.0 ? t + log1p(exp(-t)) : log1p(exp(t))) + 0.5 * s->lambda * xnorm2;
        double coef = -(double)y[idx[m]] / (1.0 + exp(-t)); /* -y sigmoid(t) */
        for (int64_t e = 0; e < s->d; ++e) gacc[e] += coef * (double)a[e] + s->lambda * (double)xhat[e];
    }
    for (int64_t e = 0; e < s->d; ++e) gacc[e] *= s->gscale;
    return loss * s->gscale;
}

/* Two-layer perceptron in_ -> hid (ReLU) -> out, softmax cross-entropy.
 * Parameters flattened as [W1 (in x hid, row-major), b1 (hid), W2 (hid x out), b2 (out)].
 * Mixed precision: the gradient sees the weights rounded to bf16 (xhat is the
 * fp32 master; it is rounded here), bf16 inputs, fp32-or-wider accumulation;
 * the hidden activations and their back-propagated error are rounded to bf16
 * before they enter the two large products, as a bf16 matrix unit would see
 * them.  The small second layer stays in full precision. */
static double grad_mlp(const grad_spec* s, const float* xhat, const uint16_t* Xin, int64_t ldin,
                       const int32_t* label, const int32_t* idx, double* gacc)
{
    const int I = s->mlp_in, H = s->mlp_hid, O = s->mlp_out, M = s->M;
    const float *W1, *b1, *W2, *b2;   /* point into the bf16-rounded copy of xhat, below */
    double* gW1 = gacc;
    double* gb1 = gW1 + (int64_t)I * H;
    double* gW2 = gb1 + H;
    double* gb2 = gW2 + (int64_t)H * O;
    float* hid = (float*)malloc(sizeof(float) * (size_t)H);      /* relu output, bf16-rounded */
    double* dhid = (double*)malloc(sizeof(double) * (size_t)H);
    double* pre = (double*)malloc(sizeof(double) * (size_t)H);
    double* logit = (double*)malloc(sizeof(double) * (size_t)O);
    double* dlogit = (double*)malloc(sizeof(double) * (size_t)O);
    /* the bf16 shadow of the weights, rounded once (the same value wherever it is used) */
    float* wq = (float*)malloc(sizeof(float) * (size_t)s->d);
    for (int64_t t = 0; t < s->d; ++t) wq[t] = round_bf16(xhat[t]);
    W1 = wq;
    b1 = W1 + (int64_t)I * H;
    W2 = b1 + H;
    b2 = W2 + (int64_t)H * O;
    double loss = 0.0;
    for (int m = 0; m < M; ++m) {
        const uint16_t* xin = Xin + (int64_t)idx[m] * ldin;
        /* forward, layer 1: pre[h] = sum_i x[i] W1[i][h], terms added in increasing i */
        for (int h = 0; h < H; ++h) pre[h] = 0.0;
        for (int i = 0; i < I; ++i) {
            const double xi = (double)bf16_to_f32(xin[i]);
            for (int h = 0; h < H; ++h) pre[h] += xi * (double)W1[(int64_t)i * H + h];
        }
        for (int h = 0; h < H; ++h) {
            float a = (float)(pre[h] + (double)b1[h]);
            hid[h] = round_bf16(a > 0.0f ? a : 0.0f);
        }
        /* forward, layer 2 + softmax cross-entropy */
        double zmax = -INFINITY;
        for (int o = 0; o < O; ++o) {
            double acc = (double)b2[o];
            for (int h = 0; h < H; ++h) acc += (double)hid[h] * (double)W2[(int64_t)h * O + o];
            logit[o] = acc;
            if (acc > zmax) zmax = acc;
        }
        double zsum = 0.0;
        for (int o = 0; o < O; ++o) zsum += exp(logit[o] - zmax);
        loss += -(logit[label[idx[m]]] - zmax - log(zsum));
        for (int o = 0; o < O; ++o)
            dlogit[o] = exp(logit[o] - zmax) / zsum - (o == label[idx[m]] ? 1.0 : 0.0);
        /* backward */
        for (int o = 0; o < O; ++o) gb2[o] += dlogit[o];
        for (int h = 0; h < H; ++h) {
            double acc = 0.0;
            for (int o = 0; o < O; ++o) {
                gW2[(int64_t)h * O + o] += (double)hid[h] * dlogit[o];
                acc += dlogit[o] * (double)W2[(int64_t)h * O + o];
            }
            /* error at the hidden pre-activation, scaled by gscale BEFORE the bf16
             * rounding so that the rounded operand of the large product already
             * carries the minibatch scale */
            float dh = hid[h] > 0.0f ? (float)(acc * s->gscale) : 0.0f;
            dhid[h] = (double)round_bf16(dh);
            gb1[h] += dhid[h];
        }
        for (int i = 0; i < I; ++i) {
            double xi = (double)bf16_to_f32(xin[i]);
            for (int h = 0; h < H; ++h) gW1[(int64_t)i * H + h] += xi * dhid[h];
        }
    }
    /* layer-1 terms already carry gscale (inside dhid); scale the layer-2 terms */
    for (int64_t t = 0; t < (int64_t)H * O; ++t) gW2[t] *= s->gscale;
    for (int o = 0; o < O; ++o) gb2[o] *= s->gscale;
    free(hid); free(dhid); free(pre); free(logit); free(dlogit); free(wq);
    return loss * s->gscale;
}

typedef struct {
    const void* const* features;  /* per worker: fp32 rows (linear) or bf16 rows (MLP) */
    const int64_t* ldf;           /* per worker: leading dimension in elements        */
    const void* const* targets;   /* per worker: fp32 b / fp32 y in {-1,+1} / int32 label */
} data_spec;

static double minibatch_gradient(const grad_spec* s, const data_spec* data, int worker,
                                 const float* xhat, const int32_t* idx, float* g)
{
    double* gacc = (double*)calloc((size_t)s->d, sizeof(double));
    double loss = 0.0;
    if (s->model == MODEL_LSQ)
        loss = grad_lsq(s, xhat, (const float*)data->features[worker], data->ldf[worker],
                        (const float*)data->targets[worker], idx, gacc);
    else if (s->model == MODEL_LOGREG)
        loss = grad_logreg(s, xhat, (const float*)data->features[worker], data->ldf[worker],
                           (const float*)data->targets[worker], idx, gacc);
    else
        loss = grad_mlp(s, xhat, (const uint16_t*)data->features[worker], data->ldf[worker],
                        (const int32_t*)data->targets[worker], idx, gacc);
    for (int64_t e = 0; e < s->d; ++e) g[e] = (float)gacc[e];
    free(gacc);
    return loss;
}

/* Exposed so that tests can pin the gradient formulas on their own. */
double oracle_minibatch_gradient(int model, int64_t d, int M, double gscale, double lambda,
                                 int mlp_in, int mlp_hid, int mlp_out, const float* xhat,
                                 const void* features, int64_t ldf, const void* targets,
                                 const int32_t* idx, float* g)
{
    grad_spec s = { model, d, M, gscale, lambda, mlp_in, mlp_hid, mlp_out };
    const void* f[1] = { features };
    const void* t[1] = { targets };
    int64_t l[1] = { ldf };
    data_spec data = { f, l, t };
    return minibatch_gradient(&s, &data, 0, xhat, idx, g);
}

/* ------------------------------------------------------------------------- */
/* Classification error of a model on one worker's rows (the quantity behind   */
/* the accuracy tables of the experiments section: error = 1 - accuracy).      */
/*   logistic regression: predicted label = +1 if a.x >= 0 else -1;           */
/*   perceptron: predicted class = the largest logit of the same forward pass  */
/*   as the gradient's (bf16 weights and inputs, hidden activations rounded to */
/*   bf16), the lowest class on ties.                                          */
/* Returns the number of rows whose prediction differs from the target, or -1 */
/* for a model without labels.                                                 */
/* ------------------------------------------------------------------------- */
int64_t oracle_count_misclassified(int model, int64_t d, int mlp_in, int mlp_hid, int mlp_out,
                                   const float* x, const void* features, int64_t ldf,
                                   const void* targets, int64_t rows)
{
    int64_t wrong = 0;
    if (model == MODEL_LOGREG) {
        const float* A = (const float*)features;
        const float* y = (const float*)targets;
        for (int64_t r = 0; r < rows; ++r) {
            double z = 0.0;
            for (int64_t e = 0; e < d; ++e) z += (double)A[r * ldf + e] * (double)x[e];
            const float predicted = z >= 0.0 ? 1.0f : -1.0f;
            wrong += predicted != y[r];
        }
        return wrong;
    }
    if (model != MODEL_MLP) return -1;
    const int I = mlp_in, H = mlp_hid, O = mlp_out;
    const uint16_t* Xin = (const uint16_t*)features;
    const int32_t* label = (const int32_t*)targets;
    float* wq = (float*)malloc(sizeof(float) * (size_t)d);
    double* pre = (double*)malloc(sizeof(double) * (size_t)H);
    float* hid = (float*)malloc(sizeof(float) * (size_t)H);
    for (int64_t t = 0; t < d; ++t) wq[t] = round_bf16(x[t]);
    const float* W1 = wq;
    const float* b1 = W1 + (int64_t)I * H;
    const float* W2 = b1 + H;
    const float* b2 = W2 + (int64_t)H * O;
    for (int64_t r = 0; r < rows; ++r) {
        const uint16_t* xin = Xin + r * ldf;
        for (int h = 0; h < H; ++h) pre[h] = 0.0;
        for (int i = 0; i < I; ++i) {
            const double xi = (double)bf16_to_f32(xin[i]);
            for (int h = 0; h < H; ++h) pre[h] += xi * (double)W1[(int64_t)i * H + h];
        }
        for (int h = 0; h < H; ++h) {
            float a = (float)(pre[h] + (double)b1[h]);
            hid[h] = round_bf16(a > 0.0f ? a : 0.0f);
        }
        int best = 0;
        double zbest = -INFINITY;
        for (int o = 0; o < O; ++o) {
            double acc = (double)b2[o];
            for (int h = 0; h < H; ++h) acc += (double)hid[h] * (double)W2[(int64_t)h * O + o];
            if (acc > zbest) { zbest = acc; best = o; }
        }
        wrong += best != label[r];
    }
    free(wq); free(pre); free(hid);
    return wrong;
}

/* ------------------------------------------------------------------------- */
/* One event's model update (Algorithm 1, averaging step then update step):   */
/*   x_{k+1/2} = X_k W_k   : rows i and j both become (x^i + x^j)/2           */
/*   x^i_{k+1} = x^i_{k+1/2} - gamma g_k ;  every other row = its k+1/2 value */
/* ------------------------------------------------------------------------- */
static void average_then_apply(float* xi, float* xj, const float* g, float gamma, int64_t d)
{
    for (int64_t e = 0; e < d; ++e) {
        float avg = (xi[e] + xj[e]) * 0.5f;
        float step = gamma * g[e];
        xj[e] = avg;
        xi[e] = avg - step;
    }
}

/* The same event with the optimizer the paper's experiments used (Sec. 5.2: momentum 0.9, weight
 * decay 1e-4).  Algorithm 1 has neither; the reading taken: each worker keeps its own momentum
 * buffer v^i (local optimizer state, never averaged), and momentum and weight decay act as in a
 * standard SGD step on the parameters being updated, i.e. on the averaged model x_{k+1/2}^i:
 *     u = g_k + wd * x_{k+1/2}^i ;   v^i <- mu * v^i + u ;   x_{k+1}^i = x_{k+1/2}^i - gamma * v^i
 * (mu = wd = 0 gives back the plain event).  fp32, one rounding per operation. */
static void average_then_apply_momentum(float* xi, float* xj, float* vi, const float* g, float gamma,
                                        float mu, float wd, int64_t d)
{
    for (int64_t e = 0; e < d; ++e) {
        float avg = (xi[e] + xj[e]) * 0.5f;
        float decay = wd * avg;
        float u = g[e] + decay;
        float carried = mu * vi[e];
        float v = carried + u;
        float step = gamma * v;
        vi[e] = v;
        xj[e] = avg;
        xi[e] = avg - step;
    }
}

/* wait-free variant: the pulled copy with the worker's own pending gradient applied (fp32, the
 * same two roundings as the update itself) */
static const float* compensate(float* out, const float* row, const float* g_pending, float gamma, int64_t d)
{
    for (int64_t e = 0; e < d; ++e) {
        float step = gamma * g_pending[e];
        out[e] = row[e] - step;
    }
    return out;
}

/* ------------------------------------------------------------------------- */
/* The event loop.                                                            */
/*   mode 0 ("literal"): keeps the last T+1 snapshots X_{k-T..k} and reads    */
/*     x^_k from snapshot k - tau_k, exactly as the matrix form states.       */
/*   mode 1 ("parked"): at the top of iteration s, evaluates the gradient of  */
/*     every event k with k - tau_k = s on the current row i_k and parks it   */
/*     until event k.  Same values (tests compare the two bit for bit), but   */
/*     memory is the in-flight gradients only, so it runs at any size.        */
/* coords != NULL (synthetic gradient only): X holds just the listed          */
/*   coordinates (n x ncoords); every coordinate of that workload evolves     */
/*   independently, so a sampled subset can be followed through a full run.   */
/* Optional outputs: loss[K] (minibatch loss at x^_k), g_log[K x d].          */
/* Returns 0, -1 bad argument, -2 out of memory.                              */
/* ------------------------------------------------------------------------- */
int oracle_run_events(int32_t n, int64_t d, float* X, int64_t ldx, int model, int M,
                      double gscale, double lambda, int mlp_in, int mlp_hid, int mlp_out,
                      const void* const* features, const int64_t* ldf,
                      const void* const* targets, float gamma, const float* gamma_k,
                      double synth_std, uint64_t synth_seed, uint64_t event_base,
                      const int64_t* coords, int64_t K, const int32_t* worker,
                      const int32_t* neighbour, const int32_t* tau, const int32_t* batch_idx,
                      int mode, double* loss, float* g_log, float momentum, float weight_decay,
                      float* V, int64_t ldv, const int64_t* extra_ptr, const int32_t* extra_a,
                      const int32_t* extra_b, int local_compensation)
{
    if (n < 1 || d < 1 || ldx < d || K < 0) return -1;
    grad_spec spec = { model, d, M, gscale, lambda, mlp_in, mlp_hid, mlp_out };
    data_spec data = { features, ldf, targets };
    int32_t T = 0;
    for (int64_t k = 0; k < K; ++k) {
        if (worker[k] < 0 || worker[k] >= n || neighbour[k] < 0 || neighbour[k] >= n) return -1;
        if (tau[k] < 0 || tau[k] > k) return -1;
        if (tau[k] > T) T = tau[k];
    }
    float* g = (float*)malloc(sizeof(float) * (size_t)d);
    if (!g) return -2;

    float* hist = NULL;        /* mode 0: ring of T+1 snapshots, each n x d */
    float** parked = NULL;     /* mode 1: parked[k] = g_k while in flight    */
    double* parked_loss = NULL;
    int64_t* bucket_head = NULL; /* mode 1: events grouped by read time s_k  */
    int64_t* bucket_next = NULL;
    if (model != MODEL_SYNTH) {
        if (mode == 0) {
            hist = (float*)malloc(sizeof(float) * (size_t)(T + 1) * (size_t)n * (size_t)d);
            if (!hist) { free(g); return -2; }
        } else {
            parked = (float**)calloc((size_t)K + 1, sizeof(float*));
            parked_loss = (double*)calloc((size_t)K + 1, sizeof(double));
            bucket_head = (int64_t*)malloc(sizeof(int64_t) * ((size_t)K + 1));
            bucket_next = (int64_t*)malloc(sizeof(int64_t) * ((size_t)K + 1));
            for (int64_t k = 0; k <= K; ++k) bucket_head[k] = -1;
            for (int64_t k = K - 1; k >= 0; --k) {   /* lists end up in increasing k */
                int64_t s = k - tau[k];
                bucket_next[k] = bucket_head[s];
                bucket_head[s] = k;
            }
        }
    }

    /* wait-free variant: prev[k] = latest earlier event of the same worker whose gradient is pending
     * (computed, not yet applied) when event k reads its model; g_keep[k'] keeps that gradient */
    int64_t* prev = NULL;
    float** g_keep = NULL;
    float* xcomp = NULL;
    if (local_compensation && model != MODEL_SYNTH) {
        prev = (int64_t*)malloc(sizeof(int64_t) * ((size_t)K + 1));
        g_keep = (float**)calloc((size_t)K + 1, sizeof(float*));
        xcomp = (float*)malloc(sizeof(float) * (size_t)d);
        int64_t* last_of = (int64_t*)malloc(sizeof(int64_t) * (size_t)n);
        for (int32_t r = 0; r < n; ++r) last_of[r] = -1;
        for (int64_t k = 0; k < K; ++k) {
            const int64_t kp = last_of[worker[k]], s = k - tau[k];
            prev[k] = (kp >= 0 && kp - tau[kp] <= s && s <= kp) ? kp : -1;
            last_of[worker[k]] = k;
        }
        free(last_of);
    }
#define COMPENSATED(row, k_) (prev && prev[k_] >= 0 ? compensate(xcomp, (row), g_keep[prev[k_]], gamma_k ? gamma_k[prev[k_]] : gamma, d) : (row))

    for (int64_t k = 0; k < K; ++k) {
        const int32_t i = worker[k], j = neighbour[k];
        double lk = 0.0;
        if (model == MODEL_SYNTH) {
            oracle_synth_grad(synth_seed, event_base + (uint64_t)k, synth_std, d, coords, g);
        } else if (mode == 0) {
            /* snapshot X_k, then read x^ from snapshot k - tau_k */
            float* snap = hist + (size_t)(k % (T + 1)) * (size_t)n * (size_t)d;
            for (int32_t r = 0; r < n; ++r) memcpy(snap + (size_t)r * d, X + (size_t)r * ldx, sizeof(float) * (size_t)d);
            const float* old = hist + (size_t)((k - tau[k]) % (T + 1)) * (size_t)n * (size_t)d;
            lk = minibatch_gradient(&spec, &data, i, COMPENSATED(old + (size_t)i * d, k), batch_idx + k * (int64_t)M, g);
        } else {
            for (int64_t q = bucket_head[k]; q >= 0; q = bucket_next[q]) {
                parked[q] = (float*)malloc(sizeof(float) * (size_t)d);
                parked_loss[q] = minibatch_gradient(&spec, &data, worker[q], COMPENSATED(X + (size_t)worker[q] * ldx, q),
                                                    batch_idx + q * (int64_t)M, parked[q]);
                if (g_keep) {   /* a later read of this worker may need it before event q applies it */
                    g_keep[q] = (float*)malloc(sizeof(float) * (size_t)d);
                    memcpy(g_keep[q], parked[q], sizeof(float) * (size_t)d);
                }
            }
            memcpy(g, parked[k], sizeof(float) * (size_t)d);
            lk = parked_loss[k];
            free(parked[k]);
            parked[k] = NULL;
        }
        if (loss) loss[k] = lk;
        if (g_log) memcpy(g_log + (size_t)k * d, g, sizeof(float) * (size_t)d);
        if (g_keep && mode == 0) {   /* literal mode evaluates g_k at event k: keep it for later stale reads */
            g_keep[k] = (float*)malloc(sizeof(float) * (size_t)d);
            memcpy(g_keep[k], g, sizeof(float) * (size_t)d);
        }

        /* general averaging matrix: W_k may average further disjoint pairs of workers in the same
         * event (Sec. 3.2, the generalisation of the averaging step to any doubly stochastic W_k); a product of disjoint
         * pairwise averagings is symmetric and doubly stochastic.  Those pairs carry no gradient. */
        if (extra_ptr) {
            for (int64_t q = extra_ptr[k]; q < extra_ptr[k + 1]; ++q) {
                float* xa = X + (size_t)extra_a[q] * ldx;
                float* xb = X + (size_t)extra_b[q] * ldx;
                for (int64_t e = 0; e < d; ++e) {
                    float avg = (xa[e] + xb[e]) * 0.5f;
                    xa[e] = avg;
                    xb[e] = avg;
                }
            }
        }
        const float gam = gamma_k ? gamma_k[k] : gamma;
        float* xi = X + (size_t)i * ldx;
        float* xj = X + (size_t)j * ldx;
        if (V)
            average_then_apply_momentum(xi, xj, V + (size_t)i * ldv, g, gam, momentum, weight_decay, d);
        else
            average_then_apply(xi, xj, g, gam, d);   /* j == i (no neighbour) degenerates to x -= gamma g */
    }
    if (g_keep) for (int64_t k = 0; k < K; ++k) free(g_keep[k]);
    free(g_keep); free(prev); free(xcomp);
    free(g); free(hist); free(parked); free(parked_loss); free(bucket_head); free(bucket_next);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Diagnostics: mean model (the algorithm's output) and the consensus         */
/* distance sum_i p_i |mean - x^i|^2 with uniform p (the quantity M_k of the  */
/* proofs appendix), both in fp64.                                            */
/* ------------------------------------------------------------------------- */
void oracle_mean_model(int32_t n, int64_t d, const float* X, int64_t ldx, double* mean)
{
    for (int64_t e = 0; e < d; ++e) {
        double s = 0.0;
        for (int32_t i = 0; i < n; ++i) s += (double)X[(size_t)i * ldx + e];
        mean[e] = s / (double)n;
    }
}

double oracle_consensus_distance(int32_t n, int64_t d, const float* X, int64_t ldx)
{
    double total = 0.0;
    for (int64_t e = 0; e < d; ++e) {
        double s = 0.0;
        for (int32_t i = 0; i < n; ++i) s += (double)X[(size_t)i * ldx + e];
        double mu = s / (double)n;
        for (int32_t i = 0; i < n; ++i) {
            double dv = (double)X[(size_t)i * ldx + e] - mu;
            total += dv * dv;
        }
    }
    return total / (double)n;
}

/* The same quantity with the workers' update probabilities as weights, as the */
/* proofs appendix defines it: sum_i p_i |mean - x^i|^2 (mean = plain average). */
double oracle_consensus_distance_weighted(int32_t n, int64_t d, const float* X, int64_t ldx, const double* p)
{
    double total = 0.0;
    for (int64_t e = 0; e < d; ++e) {
        double s = 0.0;
        for (int32_t i = 0; i < n; ++i) s += (double)X[(size_t)i * ldx + e];
        double mu = s / (double)n;
        for (int32_t i = 0; i < n; ++i) {
            double dv = (double)X[(size_t)i * ldx + e] - mu;
            total += p[i] * dv * dv;
        }
    }
    return total;
}

/* ------------------------------------------------------------------------- */
/* Synchronous comparison schedule: decentralized parallel SGD (D-PSGD) as    */
/* the related-work section describes it -- in each iteration every worker    */
/* computes a stochastic gradient at its own current model and, at the same   */
/* time, averages its model with its neighbours; then the gradient is applied */
/* to the averaged model:                                                     */
/*     X_{t+1}[i] = sum_j W[i][j] X_t[j] - gamma * g_i(X_t[i]; xi_{t,i})      */
/* W (n x n, row-major) is symmetric and doubly stochastic.  The mixing sum   */
/* is accumulated in fp64 and rounded once to fp32; gamma * g and the         */
/* subtraction are fp32 operations with separate roundings, as in an event.   */
/* Synthetic gradients: worker i at step t uses event number                  */
/* event_base + t * n + i.  batch_idx is S x n x M; loss (S x n) and g_log    */
/* (S x n x d) may be NULL.                                                   */
/* With the experiments' optimizer (V != NULL: n x ldx momentum buffers) the  */
/* mixed model takes the place of the averaged one in the event's rule:       */
/*     u = g_i + wd * mixed_i;  v^i <- mu * v^i + u;  X_{t+1}[i] = mixed_i - gamma * v^i */
/* ------------------------------------------------------------------------- */
int oracle_run_sync_steps(int32_t n, int64_t d, float* X, int64_t ldx, int model, int M,
                          double gscale, double lambda, int mlp_in, int mlp_hid, int mlp_out,
                          const void* const* features, const int64_t* ldf,
                          const void* const* targets, float gamma, const float* gamma_s,
                          double synth_std, uint64_t synth_seed, uint64_t event_base,
                          const int64_t* coords, int64_t S, const int32_t* batch_idx,
                          const float* W, double* loss, float* g_log,
                          float momentum, float weight_decay, float* V)
{
    if (n < 1 || d < 1 || ldx < d || S < 0 || !W) return -1;
    if (!V && (momentum != 0.0f || weight_decay != 0.0f)) return -1;
    grad_spec spec = { model, d, M, gscale, lambda, mlp_in, mlp_hid, mlp_out };
    data_spec data = { features, ldf, targets };
    float* G = (float*)malloc(sizeof(float) * (size_t)n * (size_t)d);
    float* Xnew = (float*)malloc(sizeof(float) * (size_t)n * (size_t)d);
    if (!G || !Xnew) { free(G); free(Xnew); return -2; }
    for (int64_t t = 0; t < S; ++t) {
        /* all gradients at the models the iteration starts from */
        for (int32_t i = 0; i < n; ++i) {
            float* gi = G + (size_t)i * d;
            double li = 0.0;
            if (model == MODEL_SYNTH)
                oracle_synth_grad(synth_seed, event_base + (uint64_t)t * (uint64_t)n + (uint64_t)i, synth_std, d, coords, gi);
            else
                li = minibatch_gradient(&spec, &data, i, X + (size_t)i * ldx,
                                        batch_idx + ((int64_t)t * n + i) * (int64_t)M, gi);
            if (loss) loss[t * n + i] = li;
            if (g_log) memcpy(g_log + ((size_t)t * n + i) * d, gi, sizeof(float) * (size_t)d);
        }
        const float gam = gamma_s ? gamma_s[t] : gamma;
        for (int32_t i = 0; i < n; ++i) {
            for (int64_t e = 0; e < d; ++e) {
                double mix = 0.0;
                for (int32_t j = 0; j < n; ++j) mix += (double)W[(size_t)i * n + j] * (double)X[(size_t)j * ldx + e];
                float mixed = (float)mix;
                if (V) {
                    float decay = weight_decay * mixed;
                    float u = G[(size_t)i * d + e] + decay;
                    float carried = momentum * V[(size_t)i * ldx + e];
                    float v = carried + u;
                    float step = gam * v;
                    V[(size_t)i * ldx + e] = v;
                    Xnew[(size_t)i * d + e] = mixed - step;
                } else {
                    float step = gam * G[(size_t)i * d + e];
                    Xnew[(size_t)i * d + e] = mixed - step;
                }
            }
        }
        for (int32_t i = 0; i < n; ++i) memcpy(X + (size_t)i * ldx, Xnew + (size_t)i * d, sizeof(float) * (size_t)d);
    }
    free(G); free(Xnew);
    return 0;
}

/* Mixing weights when none are given: W[i][j] = 1 / (1 + max(deg i, deg j)) on the edges,      */
/* W[i][i] = 1 - sum_j W[i][j] (the Metropolis rule: symmetric and doubly stochastic on any     */
/* undirected graph; on a regular graph of degree q it is the plain average over the worker and */
/* its neighbours, 1 / (q + 1)).  Computed in fp64, rounded once to fp32.                       */
int oracle_metropolis_weights(int32_t n, const int32_t* rowptr, const int32_t* col, float* W)
{
    if (n < 1 || !rowptr || !col || !W) return -1;
    for (size_t t = 0; t < (size_t)n * (size_t)n; ++t) W[t] = 0.0f;
    for (int32_t i = 0; i < n; ++i) {
        double self = 1.0;
        const int32_t di = rowptr[i + 1] - rowptr[i];
        for (int32_t q = rowptr[i]; q < rowptr[i + 1]; ++q) {
            const int32_t j = col[q];
            if (j < 0 || j >= n || j == i) return -1;
            const int32_t dj = rowptr[j + 1] - rowptr[j];
            const double w = 1.0 / (1.0 + (double)(di > dj ? di : dj));
            W[(size_t)i * n + j] = (float)w;
            self -= w;
        }
        W[(size_t)i * n + i] = (float)self;
    }
    return 0;
}
