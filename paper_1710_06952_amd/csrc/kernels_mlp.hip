// Minibatch gradient of the two-layer perceptron  in -> hid (ReLU) -> out with
// softmax cross-entropy (Algorithm 1, gradient step, for the dense-network
// workload).  Parameters are flattened as [W1 (in x hid) | b1 | W2 (hid x out) | b2];
// the gradient reads the bf16 shadow of the stale model and bf16 inputs, and
// accumulates in fp32.  The two large products are dense contractions and run
// on the matrix cores (v_mfma_f32_16x16x32_bf16, 64-lane wavefronts):
//   forward   H  = relu(Xb W1 + b1)        M x in  times  in x hid
//   backward  dW1 = Xb^T dH                in x M  times  M x hid
// The hidden activations and their back-propagated error are rounded to bf16
// before they enter those products.  The second layer (hid x out, out <= 16) is
// small and stays on the vector ALUs in fp32.
//
// Four launches per group of gradient operations; every reduction has a fixed
// order, so results do not depend on scheduling.
#include "device_common.hpp"
#include "internal.hpp"

namespace adpsgd_impl {
namespace {

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef uint16_t v8h __attribute__((ext_vector_type(8)));

constexpr int kT = 256;          // 4 wavefronts
constexpr int kMaxM = 64;        // minibatch rows held by one block (4 MFMA row tiles)
constexpr int kMaxOut = 16;
constexpr int kTileH = 64;       // hidden columns per block: 16 per wavefront

struct MlpParams {
    const uint16_t* Xb;
    int64_t ld;
    int in, hid, out;
    const GradOp* ops;
    int M;
    const int32_t* batch_idx;
    const WorkerDataDev* data;
    float* slots;
    float gscale;
    float* loss;
    uint16_t* Hb;    // [op][kMaxM][hid]  relu output, bf16
    uint16_t* dHb;   // [op][kMaxM][hid]  error at the hidden pre-activation, bf16, rows >= M zero
    float* dlogit;   // [op][kMaxM][kMaxOut]  softmax - onehot
    float* logit_part;  // [op][hid / 32][kMaxM][kMaxOut]  second-layer products of one forward tile
    float* loss_m;   // [op][kMaxM]
};

__device__ __forceinline__ v4f mfma_bf16(v8h a, v8h b, v4f c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c, 0, 0, 0);
}

// Operand layout of v_mfma_f32_16x16x32_bf16 (D = A B + C, A 16x32, B 32x16):
//   lane l supplies A[l % 16][8 (l / 16) .. +7] and B[8 (l / 16) .. +7][l % 16];
//   lane l receives D[4 (l / 16) + v][l % 16] in element v of its 4 results.

// ---- 1. forward: H = relu(Xb W1 + b1), grid = (hid / 32, n_ops) ----------------------
// One block owns a 64 (minibatch) x 32 (hidden) tile of H.  The contraction over the input
// features is split across the four wavefronts (k-steps of 32, step s goes to wavefront s % 4),
// each with its own transposed W1 tile in LDS; the next step's operands are fetched into
// registers while the current step's MFMAs run.  The four partial tiles are then added in a
// fixed order through LDS.
constexpr int kFwdTileH = 32;

struct FwdOperands {
    v8h w[2];   // W1 tile 32 (k) x 32 (h): lane holds 2 rows k, 8 columns each
    v8h a[4];   // input fragments of the four 16-row minibatch tiles
};

__global__ __launch_bounds__(kT) void mlp_forward_kernel(const MlpParams p) {
    __shared__ __attribute__((aligned(16))) unsigned char smem[16384];
    __shared__ float W2s[kFwdTileH][kMaxOut];     // this tile's rows of W2, zero beyond `out`
    const GradOp op = p.ops[blockIdx.y];
    const WorkerDataDev wd = p.data[op.worker];
    const uint16_t* __restrict__ feat = static_cast<const uint16_t*>(wd.features);
    const int32_t* __restrict__ idx = p.batch_idx + static_cast<int64_t>(op.event) * p.M;
    const uint16_t* __restrict__ W1 = p.Xb + static_cast<int64_t>(op.worker) * p.ld;
    const uint16_t* __restrict__ b1 = W1 + static_cast<int64_t>(p.in) * p.hid;
    const int h0 = blockIdx.x * kFwdTileH;
    {
        const uint16_t* __restrict__ W2 = b1 + p.hid;
        for (int t = threadIdx.x; t < kFwdTileH * kMaxOut; t += kT) {
            const int hh = t / kMaxOut, o = t % kMaxOut;
            W2s[hh][o] = o < p.out ? bf16_to_float(W2[static_cast<int64_t>(h0 + hh) * p.out + o]) : 0.0f;
        }
    }
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int li = lane & 15, kb = 8 * (lane >> 4);
    uint16_t(*Bt)[40] = reinterpret_cast<uint16_t(*)[40]>(smem + wave * (kFwdTileH * 40 * 2));   // [h][k]
    float* red = reinterpret_cast<float*>(smem);

    const uint16_t* rowp[4];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
        const int m = 16 * mt + li;
        rowp[mt] = m < p.M ? feat + static_cast<int64_t>(idx[m]) * wd.ld : nullptr;
    }
    const int skk = lane >> 2, shh = (lane & 3) * 8;   // staging role inside the wavefront
    auto fetch = [&](int step, FwdOperands& f) {
        const int k0 = 32 * step;
        const v8h zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int k = k0 + skk + 16 * r;
            f.w[r] = k < p.in ? *reinterpret_cast<const v8h*>(W1 + static_cast<int64_t>(k) * p.hid + h0 + shh) : zero;
        }
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
            f.a[mt] = (rowp[mt] && k0 + kb < p.in) ? *reinterpret_cast<const v8h*>(rowp[mt] + k0 + kb) : zero;
    };

    v4f acc[4][2];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int ht = 0; ht < 2; ++ht) acc[mt][ht] = v4f{0, 0, 0, 0};

    const int steps = (p.in + 31) / 32, iters = (steps + 3) / 4;   // same trip count for every wavefront
    FwdOperands cur, nxt;
    fetch(wave, cur);            // steps beyond the last one fetch zeros
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int e = 0; e < 8; ++e) Bt[shh + e][skk + 16 * r] = cur.w[r][e];
        if (it + 1 < iters) fetch(wave + 4 * (it + 1), nxt);
        __syncthreads();
        v8h bfrag[2];
#pragma unroll
        for (int ht = 0; ht < 2; ++ht) bfrag[ht] = *reinterpret_cast<const v8h*>(&Bt[16 * ht + li][kb]);
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int ht = 0; ht < 2; ++ht) acc[mt][ht] = mfma_bf16(cur.a[mt], bfrag[ht], acc[mt][ht]);
        __syncthreads();
        cur = nxt;
    }

    // (wave0 + wave2) + (wave1 + wave3), element q of lane l at red[half][q][l]
    auto spill = [&](int half) {
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int ht = 0; ht < 2; ++ht)
#pragma unroll
                for (int v = 0; v < 4; ++v) red[(half * 32 + (mt * 2 + ht) * 4 + v) * 64 + lane] = acc[mt][ht][v];
    };
    auto absorb = [&](int half) {
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int ht = 0; ht < 2; ++ht)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[mt][ht][v] += red[(half * 32 + (mt * 2 + ht) * 4 + v) * 64 + lane];
    };
    if (wave >= 2) spill(wave - 2);
    __syncthreads();
    if (wave < 2) absorb(wave);
    __syncthreads();
    if (wave == 1) spill(0);
    __syncthreads();
    float(*Hs)[kFwdTileH + 1] = reinterpret_cast<float(*)[kFwdTileH + 1]>(smem);   // the finished tile, as the next layer sees it
    if (wave == 0) {
        absorb(0);
#pragma unroll
        for (int ht = 0; ht < 2; ++ht) {
            const int h = h0 + 16 * ht + li;
            const float bias = bf16_to_float(b1[h]);
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int m = 16 * mt + 4 * (lane >> 4) + v;
                    float hval = 0.0f;
                    if (m < p.M) {
                        const float pre = acc[mt][ht][v] + bias;
                        const uint16_t hb = bf16_rne(pre > 0.0f ? pre : 0.0f);
                        p.Hb[(static_cast<int64_t>(blockIdx.y) * kMaxM + m) * p.hid + h] = hb;
                        hval = bf16_to_float(hb);
                    }
                    Hs[m][16 * ht + li] = hval;
                }
        }
    }
    __syncthreads();
    // this tile's share of the logits: thread (m, oq) sums over the 32 hidden units in order
    {
        const int m = threadIdx.x >> 2, oq = threadIdx.x & 3;
        float part[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll 8
        for (int hh = 0; hh < kFwdTileH; ++hh) {
            const float hv = Hs[m][hh];
#pragma unroll
            for (int q = 0; q < 4; ++q) part[q] += hv * W2s[hh][oq + 4 * q];
        }
        float* __restrict__ dst = p.logit_part + ((static_cast<int64_t>(blockIdx.y) * gridDim.x + blockIdx.x) * kMaxM + m) * kMaxOut;
#pragma unroll
        for (int q = 0; q < 4; ++q) dst[oq + 4 * q] = part[q];
    }
}

// ---- 2. logits, softmax, loss: grid = n_ops, one block per gradient --------------------
// Thread (m, oq) adds the hid / 32 tile contributions of logits oq, oq + 4, oq + 8, oq + 12 of sample
// m in tile order; one thread per sample then does the softmax.
__global__ __launch_bounds__(kT) void mlp_softmax_kernel(const MlpParams p) {
    __shared__ float logit_s[kMaxM][kMaxOut + 1];
    const GradOp op = p.ops[blockIdx.x];
    const WorkerDataDev wd = p.data[op.worker];
    const int32_t* __restrict__ idx = p.batch_idx + static_cast<int64_t>(op.event) * p.M;
    const uint16_t* __restrict__ W = p.Xb + static_cast<int64_t>(op.worker) * p.ld;
    const uint16_t* __restrict__ b2 = W + static_cast<int64_t>(p.in) * p.hid + p.hid + static_cast<int64_t>(p.hid) * p.out;
    const int tiles = p.hid / kFwdTileH;
    {
        const int m = threadIdx.x >> 2, oq = threadIdx.x & 3;
        const float* __restrict__ src = p.logit_part + (static_cast<int64_t>(blockIdx.x) * tiles * kMaxM + m) * kMaxOut + oq;
        float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        for (int t0 = 0; t0 < tiles; t0 += 8) {
            float buf[8][4];
#pragma unroll
            for (int t = 0; t < 8; ++t)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    buf[t][q] = (t0 + t < tiles) ? src[static_cast<int64_t>(t0 + t) * kMaxM * kMaxOut + 4 * q] : 0.0f;
#pragma unroll
            for (int t = 0; t < 8; ++t)
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[q] += buf[t][q];
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) logit_s[m][oq + 4 * q] = acc[q];
    }
    __syncthreads();
    if (threadIdx.x < p.M) {
        const int m = threadIdx.x;
        float logit[kMaxOut];
        float zmax = -INFINITY;
        for (int o = 0; o < p.out; ++o) {
            logit[o] = logit_s[m][o] + bf16_to_float(b2[o]);
            zmax = fmaxf(zmax, logit[o]);
        }
        float zsum = 0.0f;
        for (int o = 0; o < p.out; ++o) zsum += expf(logit[o] - zmax);
        const int label = static_cast<const int32_t*>(wd.targets)[idx[m]];
        float* dl = p.dlogit + (static_cast<int64_t>(blockIdx.x) * kMaxM + m) * kMaxOut;
        float lsel = 0.0f;
        for (int o = 0; o < p.out; ++o) {
            dl[o] = expf(logit[o] - zmax) / zsum - (o == label ? 1.0f : 0.0f);
            if (o == label) lsel = logit[o];
        }
        p.loss_m[static_cast<int64_t>(blockIdx.x) * kMaxM + m] = -(lsel - zmax - logf(zsum));
    }
}

// ---- 3. second-layer gradients and the hidden error: grid = (hid / 64, n_ops) ---------
// Thread (hl, mg): hidden unit h = 64 blockIdx.x + hl, minibatch rows [16 mg, 16 mg + 16).
// Sums over the minibatch are finished across the four row groups in a fixed order.
__global__ __launch_bounds__(kT) void mlp_backward_small_kernel(const MlpParams p) {
    __shared__ float dl_s[kMaxM][kMaxOut];
    __shared__ float red[4][kMaxOut + 1][64];
    const GradOp op = p.ops[blockIdx.y];
    const int hl = threadIdx.x & 63, mg = threadIdx.x >> 6;
    const int h = blockIdx.x * 64 + hl;
    const uint16_t* __restrict__ W = p.Xb + static_cast<int64_t>(op.worker) * p.ld;
    const uint16_t* __restrict__ W2 = W + static_cast<int64_t>(p.in) * p.hid + p.hid;
    float* __restrict__ g = p.slots + static_cast<int64_t>(op.slot) * p.ld;
    float* __restrict__ gb1 = g + static_cast<int64_t>(p.in) * p.hid;
    float* __restrict__ gW2 = gb1 + p.hid;
    float* __restrict__ gb2 = gW2 + static_cast<int64_t>(p.hid) * p.out;
    const float* __restrict__ dl0 = p.dlogit + static_cast<int64_t>(blockIdx.y) * kMaxM * kMaxOut;
    for (int t = threadIdx.x; t < kMaxM * kMaxOut; t += kT) {
        const int m = t / kMaxOut, o = t % kMaxOut;
        dl_s[m][o] = (m < p.M && o < p.out) ? dl0[t] : 0.0f;
    }
    __syncthreads();
    float w2[kMaxOut], gw2[kMaxOut];
#pragma unroll
    for (int o = 0; o < kMaxOut; ++o) {
        w2[o] = o < p.out ? bf16_to_float(W2[static_cast<int64_t>(h) * p.out + o]) : 0.0f;
        gw2[o] = 0.0f;
    }
    float sum_dh = 0.0f;
    uint16_t hraw[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {      // all 16 activations of this thread in flight at once
        const int m = 16 * mg + r;
        hraw[r] = m < p.M ? p.Hb[(static_cast<int64_t>(blockIdx.y) * kMaxM + m) * p.hid + h] : static_cast<uint16_t>(0);
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int m = 16 * mg + r;
        const int64_t at = (static_cast<int64_t>(blockIdx.y) * kMaxM + m) * p.hid + h;
        uint16_t dh = 0;
        if (m < p.M) {
            const float hv = bf16_to_float(hraw[r]);
            float back = 0.0f;
#pragma unroll
            for (int o = 0; o < kMaxOut; ++o) {     // entries o >= out are zero in dl_s and w2
                gw2[o] += hv * dl_s[m][o];
                back += dl_s[m][o] * w2[o];
            }
            dh = bf16_rne(hv > 0.0f ? back * p.gscale : 0.0f);
            sum_dh += bf16_to_float(dh);
        }
        p.dHb[at] = dh;                              // rows m >= M are the zero padding of the dW1 product
    }
#pragma unroll
    for (int o = 0; o < kMaxOut; ++o) red[mg][o][hl] = gw2[o];
    red[mg][kMaxOut][hl] = sum_dh;
    __syncthreads();
    if (mg == 0) {
#pragma unroll
        for (int o = 0; o < kMaxOut; ++o)
            if (o < p.out)
                gW2[static_cast<int64_t>(h) * p.out + o] = ((red[0][o][hl] + red[1][o][hl]) + (red[2][o][hl] + red[3][o][hl])) * p.gscale;
        gb1[h] = (red[0][kMaxOut][hl] + red[1][kMaxOut][hl]) + (red[2][kMaxOut][hl] + red[3][kMaxOut][hl]);
    }
    if (blockIdx.x == 0 && mg == 1 && hl < p.out) {
        float sdl = 0.0f;
        for (int m = 0; m < p.M; ++m) sdl += dl_s[m][hl];
        gb2[hl] = sdl * p.gscale;
    }
    if (blockIdx.x == 0 && threadIdx.x == 128 && p.loss) {
        float sl = 0.0f;
        for (int m = 0; m < p.M; ++m) sl += p.loss_m[static_cast<int64_t>(blockIdx.y) * kMaxM + m];
        p.loss[op.event] = sl * p.gscale;
    }
}

// ---- 4. dW1 = Xb^T dH: grid = (hid / 64, ceil(in / 64), n_ops) -------------------------
__global__ __launch_bounds__(kT) void mlp_dw1_kernel(const MlpParams p) {
    __shared__ __attribute__((aligned(16))) uint16_t At[64][72];   // inputs transposed:  [i][m], 64 m + pad
    __shared__ __attribute__((aligned(16))) uint16_t Bt[64][72];   // hidden error transposed: [h][m]
    const GradOp op = p.ops[blockIdx.z];
    const WorkerDataDev wd = p.data[op.worker];
    const uint16_t* __restrict__ feat = static_cast<const uint16_t*>(wd.features);
    const int32_t* __restrict__ idx = p.batch_idx + static_cast<int64_t>(op.event) * p.M;
    const int h0 = blockIdx.x * kTileH, i0 = blockIdx.y * 64;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int li = lane & 15, kb = 8 * (lane >> 4);

    {   // stage: thread handles one minibatch row m and 16 consecutive columns
        const int m = threadIdx.x >> 2, seg = (threadIdx.x & 3) * 16;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int c = seg + 8 * half;
            v8h xv = {0, 0, 0, 0, 0, 0, 0, 0};
            if (m < p.M && i0 + c < p.in) xv = *reinterpret_cast<const v8h*>(feat + static_cast<int64_t>(idx[m]) * wd.ld + i0 + c);
            const v8h dv = *reinterpret_cast<const v8h*>(p.dHb + (static_cast<int64_t>(blockIdx.z) * kMaxM + m) * p.hid + h0 + c);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                At[c + e][m] = xv[e];
                Bt[c + e][m] = dv[e];
            }
        }
    }
    __syncthreads();
    v4f acc[4];
#pragma unroll
    for (int it = 0; it < 4; ++it) acc[it] = v4f{0, 0, 0, 0};
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        const v8h bfrag = *reinterpret_cast<const v8h*>(&Bt[16 * wave + li][32 * ks + kb]);
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const v8h afrag = *reinterpret_cast<const v8h*>(&At[16 * it + li][32 * ks + kb]);
            acc[it] = mfma_bf16(afrag, bfrag, acc[it]);
        }
    }
    float* __restrict__ g = p.slots + static_cast<int64_t>(op.slot) * p.ld;
    const int h = h0 + 16 * wave + li;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int i = i0 + 16 * it + 4 * (lane >> 4) + v;
            if (i < p.in) g[static_cast<int64_t>(i) * p.hid + h] = acc[it][v];
        }
    }
}

size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

}  // namespace

size_t mlp_scratch_bytes(int32_t n_ops, int32_t M, int32_t in, int32_t hid, int32_t out) {
    if (n_ops < 1 || M < 1 || M > kMaxM || in < 8 || (in & 7) || hid < kTileH || (hid % kTileH) || out < 1 || out > kMaxOut)
        return 0;
    const size_t act = align256(static_cast<size_t>(n_ops) * kMaxM * hid * sizeof(uint16_t));
    const size_t lp = align256(static_cast<size_t>(n_ops) * (hid / kFwdTileH) * kMaxM * kMaxOut * 4);
    return 2 * act + align256(static_cast<size_t>(n_ops) * kMaxM * kMaxOut * 4) + align256(static_cast<size_t>(n_ops) * kMaxM * 4) + lp;
}

hipError_t launch_mlp_gradient(const MlpGradArgs& a, hipStream_t st, int* n_launches) {
    if (a.n_ops <= 0) return hipSuccess;
    if (mlp_scratch_bytes(a.n_ops, a.M, a.in, a.hid, a.out) == 0 || a.n_ops > 65535) return hipErrorInvalidValue;
    MlpParams p;
    p.Xb = a.Xbf16;
    p.ld = a.ld;
    p.in = a.in;
    p.hid = a.hid;
    p.out = a.out;
    p.ops = a.ops;
    p.M = a.M;
    p.batch_idx = a.batch_idx;
    p.data = a.data;
    p.slots = a.slots;
    p.gscale = a.gscale;
    p.loss = a.loss;
    char* s = static_cast<char*>(a.scratch);
    const size_t act = align256(static_cast<size_t>(a.n_ops) * kMaxM * a.hid * sizeof(uint16_t));
    p.Hb = reinterpret_cast<uint16_t*>(s);
    p.dHb = reinterpret_cast<uint16_t*>(s + act);
    p.dlogit = reinterpret_cast<float*>(s + 2 * act);
    p.loss_m = reinterpret_cast<float*>(s + 2 * act + align256(static_cast<size_t>(a.n_ops) * kMaxM * kMaxOut * 4));
    p.logit_part = reinterpret_cast<float*>(s + 2 * act + align256(static_cast<size_t>(a.n_ops) * kMaxM * kMaxOut * 4) +
                                            align256(static_cast<size_t>(a.n_ops) * kMaxM * 4));
    const uint32_t hb = static_cast<uint32_t>(a.hid / kTileH);
    hipLaunchKernelGGL(mlp_forward_kernel, dim3(a.hid / kFwdTileH, a.n_ops), dim3(kT), 0, st, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(mlp_softmax_kernel, dim3(a.n_ops), dim3(kT), 0, st, p);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(mlp_backward_small_kernel, dim3(a.hid / 64, a.n_ops), dim3(kT), 0, st, p);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(mlp_dw1_kernel, dim3(hb, (a.in + 63) / 64, a.n_ops), dim3(kT), 0, st, p);
    if (n_launches) *n_launches += 4;
    return hipGetLastError();
}

}  // namespace adpsgd_impl
