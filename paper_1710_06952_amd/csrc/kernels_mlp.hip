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
// Launches per group of gradient operations: forward; softmax with the second-layer
// gradients and the hidden error dH; and, only where a dense gradient is wanted
// (the synchronous schedule, the wait-free variant), dW1.  By default dW1
// is never written out: dH stays in the pending slot and the kernel that applies the
// event (section 4 below) forms the rank-M product tile by tile while it updates the
// model.  The kernels of a round form a serial chain of small grids, so each one
// keeps all its global loads in flight at once instead of looping over them.  Every
// reduction has a fixed order: results do not depend on scheduling.
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
    const float* X;
    const uint16_t* Xb;
    int64_t ld;
    int in, hid, out;
    const GradOp* ops;
    int M;
    const int32_t* batch_by_op;   // [op][M] minibatch indices, in the order of ops
    float* slots;
    float gscale;
    float* loss;
    uint16_t* Hb;    // [op][kMaxM][hid]  relu output, bf16
    uint16_t* dHb;   // [op][kMaxM][hid]  error at the hidden pre-activation, bf16, rows >= M zero
    int factored;    // dH goes to the start of the operation's pending slot instead (and stays there
                     // until the update kernel multiplies it with the inputs)
    float* logit_part;  // [op][hid / 32][kMaxM][kMaxOut]  second-layer products of one forward tile
    // Left by the forward kernel for the one that follows, so that its loads depend on nothing but its block index
    // (a kernel of this chain is a few memory round trips long; each dependent load it sheds is one of them):
    int32_t* labels;    // [op][kMaxM]  class of every sample of the minibatch, -1 beyond M
    float* W2f;         // [op][hid][kMaxOut]  the second layer's weights as fp32, zero beyond `out`
    float* b2f;         // [op][kMaxOut]
};

// all lanes of a wavefront have finished their LDS accesses before any of them goes on (LDS operations of one
// wavefront execute in order; this only keeps the compiler from moving accesses across)
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ v4f mfma_bf16(v8h a, v8h b, v4f c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c, 0, 0, 0);
}

// Operand layout of v_mfma_f32_16x16x32_bf16 (D = A B + C, A 16x32, B 32x16):
//   lane l supplies A[l % 16][8 (l / 16) .. +7] and B[8 (l / 16) .. +7][l % 16];
//   lane l receives D[4 (l / 16) + v][l % 16] in element v of its 4 results.

// ---- 0. wait-free variant: the compensated copy of the model a gradient reads ---------------
// For operations that carry a pending gradient g_k' (dense, in slot comp_slot):
//     xrow = bf16(x^i - gamma_k' g_k')        (two fp32 roundings, then round to nearest even)
// grid = (ceil(ld / 1024), n_ops); operations without compensation return at once.
__global__ __launch_bounds__(kT) void mlp_compensated_rows_kernel(const MlpParams p) {
    const GradOp op = p.ops[blockIdx.y];
    if (op.comp_slot < 0 || !op.xrow_bf16) return;
    const int64_t e = 4 * (static_cast<int64_t>(blockIdx.x) * kT + threadIdx.x);
    if (e >= p.ld) return;
    const v4f x = *reinterpret_cast<const v4f*>(p.X + static_cast<int64_t>(op.worker) * p.ld + e);
    const v4f g = *reinterpret_cast<const v4f*>(p.slots + static_cast<int64_t>(op.comp_slot) * p.ld + e);
    v4f c;
    {
#pragma clang fp contract(off)
        const v4f step = g * op.comp_gamma;
        c = x - step;
    }
    uint16_t* __restrict__ dst = static_cast<uint16_t*>(const_cast<void*>(op.xrow_bf16)) + e;
    *reinterpret_cast<v4h*>(dst) = v4h{bf16_rne(c.x), bf16_rne(c.y), bf16_rne(c.z), bf16_rne(c.w)};
}

// ---- 1. forward: H = relu(Xb W1 + b1), grid = (hid / 32, n_ops, ceil(M / 32)) ----------------------
// One block (512 threads) owns a 32 (minibatch) x 32 (hidden) tile of H (two blocks share a weight tile when the
// minibatch has more than 32 samples: a block then pulls 100 KB of operands through its compute unit instead
// of 150 KB, a round of four gradients fills the chip, and the two land on the same XCD).  The contraction over
// the input features is split across the eight wavefronts (k-steps of 32, step s goes to
// wavefront s % 8), each with its own transposed W1 tile in LDS; the operands of up to kFwdDepth
// steps of a wavefront (all of them for 784 inputs) are requested before the first MFMA, so the
// kernel pays the memory latency once.  The eight partial tiles are added in a fixed order
// through LDS -- (w, w + 4) first, then the four sums in sequence, every thread finishing four
// elements of the tile -- and the block adds its share of the logits, one thread per two of them.
// tile handled by block x of a row of G blocks: consecutive tiles on the same XCD (block x runs on XCD x % 8
// when G is a multiple of 8, as it is for every supported hidden size that is a multiple of 256)
__device__ __forceinline__ int xcd_neighbours(int x, int G) { return (G & 7) == 0 ? (x & 7) * (G >> 3) + (x >> 3) : x; }

constexpr int kFwdTileH = 32;
constexpr int kFwdT = 512;
constexpr int kFwdWaves = kFwdT / 64;
constexpr int kFwdDepth = 4;
constexpr int kFwdMT = 2;                  // 16-row minibatch tiles per block
constexpr int kFwdRows = 16 * kFwdMT;      // minibatch rows per block
constexpr int kFwdElems = kFwdMT * 2 * 4;  // accumulator elements per lane: (mt, ht, v)

struct FwdOperands {
    v8h w[2];        // W1 tile 32 (k) x 32 (h): lane holds 2 rows k, 8 columns each
    v8h a[kFwdMT];   // input fragments of the block's 16-row minibatch tiles
};

__global__ __launch_bounds__(kFwdT) void mlp_forward_kernel(const MlpParams p) {
    // per-wavefront W1 tiles during the contraction (8 x 2560 B), then four partial tiles (4 x 4 KiB)
    __shared__ __attribute__((aligned(16))) unsigned char smem[8 * kFwdTileH * 40 * 2];
    __shared__ float W2s[kFwdTileH][kMaxOut];     // this tile's rows of W2, zero beyond `out`
    __shared__ float Hs[kFwdRows][kFwdTileH + 1];  // the finished tile, as the next layer sees it
    const int m0 = kFwdRows * blockIdx.z;          // first minibatch row of this block
    const bool first_rows = blockIdx.z == 0;       // this block also leaves what does not depend on the rows
    const GradOp op = p.ops[blockIdx.y];
    const uint16_t* __restrict__ feat = static_cast<const uint16_t*>(op.features);
    const int32_t* __restrict__ idx = p.batch_by_op + static_cast<int64_t>(blockIdx.y) * p.M;   // independent of op
    const uint16_t* __restrict__ W1 = op.xrow_bf16 ? static_cast<const uint16_t*>(op.xrow_bf16)
                                                   : p.Xb + static_cast<int64_t>(op.worker) * p.ld;
    const uint16_t* __restrict__ b1 = W1 + static_cast<int64_t>(p.in) * p.hid;
    // Blocks go to the 8 XCDs round robin, each with an L2 of its own, and a 32-column tile of bf16 weights
    // is half a 128-byte line: neighbouring tiles are given to blocks of the same XCD, so that a line of W1
    // is fetched from memory once instead of twice (rocprofv3 FETCH_SIZE at 784-1024-10: 3.8 -> 2.35 MB per
    // gradient, of which 1.6 MB are W1 and 0.8 MB the minibatch inputs once per XCD; the time of this
    // latency-bound kernel does not change).
    const int tile = xcd_neighbours(blockIdx.x, gridDim.x);
    const int h0 = tile * kFwdTileH;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int li = lane & 15, kb = 8 * (lane >> 4);
    // small operands of the epilogue, requested now and used after the contraction
    uint16_t w2raw, b2raw = 0;
    int32_t label = -1;
    const uint16_t b1raw = b1[h0 + 16 * ((wave >> 2) & 1) + li];   // bias of the hidden unit this thread finishes
    {
        const uint16_t* __restrict__ W2 = b1 + p.hid;
        const int hh = threadIdx.x / kMaxOut, o = threadIdx.x % kMaxOut;     // 512 = 32 x 16
        w2raw = o < p.out ? W2[static_cast<int64_t>(h0 + hh) * p.out + o] : static_cast<uint16_t>(0);
        if (tile == 0 && first_rows) {   // one block also leaves the labels and the output bias for the next kernel
            if (threadIdx.x < kMaxM && static_cast<int>(threadIdx.x) < p.M)
                label = static_cast<const int32_t*>(op.targets)[idx[threadIdx.x]];
            if (threadIdx.x < kMaxOut && static_cast<int>(threadIdx.x) < p.out)
                b2raw = W2[static_cast<int64_t>(p.hid) * p.out + threadIdx.x];
        }
    }
    uint16_t(*Bt)[40] = reinterpret_cast<uint16_t(*)[40]>(smem + wave * (kFwdTileH * 40 * 2));   // [h][k]
    float* red = reinterpret_cast<float*>(smem);

    const uint16_t* rowp[kFwdMT];
#pragma unroll
    for (int mt = 0; mt < kFwdMT; ++mt) {
        const int m = m0 + 16 * mt + li;
        rowp[mt] = m < p.M ? feat + static_cast<int64_t>(idx[m]) * op.ld : nullptr;
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
        for (int mt = 0; mt < kFwdMT; ++mt)
            f.a[mt] = (rowp[mt] && k0 + kb < p.in) ? *reinterpret_cast<const v8h*>(rowp[mt] + k0 + kb) : zero;
    };

    v4f acc[kFwdMT][2];
#pragma unroll
    for (int mt = 0; mt < kFwdMT; ++mt)
#pragma unroll
        for (int ht = 0; ht < 2; ++ht) acc[mt][ht] = v4f{0, 0, 0, 0};

    const int steps = (p.in + 31) / 32, iters = (steps + kFwdWaves - 1) / kFwdWaves;   // same trip count for every wavefront
    for (int it0 = 0; it0 < iters; it0 += kFwdDepth) {
        FwdOperands f[kFwdDepth];
#pragma unroll
        for (int u = 0; u < kFwdDepth; ++u)
            if (it0 + u < iters) fetch(wave + kFwdWaves * (it0 + u), f[u]);   // steps beyond the last one fetch zeros
#pragma unroll
        for (int u = 0; u < kFwdDepth; ++u) {
            if (it0 + u < iters) {        // the same for every thread of the block
#pragma unroll
                for (int r = 0; r < 2; ++r)
#pragma unroll
                    for (int e = 0; e < 8; ++e) Bt[shh + e][skk + 16 * r] = f[u].w[r][e];
                wave_lds_sync();      // the tile is this wavefront's own: no other wavefront has to wait
                v8h bfrag[2];
#pragma unroll
                for (int ht = 0; ht < 2; ++ht) bfrag[ht] = *reinterpret_cast<const v8h*>(&Bt[16 * ht + li][kb]);
#pragma unroll
                for (int mt = 0; mt < kFwdMT; ++mt)
#pragma unroll
                    for (int ht = 0; ht < 2; ++ht) acc[mt][ht] = mfma_bf16(f[u].a[mt], bfrag[ht], acc[mt][ht]);
                wave_lds_sync();
            }
        }
    }
    {
        const float w2 = bf16_to_float(w2raw);
        W2s[threadIdx.x / kMaxOut][threadIdx.x % kMaxOut] = w2;
        if (first_rows) p.W2f[(static_cast<int64_t>(blockIdx.y) * p.hid + h0) * kMaxOut + threadIdx.x] = w2;     // 32 x 16 floats, contiguous
        if (tile == 0 && first_rows) {
            if (threadIdx.x < kMaxM) p.labels[static_cast<int64_t>(blockIdx.y) * kMaxM + threadIdx.x] = label;
            if (threadIdx.x < kMaxOut) p.b2f[static_cast<int64_t>(blockIdx.y) * kMaxOut + threadIdx.x] = bf16_to_float(b2raw);
        }
    }
    __syncthreads();      // the partial tiles below reuse the memory of the wavefronts' weight tiles

    // element q = (mt, ht, v) of lane l of partial tile w at red[(w * kFwdElems + q) * 64 + l]
    auto spill = [&](int w) {
#pragma unroll
        for (int mt = 0; mt < kFwdMT; ++mt)
#pragma unroll
            for (int ht = 0; ht < 2; ++ht)
#pragma unroll
                for (int v = 0; v < 4; ++v) red[(w * kFwdElems + (mt * 2 + ht) * 4 + v) * 64 + lane] = acc[mt][ht][v];
    };
    if (wave >= 4) spill(wave - 4);
    __syncthreads();
    if (wave < 4) {
#pragma unroll
        for (int mt = 0; mt < kFwdMT; ++mt)
#pragma unroll
            for (int ht = 0; ht < 2; ++ht)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[mt][ht][v] += red[((wave * kFwdElems) + (mt * 2 + ht) * 4 + v) * 64 + lane];
    }
    __syncthreads();
    if (wave < 4) spill(wave);
    __syncthreads();
    // every thread finishes kFwdElems / 8 elements: q = wave + 8 j
#pragma unroll
    for (int j = 0; j < kFwdElems / kFwdWaves; ++j) {
        const int q = wave + kFwdWaves * j;
        const float sum = ((red[(0 * kFwdElems + q) * 64 + lane] + red[(1 * kFwdElems + q) * 64 + lane]) +
                           red[(2 * kFwdElems + q) * 64 + lane]) + red[(3 * kFwdElems + q) * 64 + lane];
        const int mt = q >> 3, ht = (q >> 2) & 1, v = q & 3;
        const int ml = 16 * mt + 4 * (lane >> 4) + v, m = m0 + ml, hh = 16 * ht + li;    // row inside the block, and of the minibatch
        float hval = 0.0f;
        if (m < p.M) {
            const float pre = sum + bf16_to_float(b1raw);
            const uint16_t hb = bf16_rne(pre > 0.0f ? pre : 0.0f);
            p.Hb[(static_cast<int64_t>(blockIdx.y) * kMaxM + m) * p.hid + h0 + hh] = hb;
            hval = bf16_to_float(hb);
        }
        Hs[ml][hh] = hval;
    }
    __syncthreads();
    // this tile's share of the logits: thread (m, o) sums over the 32 hidden units in order
    {
        const int ml = threadIdx.x >> 4, o = threadIdx.x & 15;       // 512 = 32 rows x 16 outputs
        float part = 0.0f;
#pragma unroll 8
        for (int hh = 0; hh < kFwdTileH; ++hh) part += Hs[ml][hh] * W2s[hh][o];
        p.logit_part[((static_cast<int64_t>(blockIdx.y) * gridDim.x + tile) * kMaxM + m0 + ml) * kMaxOut + o] = part;
    }
}

// ---- 2. softmax, second-layer gradients and the hidden error: grid = (hid / 64, n_ops) ----
// 1024 threads.  The grid is small and the work per block is a chain of short dependent steps,
// so the block is wide: every step is spread over 16 wavefronts and every global operand is
// requested before the first one is used.
//   a. thread (m, o) finishes logit o of sample m (sum of the hid / 32 forward-tile contributions
//      in tile order); the 16 lanes of a sample take the softmax together (butterfly max and sum).
//      The 16 blocks of a gradient repeat this small step rather than wait for a kernel of its own.
//   b. thread (hl, mg): hidden unit h = 64 blockIdx.x + hl, minibatch rows [4 mg, 4 mg + 4):
//      its share of dW2 and db1, and the hidden error dH (rounded to bf16) of its four rows.
//   c. the 16 row groups are added pairwise in a fixed tree through LDS.
constexpr int kBwdT = 1024;
constexpr int kBwdGroups = kBwdT / 64;            // 16 row groups
constexpr int kBwdRows = kMaxM / kBwdGroups;      // 4 minibatch rows per thread

__global__ __launch_bounds__(kBwdT) void mlp_backward_small_kernel(const MlpParams p) {
    __shared__ __attribute__((aligned(16))) float dl_s[kMaxM][kMaxOut];   // softmax - onehot, zero beyond M and out
    __shared__ float loss_s[kMaxM];
    __shared__ float red[kBwdGroups / 2][kMaxOut + 1][64];
    const GradOp op = p.ops[blockIdx.y];     // needed for the stores only: no load below waits for it
    uint16_t* __restrict__ dH = p.factored ? reinterpret_cast<uint16_t*>(p.slots + static_cast<int64_t>(op.slot) * p.ld)
                                           : p.dHb + static_cast<int64_t>(blockIdx.y) * kMaxM * p.hid;
    const int hl = threadIdx.x & 63, mg = threadIdx.x >> 6;
    const int h = blockIdx.x * 64 + hl;
    const int sm = threadIdx.x >> 4, so = threadIdx.x & 15;       // step a: sample and logit

    // ---- all global loads (everything the forward kernel left in the scratch memory, addressed by block index)
    const int label = p.labels[static_cast<int64_t>(blockIdx.y) * kMaxM + sm];      // -1 beyond M
    const int tiles = p.hid / kFwdTileH;
    const float* __restrict__ src = p.logit_part + (static_cast<int64_t>(blockIdx.y) * tiles * kMaxM + sm) * kMaxOut + so;
    constexpr int kTileBatch = 32;
    float part[kTileBatch];
#pragma unroll
    for (int t = 0; t < kTileBatch; ++t) part[t] = t < tiles ? src[static_cast<int64_t>(t) * kMaxM * kMaxOut] : 0.0f;
    const float b2v = p.b2f[static_cast<int64_t>(blockIdx.y) * kMaxOut + so];         // zero beyond `out`
    v4f w2q[kMaxOut / 4];
    uint16_t hraw[kBwdRows];
    {
        const v4f* __restrict__ w2p = reinterpret_cast<const v4f*>(p.W2f + (static_cast<int64_t>(blockIdx.y) * p.hid + h) * kMaxOut);
#pragma unroll
        for (int q = 0; q < kMaxOut / 4; ++q) w2q[q] = w2p[q];
    }
#pragma unroll
    for (int r = 0; r < kBwdRows; ++r) {
        const int m = kBwdRows * mg + r;
        hraw[r] = m < p.M ? p.Hb[(static_cast<int64_t>(blockIdx.y) * kMaxM + m) * p.hid + h] : static_cast<uint16_t>(0);
    }

    // ---- a. logits and softmax
    {
        float z = 0.0f;
#pragma unroll
        for (int t = 0; t < kTileBatch; ++t) z += part[t];
        for (int t0 = kTileBatch; t0 < tiles; t0 += kTileBatch) {      // hidden layers wider than 1024
#pragma unroll
            for (int t = 0; t < kTileBatch; ++t) part[t] = (t0 + t < tiles) ? src[static_cast<int64_t>(t0 + t) * kMaxM * kMaxOut] : 0.0f;
#pragma unroll
            for (int t = 0; t < kTileBatch; ++t) z += part[t];
        }
        const bool live = so < p.out;
        const float logit = live ? z + b2v : -INFINITY;
        float zmax = logit;
#pragma unroll
        for (int off = 8; off > 0; off >>= 1) zmax = fmaxf(zmax, __shfl_xor(zmax, off, 64));
        const float ez = live ? expf(logit - zmax) : 0.0f;
        float zsum = ez;
#pragma unroll
        for (int off = 8; off > 0; off >>= 1) zsum += __shfl_xor(zsum, off, 64);
        const int lsrc = (threadIdx.x & 48) + (label >= 0 && label < p.out ? label : 0);   // lane of the labelled class
        const float lsel = __shfl(logit, lsrc, 64);
        dl_s[sm][so] = (live && sm < p.M) ? ez / zsum - (so == label ? 1.0f : 0.0f) : 0.0f;
        if (so == 0) loss_s[sm] = sm < p.M ? -(lsel - zmax - logf(zsum)) : 0.0f;
    }
    __syncthreads();

    // ---- b. this thread's hidden unit and rows
    float* __restrict__ g = p.slots + static_cast<int64_t>(op.slot) * p.ld;
    float* __restrict__ gb1 = g + static_cast<int64_t>(p.in) * p.hid;
    float* __restrict__ gW2 = gb1 + p.hid;
    float* __restrict__ gb2 = gW2 + static_cast<int64_t>(p.hid) * p.out;
    float w2[kMaxOut], gw2[kMaxOut];
#pragma unroll
    for (int q = 0; q < kMaxOut / 4; ++q) {
        w2[4 * q] = w2q[q].x; w2[4 * q + 1] = w2q[q].y; w2[4 * q + 2] = w2q[q].z; w2[4 * q + 3] = w2q[q].w;
    }
#pragma unroll
    for (int o = 0; o < kMaxOut; ++o) gw2[o] = 0.0f;
    float sum_dh = 0.0f;
#pragma unroll
    for (int r = 0; r < kBwdRows; ++r) {
        const int m = kBwdRows * mg + r;
        float dl[kMaxOut];
#pragma unroll
        for (int q = 0; q < kMaxOut / 4; ++q) {
            const v4f t4 = *reinterpret_cast<const v4f*>(&dl_s[m][4 * q]);
            dl[4 * q] = t4.x; dl[4 * q + 1] = t4.y; dl[4 * q + 2] = t4.z; dl[4 * q + 3] = t4.w;
        }
        const float hv = bf16_to_float(hraw[r]);       // zero for rows m >= M, whose dl is zero as well
        float back = 0.0f;
#pragma unroll
        for (int o = 0; o < kMaxOut; ++o) {             // entries o >= out are zero in dl_s and w2
            gw2[o] += hv * dl[o];
            back += dl[o] * w2[o];
        }
        const uint16_t dh = (m < p.M && hv > 0.0f) ? bf16_rne(back * p.gscale) : static_cast<uint16_t>(0);
        sum_dh += bf16_to_float(dh);
        dH[static_cast<int64_t>(m) * p.hid + h] = dh;    // rows m >= M are the zero padding of the dW1 product
    }

    // ---- c. fixed pairwise tree over the 16 row groups: (g, g + 8), then (g, g + 4), (g, g + 2), (g, g + 1)
#pragma unroll
    for (int half = kBwdGroups / 2; half > 0; half >>= 1) {
        if (mg >= half && mg < 2 * half) {
#pragma unroll
            for (int o = 0; o < kMaxOut; ++o) red[mg - half][o][hl] = gw2[o];
            red[mg - half][kMaxOut][hl] = sum_dh;
        }
        __syncthreads();
        if (mg < half) {
#pragma unroll
            for (int o = 0; o < kMaxOut; ++o) gw2[o] += red[mg][o][hl];
            sum_dh += red[mg][kMaxOut][hl];
        }
        __syncthreads();
    }
    if (mg == 0) {
#pragma unroll
        for (int o = 0; o < kMaxOut; ++o)
            if (o < p.out) gW2[static_cast<int64_t>(h) * p.out + o] = gw2[o] * p.gscale;
        gb1[h] = sum_dh;
    }
    if (blockIdx.x == 0 && mg == 1 && hl < p.out) {
        float sdl = 0.0f;
        for (int m = 0; m < p.M; ++m) sdl += dl_s[m][hl];
        gb2[hl] = sdl * p.gscale;
    }
    if (blockIdx.x == 0 && threadIdx.x == 128 && p.loss) {
        float sl = 0.0f;
        for (int m = 0; m < p.M; ++m) sl += loss_s[m];
        p.loss[op.event] = sl * p.gscale;
    }
}

// ---- 2b. loss only (evaluation of the objective): grid = n_ops, 1024 threads ------------------
// Step a of the backward kernel without the rest: logits, softmax, cross-entropy of the first
// `count` samples of each operation, summed in sample order in fp64.  count_errors: a sample
// contributes 1 when its largest logit (the lowest class on ties) is not its label, else 0.
__global__ __launch_bounds__(kBwdT) void mlp_loss_kernel(const MlpParams p, double* loss_sum, int count_errors) {
    __shared__ float loss_s[kMaxM];
    const GradOp op = p.ops[blockIdx.x];
    const int sm = threadIdx.x >> 4, so = threadIdx.x & 15;
    const int label = p.labels[static_cast<int64_t>(blockIdx.x) * kMaxM + sm];       // left by the forward kernel, -1 beyond M
    const int tiles = p.hid / kFwdTileH;
    const float* __restrict__ src = p.logit_part + (static_cast<int64_t>(blockIdx.x) * tiles * kMaxM + sm) * kMaxOut + so;
    float z = 0.0f;
    for (int t0 = 0; t0 < tiles; t0 += 32) {
        float part[32];
#pragma unroll
        for (int t = 0; t < 32; ++t) part[t] = (t0 + t < tiles) ? src[static_cast<int64_t>(t0 + t) * kMaxM * kMaxOut] : 0.0f;
#pragma unroll
        for (int t = 0; t < 32; ++t) z += part[t];
    }
    const bool live = so < p.out;
    const float logit = live ? z + p.b2f[static_cast<int64_t>(blockIdx.x) * kMaxOut + so] : -INFINITY;
    float zmax = logit;
#pragma unroll
    for (int off = 8; off > 0; off >>= 1) zmax = fmaxf(zmax, __shfl_xor(zmax, off, 64));
    float zsum = live ? expf(logit - zmax) : 0.0f;
#pragma unroll
    for (int off = 8; off > 0; off >>= 1) zsum += __shfl_xor(zsum, off, 64);
    const int lsrc = (threadIdx.x & 48) + (label >= 0 && label < p.out ? label : 0);
    const float lsel = __shfl(logit, lsrc, 64);
    int best = live && logit == zmax ? so : kMaxOut;
#pragma unroll
    for (int off = 8; off > 0; off >>= 1) best = min(best, __shfl_xor(best, off, 64));
    if (so == 0) loss_s[sm] = count_errors ? (best != label ? 1.0f : 0.0f) : -(lsel - zmax - logf(zsum));
    __syncthreads();
    if (threadIdx.x == 0) {
        const int count = op.count > 0 ? (op.count < p.M ? op.count : p.M) : p.M;
        double s = 0.0;
        for (int m = 0; m < count; ++m) s += loss_s[m];
        loss_sum[blockIdx.x] = s;
    }
}

// ---- 3. dW1 = Xb^T dH ------------------------------------------------------------------
// One 64 (inputs) x 64 (hidden) tile of the product: the minibatch rows of the inputs and of dH
// ([kMaxM][hid] bf16, rows >= M zero) are transposed through LDS, then wavefront w multiplies the
// four 16-row input tiles with hidden columns [16 w, 16 w + 16).  Lane l ends up with
// acc[it][v] = dW1[i0 + 16 it + 4 (l / 16) + v][h0 + 16 w + l % 16].
__device__ __forceinline__ void dw1_tile(const uint16_t* __restrict__ feat, int64_t feat_ld, const int32_t* __restrict__ idx,
                                         int M, int in, const uint16_t* __restrict__ dH, int hid, int h0, int i0,
                                         uint16_t (*At)[72], uint16_t (*Bt)[72], v4f acc[4]) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int li = lane & 15, kb = 8 * (lane >> 4);
    {   // stage: thread handles one minibatch row m and 16 consecutive columns
        const int m = threadIdx.x >> 2, seg = (threadIdx.x & 3) * 16;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int c = seg + 8 * half;
            v8h xv = {0, 0, 0, 0, 0, 0, 0, 0};
            if (m < M && i0 + c < in) xv = *reinterpret_cast<const v8h*>(feat + static_cast<int64_t>(idx[m]) * feat_ld + i0 + c);
            const v8h dv = *reinterpret_cast<const v8h*>(dH + static_cast<int64_t>(m) * hid + h0 + c);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                At[c + e][m] = xv[e];
                Bt[c + e][m] = dv[e];
            }
        }
    }
    __syncthreads();
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
}

// dW1 written out as a dense gradient: grid = (hid / 64, ceil(in / 64), n_ops)
__global__ __launch_bounds__(kT) void mlp_dw1_kernel(const MlpParams p) {
    __shared__ __attribute__((aligned(16))) uint16_t At[64][72];   // inputs transposed:  [i][m], 64 m + pad
    __shared__ __attribute__((aligned(16))) uint16_t Bt[64][72];   // hidden error transposed: [h][m]
    const GradOp op = p.ops[blockIdx.z];
    const int h0 = blockIdx.x * kTileH, i0 = blockIdx.y * 64;
    v4f acc[4];
    dw1_tile(static_cast<const uint16_t*>(op.features), op.ld, p.batch_by_op + static_cast<int64_t>(blockIdx.z) * p.M, p.M, p.in,
             p.dHb + static_cast<int64_t>(blockIdx.z) * kMaxM * p.hid, p.hid, h0, i0, At, Bt, acc);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    float* __restrict__ g = p.slots + static_cast<int64_t>(op.slot) * p.ld;
    const int h = h0 + 16 * wave + (lane & 15);
#pragma unroll
    for (int it = 0; it < 4; ++it) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int i = i0 + 16 * it + 4 * (lane >> 4) + v;
            if (i < p.in) g[static_cast<int64_t>(i) * p.hid + h] = acc[it][v];
        }
    }
}

// ---- 4. model update with dW1 in factored form ----------------------------------------------
// The event's update  avg = (x^i + x^j) / 2;  x^j <- avg;  x^i <- avg - gamma g  for the
// perceptron, with the first-layer part of g formed here from its factors (the same tile product
// as above, so the values are those of the dense gradient) and only the small remainder
// (b1, W2, b2) read from the pending slot.  The bf16 shadow of both rows is rewritten.
//   grid = (hid / 64, ceil(in / 64) + tail rows, events of the round)
//   blockIdx.y <  ceil(in / 64): one 64 x 64 tile of W1.  The tile of g goes through LDS so that
//                 each thread updates float4 pieces of contiguous rows (16 lanes per 256-byte row);
//   blockIdx.y >= ceil(in / 64): 1024 consecutive floats of the remainder, elementwise.
struct MlpApplyParams {
    float* X;
    int64_t ld;
    int64_t d;
    int in, hid, M;
    const PairOp* ops;
    const float* slots;
    uint16_t* Xbf16;
    const int32_t* batch_by_op;   // [op][M]
    float* V;                // momentum buffers (MOM), else nullptr
    float momentum, weight_decay;
};

// vold: the worker's momentum entries (MOM and not average_only), else unused
template <bool MOM>
__device__ __forceinline__ void apply4(const MlpApplyParams& p, const PairOp& op, int64_t e, v4f a, v4f b, v4f g, v4f vold,
                                       bool average_only, bool pair, int valid) {
    float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w}, gv[4] = {g.x, g.y, g.z, g.w};
    float ni[4], nj[4];
    if (MOM && !average_only) {       // an averaging-only pair leaves the momentum buffers alone
        const float vo[4] = {vold.x, vold.y, vold.z, vold.w};
        float vn[4];
#pragma unroll
        for (int c = 0; c < 4; ++c)
            average_then_apply_momentum(av[c], bv[c], gv[c], vo[c], op.gamma, p.momentum, p.weight_decay, ni[c], nj[c], vn[c]);
        float* __restrict__ vi = p.V + static_cast<int64_t>(op.i) * p.ld + e;
        if (valid == 4) *reinterpret_cast<v4f*>(vi) = v4f{vn[0], vn[1], vn[2], vn[3]};
        else
            for (int c = 0; c < valid; ++c) vi[c] = vn[c];
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c)
            average_then_apply(av[c], bv[c], average_only ? 0.0f : gv[c], average_only ? 0.0f : op.gamma, ni[c], nj[c]);
    }
    float* __restrict__ xi = p.X + static_cast<int64_t>(op.i) * p.ld + e;
    float* __restrict__ xj = p.X + static_cast<int64_t>(op.j) * p.ld + e;
    uint16_t* __restrict__ si = p.Xbf16 + static_cast<int64_t>(op.i) * p.ld + e;
    uint16_t* __restrict__ sj = p.Xbf16 + static_cast<int64_t>(op.j) * p.ld + e;
    if (valid == 4) {
        *reinterpret_cast<v4f*>(xi) = v4f{ni[0], ni[1], ni[2], ni[3]};
        *reinterpret_cast<v4h*>(si) = v4h{bf16_rne(ni[0]), bf16_rne(ni[1]), bf16_rne(ni[2]), bf16_rne(ni[3])};
        if (pair) {
            *reinterpret_cast<v4f*>(xj) = v4f{nj[0], nj[1], nj[2], nj[3]};
            *reinterpret_cast<v4h*>(sj) = v4h{bf16_rne(nj[0]), bf16_rne(nj[1]), bf16_rne(nj[2]), bf16_rne(nj[3])};
        }
    } else {                      // ragged end of the parameter vector: entries at and beyond d stay untouched
        for (int c = 0; c < valid; ++c) {
            xi[c] = ni[c];
            si[c] = bf16_rne(ni[c]);
            if (pair) {
                xj[c] = nj[c];
                sj[c] = bf16_rne(nj[c]);
            }
        }
    }
}

template <bool MOM>
__global__ __launch_bounds__(kT) void mlp_apply_factored_kernel(const MlpApplyParams p) {
    __shared__ __attribute__((aligned(16))) uint16_t At[64][72];
    __shared__ __attribute__((aligned(16))) uint16_t Bt[64][72];
    __shared__ __attribute__((aligned(16))) float Gs[64][68];       // the tile of g, [input][hidden]
    const PairOp op = p.ops[blockIdx.z];
    const bool average_only = (op.flags & 1) != 0;    // extra pair of a general W_k: no gradient, no step
    const bool pair = op.i != op.j;
    const float* __restrict__ xi = p.X + static_cast<int64_t>(op.i) * p.ld;
    const float* __restrict__ xj = p.X + static_cast<int64_t>(op.j) * p.ld;
    const float* __restrict__ slot = p.slots + static_cast<int64_t>(op.slot) * p.ld;
    const int in_tiles = (p.in + 63) / 64;
    if (static_cast<int>(blockIdx.y) >= in_tiles) {
        // remainder of the parameter vector (b1, W2, b2): dense gradient from the slot
        const int64_t tb = static_cast<int64_t>(blockIdx.y - in_tiles) * gridDim.x + blockIdx.x;
        const int64_t e = static_cast<int64_t>(p.in) * p.hid + 4 * (tb * kT + threadIdx.x);
        if (e >= p.d) return;
        const int valid = p.d - e >= 4 ? 4 : static_cast<int>(p.d - e);
        const v4f a = *reinterpret_cast<const v4f*>(xi + e), b = *reinterpret_cast<const v4f*>(xj + e);   // rows are padded
        v4f g = {0, 0, 0, 0}, vold = {0, 0, 0, 0};
        if (!average_only) g = *reinterpret_cast<const v4f*>(slot + e);
        if (MOM && !average_only) vold = *reinterpret_cast<const v4f*>(p.V + static_cast<int64_t>(op.i) * p.ld + e);
        apply4<MOM>(p, op, e, a, b, g, vold, average_only, pair, valid);
        return;
    }
    const int h0 = blockIdx.x * kTileH, i0 = blockIdx.y * 64;
    const int rr = threadIdx.x >> 4, hq = (threadIdx.x & 15) * 4;      // this thread's rows 16 r + rr, columns hq .. hq + 3
    v4f a[4], b[4], vold[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {        // the model rows are requested before the product is formed
        const int i = i0 + 16 * r + rr;
        vold[r] = v4f{0, 0, 0, 0};
        if (i < p.in) {
            const int64_t e = static_cast<int64_t>(i) * p.hid + h0 + hq;
            a[r] = *reinterpret_cast<const v4f*>(xi + e);
            b[r] = *reinterpret_cast<const v4f*>(xj + e);
            if (MOM && !average_only) vold[r] = *reinterpret_cast<const v4f*>(p.V + static_cast<int64_t>(op.i) * p.ld + e);
        }
    }
    if (!average_only) {                  // uniform over the block
        v4f acc[4];
        dw1_tile(static_cast<const uint16_t*>(op.features), op.feat_ld, p.batch_by_op + static_cast<int64_t>(blockIdx.z) * p.M, p.M,
                 p.in, reinterpret_cast<const uint16_t*>(slot), p.hid, h0, i0, At, Bt, acc);
        const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
        for (int it = 0; it < 4; ++it)
#pragma unroll
            for (int v = 0; v < 4; ++v) Gs[16 * it + 4 * (lane >> 4) + v][16 * wave + (lane & 15)] = acc[it][v];
        __syncthreads();
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int i = i0 + 16 * r + rr;
        if (i >= p.in) continue;
        v4f g = {0, 0, 0, 0};
        if (!average_only) g = *reinterpret_cast<const v4f*>(&Gs[16 * r + rr][hq]);
        apply4<MOM>(p, op, static_cast<int64_t>(i) * p.hid + h0 + hq, a[r], b[r], g, vold[r], average_only, pair, 4);
    }
}

size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

// scratch memory of a launch group: [Hb][dHb][logit_part][W2f][labels][b2f]
struct ScratchLayout {
    size_t dHb, logit_part, W2f, labels, b2f, total;
};
ScratchLayout scratch_layout(int32_t n_ops, int32_t hid) {
    const size_t ops = static_cast<size_t>(n_ops);
    const size_t act = align256(ops * kMaxM * hid * sizeof(uint16_t));
    ScratchLayout L;
    L.dHb = act;
    L.logit_part = 2 * act;
    L.W2f = L.logit_part + align256(ops * (hid / kFwdTileH) * kMaxM * kMaxOut * 4);
    L.labels = L.W2f + align256(ops * hid * kMaxOut * 4);
    L.b2f = L.labels + align256(ops * kMaxM * 4);
    L.total = L.b2f + align256(ops * kMaxOut * 4);
    return L;
}
void set_scratch(MlpParams& p, void* scratch, int32_t n_ops, int32_t hid) {
    const ScratchLayout L = scratch_layout(n_ops, hid);
    char* s = static_cast<char*>(scratch);
    p.Hb = reinterpret_cast<uint16_t*>(s);
    p.dHb = reinterpret_cast<uint16_t*>(s + L.dHb);
    p.logit_part = reinterpret_cast<float*>(s + L.logit_part);
    p.W2f = reinterpret_cast<float*>(s + L.W2f);
    p.labels = reinterpret_cast<int32_t*>(s + L.labels);
    p.b2f = reinterpret_cast<float*>(s + L.b2f);
}

}  // namespace

size_t mlp_scratch_bytes(int32_t n_ops, int32_t M, int32_t in, int32_t hid, int32_t out) {
    if (n_ops < 1 || M < 1 || M > kMaxM || in < 8 || (in & 7) || hid < kTileH || (hid % kTileH) || out < 1 || out > kMaxOut)
        return 0;
    return scratch_layout(n_ops, hid).total;
}

hipError_t launch_mlp_loss(const MlpGradArgs& a, double* loss_sum, bool count_errors, hipStream_t st) {
    if (a.n_ops <= 0) return hipSuccess;
    if (mlp_scratch_bytes(a.n_ops, a.M, a.in, a.hid, a.out) == 0 || a.n_ops > 65535) return hipErrorInvalidValue;
    MlpParams p{};
    p.X = a.X;
    p.Xb = a.Xbf16;
    p.ld = a.ld;
    p.in = a.in;
    p.hid = a.hid;
    p.out = a.out;
    p.ops = a.ops;
    p.M = a.M;
    p.batch_by_op = a.batch_by_op;
    p.slots = a.slots;
    p.gscale = a.gscale;
    p.loss = nullptr;
    set_scratch(p, a.scratch, a.n_ops, a.hid);
    hipLaunchKernelGGL(mlp_forward_kernel, dim3(a.hid / kFwdTileH, a.n_ops, (a.M + kFwdRows - 1) / kFwdRows), dim3(kFwdT), 0, st, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(mlp_loss_kernel, dim3(a.n_ops), dim3(kBwdT), 0, st, p, loss_sum, count_errors ? 1 : 0);
    return hipGetLastError();
}

bool mlp_can_factor(int32_t in, int32_t hid, int32_t M) {
    // dH (kMaxM x hid bf16) must fit the first-layer part of a pending slot (in x hid fp32)
    return M >= 1 && M <= kMaxM && in >= 32 && (in & 7) == 0 && hid >= kTileH && hid % kTileH == 0;
}

hipError_t launch_mlp_apply_factored(const MlpApplyArgs& a, hipStream_t st) {
    if (a.n_ops <= 0) return hipSuccess;
    if (!mlp_can_factor(a.in, a.hid, a.M) || a.n_ops > 65535 || !a.Xbf16) return hipErrorInvalidValue;
    MlpApplyParams p;
    p.X = a.X;
    p.ld = a.ld;
    p.d = a.d;
    p.in = a.in;
    p.hid = a.hid;
    p.M = a.M;
    p.ops = a.ops;
    p.slots = a.slots;
    p.Xbf16 = a.Xbf16;
    p.batch_by_op = a.batch_by_op;
    p.V = a.V;
    p.momentum = a.momentum;
    p.weight_decay = a.weight_decay;
    const int64_t tail = a.d - static_cast<int64_t>(a.in) * a.hid;            // floats after W1
    const uint32_t bx = static_cast<uint32_t>(a.hid / kTileH);
    const int64_t per_row = static_cast<int64_t>(bx) * kT * 4;                  // floats one grid row of blocks covers
    const int64_t tail_rows = tail > 0 ? (tail + per_row - 1) / per_row : 0;
    const int64_t by = (a.in + 63) / 64 + tail_rows;
    if (by > 65535) return hipErrorInvalidValue;
    const dim3 grid(bx, static_cast<uint32_t>(by), a.n_ops);
    if (a.V) hipLaunchKernelGGL(mlp_apply_factored_kernel<true>, grid, dim3(kT), 0, st, p);
    else hipLaunchKernelGGL(mlp_apply_factored_kernel<false>, grid, dim3(kT), 0, st, p);
    return hipGetLastError();
}

hipError_t launch_mlp_gradient(const MlpGradArgs& a, hipStream_t st, int* n_launches) {
    if (a.n_ops <= 0) return hipSuccess;
    if (mlp_scratch_bytes(a.n_ops, a.M, a.in, a.hid, a.out) == 0 || a.n_ops > 65535) return hipErrorInvalidValue;
    MlpParams p;
    p.X = a.X;
    p.Xb = a.Xbf16;
    p.ld = a.ld;
    p.in = a.in;
    p.hid = a.hid;
    p.out = a.out;
    p.ops = a.ops;
    p.M = a.M;
    p.batch_by_op = a.batch_by_op;
    p.slots = a.slots;
    p.gscale = a.gscale;
    p.loss = a.loss;
    p.factored = a.factored ? 1 : 0;
    if (a.factored && !mlp_can_factor(a.in, a.hid, a.M)) return hipErrorInvalidValue;
    set_scratch(p, a.scratch, a.n_ops, a.hid);
    const uint32_t hb = static_cast<uint32_t>(a.hid / kTileH);
    if (a.compensate) {
        if (!a.X || a.factored) return hipErrorInvalidValue;
        const int64_t cb = (a.ld / 4 + kT - 1) / kT;
        hipLaunchKernelGGL(mlp_compensated_rows_kernel, dim3(static_cast<uint32_t>(cb), a.n_ops), dim3(kT), 0, st, p);
        const hipError_t ec = hipGetLastError();
        if (ec != hipSuccess) return ec;
        if (n_launches) *n_launches += 1;
    }
    hipLaunchKernelGGL(mlp_forward_kernel, dim3(a.hid / kFwdTileH, a.n_ops, (a.M + kFwdRows - 1) / kFwdRows), dim3(kFwdT), 0, st, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(mlp_backward_small_kernel, dim3(a.hid / 64, a.n_ops), dim3(kBwdT), 0, st, p);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (a.factored) {
        if (n_launches) *n_launches += 2;
        return hipSuccess;
    }
    hipLaunchKernelGGL(mlp_dw1_kernel, dim3(hb, (a.in + 63) / 64, a.n_ops), dim3(kT), 0, st, p);
    if (n_launches) *n_launches += 3;
    return hipGetLastError();
}

}  // namespace adpsgd_impl
