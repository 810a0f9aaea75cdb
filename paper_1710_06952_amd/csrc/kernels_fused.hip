// Fused gossip-average + gradient-apply kernel: the model update of one round
// of row-disjoint events (Algorithm 1, averaging step X W_k followed by the
// update step on row i_k):
//     avg = (x^i + x^j) / 2;   x^j <- avg;   x^i <- avg - gamma * g_k
// Four HBM streams per event (read x^i, x^j, write x^i, x^j) plus one read of
// g_k from its pending slot, or no fifth stream when g_k is synthetic and is
// generated in registers.  Pure streaming, no reuse, so caches are bypassed
// when the models do not fit them.
//
// Access shape (chosen by measurement on MI355X, 13 GB working set, in-place
// update of ~30 row pairs): each wavefront instruction moves 256 contiguous
// bytes (one dword per lane) and every lane keeps 4 loads per row in flight;
// this sustains 6.4 TB/s, against 5.8 TB/s for 128-bit accesses of any unroll
// and 5.3-5.9 TB/s for deeper or shallower unrolls of the dword shape.
#include "device_common.hpp"
#include "internal.hpp"

namespace adpsgd_impl {
namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 4;                          // dwords per thread, per row, per tile
constexpr int64_t kTileElems = kThreads * kUnroll;  // 1024 floats = 4 KiB of each row

struct FusedParams {
    float* X;
    int64_t ld;
    int64_t d;
    const PairOp* ops;
    const float* slots;
    uint16_t* Xbf16;
    float synth_std;
    uint32_t key0, key1;
    float* V;
    float momentum, weight_decay;
};

template <bool STREAM>
__device__ __forceinline__ float load1(const float* p) {
    return STREAM ? __builtin_nontemporal_load(p) : *p;
}
template <bool STREAM>
__device__ __forceinline__ void store1(float* p, float v) {
    if (STREAM) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// grid = (ceil(d / 1024), events of the round).  Pass u of thread t touches element
// 1024 blockIdx.x + 256 u + t of both rows.
// SOLO = the round contains an event without a partner (i == j: a worker with no neighbour takes a
// plain SGD step); all other rounds run the variant without the per-store test (1.3 % faster).
template <bool SYNTH, bool SHADOW, bool STREAM, bool SOLO, bool MOM>
__global__ __launch_bounds__(kThreads) void fused_gossip_apply_kernel(const FusedParams p) {
    __shared__ __attribute__((aligned(16))) float zs[SYNTH ? kTileElems : 4];
    const PairOp op = p.ops[blockIdx.y];   // uniform address: scalar loads, no LDS staging needed
    float* __restrict__ xi = p.X + static_cast<int64_t>(op.i) * p.ld;
    float* __restrict__ xj = p.X + static_cast<int64_t>(op.j) * p.ld;
    const float* __restrict__ gs = SYNTH ? nullptr : p.slots + static_cast<int64_t>(op.slot) * p.ld;
    const bool pair = !SOLO || op.i != op.j;
    const bool average_only = (op.flags & 1) != 0;   // extra pair of a general W_k: no gradient, no step
    const int64_t tile = static_cast<int64_t>(blockIdx.x) * kTileElems;
    const int64_t e0 = tile + threadIdx.x;

    float* __restrict__ vi = MOM ? p.V + static_cast<int64_t>(op.i) * p.ld : nullptr;
    float a[kUnroll], b[kUnroll], g[kUnroll], vold[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const int64_t e = e0 + u * kThreads;
        if (e < p.d) {     // (no default values: initialising a/b/g costs 3.5 % of the bandwidth)
            a[u] = load1<STREAM>(xi + e);
            b[u] = load1<STREAM>(xj + e);
            if (!SYNTH && !average_only) g[u] = load1<STREAM>(gs + e);
            if (MOM && !average_only) vold[u] = load1<STREAM>(vi + e);
        }
    }
    if (average_only) {       // uniform over the block
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int64_t e = e0 + u * kThreads;
            if (e >= p.d) continue;
            const float avg = (a[u] + b[u]) * 0.5f;
            store1<STREAM>(xi + e, avg);
            store1<STREAM>(xj + e, avg);
            if (SHADOW) {
                p.Xbf16[static_cast<int64_t>(op.i) * p.ld + e] = bf16_rne(avg);
                p.Xbf16[static_cast<int64_t>(op.j) * p.ld + e] = bf16_rne(avg);
            }
        }
        return;
    }
    if (SYNTH) {
        // One generator call yields the gradient of 4 consecutive elements.  Lane c of wavefront w
        // produces the c-th of the 64 quads that wavefront touches (quad c lies in pass c / 16) and
        // parks it in LDS in element order, so that pass u of lane l finds its value at 64 u + l.
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        const int64_t eq = tile + (lane >> 4) * kThreads + 64 * wave + 4 * (lane & 15);
        const int64_t q = eq >> 2;
        const v4f z = synth_normals4(static_cast<uint32_t>(q), static_cast<uint32_t>(q >> 32), op.k_lo, op.k_hi,
                                     p.key0, p.key1) * p.synth_std;
        *reinterpret_cast<v4f*>(&zs[wave * 256 + 4 * lane]) = z;
        __syncthreads();
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) g[u] = zs[wave * 256 + 64 * u + lane];
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const int64_t e = e0 + u * kThreads;
        if (e >= p.d) continue;            // entries at and beyond d are never touched: they stay zero
        float ni, nj;
        if (MOM) {
            float vnew;
            average_then_apply_momentum(a[u], b[u], g[u], vold[u], op.gamma, p.momentum, p.weight_decay, ni, nj, vnew);
            store1<STREAM>(vi + e, vnew);
        } else {
            average_then_apply(a[u], b[u], g[u], op.gamma, ni, nj);
        }
        store1<STREAM>(xi + e, ni);
        if (pair) store1<STREAM>(xj + e, nj);
        if (SHADOW) {
            p.Xbf16[static_cast<int64_t>(op.i) * p.ld + e] = bf16_rne(ni);
            if (pair) p.Xbf16[static_cast<int64_t>(op.j) * p.ld + e] = bf16_rne(nj);
        }
    }
}

__global__ __launch_bounds__(kThreads) void synth_gradient_kernel(float* out, int64_t d, float std, uint32_t k_lo,
                                                                  uint32_t k_hi, uint32_t key0, uint32_t key1) {
    const int64_t v = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (4 * v >= d) return;
    const v4f g = synth_normals4(static_cast<uint32_t>(v), static_cast<uint32_t>(v >> 32), k_lo, k_hi, key0, key1) * std;
    const float gv[4] = {g.x, g.y, g.z, g.w};
    for (int t = 0; t < 4; ++t)
        if (4 * v + t < d) out[4 * v + t] = gv[t];
}

template <bool SYNTH, bool SHADOW, bool STREAM, bool SOLO>
hipError_t launch_mom(const FusedParams& p, dim3 grid, hipStream_t st) {
    if (p.V) hipLaunchKernelGGL((fused_gossip_apply_kernel<SYNTH, SHADOW, STREAM, SOLO, true>), grid, dim3(kThreads), 0, st, p);
    else hipLaunchKernelGGL((fused_gossip_apply_kernel<SYNTH, SHADOW, STREAM, SOLO, false>), grid, dim3(kThreads), 0, st, p);
    return hipGetLastError();
}
template <bool SYNTH, bool SHADOW, bool STREAM>
hipError_t launch_solo(const FusedParams& p, dim3 grid, bool solo, hipStream_t st) {
    if (solo) return launch_mom<SYNTH, SHADOW, STREAM, true>(p, grid, st);
    return launch_mom<SYNTH, SHADOW, STREAM, false>(p, grid, st);
}
template <bool SYNTH, bool SHADOW>
hipError_t launch_variant(const FusedParams& p, dim3 grid, bool streaming, bool solo, hipStream_t st) {
    if (streaming) return launch_solo<SYNTH, SHADOW, true>(p, grid, solo, st);
    return launch_solo<SYNTH, SHADOW, false>(p, grid, solo, st);
}

}  // namespace

hipError_t launch_fused_gossip_apply(const FusedArgs& a, hipStream_t st) {
    if (a.n_ops <= 0) return hipSuccess;
    FusedParams p;
    p.X = a.X;
    p.ld = a.ld;
    p.d = a.d;
    p.ops = a.ops;
    p.slots = a.slots;
    p.Xbf16 = a.Xbf16;
    p.synth_std = a.synth_std;
    p.key0 = static_cast<uint32_t>(a.synth_seed);
    p.key1 = static_cast<uint32_t>(a.synth_seed >> 32);
    p.V = a.V;
    p.momentum = a.momentum;
    p.weight_decay = a.weight_decay;
    const int64_t tiles = (p.d + kTileElems - 1) / kTileElems;
    if (tiles > 0x7FFFFFFF || a.n_ops > 65535) return hipErrorInvalidValue;
    const dim3 grid(static_cast<uint32_t>(tiles), static_cast<uint32_t>(a.n_ops));
    if (a.synth) return launch_variant<true, false>(p, grid, a.streaming, a.has_solo, st);
    if (a.Xbf16) return launch_variant<false, true>(p, grid, a.streaming, a.has_solo, st);
    return launch_variant<false, false>(p, grid, a.streaming, a.has_solo, st);
}

hipError_t launch_synth_gradient(uint64_t seed, uint64_t k, float std, int64_t d, float* out, hipStream_t st) {
    if (d <= 0) return hipSuccess;
    const int64_t n_vec = (d + 3) / 4;
    const int64_t blocks = (n_vec + kThreads - 1) / kThreads;
    if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    hipLaunchKernelGGL(synth_gradient_kernel, dim3(static_cast<uint32_t>(blocks)), dim3(kThreads), 0, st, out, d, std,
                       static_cast<uint32_t>(k), static_cast<uint32_t>(k >> 32), static_cast<uint32_t>(seed),
                       static_cast<uint32_t>(seed >> 32));
    return hipGetLastError();
}

}  // namespace adpsgd_impl
