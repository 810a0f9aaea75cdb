// Fused gossip-average + gradient-apply kernel: the model update of one round
// of row-disjoint events (Algorithm 1, averaging step X W_k followed by the
// update step on row i_k):
//     avg = (x^i + x^j) / 2;   x^j <- avg;   x^i <- avg - gamma * g_k
// Four HBM streams per event (read x^i, x^j, write x^i, x^j) plus one read of
// g_k from its pending slot, or no fifth stream when g_k is synthetic and is
// generated in registers.  Pure streaming: 128-bit accesses, every load of a
// tile issued before the first use, no reuse, so caches are bypassed when the
// models do not fit them.
#include "device_common.hpp"
#include "internal.hpp"

namespace adpsgd_impl {
namespace {

#ifndef ADPSGD_FUSED_THREADS
#define ADPSGD_FUSED_THREADS 256
#endif
#ifndef ADPSGD_FUSED_UNROLL
#define ADPSGD_FUSED_UNROLL 4
#endif
constexpr int kThreads = ADPSGD_FUSED_THREADS;
constexpr int kUnroll = ADPSGD_FUSED_UNROLL;      // float4 per thread, per row, per tile
constexpr int64_t kTileVec = kThreads * kUnroll;  // 1024 float4 = 16 KiB of each row

struct FusedParams {
    float* X;
    int64_t ld;
    int64_t d;
    int64_t n_vec;      // ceil(d / 4)
    const PairOp* ops;
    const float* slots;
    uint16_t* Xbf16;
    float synth_std;
    uint32_t key0, key1;
};

// The three fp32 operations of the update keep their separate roundings: the
// product gamma*g and the subtraction must not be contracted into an FMA.
__device__ __forceinline__ void average_then_apply(v4f a, v4f b, v4f g, float gamma, v4f& new_i, v4f& new_j) {
#pragma clang fp contract(off)
    const v4f avg = (a + b) * 0.5f;
    const v4f step = g * gamma;
    new_j = avg;
    new_i = avg - step;
}

template <bool SYNTH, bool SHADOW, bool STREAM>
__global__ __launch_bounds__(kThreads) void fused_gossip_apply_kernel(const FusedParams p) {
    const PairOp op = p.ops[blockIdx.y];   // uniform address: scalar loads
    float* __restrict__ xi = p.X + static_cast<int64_t>(op.i) * p.ld;
    float* __restrict__ xj = p.X + static_cast<int64_t>(op.j) * p.ld;
    const float* __restrict__ gs = SYNTH ? nullptr : p.slots + static_cast<int64_t>(op.slot) * p.ld;
    const bool pair = op.i != op.j;
    const int64_t v0 = static_cast<int64_t>(blockIdx.x) * kTileVec + threadIdx.x;

    v4f a[kUnroll], b[kUnroll], g[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const int64_t v = v0 + static_cast<int64_t>(u) * kThreads;
        if (v < p.n_vec) {
            a[u] = load4<STREAM>(xi + 4 * v);
            b[u] = load4<STREAM>(xj + 4 * v);
            if (!SYNTH) g[u] = load4<STREAM>(gs + 4 * v);
        }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const int64_t v = v0 + static_cast<int64_t>(u) * kThreads;
        if (v >= p.n_vec) continue;
        if (SYNTH) {
#ifdef ADPSGD_EXPERIMENT_NO_RNG
            g[u] = v4f{1.0f, 1.0f, 1.0f, 1.0f} * p.synth_std;
#else
            g[u] = synth_normals4(static_cast<uint32_t>(v), static_cast<uint32_t>(v >> 32), op.k_lo, op.k_hi,
                                  p.key0, p.key1) * p.synth_std;
#endif
        }
        if (4 * v + 4 > p.d) {   // ragged tail: entries at and beyond d stay zero
            const int64_t e = 4 * v;
            if (e + 1 >= p.d) g[u].y = 0.0f;
            if (e + 2 >= p.d) g[u].z = 0.0f;
            if (e + 3 >= p.d) g[u].w = 0.0f;
        }
        v4f ni, nj;
        average_then_apply(a[u], b[u], g[u], op.gamma, ni, nj);
        store4<STREAM>(xi + 4 * v, ni);
        if (pair) store4<STREAM>(xj + 4 * v, nj);
        if (SHADOW) {
            v4h hi = {bf16_rne(ni.x), bf16_rne(ni.y), bf16_rne(ni.z), bf16_rne(ni.w)};
            *reinterpret_cast<v4h*>(p.Xbf16 + static_cast<int64_t>(op.i) * p.ld + 4 * v) = hi;
            if (pair) {
                v4h hj = {bf16_rne(nj.x), bf16_rne(nj.y), bf16_rne(nj.z), bf16_rne(nj.w)};
                *reinterpret_cast<v4h*>(p.Xbf16 + static_cast<int64_t>(op.j) * p.ld + 4 * v) = hj;
            }
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

template <bool SYNTH, bool SHADOW>
hipError_t launch_variant(const FusedParams& p, dim3 grid, bool streaming, hipStream_t st) {
    if (streaming) hipLaunchKernelGGL((fused_gossip_apply_kernel<SYNTH, SHADOW, true>), grid, dim3(kThreads), 0, st, p);
    else hipLaunchKernelGGL((fused_gossip_apply_kernel<SYNTH, SHADOW, false>), grid, dim3(kThreads), 0, st, p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_fused_gossip_apply(const FusedArgs& a, hipStream_t st) {
    if (a.n_ops <= 0) return hipSuccess;
    FusedParams p;
    p.X = a.X;
    p.ld = a.ld;
    p.d = a.d;
    p.n_vec = (a.d + 3) / 4;
    p.ops = a.ops;
    p.slots = a.slots;
    p.Xbf16 = a.Xbf16;
    p.synth_std = a.synth_std;
    p.key0 = static_cast<uint32_t>(a.synth_seed);
    p.key1 = static_cast<uint32_t>(a.synth_seed >> 32);
    const int64_t tiles = (p.n_vec + kTileVec - 1) / kTileVec;
    if (tiles > 0x7FFFFFFF || a.n_ops > 65535) return hipErrorInvalidValue;
    const dim3 grid(static_cast<uint32_t>(tiles), static_cast<uint32_t>(a.n_ops));
    if (a.synth) return launch_variant<true, false>(p, grid, a.streaming, st);
    if (a.Xbf16) return launch_variant<false, true>(p, grid, a.streaming, st);
    return launch_variant<false, false>(p, grid, a.streaming, st);
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
