// Device helpers shared by the HIP kernels: 128-bit vector types, the
// counter-based generator, the synthetic normal gradient, bf16 rounding and
// wavefront reductions (64 lanes on CDNA).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace adpsgd_impl {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));
typedef uint16_t v4h __attribute__((ext_vector_type(4)));

template <bool STREAM>
__device__ __forceinline__ v4f load4(const float* p) {
    if (STREAM) return __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p));
    return *reinterpret_cast<const v4f*>(p);
}
template <bool STREAM>
__device__ __forceinline__ void store4(float* p, v4f v) {
    if (STREAM) __builtin_nontemporal_store(v, reinterpret_cast<v4f*>(p));
    else *reinterpret_cast<v4f*>(p) = v;
}

// Philox4x32, 10 rounds (Salmon et al., SC'11).  The key and the upper counter
// words are uniform over a workgroup, so the key schedule lives in scalar registers.
__device__ __forceinline__ v4u philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                             uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t pa = static_cast<uint64_t>(0xD2511F53u) * c0;
        const uint64_t pb = static_cast<uint64_t>(0xCD9E8D57u) * c2;
        const uint32_t n0 = static_cast<uint32_t>(pb >> 32) ^ c1 ^ k0;
        const uint32_t n2 = static_cast<uint32_t>(pa >> 32) ^ c3 ^ k1;
        c1 = static_cast<uint32_t>(pb);
        c3 = static_cast<uint32_t>(pa);
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    v4u out = {c0, c1, c2, c3};
    return out;
}

constexpr uint32_t kStreamGrad = 2u << 24;

// Box-Muller on two 32-bit words: u1 = ((wa >> 9) + 1/2) 2^-23 in (0,1) and
// u2 = (wb >> 8) 2^-24 in [0,1) are exact in fp32; returns r cos(2 pi u2), r sin(2 pi u2).
__device__ __forceinline__ void box_muller(uint32_t wa, uint32_t wb, float& zc, float& zs) {
    const float u1 = (static_cast<float>(wa >> 9) + 0.5f) * 0x1p-23f;
    const float u2 = static_cast<float>(wb >> 8) * 0x1p-24f;
    // accurate library functions: the hardware approximations (v_log / v_sin / v_cos) were measured
    // and buy nothing, the kernel being bound by memory at the same time
    const float r = sqrtf(-2.0f * logf(u1));
    float s, c;
    sincospif(2.0f * u2, &s, &c);
    zc = r * c;
    zs = r * s;
}

// Four standard normals for elements 4q .. 4q+3 of the synthetic gradient of event k.
__device__ __forceinline__ v4f synth_normals4(uint32_t q_lo, uint32_t q_hi, uint32_t k_lo, uint32_t k_hi,
                                              uint32_t key0, uint32_t key1) {
    const v4u w = philox4x32_10(q_lo, q_hi, k_lo, (k_hi & 0x00FFFFFFu) | kStreamGrad, key0, key1);
    v4f z;
    float a, b;
    box_muller(w.x, w.y, a, b);
    z.x = a; z.y = b;
    box_muller(w.z, w.w, a, b);
    z.z = a; z.w = b;
    return z;
}

__device__ __forceinline__ uint16_t bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return static_cast<uint16_t>((u >> 16) | 0x0040u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}
__device__ __forceinline__ float bf16_to_float(uint16_t h) {
    return __uint_as_float(static_cast<uint32_t>(h) << 16);
}

// The three fp32 operations of the update keep their separate roundings: the
// product gamma*g and the subtraction must not be contracted into an FMA.
__device__ __forceinline__ void average_then_apply(float a, float b, float g, float gamma, float& new_i, float& new_j) {
#pragma clang fp contract(off)
    const float avg = (a + b) * 0.5f;
    const float step = g * gamma;
    new_j = avg;
    new_i = avg - step;
}

// The event with the experiments' optimizer (Sec. 5.2): per-worker momentum buffer v, weight decay on
// the averaged model;  u = g + wd * avg;  v <- mu * v + u;  x^i <- avg - gamma * v.  One rounding per
// operation, in this order.
__device__ __forceinline__ void average_then_apply_momentum(float a, float b, float g, float v_old, float gamma, float mu,
                                                            float wd, float& new_i, float& new_j, float& v_new) {
#pragma clang fp contract(off)
    const float avg = (a + b) * 0.5f;
    const float decay = wd * avg;
    const float u = g + decay;
    const float carried = mu * v_old;
    v_new = carried + u;
    const float step = gamma * v_new;
    new_j = avg;
    new_i = avg - step;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

}  // namespace adpsgd_impl
