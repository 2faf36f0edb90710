// Device-side helpers shared by the HIP kernels of the V-ABFT path (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "vabft.h"

namespace vabft {

constexpr int WAVE = 64;

// ---------------------------------------------------------------------------
// element types
// ---------------------------------------------------------------------------
struct bf16_t { uint16_t bits; };
struct f16_t { _Float16 v; };
struct f8_t { uint8_t bits; };   // OCP FP8 E4M3
struct bf8_t { uint8_t bits; };  // OCP FP8 E5M2

template <typename T> struct Elem;

template <> struct Elem<bf16_t> {
    using acc_t = float;
    static constexpr int bytes = 2;
    static constexpr int vec = 8;  // elements per 16-byte chunk
    static __device__ __forceinline__ float to_acc(uint16_t raw) { return __uint_as_float(((uint32_t)raw) << 16); }
    // float -> bf16 bit pattern, round to nearest even; NaN stays NaN
    static __device__ __forceinline__ uint16_t from_acc(float x) {
        uint32_t u = __float_as_uint(x);
        if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
        u += 0x7fffu + ((u >> 16) & 1u);
        return (uint16_t)(u >> 16);
    }
};

template <> struct Elem<f16_t> {
    using acc_t = float;
    static constexpr int bytes = 2;
    static constexpr int vec = 8;
    static __device__ __forceinline__ float to_acc(uint16_t raw) {
        _Float16 h;
        __builtin_memcpy(&h, &raw, 2);
        return (float)h;
    }
    static __device__ __forceinline__ uint16_t from_acc(float x) {
        _Float16 h = (_Float16)x;  // v_cvt_f16_f32, round to nearest even
        uint16_t r;
        __builtin_memcpy(&r, &h, 2);
        return r;
    }
};

template <> struct Elem<f8_t> {
    using acc_t = float;
    static constexpr int bytes = 1;
    static constexpr int vec = 16;  // elements per 16-byte chunk
    static __device__ __forceinline__ float to_acc(uint8_t raw) { return __builtin_amdgcn_cvt_f32_fp8((int)raw, 0); }
};

template <> struct Elem<bf8_t> {
    using acc_t = float;
    static constexpr int bytes = 1;
    static constexpr int vec = 16;
    static __device__ __forceinline__ float to_acc(uint8_t raw) { return __builtin_amdgcn_cvt_f32_bf8((int)raw, 0); }
};

template <> struct Elem<float> {
    using acc_t = float;
    static constexpr int bytes = 4;
    static constexpr int vec = 4;
};

template <> struct Elem<double> {
    using acc_t = double;
    static constexpr int bytes = 8;
    static constexpr int vec = 2;
};

// ---------------------------------------------------------------------------
// wave-level reductions (all 64 lanes end with the result)
// ---------------------------------------------------------------------------
template <typename T> __device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, WAVE);
    return v;
}
template <typename T> __device__ __forceinline__ T wave_max(T v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        T o = __shfl_xor(v, off, WAVE);
        v = v > o ? v : o;
    }
    return v;
}
template <typename T> __device__ __forceinline__ T wave_min(T v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        T o = __shfl_xor(v, off, WAVE);
        v = v < o ? v : o;
    }
    return v;
}

// Fold of the per-workgroup partials [count][3] of (S1, S2, S3) (Algorithm 1, k-loop) by the first 256
// threads of a workgroup, in the order the encode kernels use when they fold them themselves:
// thread t adds partials t, t + 256, ... in increasing order, a butterfly inside each of the four
// wavefronts, and (after a workgroup barrier) the four wavefront results in order.
// s_red: 12 doubles of LDS, [3][4].
__device__ __forceinline__ void fold_s_partials_to_lds(const double* __restrict__ partial, int count, int t,
                                                       double* s_red) {
    if (t < 256) {
        double a1 = 0, a2 = 0, a3 = 0;
        // four partials per round: their twelve loads are in flight together (one trip to memory per round, not per
        // partial), the additions stay in increasing order of b
        for (int b0 = t; b0 < count; b0 += 4 * 256) {
            double q[4][3];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int b = b0 + u * 256;
                const double* src = partial + 3 * (int64_t)(b < count ? b : t);
                q[u][0] = src[0];
                q[u][1] = src[1];
                q[u][2] = src[2];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const bool ok = b0 + u * 256 < count;
                a1 = ok ? a1 + q[u][0] : a1;
                a2 = ok ? a2 + q[u][1] : a2;
                a3 = ok ? a3 + q[u][2] : a3;
            }
        }
        a1 = wave_sum(a1);
        a2 = wave_sum(a2);
        a3 = wave_sum(a3);
        if ((t & 63) == 0) {
            s_red[0 * 4 + (t >> 6)] = a1;
            s_red[1 * 4 + (t >> 6)] = a2;
            s_red[2 * 4 + (t >> 6)] = a3;
        }
    }
}
__device__ __forceinline__ double folded_s(const double* s_red, int q) {
    double v = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) v += s_red[q * 4 + w];
    return v;
}

template <typename T> __device__ __forceinline__ T type_max();
template <> __device__ __forceinline__ float type_max<float>() { return 3.402823466e+38f; }
template <> __device__ __forceinline__ double type_max<double>() { return 1.7976931348623157e+308; }

// 16-byte global load of raw bits
struct alignas(16) raw16 { uint32_t w[4]; };

__device__ __forceinline__ raw16 ld16(const void* p) { return *reinterpret_cast<const raw16*>(p); }

// splitmix64 output for counter `index` of the stream seeded with `seed`
__device__ __forceinline__ uint64_t splitmix64_at(uint64_t seed, uint64_t index) {
    uint64_t z = seed + (index + 1ull) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

}  // namespace vabft
