// 16 raw bytes -> accumulator-typed values, for the streaming kernels.
#pragma once
#include "vabft_device.h"

namespace vabft {

// ---------------------------------------------------------------------------
// chunk unpacking: 16 raw bytes -> vec accumulator-typed values
// ---------------------------------------------------------------------------
template <typename T> struct Unpack;
template <> struct Unpack<bf16_t> {
    static __device__ __forceinline__ void run(const raw16& r, float (&v)[8]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(r.w[i] << 16);
            v[2 * i + 1] = __uint_as_float(r.w[i] & 0xffff0000u);
        }
    }
    static __device__ __forceinline__ float one(const void* base, int64_t idx) {
        return Elem<bf16_t>::to_acc(reinterpret_cast<const uint16_t*>(base)[idx]);
    }
};
template <> struct Unpack<f16_t> {
    static __device__ __forceinline__ void run(const raw16& r, float (&v)[8]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = Elem<f16_t>::to_acc((uint16_t)(r.w[i] & 0xffffu));
            v[2 * i + 1] = Elem<f16_t>::to_acc((uint16_t)(r.w[i] >> 16));
        }
    }
    static __device__ __forceinline__ float one(const void* base, int64_t idx) {
        return Elem<f16_t>::to_acc(reinterpret_cast<const uint16_t*>(base)[idx]);
    }
};
template <> struct Unpack<f8_t> {
    static __device__ __forceinline__ void run(const raw16& r, float (&v)[16]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[4 * i + 0] = __builtin_amdgcn_cvt_f32_fp8((int)r.w[i], 0);
            v[4 * i + 1] = __builtin_amdgcn_cvt_f32_fp8((int)r.w[i], 1);
            v[4 * i + 2] = __builtin_amdgcn_cvt_f32_fp8((int)r.w[i], 2);
            v[4 * i + 3] = __builtin_amdgcn_cvt_f32_fp8((int)r.w[i], 3);
        }
    }
    static __device__ __forceinline__ float one(const void* base, int64_t idx) {
        return Elem<f8_t>::to_acc(reinterpret_cast<const uint8_t*>(base)[idx]);
    }
};
template <> struct Unpack<bf8_t> {
    static __device__ __forceinline__ void run(const raw16& r, float (&v)[16]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[4 * i + 0] = __builtin_amdgcn_cvt_f32_bf8((int)r.w[i], 0);
            v[4 * i + 1] = __builtin_amdgcn_cvt_f32_bf8((int)r.w[i], 1);
            v[4 * i + 2] = __builtin_amdgcn_cvt_f32_bf8((int)r.w[i], 2);
            v[4 * i + 3] = __builtin_amdgcn_cvt_f32_bf8((int)r.w[i], 3);
        }
    }
    static __device__ __forceinline__ float one(const void* base, int64_t idx) {
        return Elem<bf8_t>::to_acc(reinterpret_cast<const uint8_t*>(base)[idx]);
    }
};
template <> struct Unpack<float> {
    static __device__ __forceinline__ void run(const raw16& r, float (&v)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = __uint_as_float(r.w[i]);
    }
    static __device__ __forceinline__ float one(const void* base, int64_t idx) {
        return reinterpret_cast<const float*>(base)[idx];
    }
};
template <> struct Unpack<double> {
    static __device__ __forceinline__ void run(const raw16& r, double (&v)[2]) {
        v[0] = __hiloint2double((int)r.w[1], (int)r.w[0]);
        v[1] = __hiloint2double((int)r.w[3], (int)r.w[2]);
    }
    static __device__ __forceinline__ double one(const void* base, int64_t idx) {
        return reinterpret_cast<const double*>(base)[idx];
    }
};


static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace vabft
