// Pieces shared by the GEMM kernels: block -> tile mapping, guarded loads, the fault
// injector applied to accumulator registers (paper section 6.1 "Error injection").
#pragma once
#include <type_traits>

#include "vabft_device.h"
#include "vabft_host.h"

namespace vabft {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) double f64x4_t;

// Workgroups are dealt round-robin to the 8 XCDs (each with a private L2).  Give every XCD
// a contiguous run of logical tile ids, and walk tiles in groups of GM tile-rows so that the
// tiles resident on one XCD share A row-panels and B column-panels.
__device__ __forceinline__ void tile_of_block(int b, int tiles_m, int tiles_n, int& bm, int& bn) {
    const int nb = tiles_m * tiles_n;
    const int xcd = b & 7, q = b >> 3;
    const int base = nb >> 3, rem = nb & 7;
    const int L = xcd * base + (xcd < rem ? xcd : rem) + q;
    constexpr int GM = 4;
    const int group = L / (GM * tiles_n);
    const int first_m = group * GM;
    const int gsize = (tiles_m - first_m) < GM ? (tiles_m - first_m) : GM;
    const int in = L - group * GM * tiles_n;
    bm = first_m + in % gsize;
    bn = in / gsize;
}

// 16-byte chunk of a row-major matrix of 2-byte elements, zero-filled outside [nr) x [nc)
__device__ __forceinline__ raw16 guarded_chunk2(const uint16_t* base, int r, int nr, int c, int nc, int64_t ld,
                                                int vec_ok) {
    raw16 out = {{0u, 0u, 0u, 0u}};
    if (r < nr && c < nc) {
        const uint16_t* p = base + (int64_t)r * ld + c;
        if (vec_ok && c + 8 <= nc) {
            out = ld16(p);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (c + e < nc) out.w[e >> 1] |= ((uint32_t)p[e]) << ((e & 1) * 16);
        }
    }
    return out;
}

// same for 4- and 8-byte elements (V elements per chunk)
template <typename T, int V>
__device__ __forceinline__ void guarded_chunk_wide(const T* base, int r, int nr, int c, int nc, int64_t ld,
                                                   int vec_ok, T (&out)[V]) {
#pragma unroll
    for (int e = 0; e < V; ++e) out[e] = 0;
    if (r < nr && c < nc) {
        const T* p = base + (int64_t)r * ld + c;
        if (vec_ok && c + V <= nc) {
            raw16 v = ld16(p);
            __builtin_memcpy(out, &v, 16);
        } else {
#pragma unroll
            for (int e = 0; e < V; ++e)
                if (c + e < nc) out[e] = p[e];
        }
    }
}

// --- bit flips on accumulator words ----------------------------------------
__device__ __forceinline__ float flip_bit(float v, int bit) { return __uint_as_float(__float_as_uint(v) ^ (1u << bit)); }
__device__ __forceinline__ double flip_bit(double v, int bit) {
    return __longlong_as_double(__double_as_longlong(v) ^ (long long)(1ull << bit));
}
template <typename acc_t> __device__ __forceinline__ constexpr int acc_bits() { return sizeof(acc_t) * 8; }

__device__ __forceinline__ void log_fault(const InjectArgs& inj, int row, int col, int bit, double before,
                                          double after) {
    const int slot = atomicAdd(inj.d_ninj, 1);
    if (slot < inj.log_capacity) {
        vabft_inject_rec rec;
        rec.row = row;
        rec.col = col;
        rec.bit = bit;
        rec.pad = 0;
        rec.before = before;
        rec.after = after;
        inj.d_log[slot] = rec;
    }
}

// Flip `bit` of an accumulator value and append the record (rare path, kept out of line).
template <typename acc_t>
__device__ __noinline__ acc_t flip_and_log(const InjectArgs& inj, acc_t before, int row, int col, int bit) {
    const acc_t after = flip_bit(before, bit);
    log_fault(inj, row, col, bit, (double)before, (double)after);
    return after;
}

// Compile-time loop: the body receives std::integral_constant indices, so accumulator
// registers are always addressed statically (a run-time index would push them to scratch).
template <int I, int N, typename F> __device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// Bernoulli draw for element (gi, gj); returns the bit to flip or -1
__device__ __forceinline__ int bernoulli_bit(const InjectArgs& inj, int gi, int gj, int N) {
    const uint64_t z = splitmix64_at(inj.seed, (uint64_t)gi * (uint64_t)N + (uint64_t)gj);
    if ((z >> 11) < inj.hit_limit) return inj.bit_lo + (int)((uint32_t)(z & 0x7FFull) % (uint32_t)inj.bit_span);
    return -1;
}

}  // namespace vabft
