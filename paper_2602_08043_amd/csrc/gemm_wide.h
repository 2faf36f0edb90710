// FP32 / FP64 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x2f32, v_mfma_f64_16x16x4f64)
// with the fused V-ABFT epilogue (paper section 2.2 C^{r1'} = C r1 on the accumulator tile;
// section 5.1 injector).  These MFMAs take one element per lane and are 16 passes long, so
// the kernel is matrix-core bound with a simple LDS staging.
//
// Tile 128 x 128 x 16 per workgroup of 4 wavefronts (2 x 2), 64 x 64 per wavefront.
// Result layout per MFMA tile (probed on the device): lane l owns column (l % MT);
//   32x32 (FP32): register r is row 8*(r/4) + 4*(l/32) + r%4
//   16x16 (FP64): register r is row (l/16) + 4*r
// so a row sum needs a butterfly over the MT lanes that share the row.
#pragma once
#include "gemm_common.h"

namespace vabft {

template <typename T> struct WideCfg;
template <> struct WideCfg<float> {
    static constexpr int MT = 32, KM = 2, NR = 16, V = 4;
    using accv_t = f32x16_t;
    static __device__ __forceinline__ accv_t mfma(float a, float b, accv_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int row_of(int r, int lane) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }
};
template <> struct WideCfg<double> {
    static constexpr int MT = 16, KM = 4, NR = 4, V = 2;
    using accv_t = f64x4_t;
    static __device__ __forceinline__ accv_t mfma(double a, double b, accv_t c) {
        return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int row_of(int r, int lane) { return (lane >> 4) + 4 * r; }
};

namespace gw {
constexpr int BM = 128, BN = 128, BK = 16;
constexpr int LDK = BK + 1;  // [row][k] layout, padded
template <typename T> constexpr int ldn() { return BN + 16 / (int)sizeof(T); }  // [k][n] layout, padded, 16 B aligned
template <typename T> constexpr int a_elems() { return BM * LDK; }
template <typename T> constexpr int b_elems() { return (BN * LDK) > (BK * ldn<T>()) ? (BN * LDK) : (BK * ldn<T>()); }
template <typename T> constexpr int stage_elems() { return a_elems<T>() + b_elems<T>(); }
template <typename T> constexpr int lds_bytes() { return 2 * stage_elems<T>() * (int)sizeof(T); }
}  // namespace gw

// MODE 0: plain GEMM; 1: fused row-sum check; 2: check plus the fault injector.
template <typename T, int TRANSB, int MODE, bool EDGE>
__global__ __launch_bounds__(256) void gemmw_kernel(const GemmArgs g) {
    using namespace gw;
    constexpr bool VERIFY = MODE >= 1, INJECT = MODE == 2;
    using Cfg = WideCfg<T>;
    using accv_t = typename Cfg::accv_t;
    constexpr int MT = Cfg::MT, KM = Cfg::KM, NR = Cfg::NR, V = Cfg::V;
    constexpr int TM = 64 / MT;  // MFMA tiles per wavefront in each direction
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    T* smem = reinterpret_cast<T*>(smem_raw);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int lm = lane % MT, lk = lane / MT;
    int bm, bn;
    tile_of_block(blockIdx.x, g.tiles_m, g.tiles_n, bm, bn);
    if (VERIFY && blockIdx.x == 0 && tid == 0) *g.d_nflag = 0;
    const int row0 = bm * BM, col0 = bn * BN;
    const T* __restrict__ A = reinterpret_cast<const T*>(g.A);
    const T* __restrict__ B = reinterpret_cast<const T*>(g.B);

    accv_t acc[TM][TM];
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
        for (int ni = 0; ni < TM; ++ni)
#pragma unroll
            for (int r = 0; r < NR; ++r) acc[mi][ni][r] = 0;

    constexpr int CPR = BK / V;                // chunks per row in a [row][k] tile
    constexpr int NCH_A = BM * CPR / 256;      // chunks per thread
    constexpr int CPK = BN / V;                // chunks per k-row in a [k][n] tile
    constexpr int NCH_B = BK * CPK / 256;
    static_assert(NCH_A == NCH_B, "tile shape");
    T ra[NCH_A][V], rb[NCH_B][V];

    // one 16-byte chunk; whole-tile problems need no guards
    auto load_chunk = [&](const T* base, int r, int nr, int c, int nc, int64_t ld, int vec_ok, T (&out)[V]) {
        if (!EDGE) {
            const raw16 v = ld16(base + (int64_t)r * ld + c);
            __builtin_memcpy(out, &v, 16);
        } else {
            guarded_chunk_wide<T, V>(base, r, nr, c, nc, ld, vec_ok, out);
        }
    };
    auto load_tiles = [&](int kt) {
        const int kbase = kt * BK;
#pragma unroll
        for (int p = 0; p < NCH_A; ++p) {
            const int id = tid + 256 * p, r = id / CPR, c = id % CPR;
            load_chunk(A, row0 + r, g.M, kbase + c * V, g.K, g.lda, g.a_vec_ok, ra[p]);
        }
        if (TRANSB) {
#pragma unroll
            for (int p = 0; p < NCH_B; ++p) {
                const int id = tid + 256 * p, r = id / CPR, c = id % CPR;
                load_chunk(B, col0 + r, g.N, kbase + c * V, g.K, g.ldb, g.b_vec_ok, rb[p]);
            }
        } else {
#pragma unroll
            for (int p = 0; p < NCH_B; ++p) {
                const int id = tid + 256 * p, kr = id / CPK, c = id % CPK;
                load_chunk(B, kbase + kr, g.K, col0 + c * V, g.N, g.ldb, g.b_vec_ok, rb[p]);
            }
        }
    };

    auto store_tiles = [&](int s) {
        T* As = smem + s * stage_elems<T>();
        T* Bs = As + a_elems<T>();
#pragma unroll
        for (int p = 0; p < NCH_A; ++p) {
            const int id = tid + 256 * p, r = id / CPR, c = id % CPR;
#pragma unroll
            for (int e = 0; e < V; ++e) As[r * LDK + c * V + e] = ra[p][e];
        }
        if (TRANSB) {
#pragma unroll
            for (int p = 0; p < NCH_B; ++p) {
                const int id = tid + 256 * p, r = id / CPR, c = id % CPR;
#pragma unroll
                for (int e = 0; e < V; ++e) Bs[r * LDK + c * V + e] = rb[p][e];
            }
        } else {
#pragma unroll
            for (int p = 0; p < NCH_B; ++p) {
                const int id = tid + 256 * p, kr = id / CPK, c = id % CPK;
#pragma unroll
                for (int e = 0; e < V; ++e) Bs[kr * ldn<T>() + c * V + e] = rb[p][e];
            }
        }
    };

    auto compute = [&](int s) {
        const T* As = smem + s * stage_elems<T>();
        const T* Bs = As + a_elems<T>();
#pragma unroll
        for (int ks = 0; ks < BK / KM; ++ks) {
            T af[TM], bf[TM];
            const int k = ks * KM + lk;
#pragma unroll
            for (int mi = 0; mi < TM; ++mi) af[mi] = As[(wm * 64 + mi * MT + lm) * LDK + k];
#pragma unroll
            for (int ni = 0; ni < TM; ++ni)
                bf[ni] = TRANSB ? Bs[(wn * 64 + ni * MT + lm) * LDK + k] : Bs[k * ldn<T>() + wn * 64 + ni * MT + lm];
#pragma unroll
            for (int mi = 0; mi < TM; ++mi)
#pragma unroll
                for (int ni = 0; ni < TM; ++ni) acc[mi][ni] = Cfg::mfma(af[mi], bf[ni], acc[mi][ni]);
        }
    };

    const int nk = (g.K + BK - 1) / BK;
    load_tiles(0);
    store_tiles(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const bool more = kt + 1 < nk;
        if (more) load_tiles(kt + 1);
        compute(kt & 1);
        if (more) store_tiles((kt + 1) & 1);
        __syncthreads();
    }

    // accumulator element (mi, ni, r): row = row0 + wm*64 + mi*MT + row_of(r, lane), col = col0 + wn*64 + ni*MT + lm
    if (INJECT) {
        const InjectArgs& inj = g.inj;
        if (inj.mode == 1) {
            for (int e = 0; e < inj.n_list; ++e) {
                const int fr = inj.d_list[3 * e], fc = inj.d_list[3 * e + 1], fb = inj.d_list[3 * e + 2];
                if (fr < row0 || fr >= row0 + BM || fc < col0 || fc >= col0 + BN) continue;
                if (fr >= g.M || fc >= g.N || fb < 0 || fb >= acc_bits<T>()) continue;
                const int rl = fr - row0, cl = fc - col0;
                if ((rl >> 6) != wm || (cl >> 6) != wn || (cl % MT) != lm) continue;
                const int fmi = (rl & 63) / MT, fni = (cl & 63) / MT, rin = rl % MT;
                T before = 0, after = 0;
                bool mine = false;
                static_for<0, TM>([&](auto mi_c) {
                    static_for<0, TM>([&](auto ni_c) {
                        static_for<0, NR>([&](auto r_c) {
                            constexpr int mi = decltype(mi_c)::value, ni = decltype(ni_c)::value,
                                          r = decltype(r_c)::value;
                            if (mi == fmi && ni == fni && Cfg::row_of(r, lane) == rin) {
                                before = acc[mi][ni][r];
                                after = flip_bit(before, fb);
                                acc[mi][ni][r] = after;
                                mine = true;
                            }
                        });
                    });
                });
                if (mine) log_fault(inj, fr, fc, fb, (double)before, (double)after);
            }
        } else if (inj.mode == 2) {
            static_for<0, TM>([&](auto mi_c) {
                static_for<0, TM>([&](auto ni_c) {
                    static_for<0, NR>([&](auto r_c) {
                        constexpr int mi = decltype(mi_c)::value, ni = decltype(ni_c)::value, r = decltype(r_c)::value;
                        const int gi = row0 + wm * 64 + mi * MT + Cfg::row_of(r, lane);
                        const int gj = col0 + wn * 64 + ni * MT + lm;
                        if (gi < g.M && gj < g.N) {
                            const int bit = bernoulli_bit(inj, gi, gj, g.N);
                            if (bit >= 0) acc[mi][ni][r] = flip_and_log<T>(inj, acc[mi][ni][r], gi, gj, bit);
                        }
                    });
                });
            });
        }
    }

    if (VERIFY) {
        T* red = smem;  // [2][128]
#pragma unroll
        for (int mi = 0; mi < TM; ++mi)
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                T s = 0;
#pragma unroll
                for (int ni = 0; ni < TM; ++ni) s += acc[mi][ni][r];
#pragma unroll
                for (int off = MT / 2; off >= 1; off >>= 1) s += __shfl_xor(s, off, WAVE);
                if (lm == 0) red[wn * BM + wm * 64 + mi * MT + Cfg::row_of(r, lane)] = s;
            }
        __syncthreads();
        if (tid < BM) {
            const int gi = row0 + tid;
            if (gi < g.M) reinterpret_cast<T*>(g.rowpart)[(int64_t)bn * g.M + gi] = red[tid] + red[BM + tid];
        }
    }

    T* __restrict__ C = reinterpret_cast<T*>(g.C);
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
        for (int ni = 0; ni < TM; ++ni)
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                const int gi = row0 + wm * 64 + mi * MT + Cfg::row_of(r, lane);
                const int gj = col0 + wn * 64 + ni * MT + lm;
                if (!EDGE || (gi < g.M && gj < g.N)) C[(int64_t)gi * g.ldc + gj] = acc[mi][ni][r];
            }
}

template <typename T>
static int gemmw_launch(const GemmArgs& a, int transB, int mode, bool edge, hipStream_t st) {
    const dim3 grid(a.tiles_m * a.tiles_n), block(256);
    const size_t lds = gw::lds_bytes<T>();
#define VABFT_GW_CASE(TB, VF, ED)                                                                          \
    if (transB == TB && mode == VF && edge == ED) {                                               \
        auto kern = gemmw_kernel<T, TB, VF, ED>;                                                           \
        static bool attr_set = false;                                                                      \
        if (!attr_set) {                                                                                   \
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                                   \
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)   \
                return VABFT_EDEVICE;                                                                      \
            attr_set = true;                                                                               \
        }                                                                                                  \
        kern<<<grid, block, lds, st>>>(a);                                                                 \
        return hipGetLastError() == hipSuccess ? VABFT_OK : VABFT_EDEVICE;                                 \
    }
    VABFT_GW_CASE(0, 0, false)
    VABFT_GW_CASE(0, 0, true)
    VABFT_GW_CASE(0, 1, false)
    VABFT_GW_CASE(0, 1, true)
    VABFT_GW_CASE(0, 2, false)
    VABFT_GW_CASE(0, 2, true)
    VABFT_GW_CASE(1, 0, false)
    VABFT_GW_CASE(1, 0, true)
    VABFT_GW_CASE(1, 1, false)
    VABFT_GW_CASE(1, 1, true)
    VABFT_GW_CASE(1, 2, false)
    VABFT_GW_CASE(1, 2, true)
#undef VABFT_GW_CASE
    return VABFT_EINVAL;
}

}  // namespace vabft
