// FP32 / FP64 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x2f32, v_mfma_f64_16x16x4f64)
// with the fused V-ABFT epilogue (paper section 2.2 C^{r1'} = C r1 on the accumulator tile;
// section 5.1 injector).  These MFMAs take one element per lane and are 16 passes long, so
// the kernel is matrix-core bound with a simple LDS staging.
//
// Tile 128 x 128 x 16 per workgroup of 4 wavefronts (2 x 2), 64 x 64 per wavefront.
// Result layout per MFMA tile (probed on the device): lane l owns column (l % MT);
//   32x32 (FP32): register r is row 8*(r/4) + 4*(l/32) + r%4
//   16x16 (FP64): register r is row (l/16) + 4*r
// The epilogue goes through LDS: each wavefront parks its tile there, one lane per row adds
// the row in column order (two partial row sums per tile-column, one per wavefront), and C
// leaves in 16-byte pieces contiguous along rows.
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
template <typename T> constexpr int loop_bytes() { return 2 * stage_elems<T>() * (int)sizeof(T); }
template <typename T> constexpr int epi_bytes() { return 4 * 64 * (64 + 16 / (int)sizeof(T)) * (int)sizeof(T); }
template <typename T> constexpr int lds_bytes() { return loop_bytes<T>() > epi_bytes<T>() ? loop_bytes<T>() : epi_bytes<T>(); }
}  // namespace gw

// MODE 0: plain GEMM; 1: fused row-sum check; 2: check plus the fault injector.
template <typename T, int TRANSB, int MODE, bool EDGE>
__global__ __launch_bounds__(256) void gemmw_kernel(const GemmArgs g) {
    using namespace gw;
    constexpr bool VERIFY = MODE >= 1, INJECT = MODE == 2, WSUM = MODE == 2 || MODE == 3;
    constexpr bool CSUM = MODE == 2 || MODE == 4;
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
    if (VERIFY && blockIdx.x == 0 && tid == 0 && g.block_mode) *g.d_nblockflag = 0;
    if (CSUM && blockIdx.x == 0 && tid == 0 && g.d_ncolflag) *g.d_ncolflag = 0;
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

    // ---- epilogue through LDS ------------------------------------------------------------
    // Each wavefront parks its 64 x 64 accumulator tile in a private, padded LDS buffer (the
    // accumulators are only stored, never used as vector operands, so they stay in the
    // accumulation registers through the main loop).  Element (mi, ni, r) is tile row
    // mi*MT + row_of(r, lane), tile column ni*MT + lane%MT.  From there: the injector edits
    // elements in place, lane l sums row l in column order, and rows are copied to C in
    // 16-byte pieces that are contiguous along a row.
    constexpr int PITCH = 64 + 16 / (int)sizeof(T);  // elements; 4 banks of skew per row
    T* tile = smem + wave * (64 * PITCH);
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
        for (int ni = 0; ni < TM; ++ni)
#pragma unroll
            for (int r = 0; r < NR; ++r)
                tile[(mi * MT + Cfg::row_of(r, lane)) * PITCH + ni * MT + lm] = acc[mi][ni][r];
    // LDS operations of one wavefront complete in order; the compiler must keep that order too
    asm volatile("" ::: "memory");
    const int trow0 = row0 + wm * 64, tcol0 = col0 + wn * 64;

    if (INJECT) {
        const InjectArgs& inj = g.inj;
        if (inj.mode == 1) {
            for (int e = 0; e < inj.n_list; ++e) {
                const int fr = inj.d_list[3 * e], fc = inj.d_list[3 * e + 1], fb = inj.d_list[3 * e + 2];
                if (fr < trow0 || fr >= trow0 + 64 || fc < tcol0 || fc >= tcol0 + 64) continue;
                if (fr >= g.M || fc >= g.N || fb < 0 || fb >= acc_bits<T>()) continue;
                if (lane == 0) {
                    T* p = tile + (fr - trow0) * PITCH + (fc - tcol0);
                    const T before = *p, after = flip_bit(before, fb);
                    *p = after;
                    log_fault(inj, fr, fc, fb, (double)before, (double)after);
                }
            }
        } else if (inj.mode == 2) {
            const int gi = trow0 + lane;  // lane l walks row l of the tile
            if (gi < g.M) {
                for (int c = 0; c < 64; ++c) {
                    const int gj = tcol0 + c;
                    if (gj >= g.N) break;
                    const int bit = bernoulli_bit(inj, gi, gj, g.N);
                    if (bit >= 0) {
                        T* p = tile + lane * PITCH + c;
                        const T before = *p, after = flip_bit(before, bit);
                        *p = after;
                        log_fault(inj, gi, gj, bit, (double)before, (double)after);
                    }
                }
            }
        }
        asm volatile("" ::: "memory");
    }

    if (VERIFY) {
        // row sum of the accumulator tile (section 2.2 C^{r1'} = C r1, before any rounding of C):
        // lane l adds the 64 columns of row l; partial index 2*bn + wn
        // (pairwise inside each 16-byte chunk, chunk sums into four rotating accumulators that
        // are folded pairwise at the end: a short error chain instead of 64 sequential adds)
        const T* rowp = tile + lane * PITCH;
        T part[4] = {0, 0, 0, 0};
#pragma unroll
        for (int c = 0; c < 64; c += V) {
            T v[V];
            const raw16 q = *reinterpret_cast<const raw16*>(rowp + c);
            __builtin_memcpy(v, &q, 16);
            T cs;
            if constexpr (V == 2)
                cs = v[0] + v[1];
            else
                cs = (v[0] + v[1]) + (v[2] + v[3]);
            part[(c / V) & 3] += cs;
        }
        const T s = (part[0] + part[1]) + (part[2] + part[3]);
        const int gi = trow0 + lane;
        if (gi < g.M) reinterpret_cast<T*>(g.rowpart)[(int64_t)(2 * bn + wn) * g.M + gi] = s;
        if (WSUM) {
            // position-weighted row sum (section 2.2 C^{r2'} = C r2, r2 = [1..N]): weights 0..63
            // inside the tile, the offset of the tile's first column applied once to s
            T part2[4] = {0, 0, 0, 0};
#pragma unroll
            for (int c = 0; c < 64; c += V) {
                T v[V];
                const raw16 q = *reinterpret_cast<const raw16*>(rowp + c);
                __builtin_memcpy(v, &q, 16);
                T cs = 0;
#pragma unroll
                for (int e = 0; e < V; ++e) cs = fma((T)(c + e), v[e], cs);
                part2[(c / V) & 3] += cs;
            }
            const T s2 = fma((T)(tcol0 + 1), s, (part2[0] + part2[1]) + (part2[2] + part2[3]));
            if (gi < g.M) reinterpret_cast<T*>(g.rowpart2)[(int64_t)(2 * bn + wn) * g.M + gi] = s2;
        }
    }

    if (CSUM) {
        // column sums of the accumulator tile (section 2.2 C^{c1'} = c1 C): lane c adds the 64 rows of
        // column c (consecutive lanes read consecutive LDS words); partial index 2*bm + wm
        T part[4] = {0, 0, 0, 0};
#pragma unroll
        for (int r = 0; r < 64; ++r) part[r & 3] += tile[r * PITCH + lane];
        const int gj = tcol0 + lane;
        if (gj < g.N)
            reinterpret_cast<T*>(g.colpart)[(int64_t)(2 * bm + wm) * g.N + gj] = (part[0] + part[1]) + (part[2] + part[3]);
    }

    T* __restrict__ C = reinterpret_cast<T*>(g.C);
    constexpr int CPRW = 64 / V;  // 16-byte chunks per tile row
#pragma unroll 4
    for (int it = 0; it < 64 * CPRW / 64; ++it) {
        const int idx = lane + 64 * it, r = idx / CPRW, c = (idx % CPRW) * V;
        const raw16 q = *reinterpret_cast<const raw16*>(tile + r * PITCH + c);
        const int gi = trow0 + r, gj = tcol0 + c;
        if (!EDGE) {
            typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_st;
            __builtin_nontemporal_store(__builtin_bit_cast(u32x4_st, q),
                                        reinterpret_cast<u32x4_st*>(C + (int64_t)gi * g.ldc + gj));
        } else if (gi < g.M) {
            if (g.c_vec_ok && gj + V <= g.N) {
                *reinterpret_cast<raw16*>(C + (int64_t)gi * g.ldc + gj) = q;
            } else {
                T v[V];
                __builtin_memcpy(v, &q, 16);
#pragma unroll
                for (int e = 0; e < V; ++e)
                    if (gj + e < g.N) C[(int64_t)gi * g.ldc + gj + e] = v[e];
            }
        }
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
    VABFT_GW_CASE(0, 3, false)
    VABFT_GW_CASE(0, 3, true)
    VABFT_GW_CASE(0, 4, false)
    VABFT_GW_CASE(0, 4, true)
    VABFT_GW_CASE(1, 0, false)
    VABFT_GW_CASE(1, 0, true)
    VABFT_GW_CASE(1, 1, false)
    VABFT_GW_CASE(1, 1, true)
    VABFT_GW_CASE(1, 2, false)
    VABFT_GW_CASE(1, 2, true)
    VABFT_GW_CASE(1, 3, false)
    VABFT_GW_CASE(1, 3, true)
    VABFT_GW_CASE(1, 4, false)
    VABFT_GW_CASE(1, 4, true)
#undef VABFT_GW_CASE
    return VABFT_EINVAL;
}

}  // namespace vabft
