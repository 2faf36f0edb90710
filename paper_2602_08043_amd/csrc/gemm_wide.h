// FP32 / FP64 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x2f32, v_mfma_f64_16x16x4f64)
// with the fused V-ABFT epilogue (paper section 2.2 C^{r1'} = C r1 on the accumulator tile;
// section 6.1 injector).  These MFMAs take one element per lane and are 16 passes long, so
// the kernel is matrix-core bound with a simple LDS staging.
//
// Tile 128 x 128 x 16 per workgroup of 4 wavefronts (2 x 2), 64 x 64 per wavefront (WT = 64); problems with so
// few such tiles that most compute units would idle run 64 x 64 x 16 tiles, 32 x 32 per wavefront (WT = 32).
// Result layout per MFMA tile (probed on the device): lane l owns column (l % MT);
//   32x32 (FP32): register r is row 8*(r/4) + 4*(l/32) + r%4
//   16x16 (FP64): register r is row (l/16) + 4*r
// The epilogue goes through LDS: each wavefront parks its tile there, one lane per row adds
// the row in column order (two partial row sums per tile-column, one per wavefront), and C
// leaves in 16-byte pieces contiguous along rows.
//
// Whole-tile problems (EDGE == false) also finish the check inside this kernel, the way the
// 16-bit kernels do: the partials are published with device-scope stores, the last workgroup
// to finish a tile-row (an arrival ticket per tile-row) folds them in a fixed order, compares
// with the threshold and writes rowsum, E and flags; the last row block writes nflag.  With
// FUSED the A-side of Algorithm 1 rides along: every A tile passes through registers on its
// way to LDS, and tile-column bn folds the k-tiles kt with kt % tiles_n == bn into
// (sum, dot with Be, max, min) per row of A, from which the last workgroup forms the row's
// mean, extrema-variance bound, expected checksum A (B r1) and threshold.
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
constexpr int BK = 16;
constexpr int LDK = BK + 1;  // [row][k] layout, padded
// WT: rows = columns of a wavefront's tile; the workgroup's tile is 2 WT x 2 WT
template <typename T, int WT> constexpr int ldn() { return 2 * WT + 16 / (int)sizeof(T); }  // [k][n] layout, padded, 16 B aligned
template <typename T, int WT> constexpr int a_elems() { return 2 * WT * LDK; }
template <typename T, int WT> constexpr int b_elems() {
    return (2 * WT * LDK) > (BK * ldn<T, WT>()) ? (2 * WT * LDK) : (BK * ldn<T, WT>());
}
template <typename T, int WT> constexpr int stage_elems() { return a_elems<T, WT>() + b_elems<T, WT>(); }
template <typename T, int WT> constexpr int loop_bytes() { return 2 * stage_elems<T, WT>() * (int)sizeof(T); }
template <typename T, int WT> constexpr int epi_bytes() { return 4 * WT * (WT + 16 / (int)sizeof(T)) * (int)sizeof(T); }
// 16 more bytes behind the larger of the two for the "last workgroup of the tile-row" flag
template <typename T, int WT> constexpr int flag_offset() {
    return loop_bytes<T, WT>() > epi_bytes<T, WT>() ? loop_bytes<T, WT>() : epi_bytes<T, WT>();
}
// ... and 12 doubles for the fold of the S1..S3 partials of an encode that deferred it
template <typename T, int WT> constexpr int lds_bytes() { return flag_offset<T, WT>() + 16 + 96; }

// Partials exchanged between workgroups (possibly on different XCDs, each with a private L2) go
// through device-scope relaxed atomic stores and loads, performed at the device's coherence
// point: no cache write-back / invalidate is needed around the ticket.
__device__ __forceinline__ float ld_dev(const float* p) {
    return __builtin_bit_cast(float, __hip_atomic_load(reinterpret_cast<const uint32_t*>(p), __ATOMIC_RELAXED,
                                                        __HIP_MEMORY_SCOPE_AGENT));
}
__device__ __forceinline__ double ld_dev(const double* p) {
    return __builtin_bit_cast(double, __hip_atomic_load(reinterpret_cast<const uint64_t*>(p), __ATOMIC_RELAXED,
                                                         __HIP_MEMORY_SCOPE_AGENT));
}
__device__ __forceinline__ void st_dev(float* p, float v) {
    __hip_atomic_store(reinterpret_cast<uint32_t*>(p), __builtin_bit_cast(uint32_t, v), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev(double* p, double v) {
    __hip_atomic_store(reinterpret_cast<uint64_t*>(p), __builtin_bit_cast(uint64_t, v), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T> __device__ __forceinline__ constexpr T lowest();
template <> __device__ __forceinline__ constexpr float lowest<float>() { return -3.402823466e+38f; }
template <> __device__ __forceinline__ constexpr double lowest<double>() { return -1.7976931348623157e+308; }
}  // namespace gw

// MODE 0: plain GEMM; 1: fused row-sum check; 2: check, fault injector, weighted row sums and
// column sums; 3: check and weighted row sums; 4: check and column sums.
// FUSED (whole tiles only): also the A-side statistics, expected checksum and thresholds.
template <typename T, int WT, int TRANSB, int MODE, bool EDGE, bool FUSED>
__global__ __launch_bounds__(256) void gemmw_kernel(const GemmArgs g) {
    using namespace gw;
    constexpr int BM = 2 * WT, BN = 2 * WT;
    constexpr bool VERIFY = MODE >= 1, INJECT = MODE == 2, WSUM = MODE == 2 || MODE == 3;
    constexpr bool CSUM = MODE == 2 || MODE == 4;
    static_assert(!FUSED || (VERIFY && !EDGE), "fused statistics belong to the whole-tile verified kernel");
    using Cfg = WideCfg<T>;
    using accv_t = typename Cfg::accv_t;
    constexpr int MT = Cfg::MT, KM = Cfg::KM, NR = Cfg::NR, V = Cfg::V;
    constexpr int TM = WT / MT;  // MFMA tiles per wavefront in each direction
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    T* smem = reinterpret_cast<T*>(smem_raw);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int lm = lane % MT, lk = lane / MT;
    int bm, bn;
    tile_of_block(blockIdx.x, g.tiles_m, g.tiles_n, bm, bn);
    // a compare kernel that follows this one counts into nflag; the in-kernel compare writes it itself
    if (VERIFY && (EDGE || g.block_mode) && blockIdx.x == 0 && tid == 0) *g.d_nflag = 0;
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
    // PD k-tiles are in flight from global memory at a time, each in a register slot of its own.  The small tile
    // serves problems of a few dozen workgroups, whose time is a chain of global-memory latencies, one per k-tile
    // with a single slot (FP32 256^3: 16 k-tiles of 16); four slots take three of every four out of the chain.
    constexpr int PD = WT == 32 ? 4 : 1;
    T ra[PD][NCH_A][V], rb[PD][NCH_B][V];

    // one 16-byte chunk; whole-tile problems need no guards
    auto load_chunk = [&](const T* base, int r, int nr, int c, int nc, int64_t ld, int vec_ok, T (&out)[V]) {
        if (!EDGE) {
            const raw16 v = ld16(base + (int64_t)r * ld + c);
            __builtin_memcpy(out, &v, 16);
        } else {
            guarded_chunk_wide<T, V>(base, r, nr, c, nc, ld, vec_ok, out);
        }
    };
    // (the register slot is a compile-time constant everywhere: a runtime index would put the slots in scratch)
    auto load_tiles = [&](int kt, auto slot_c) {
        constexpr int SL = decltype(slot_c)::value;
        const int kbase = kt * BK;
#pragma unroll
        for (int p = 0; p < NCH_A; ++p) {
            const int id = tid + 256 * p, r = id / CPR, c = id % CPR;
            load_chunk(A, row0 + r, g.M, kbase + c * V, g.K, g.lda, g.a_vec_ok, ra[SL][p]);
        }
        if (TRANSB) {
#pragma unroll
            for (int p = 0; p < NCH_B; ++p) {
                const int id = tid + 256 * p, r = id / CPR, c = id % CPR;
                load_chunk(B, col0 + r, g.N, kbase + c * V, g.K, g.ldb, g.b_vec_ok, rb[SL][p]);
            }
        } else {
#pragma unroll
            for (int p = 0; p < NCH_B; ++p) {
                const int id = tid + 256 * p, kr = id / CPK, c = id % CPK;
                load_chunk(B, kbase + kr, g.K, col0 + c * V, g.N, g.ldb, g.b_vec_ok, rb[SL][p]);
            }
        }
    };

    auto store_tiles = [&](int s, auto slot_c) {
        constexpr int SL = decltype(slot_c)::value;
        T* As = smem + s * stage_elems<T, WT>();
        T* Bs = As + a_elems<T, WT>();
#pragma unroll
        for (int p = 0; p < NCH_A; ++p) {
            const int id = tid + 256 * p, r = id / CPR, c = id % CPR;
#pragma unroll
            for (int e = 0; e < V; ++e) As[r * LDK + c * V + e] = ra[SL][p][e];
        }
        if (TRANSB) {
#pragma unroll
            for (int p = 0; p < NCH_B; ++p) {
                const int id = tid + 256 * p, r = id / CPR, c = id % CPR;
#pragma unroll
                for (int e = 0; e < V; ++e) Bs[r * LDK + c * V + e] = rb[SL][p][e];
            }
        } else {
#pragma unroll
            for (int p = 0; p < NCH_B; ++p) {
                const int id = tid + 256 * p, kr = id / CPK, c = id % CPK;
#pragma unroll
                for (int e = 0; e < V; ++e) Bs[kr * ldn<T, WT>() + c * V + e] = rb[SL][p][e];
            }
        }
    };

    // ---- fused A-side statistics (FUSED) ------------------------------------------------
    // Chunk p of this thread is V consecutive k of row (tid + 256 p) / CPR of the tile; the
    // chunk's position in the k-tile, tid % CPR, is the same for every p, so one 16-byte
    // piece of Be serves all of them.  st[p] = (sum, dot with Be, max, min).
    T st[NCH_A][4];
    raw16 be_raw[PD];
#pragma unroll
    for (int q = 0; q < PD; ++q) be_raw[q] = raw16{{0u, 0u, 0u, 0u}};
#pragma unroll
    for (int p = 0; p < NCH_A; ++p) {
        st[p][0] = 0;
        st[p][1] = 0;
        st[p][2] = lowest<T>();
        st[p][3] = -lowest<T>();
    }
    auto load_be = [&](int kt, auto slot_c) {
        be_raw[decltype(slot_c)::value] = ld16(reinterpret_cast<const T*>(g.Be) + kt * BK + (tid % CPR) * V);
    };
    auto fold_stats = [&](auto slot_c) {
        constexpr int SL = decltype(slot_c)::value;
        T bev[V];
        __builtin_memcpy(bev, &be_raw[SL], 16);
        // the chunk's sum and dot product are formed pairwise and then added to the running values, so the
        // sequential rounding chain of a thread is one add per folded k-tile, not one per element
#pragma unroll
        for (int p = 0; p < NCH_A; ++p) {
            T cs, cd;
            if constexpr (V == 2) {
                cs = ra[SL][p][0] + ra[SL][p][1];
                cd = fma(ra[SL][p][1], bev[1], ra[SL][p][0] * bev[0]);
            } else {
                cs = (ra[SL][p][0] + ra[SL][p][1]) + (ra[SL][p][2] + ra[SL][p][3]);
                cd = fma(ra[SL][p][1], bev[1], ra[SL][p][0] * bev[0]) + fma(ra[SL][p][3], bev[3], ra[SL][p][2] * bev[2]);
            }
            st[p][0] += cs;
            st[p][1] += cd;
#pragma unroll
            for (int e = 0; e < V; ++e) {
                st[p][2] = fmax(st[p][2], ra[SL][p][e]);
                st[p][3] = fmin(st[p][3], ra[SL][p][e]);
            }
        }
    };

    auto compute = [&](int s) {
        const T* As = smem + s * stage_elems<T, WT>();
        const T* Bs = As + a_elems<T, WT>();
#pragma unroll
        for (int ks = 0; ks < BK / KM; ++ks) {
            T af[TM], bf[TM];
            const int k = ks * KM + lk;
#pragma unroll
            for (int mi = 0; mi < TM; ++mi) af[mi] = As[(wm * WT + mi * MT + lm) * LDK + k];
#pragma unroll
            for (int ni = 0; ni < TM; ++ni)
                bf[ni] = TRANSB ? Bs[(wn * WT + ni * MT + lm) * LDK + k] : Bs[k * ldn<T, WT>() + wn * WT + ni * MT + lm];
#pragma unroll
            for (int mi = 0; mi < TM; ++mi)
#pragma unroll
                for (int ni = 0; ni < TM; ++ni) acc[mi][ni] = Cfg::mfma(af[mi], bf[ni], acc[mi][ni]);
        }
    };

    const int nk = (g.K + BK - 1) / BK;
    int next_fold = bn;  // FUSED: the next k-tile this tile-column folds into the statistics
    using SL0 = std::integral_constant<int, 0>;
    // k-tile t travels in register slot t % PD: the first PD tiles go out at once
    static_for<0, PD>([&](auto q_c) {
        constexpr int q = decltype(q_c)::value;
        if (q < nk) {
            // the 16 bytes of Be are fetched for every k-tile, in front of the tile's own loads: loads
            // return in order, so the waits of store_tiles cover them, and a conditional load here
            // would make the compiler drain the whole load queue in front of it
            if (FUSED) load_be(q, q_c);
            load_tiles(q, q_c);
        }
    });
    if (FUSED && !g.S)
        fold_s_partials_to_lds(g.s_partial, g.s_nparts, tid, reinterpret_cast<double*>(smem_raw + flag_offset<T, WT>() + 16));
    store_tiles(0, SL0{});
    if (FUSED && next_fold == 0) {
        fold_stats(SL0{});
        next_fold += g.tiles_n;
    }
    __syncthreads();
    for (int kt0 = 0; kt0 < nk; kt0 += PD) {
        static_for<0, PD>([&](auto j_c) {
            constexpr int j = decltype(j_c)::value;
            using NEXT = std::integral_constant<int, (j + 1) % PD>;
            const int kt = kt0 + j;
            if (kt < nk) {  // workgroup-uniform
                const bool more = kt + 1 < nk;
                const bool fold = FUSED && more && kt + 1 == next_fold;  // workgroup-uniform
                // slot j held k-tile kt, which is in LDS by now: it takes k-tile kt + PD
                if (kt + PD < nk) {
                    if (FUSED) load_be(kt + PD, j_c);
                    load_tiles(kt + PD, j_c);
                }
                compute(kt & 1);
                if (more) store_tiles((kt + 1) & 1, NEXT{});
                if (fold) {
                    fold_stats(NEXT{});
                    next_fold += g.tiles_n;
                }
                __syncthreads();
            }
        });
    }

    if constexpr (FUSED) {
        // Publish this tile-column's A statistics while the operand stages of LDS are free: the
        // CPR threads that share a row of the A tile are neighbouring lanes; after their
        // exchange the row's four values pass through LDS so that the device-scope stores are
        // contiguous along the rows (64 consecutive words per wavefront and store).
        T* sred = smem;  // [4][BM]
#pragma unroll
        for (int p = 0; p < NCH_A; ++p) {
#pragma unroll
            for (int d = 1; d < CPR; d <<= 1) {
                st[p][0] += __shfl_xor(st[p][0], d, 64);
                st[p][1] += __shfl_xor(st[p][1], d, 64);
                st[p][2] = fmax(st[p][2], __shfl_xor(st[p][2], d, 64));
                st[p][3] = fmin(st[p][3], __shfl_xor(st[p][3], d, 64));
            }
            if (tid % CPR == 0) {
                const int r = (tid + 256 * p) / CPR;
#pragma unroll
                for (int q = 0; q < 4; ++q) sred[q * BM + r] = st[p][q];
            }
        }
        __syncthreads();
        T* ap = reinterpret_cast<T*>(g.apart) + (int64_t)bn * 4 * g.M + row0;
        constexpr int QPT = 4 * BM / 256;  // values per thread: 256 threads publish 4 x BM values
#pragma unroll
        for (int h = 0; h < QPT; ++h) {
            const int q = QPT * (tid / BM) + h, r = tid % BM;
            st_dev(ap + q * (int64_t)g.M + r, sred[q * BM + r]);
        }
        __syncthreads();  // the accumulator tiles are parked over this area next
    }

    // ---- epilogue through LDS ------------------------------------------------------------
    // Each wavefront parks its WT x WT accumulator tile in a private, padded LDS buffer (the
    // accumulators are only stored, never used as vector operands, so they stay in the
    // accumulation registers through the main loop).  Element (mi, ni, r) is tile row
    // mi*MT + row_of(r, lane), tile column ni*MT + lane%MT.  From there: the injector edits
    // elements in place, lane l sums row l in column order, and rows are copied to C in
    // 16-byte pieces that are contiguous along a row.
    constexpr int PITCH = WT + 16 / (int)sizeof(T);  // elements; 4 banks of skew per row
    T* tile = smem + wave * (WT * PITCH);
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
        for (int ni = 0; ni < TM; ++ni)
#pragma unroll
            for (int r = 0; r < NR; ++r)
                tile[(mi * MT + Cfg::row_of(r, lane)) * PITCH + ni * MT + lm] = acc[mi][ni][r];
    // LDS operations of one wavefront complete in order; the compiler must keep that order too
    asm volatile("" ::: "memory");
    const int trow0 = row0 + wm * WT, tcol0 = col0 + wn * WT;

    if (INJECT) {
        const InjectArgs& inj = g.inj;
        if (inj.mode == 1) {
            for (int e = 0; e < inj.n_list; ++e) {
                const int fr = inj.d_list[3 * e], fc = inj.d_list[3 * e + 1], fb = inj.d_list[3 * e + 2];
                if (fr < trow0 || fr >= trow0 + WT || fc < tcol0 || fc >= tcol0 + WT) continue;
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
            if (lane < WT && gi < g.M) {
                for (int c = 0; c < WT; ++c) {
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
        // lane l < WT adds the WT columns of row l; partial index 2*bn + wn
        // (pairwise inside each 16-byte chunk, chunk sums into four rotating accumulators that
        // are folded pairwise at the end: a short error chain instead of WT sequential adds)
        const bool has_row = WT == 64 || lane < WT;
        const T* rowp = tile + (has_row ? lane : 0) * PITCH;
        T part[4] = {0, 0, 0, 0};
#pragma unroll
        for (int c = 0; c < WT; c += V) {
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
        if (!EDGE) {
            if (has_row) st_dev(reinterpret_cast<T*>(g.rowpart) + (int64_t)(2 * bn + wn) * g.M + gi, s);
        } else if (has_row && gi < g.M) {
            reinterpret_cast<T*>(g.rowpart)[(int64_t)(2 * bn + wn) * g.M + gi] = s;
        }
        if (WSUM) {
            // position-weighted row sum (section 2.2 C^{r2'} = C r2, r2 = [1..N]): weights 0..WT-1
            // inside the tile, the offset of the tile's first column applied once to s
            T part2[4] = {0, 0, 0, 0};
#pragma unroll
            for (int c = 0; c < WT; c += V) {
                T v[V];
                const raw16 q = *reinterpret_cast<const raw16*>(rowp + c);
                __builtin_memcpy(v, &q, 16);
                T cs = 0;
#pragma unroll
                for (int e = 0; e < V; ++e) cs = fma((T)(c + e), v[e], cs);
                part2[(c / V) & 3] += cs;
            }
            const T s2 = fma((T)(tcol0 + 1), s, (part2[0] + part2[1]) + (part2[2] + part2[3]));
            if (!EDGE) {
                if (has_row) st_dev(reinterpret_cast<T*>(g.rowpart2) + (int64_t)(2 * bn + wn) * g.M + gi, s2);
            } else if (has_row && gi < g.M) {
                reinterpret_cast<T*>(g.rowpart2)[(int64_t)(2 * bn + wn) * g.M + gi] = s2;
            }
        }
    }

    if (CSUM) {
        // column sums of the accumulator tile (section 2.2 C^{c1'} = c1 C): lane c < WT adds the WT rows of
        // column c (consecutive lanes read consecutive LDS words); partial index 2*bm + wm
        const bool has_col = WT == 64 || lane < WT;
        T part[4] = {0, 0, 0, 0};
#pragma unroll
        for (int r = 0; r < WT; ++r) part[r & 3] += tile[r * PITCH + (has_col ? lane : 0)];
        const int gj = tcol0 + lane;
        if (has_col && gj < g.N)
            reinterpret_cast<T*>(g.colpart)[(int64_t)(2 * bm + wm) * g.N + gj] = (part[0] + part[1]) + (part[2] + part[3]);
    }

    if constexpr (VERIFY && !EDGE) {
        T* const rowpart = reinterpret_cast<T*>(g.rowpart);
        T* const rowpart2 = reinterpret_cast<T*>(g.rowpart2);
        T* const apart = reinterpret_cast<T*>(g.apart);
        // block-wise check: the partials are all this kernel leaves; a later kernel compares them per block
        if (!g.block_mode) {
            // Every thread's partials are performed (vmcnt(0)) before the workgroup takes this
            // tile-row's arrival ticket; the check runs before the store of C because behind that
            // burst of stores each of these round trips would cost several microseconds.
            int* s_last = reinterpret_cast<int*>(smem_raw + flag_offset<T, WT>());
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
            if (tid == 0) *s_last = (atomicAdd(&g.tickets[bm], 1) == g.tiles_n - 1);
            __syncthreads();
            if (*s_last) {
                // fold the partials in tile order (loads issued in batches so their latencies
                // overlap; absent entries count as the neutral element)
                const bool act = tid < BM;
                const int gi = row0 + (act ? tid : 0);
                const int np = 2 * g.tiles_n;
                // every batch is folded as a tree and lands in one of four rotating accumulators, themselves
                // folded pairwise at the end: the rounding chain of a sum is log-like in the number of partials
                T rs4[4] = {0, 0, 0, 0}, rs24[4] = {0, 0, 0, 0}, sum4[4] = {0, 0, 0, 0}, dot4[4] = {0, 0, 0, 0};
                T mx = lowest<T>(), mn = -lowest<T>();
                if (act) {
                    for (int t0 = 0; t0 < np; t0 += 16) {
                        T v[16], v2[16];
#pragma unroll
                        for (int j = 0; j < 16; ++j) {
                            const int t = t0 + j < np ? t0 + j : np - 1;
                            v[j] = ld_dev(rowpart + (int64_t)t * g.M + gi);
                            if (WSUM) v2[j] = ld_dev(rowpart2 + (int64_t)t * g.M + gi);
                        }
#pragma unroll
                        for (int j = 0; j < 16; ++j)
                            if (!(t0 + j < np)) {
                                v[j] = 0;
                                if (WSUM) v2[j] = 0;
                            }
                        T q[4], q2[4];
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            q[j] = (v[4 * j] + v[4 * j + 1]) + (v[4 * j + 2] + v[4 * j + 3]);
                            if (WSUM) q2[j] = (v2[4 * j] + v2[4 * j + 1]) + (v2[4 * j + 2] + v2[4 * j + 3]);
                        }
                        const T b = (q[0] + q[1]) + (q[2] + q[3]), b2 = WSUM ? (q2[0] + q2[1]) + (q2[2] + q2[3]) : (T)0;
                        const int slot = (t0 >> 4) & 3;  // x + 0 is exact: the other three stay as they are
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            rs4[k] += slot == k ? b : (T)0;
                            if (WSUM) rs24[k] += slot == k ? b2 : (T)0;
                        }
                    }
                    if (FUSED) {
                        for (int t0 = 0; t0 < g.tiles_n; t0 += 8) {
                            T v[8][4];
#pragma unroll
                            for (int j = 0; j < 8; ++j) {
                                const int t = t0 + j < g.tiles_n ? t0 + j : g.tiles_n - 1;
                                const T* ap = apart + (int64_t)t * 4 * g.M + gi;
#pragma unroll
                                for (int q = 0; q < 4; ++q) v[j][q] = ld_dev(ap + q * (int64_t)g.M);
                            }
#pragma unroll
                            for (int j = 0; j < 8; ++j)
                                if (!(t0 + j < g.tiles_n)) {
                                    v[j][0] = 0;
                                    v[j][1] = 0;
                                    v[j][2] = lowest<T>();
                                    v[j][3] = -lowest<T>();
                                }
                            const T bs = ((v[0][0] + v[1][0]) + (v[2][0] + v[3][0])) +
                                         ((v[4][0] + v[5][0]) + (v[6][0] + v[7][0]));
                            const T bd = ((v[0][1] + v[1][1]) + (v[2][1] + v[3][1])) +
                                         ((v[4][1] + v[5][1]) + (v[6][1] + v[7][1]));
                            const int slot = (t0 >> 3) & 3;
#pragma unroll
                            for (int k = 0; k < 4; ++k) {
                                sum4[k] += slot == k ? bs : (T)0;
                                dot4[k] += slot == k ? bd : (T)0;
                            }
#pragma unroll
                            for (int j = 0; j < 8; j += 4) {
                                mx = fmax(mx, fmax(fmax(v[j][2], v[j + 1][2]), fmax(v[j + 2][2], v[j + 3][2])));
                                mn = fmin(mn, fmin(fmin(v[j][3], v[j + 1][3]), fmin(v[j + 2][3], v[j + 3][3])));
                            }
                        }
                    }
                }
                const T rs = (rs4[0] + rs4[1]) + (rs4[2] + rs4[3]), rs2 = (rs24[0] + rs24[1]) + (rs24[2] + rs24[3]);
                const T sum = (sum4[0] + sum4[1]) + (sum4[2] + sum4[3]), dot = (dot4[0] + dot4[1]) + (dot4[2] + dot4[3]);
                int f = 0;
                if (act) {
                    T expv, thr;
                    if (FUSED) {
                        // Algorithm 1 for this row of A, in double precision
                        const double mu = (double)sum / (double)g.K;
                        double var = ((double)mx - mu) * (mu - (double)mn);
                        var = var > 0 ? var : 0;
                        const double* s_red = reinterpret_cast<const double*>(smem_raw + flag_offset<T, WT>() + 16);
                        const double S1 = g.S ? g.S[0] : folded_s(s_red, 0), S2 = g.S ? g.S[1] : folded_s(s_red, 1),
                                     S3 = g.S ? g.S[2] : folded_s(s_red, 2), dN = (double)g.N;
                        const double t_det = dN * fabs(mu) * S1;
                        const double t_var23 = g.c_sigma * sqrt(dN * mu * mu * S2 + dN * dN * var * S3);
                        const double t_var4 = g.c_sigma * sqrt(dN) * sqrt(var) * sqrt(S2);
                        expv = dot;
                        thr = (T)(g.e_max * (t_det + t_var23 + t_var4));
                        T* astat = reinterpret_cast<T*>(g.astat);
                        astat[3 * (int64_t)gi + 0] = mx;
                        astat[3 * (int64_t)gi + 1] = mn;
                        astat[3 * (int64_t)gi + 2] = (T)mu;
                        reinterpret_cast<T*>(const_cast<void*>(g.expected))[gi] = expv;
                        reinterpret_cast<T*>(const_cast<void*>(g.T))[gi] = thr;
                    } else {
                        expv = reinterpret_cast<const T*>(g.expected)[gi];
                        thr = reinterpret_cast<const T*>(g.T)[gi];
                    }
                    const T e = expv - rs;
                    f = !(fabs(e) <= thr);
                    reinterpret_cast<T*>(g.rowsum)[gi] = rs;
                    if (WSUM && g.rowsum2) reinterpret_cast<T*>(g.rowsum2)[gi] = rs2;
                    reinterpret_cast<T*>(g.E)[gi] = e;
                    g.flags[gi] = f;
                }
                const int cnt = __syncthreads_count(f);
                if (tid == 0) {
                    // this tile-row is done: reset its ticket, then one 64-bit atomic both counts the
                    // finished row blocks (high word) and accumulates the flagged rows (low word);
                    // whoever completes the count publishes nflag and leaves the counter zero
                    __hip_atomic_store(&g.tickets[bm], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    unsigned long long* done = reinterpret_cast<unsigned long long*>(g.tickets + ((g.tiles_m + 1) & ~1));
                    const unsigned long long old = atomicAdd(done, (1ull << 32) | (unsigned long long)(unsigned)cnt);
                    if ((int)(old >> 32) == g.tiles_m - 1) {
                        *g.d_nflag = (int)(unsigned)(old & 0xffffffffull) + cnt;
                        __hip_atomic_store(done, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                }
            }
        }
    }

    T* __restrict__ C = reinterpret_cast<T*>(g.C);
    constexpr int CPRW = WT / V;  // 16-byte chunks per tile row
#pragma unroll 4
    for (int it = 0; it < WT * CPRW / 64; ++it) {
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

// WT: 64 (128 x 128 tiles) or 32 (64 x 64 tiles); a.tiles_m / a.tiles_n count tiles of that size
template <typename T, int WT>
static int gemmw_launch_wt(const GemmArgs& a, int transB, int mode, bool edge, hipStream_t st) {
    const bool fused = a.fused_stats != 0;
    const dim3 grid(a.tiles_m * a.tiles_n), block(256);
    const size_t lds = gw::lds_bytes<T, WT>();
#define VABFT_GW_CASE(TB, VF, ED, FU)                                                                      \
    if (transB == TB && mode == VF && edge == ED && fused == FU) {                                         \
        auto kern = gemmw_kernel<T, WT, TB, VF, ED, FU>;                                                   \
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
    VABFT_GW_CASE(0, 0, false, false)
    VABFT_GW_CASE(0, 0, true, false)
    VABFT_GW_CASE(0, 1, false, false)
    VABFT_GW_CASE(0, 1, true, false)
    VABFT_GW_CASE(0, 2, false, false)
    VABFT_GW_CASE(0, 2, true, false)
    VABFT_GW_CASE(0, 3, false, false)
    VABFT_GW_CASE(0, 3, true, false)
    VABFT_GW_CASE(0, 4, false, false)
    VABFT_GW_CASE(0, 4, true, false)
    VABFT_GW_CASE(1, 0, false, false)
    VABFT_GW_CASE(1, 0, true, false)
    VABFT_GW_CASE(1, 1, false, false)
    VABFT_GW_CASE(1, 1, true, false)
    VABFT_GW_CASE(1, 2, false, false)
    VABFT_GW_CASE(1, 2, true, false)
    VABFT_GW_CASE(1, 3, false, false)
    VABFT_GW_CASE(1, 3, true, false)
    VABFT_GW_CASE(1, 4, false, false)
    VABFT_GW_CASE(1, 4, true, false)
    // with the A-side statistics: the check alone, and the injector runs
    VABFT_GW_CASE(0, 1, false, true)
    VABFT_GW_CASE(0, 2, false, true)
    VABFT_GW_CASE(1, 1, false, true)
    VABFT_GW_CASE(1, 2, false, true)
#undef VABFT_GW_CASE
    return VABFT_EINVAL;
}

template <typename T>
static int gemmw_launch(const GemmArgs& a, int transB, int mode, bool edge, int wave_tile, hipStream_t st) {
    return wave_tile == 32 ? gemmw_launch_wt<T, 32>(a, transB, mode, edge, st)
                           : gemmw_launch_wt<T, 64>(a, transB, mode, edge, st);
}

}  // namespace vabft
