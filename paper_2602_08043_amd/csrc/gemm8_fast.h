// FP8 (OCP E4M3 or E5M2) GEMM with FP32 accumulation and FP16 output on the gfx950 matrix cores
// (v_mfma_f32_32x32x64_f8f6f4; the instruction's format selectors choose between the two encodings, and
// the conversion instruction of the fused statistics follows), for whole-tile problems with B stored N x K:
// M % 256 == 0, N % 256 == 0, K % 256 == 0, 16-byte aligned rows.
//
// The paper treats FP8 as one more input precision of the same accumulation strategy ("FP8 inputs ->
// FP32 accumulation -> FP16 output", section 3.6): the fused check works on the FP32 accumulators exactly
// as for BF16 / FP16, so this kernel is the 16-bit whole-tile kernel with one-byte elements:
//   * the same 256 x 256 tile per workgroup of 4 wavefronts, 128 x 128 per wavefront, 4 x 4 MFMA tiles;
//   * the same LDS image per stage, [256 rows][128 bytes] per operand with chunk c of row r at position
//     c ^ ((r >> 1) & 7), filled by global_load_lds_dwordx4; a row now holds 128 k-values, i.e. two
//     k-steps of 64;
//   * a fragment is 32 bytes per lane (two ds_read_b128): lane l of an MFMA operand holds row l % 32 and
//     the half l / 32 of the k-step's 64 bytes.  Which byte the hardware takes for which k inside an
//     operand does not matter: A and B fragments are cut the same way, so every product pairs equal k;
//   * per k-step 16 MFMAs of 64 cycles; each slot also issues one fragment read of the next k-step and,
//     in the first k-step after the barrier, one of the 16 loads of the next tile;
//   * the epilogue (row sums before quantisation, compare-and-flag, injector, weighted and column sums,
//     FP16 store) is the 16-bit kernel's;
//   * FUSED: the A-side of Algorithm 1 as in the 16-bit kernel.  Tile-column bn folds the units (two k-tiles,
//     256 k) u with u % tiles_n == bn; a lane's 32 fragment bytes are consecutive k of its row, wavefront wn
//     takes 16 of them, four per slot (convert, sum, FMA with Be, max, min); the Be values of a k-step are read
//     from the LDS cache when the k-step starts.
#pragma once
#include "gemm_tile32.h"

namespace vabft {

typedef __attribute__((ext_vector_type(8))) int i32x8_t;

namespace g8f {
using namespace g16f;
constexpr int BKB = 128;  // bytes (= k-values) per tile row
struct alignas(16) raw32 {
    raw16 lo, hi;
};
// FMT: 0 = E4M3, 1 = E5M2 (the instruction's cbsz / blgp format codes), both operands alike; no block scaling
template <int FMT> __device__ __forceinline__ f32x16_t mfma_f8(const raw32& a, const raw32& b, f32x16_t c) {
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(__builtin_bit_cast(i32x8_t, a), __builtin_bit_cast(i32x8_t, b),
                                                           c, FMT, FMT, 0, 0, 0, 0);
}
template <int FMT, int BYTE> __device__ __forceinline__ float cvt_f8(int w) {
    if constexpr (FMT == 0) return __builtin_amdgcn_cvt_f32_fp8(w, BYTE);
    else return __builtin_amdgcn_cvt_f32_bf8(w, BYTE);
}
}  // namespace g8f

template <int FMT, int MODE, bool FUSED>
__global__ __launch_bounds__(256) void gemm8_fast_kernel(const GemmArgs g) {
    using namespace g8f;
    constexpr bool CSUM = MODE == 2 || MODE == 4;
    static_assert(!FUSED || MODE == 1 || MODE == 2, "fused statistics belong to the verified kernel");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    lds_u8* const lds = (lds_u8*)smem;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lh = lane >> 5;
    int bm, bn;
    tile_of_block(blockIdx.x, g.tiles_m, g.tiles_n, bm, bn);
    if (CSUM && blockIdx.x == 0 && tid == 0 && g.d_ncolflag) *g.d_ncolflag = 0;
    if ((MODE == 5 || MODE == 2) && blockIdx.x == 0 && tid == 0 && g.block_mode) {
        *g.d_nflag = 0;
        *g.d_nblockflag = 0;
    }
    const int row0 = bm * BM, col0 = bn * BN;
    const unsigned char* __restrict__ A = reinterpret_cast<const unsigned char*>(g.A);
    const unsigned char* __restrict__ B = reinterpret_cast<const unsigned char*>(g.B);

    f32x16_t acc[4][4];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

    // ---- global -> LDS: each wavefront issues 8 + 8 loads of 1 KiB per k-tile (64 rows x 128 bytes of A,
    // 64 rows x 128 bytes of B).  Load i covers rows wave*64 + i*8 .. +7; lane l sits at row l/8, chunk
    // position l%8, and fetches chunk (l%8) ^ ((row>>1)&7) with (row>>1)&7 = 4*(i&1) + l/16.
    const uint32_t rk_e = ((lane & 7) ^ (lane >> 4)) << 4, rk_o = ((lane & 7) ^ (lane >> 4) ^ 4) << 4;
    const unsigned char* const a_base = A + (int64_t)(row0 + wave * 64) * g.lda;
    const uint32_t a_lane_e = (uint32_t)(lane >> 3) * (uint32_t)g.lda + rk_e;
    const uint32_t a_lane_o = (uint32_t)(lane >> 3) * (uint32_t)g.lda + rk_o;
    const int64_t a_step = 8 * g.lda;
    const unsigned char* const b_base = B + (int64_t)(col0 + wave * 64) * g.ldb;
    const uint32_t b_lane_e = (uint32_t)(lane >> 3) * (uint32_t)g.ldb + rk_e;
    const uint32_t b_lane_o = (uint32_t)(lane >> 3) * (uint32_t)g.ldb + rk_o;
    const int64_t b_step = 8 * g.ldb;
    lds_u8* const a_dst = lds + wave * (64 * 128);
    lds_u8* const b_dst = lds + A_BYTES + wave * (64 * 128);

    auto issue_load = [&](auto ls_c, auto l_c, const unsigned char* ap, const unsigned char* bp) {
        constexpr int LS = decltype(ls_c)::value, l = decltype(l_c)::value;
        if constexpr (l < 8)
            g2l16(ap + l * a_step + ((l & 1) ? a_lane_o : a_lane_e), a_dst + LS * STAGE + l * 1024);
        else
            g2l16(bp + (l - 8) * b_step + ((l & 1) ? b_lane_o : b_lane_e), b_dst + LS * STAGE + (l - 8) * 1024);
    };

    // ---- LDS -> fragments: k-step q (0, 1) of a stage is the 64 bytes 64q .. 64q+63 of every row; lane half
    // lh takes chunks 4q + 2lh and 4q + 2lh + 1
    const int f_swz = (l32 >> 1) & 7;
    lds_u8* a_rd[2][2][2];  // [stage][k-step][chunk of the pair]
    lds_u8* b_rd[2][2][2];
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const int pos = ((4 * q + 2 * lh + c) ^ f_swz) << 4;
                a_rd[st][q][c] = lds + st * STAGE + (wm * 128 + l32) * 128 + pos;
                b_rd[st][q][c] = lds + st * STAGE + A_BYTES + (wn * 128 + l32) * 128 + pos;
            }

    // read operation op (0..15) of k-step KS of stage S: ops 0..7 fill af[op/2] (lo, hi), 8..15 bf
    auto frag_op = [&](auto s_c, auto ks_c, auto op_c, raw32 (&af)[4], raw32 (&bf)[4]) {
        constexpr int S = decltype(s_c)::value, KS = decltype(ks_c)::value, op = decltype(op_c)::value;
        constexpr int t = (op & 7) >> 1, c = op & 1;
        if constexpr (op < 8) {
            const raw16 v = lds_read16(a_rd[S][KS][c] + t * 4096);
            if constexpr (c == 0) af[t].lo = v; else af[t].hi = v;
        } else {
            const raw16 v = lds_read16(b_rd[S][KS][c] + t * 4096);
            if constexpr (c == 0) bf[t].lo = v; else bf[t].hi = v;
        }
    };

    // ---- fused A-side statistics (FUSED) ----------------------------------------------------------------
    // st[mi] = (sum, dot with Be, max, min) of rows wm*128 + mi*32 + l32 over the k this lane folds.  A unit is
    // two k-tiles; its four k-steps, in the order the bodies multiply them, cover k = 256u - 64 + 64 s .. + 63
    // (s = 0..3; the first belongs to the previous tile because fragments run one k-step ahead).  The lane's
    // 16 bytes of a k-step are k = 256u - 64 + 64 s + 32 lh + 16 wn + 0..15; bev holds their Be values.
    float st[4][4];
    f32x4_t bev[4];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
        st[mi][0] = 0.f;
        st[mi][1] = 0.f;
        st[mi][2] = -3.402823466e+38f;
        st[mi][3] = 3.402823466e+38f;
    }
    // Be cache: slot j (256 floats) holds the unit u = bn + j * tiles_n
    auto load_bev = [&](int j, auto sidx_c) {
        constexpr int SIDX = decltype(sidx_c)::value;
        const float* p = reinterpret_cast<const float*>(smem + BE_CACHE_OFFSET) + j * 256 + 64 * SIDX + 32 * lh + 16 * wn;
#pragma unroll
        for (int d = 0; d < 4; ++d) bev[d] = *reinterpret_cast<const f32x4_t*>(p + 4 * d);
    };
    // slot (mi, d) folds dword d of this wavefront's half of fragment mi: four consecutive k
    auto stats_slot = [&](const raw32 (&af)[4], auto slot_c, auto sidx_c, bool skip) {
        constexpr int slot = decltype(slot_c)::value, SIDX = decltype(sidx_c)::value;
        constexpr int mi = slot >> 2, d = slot & 3;
        const uint32_t lo = af[mi].lo.w[d], hi = af[mi].hi.w[d];
        const int w = (int)(wn ? hi : lo);
        const float x0 = cvt_f8<FMT, 0>(w), x1 = cvt_f8<FMT, 1>(w), x2 = cvt_f8<FMT, 2>(w), x3 = cvt_f8<FMT, 3>(w);
        st[mi][0] += (x0 + x1) + (x2 + x3);
        st[mi][1] += fmaf(x1, bev[d][1], x0 * bev[d][0]) + fmaf(x3, bev[d][3], x2 * bev[d][2]);
        st[mi][2] = fmaxf(fmaxf(fmaxf(st[mi][2], x0), x1), fmaxf(x2, x3));
        st[mi][3] = fminf(fminf(fminf(st[mi][3], x0), x1), fminf(x2, x3));
        if constexpr (SIDX == 0 && d == 3) {
            // `skip` (wave-uniform): the all-zero fragments of the very first pass; it can only be the first
            // k-step this workgroup folds, so max / min go back to their initial values behind it
            st[mi][2] = skip ? -3.402823466e+38f : st[mi][2];
            st[mi][3] = skip ? 3.402823466e+38f : st[mi][3];
        }
    };

    // One k-step = 16 slots of one MFMA (64 cycles).  Slot i also issues fragment read i of the NEXT k-step
    // and, when LOADS, global -> LDS load i of the next tile into stage S^1; with SIDX >= 0 it also folds four
    // elements of the fragments being multiplied into the A statistics (k-step SIDX of folded unit number hj).
    auto kstep = [&](auto s_c, auto ks_c, auto loads_c, auto sidx_c, const raw32 (&af)[4], const raw32 (&bf)[4],
                     raw32 (&naf)[4], raw32 (&nbf)[4], const unsigned char* ap, const unsigned char* bp, int hj,
                     bool skip) {
        constexpr int S = decltype(s_c)::value, SIDX = decltype(sidx_c)::value;
        constexpr bool LOADS = decltype(loads_c)::value != 0;
        if constexpr (FUSED && SIDX >= 0) load_bev(hj, sidx_c);
        static_for<0, 16>([&](auto slot_c) {
            constexpr int slot = decltype(slot_c)::value;
            constexpr int mi = slot >> 2, ni = slot & 3;
            acc[mi][ni] = mfma_f8<FMT>(bf[ni], af[mi], acc[mi][ni]);
            __builtin_amdgcn_sched_barrier(0);  // MFMA first, the rest of the slot in its shadow
            frag_op(s_c, ks_c, slot_c, naf, nbf);
            if constexpr (LOADS) issue_load(std::integral_constant<int, S ^ 1>{}, slot_c, ap, bp);
            if constexpr (FUSED && SIDX >= 0) stats_slot(af, slot_c, sidx_c, skip);
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;

    const int nk = g.K / BKB;
    raw32 af0[4], bf0[4], af1[4], bf1[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        af1[i].lo = af1[i].hi = raw16{{0u, 0u, 0u, 0u}};
        bf1[i].lo = bf1[i].hi = raw16{{0u, 0u, 0u, 0u}};
    }
    static_for<0, 16>([&](auto l_c) { issue_load(I0{}, l_c, a_base, b_base); });
    if (FUSED) {
        // cache the Be slices of every unit this tile-column folds (the host guarantees they fit)
        float* cache = reinterpret_cast<float*>(smem + BE_CACHE_OFFSET);
        const float* const Be = reinterpret_cast<const float*>(g.Be);
        const int nunits = nk >> 1;
        for (int j = 0, u = bn; u <= nunits && j < BE_CACHE_SLOTS / 2; ++j, u += g.tiles_n) {
            const int k = 256 * u - 64 + tid;
            cache[j * 256 + tid] = (k >= 0 && k < g.K) ? Be[k] : 0.f;
        }
        // S1..S3 still in partials: every workgroup folds them here, under the latency of its first tile
        if (!g.S) fold_s_partials_to_lds(g.s_partial, g.s_nparts, tid, reinterpret_cast<double*>(smem + S_RED_OFFSET));
    }
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    // One body per k-tile, from barrier to barrier: the last k-step of tile kt-1 (its fragments are already
    // in registers; the very first pass multiplies zeros) and the first k-step of tile kt.  The 16 loads of
    // tile kt+1 (clamped at the last tile; the reload is harmless) ride in the first of the two, into the
    // stage that held tile kt-1, whose last reads completed before the previous barrier.
    using IN = std::integral_constant<int, -1>;
    using I2 = std::integral_constant<int, 2>;
    using I3 = std::integral_constant<int, 3>;
    // stc: 0 plain, 1 with the statistics (the two k-steps of the body are k-steps 2S and 2S+1 of the unit)
    auto tile_body = [&](auto s_c, auto stc, int kt, int hj, bool skip) {
        constexpr int S = decltype(s_c)::value;
        constexpr bool STATS = decltype(stc)::value != 0;
        using SA = std::integral_constant<int, STATS ? 2 * S : -1>;
        using SB = std::integral_constant<int, STATS ? 2 * S + 1 : -1>;
        const int ktn = kt + 1 < nk ? kt + 1 : nk - 1;
        const unsigned char* ap = a_base + (int64_t)ktn * BKB;
        const unsigned char* bp = b_base + (int64_t)ktn * BKB;
        kstep(s_c, I0{}, I1{}, SA{}, af1, bf1, af0, bf0, ap, bp, hj, skip);   // step (kt-1, 1); reads (kt, 0)
        kstep(s_c, I1{}, I0{}, SB{}, af0, bf0, af1, bf1, ap, bp, hj, false);  // step (kt, 0);   reads (kt, 1)
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
    };
    // K is a multiple of 256 (the host checks): tiles come in pairs (units), so the stage parity is a
    // compile-time constant and there is no odd tail (a branch here makes the compiler shuffle the 256
    // accumulators)
    if constexpr (FUSED) {
        // plain units run in a branch-free inner loop, the folded unit in straight-line code between two such loops
        const int nunits = nk >> 1;
        int hu = bn, hj = 0, u = 0;
        for (;;) {
            const int stop = hu < nunits ? hu : nunits;
            for (; u < stop; ++u) {
                tile_body(I0{}, I0{}, 2 * u, 0, false);
                tile_body(I1{}, I0{}, 2 * u + 1, 0, false);
            }
            if (u >= nunits) break;
            tile_body(I0{}, I1{}, 2 * u, hj, u == 0);
            tile_body(I1{}, I1{}, 2 * u + 1, hj, false);
            ++u;
            hu += g.tiles_n;
            ++hj;
        }
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int ni = 0; ni < 4; ++ni) acc[mi][ni] = mfma_f8<FMT>(bf1[ni], af1[mi], acc[mi][ni]);  // step (nk-1, 1)
        // ... which is k-step 0 of the unit that would follow the last one
        if (hu == nunits) {
            load_bev(hj, I0{});
            static_for<0, 16>([&](auto slot_c) { stats_slot(af1, slot_c, I0{}, false); });
        }
    } else {
        for (int kt = 0; kt < nk; kt += 2) {
            tile_body(I0{}, I0{}, kt, 0, false);
            tile_body(I1{}, I0{}, kt + 1, 0, false);
        }
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int ni = 0; ni < 4; ++ni) acc[mi][ni] = mfma_f8<FMT>(bf1[ni], af1[mi], acc[mi][ni]);  // step (nk-1, 1)
    }

    gemm16_fast_epilogue<f16_t, MODE, FUSED>(g, acc, st, smem, bm, bn, row0, col0, tid, lane, wm, wn, l32, lh);
}

template <int FMT> static int gemm8_fast_launch(const GemmArgs& a, int mode, hipStream_t st) {
    const dim3 grid(a.tiles_m * a.tiles_n), block(256);
    const bool fused = a.fused_stats != 0;
    const size_t lds = fused ? g16f::LDS_BYTES_FUSED : g16::LDS_BYTES;
#define VABFT_G8F_CASE(VF, FU)                                                                             \
    if (mode == VF && fused == FU) {                                                                       \
        auto kern = gemm8_fast_kernel<FMT, VF, FU>;                                                             \
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
    VABFT_G8F_CASE(0, false)
    VABFT_G8F_CASE(1, false)
    VABFT_G8F_CASE(2, false)
    VABFT_G8F_CASE(3, false)
    VABFT_G8F_CASE(4, false)
    VABFT_G8F_CASE(5, false)
    VABFT_G8F_CASE(1, true)
    VABFT_G8F_CASE(2, true)
#undef VABFT_G8F_CASE
    return VABFT_EINVAL;
}

}  // namespace vabft
