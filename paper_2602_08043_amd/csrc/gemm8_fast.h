// FP8 (OCP E4M3) GEMM with FP32 accumulation and FP16 output on the gfx950 matrix cores
// (v_mfma_f32_32x32x64_f8f6f4), for whole-tile problems with B stored N x K:
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
//     FP16 store) is the 16-bit kernel's.
#pragma once
#include "gemm16_fast.h"

namespace vabft {

typedef __attribute__((ext_vector_type(8))) int i32x8_t;

namespace g8f {
using namespace g16f;
constexpr int BKB = 128;  // bytes (= k-values) per tile row
struct alignas(16) raw32 {
    raw16 lo, hi;
};
__device__ __forceinline__ f32x16_t mfma_f8(const raw32& a, const raw32& b, f32x16_t c) {
    // cbsz = blgp = 0: both operands E4M3; no block scaling
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(__builtin_bit_cast(i32x8_t, a), __builtin_bit_cast(i32x8_t, b),
                                                           c, 0, 0, 0, 0, 0, 0);
}
}  // namespace g8f

template <int MODE>
__global__ __launch_bounds__(256) void gemm8_fast_kernel(const GemmArgs g) {
    using namespace g8f;
    constexpr bool CSUM = MODE == 2 || MODE == 4;
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

    // One k-step = 16 slots of one MFMA (64 cycles).  Slot i also issues fragment read i of the NEXT k-step
    // and, when LOADS, global -> LDS load i of the next tile into stage S^1.
    auto kstep = [&](auto s_c, auto ks_c, auto loads_c, const raw32 (&af)[4], const raw32 (&bf)[4], raw32 (&naf)[4],
                     raw32 (&nbf)[4], const unsigned char* ap, const unsigned char* bp) {
        constexpr int S = decltype(s_c)::value;
        constexpr bool LOADS = decltype(loads_c)::value != 0;
        static_for<0, 16>([&](auto slot_c) {
            constexpr int slot = decltype(slot_c)::value;
            constexpr int mi = slot >> 2, ni = slot & 3;
            acc[mi][ni] = mfma_f8(bf[ni], af[mi], acc[mi][ni]);
            __builtin_amdgcn_sched_barrier(0);  // MFMA first, the rest of the slot in its shadow
            frag_op(s_c, ks_c, slot_c, naf, nbf);
            if constexpr (LOADS) issue_load(std::integral_constant<int, S ^ 1>{}, slot_c, ap, bp);
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
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    // One body per k-tile, from barrier to barrier: the last k-step of tile kt-1 (its fragments are already
    // in registers; the very first pass multiplies zeros) and the first k-step of tile kt.  The 16 loads of
    // tile kt+1 (clamped at the last tile; the reload is harmless) ride in the first of the two, into the
    // stage that held tile kt-1, whose last reads completed before the previous barrier.
    auto tile_body = [&](auto s_c, int kt) {
        const int ktn = kt + 1 < nk ? kt + 1 : nk - 1;
        const unsigned char* ap = a_base + (int64_t)ktn * BKB;
        const unsigned char* bp = b_base + (int64_t)ktn * BKB;
        kstep(s_c, I0{}, I1{}, af1, bf1, af0, bf0, ap, bp);  // step (kt-1, 1); reads (kt, 0)
        kstep(s_c, I1{}, I0{}, af0, bf0, af1, bf1, ap, bp);  // step (kt, 0);   reads (kt, 1)
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
    };
    // K is a multiple of 256 (the host checks): tiles come in pairs, so the stage parity is a compile-time
    // constant and there is no odd tail (a branch here makes the compiler shuffle the 256 accumulators)
    for (int kt = 0; kt < nk; kt += 2) {
        tile_body(I0{}, kt);
        tile_body(I1{}, kt + 1);
    }
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni) acc[mi][ni] = mfma_f8(bf1[ni], af1[mi], acc[mi][ni]);  // step (nk-1, 1)

    float st[4][4] = {};
    gemm16_fast_epilogue<f16_t, MODE, false>(g, acc, st, smem, bm, bn, row0, col0, tid, lane, wm, wn, l32, lh);
}

static int gemm8_fast_launch(const GemmArgs& a, int mode, hipStream_t st) {
    const dim3 grid(a.tiles_m * a.tiles_n), block(256);
    const size_t lds = g16::LDS_BYTES;
#define VABFT_G8F_CASE(VF)                                                                                 \
    if (mode == VF) {                                                                                      \
        auto kern = gemm8_fast_kernel<VF>;                                                                 \
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
    VABFT_G8F_CASE(0)
    VABFT_G8F_CASE(1)
    VABFT_G8F_CASE(2)
    VABFT_G8F_CASE(3)
    VABFT_G8F_CASE(4)
    VABFT_G8F_CASE(5)
#undef VABFT_G8F_CASE
    return VABFT_EINVAL;
}

}  // namespace vabft
