// BF16 / FP16 GEMM main loop for whole-tile problems (M % 256 == 0, N % 256 == 0,
// K % 64 == 0, 16-byte aligned rows): global memory -> LDS without passing through
// registers (global_load_lds_dwordx4), fragments software-pipelined one k-step ahead of the
// MFMAs, one workgroup barrier per 64-wide k-tile, and the loads of the tile after next
// spread between the MFMAs so that the texture path never backs up into the MFMA issue.
//
// LDS has 64 banks on gfx950 and serves 16 lanes of a ds_read_b128 per cycle, so 16
// consecutive rows must land on 16 distinct 16-byte slots of a 256-byte window.
// Layouts (per stage, 64 KiB, two stages):
//   A tile, and B tile when B is stored N x K:  [256 rows][8 chunks of 16 B], chunk c of row r
//       at position c ^ ((r >> 1) & 7); fragments by ds_read_b128.
//   B tile when B is stored K x N:  [64 k][32 chunks of 16 B] (n contiguous), chunk c of row k
//       at position c ^ (4 * (k & 3)); fragments by ds_read_b64_tr_b16, which hands lane i of a
//       16-lane block the 4 k-consecutive values of column i of a 4(k) x 16(n) sub-tile.
// Check-side work fused into this kernel (MODE >= 1):
//   * row sums of the accumulator tile before quantisation (section 3.6 fused check);
//   * optionally (FUSED) the A-side of Algorithm 1: every A fragment passes through registers
//     on its way to the MFMA, so tile-column bn accumulates sum / max / min / dot-with-Be of
//     the k-steps whose body index is congruent to bn modulo the number of tile-columns;
//   * the compare-and-flag step: the last workgroup to finish a tile-row (an arrival ticket per
//     tile-row) combines that row block's partials in a fixed order, evaluates the threshold
//     in double precision, and writes rowsum, E, flags; the last row block writes nflag;
//   * (MODE 2, 3) the position-weighted row sums C r2 of section 2.2, through the same partials;
//   * (MODE 2, 4) the column sums c1 C of section 2.2, as per-tile-row partials for a later compare.
#pragma once
#include "gemm16.h"

namespace vabft {

typedef __attribute__((ext_vector_type(4))) short s16x4_t;

namespace g16f {
using namespace g16;
typedef __attribute__((address_space(3))) unsigned char lds_u8;
typedef const __attribute__((address_space(1))) unsigned char glb_u8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

__device__ __forceinline__ raw16 lds_read16(const lds_u8* p) {
    const u32x4_t v = *reinterpret_cast<const __attribute__((address_space(3))) u32x4_t*>(p);
    return __builtin_bit_cast(raw16, v);
}

// s_waitcnt lgkmcnt(0) only (vmcnt and expcnt fields left at their maxima)
__device__ __forceinline__ void wait_lgkmcnt0() { __builtin_amdgcn_s_waitcnt(0xC07F); }

// Transposing 8-byte LDS read, issued as inline assembly: the compiler treats the intrinsic
// form as possibly aliasing the asynchronous global -> LDS loads and would wait for ALL of
// them (vmcnt(0)) in front of every such read.  The caller must wait for lgkmcnt before it
// uses the result (LDS operations of a wavefront complete in order).
template <int OFFSET> __device__ __forceinline__ uint64_t lds_read_tr16_b64(const lds_u8* p) {
    static_assert(OFFSET >= 0 && OFFSET < 65536, "ds offset field is 16 bits");
    uint64_t v;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2"
                 : "=v"(v)
                 : "v"((uint32_t) reinterpret_cast<uintptr_t>(p)), "n"(OFFSET));
    return v;
}

// 16 bytes per lane, global -> LDS at (wave-uniform) lds_base + lane * 16
__device__ __forceinline__ void g2l16(const void* gptr, lds_u8* lds_base) {
    __builtin_amdgcn_global_load_lds((glb_u8*)gptr, (__attribute__((address_space(3))) void*)lds_base, 16, 0, 0);
}

// Partials exchanged between workgroups (which may sit on different XCDs with private L2s) go
// through device-scope relaxed atomic stores and loads: they are performed at the device's
// coherence point, so no cache write-back / invalidate fence is needed around the ticket.
__device__ __forceinline__ float ld_agent(const float* p) {
    return __builtin_bit_cast(float, __hip_atomic_load(reinterpret_cast<const uint32_t*>(p), __ATOMIC_RELAXED,
                                                        __HIP_MEMORY_SCOPE_AGENT));
}
__device__ __forceinline__ void st_agent(float* p, float v) {
    __hip_atomic_store(reinterpret_cast<uint32_t*>(p), __builtin_bit_cast(uint32_t, v), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}

// element e (0..3) of the two selected dwords of a 16-byte fragment, as float
template <typename T> __device__ __forceinline__ float frag_elem(uint32_t d0, uint32_t d1, int e);
template <> __device__ __forceinline__ float frag_elem<bf16_t>(uint32_t d0, uint32_t d1, int e) {
    const uint32_t d = e < 2 ? d0 : d1;
    return __uint_as_float((e & 1) ? (d & 0xffff0000u) : (d << 16));
}
template <> __device__ __forceinline__ float frag_elem<f16_t>(uint32_t d0, uint32_t d1, int e) {
    const uint32_t d = e < 2 ? d0 : d1;
    return Elem<f16_t>::to_acc((uint16_t)((e & 1) ? (d >> 16) : (d & 0xffffu)));
}

// Be values the workgroup will need, cached in LDS behind the two operand stages: one slot of
// 128 floats per folded unit u (k = 128*u - 16 .. 128*u + 111).
constexpr int BE_CACHE_OFFSET = LDS_BYTES;
constexpr int BE_CACHE_SLOTS = 16;
// behind the cache: 12 doubles for the fold of the S1..S3 partials of an encode that deferred it
constexpr int S_RED_OFFSET = LDS_BYTES + BE_CACHE_SLOTS * 128 * 4;
constexpr int LDS_BYTES_FUSED = S_RED_OFFSET + 128;
}  // namespace g16f

// Epilogue shared by the whole-tile kernels (16-bit and FP8 inputs; T is the OUTPUT element type): injector,
// row sums (and weighted / column sums), publication of the partials, the compare-and-flag step in the last
// workgroup of the tile-row, and the store of C.  st[mi] = (sum, dot with Be, max, min) of the A rows when FUSED.
template <typename T, int MODE, bool FUSED>
__device__ __forceinline__ void gemm16_fast_epilogue(const GemmArgs& g, f32x16_t (&acc)[4][4], float (&st)[4][4],
                                                     unsigned char* smem, int bm, int bn, int row0, int col0, int tid,
                                                     int lane, int wm, int wn, int l32, int lh) {
    using namespace g16f;
    constexpr bool VERIFY = MODE >= 1, INJECT = MODE == 2, WSUM = MODE == 2 || MODE == 3;
    constexpr bool CSUM = MODE == 2 || MODE == 4;
    gemm16_inject<INJECT>(g, acc, row0, col0, wm, wn, l32, lh);
    if (VERIFY) {
        float* red = reinterpret_cast<float*>(smem);                 // [2 wn][256 rows]
        float* sred = reinterpret_cast<float*>(smem + SRED_OFFSET);  // [2 wn][4][256 rows]
        float* red2 = reinterpret_cast<float*>(smem + RED2_OFFSET);  // [2 wn][256 rows]
        int* s_last = reinterpret_cast<int*>(smem + 2048);
        gemm16_rowsum_to_lds(acc, red, wm, wn, l32, lh);
        if (WSUM) gemm16_rowsum2_to_lds(acc, red2, col0, wm, wn, l32, lh);
        float* cred = reinterpret_cast<float*>(smem + CRED_OFFSET);  // [2 wm][256 columns]
        if (CSUM) gemm16_colsum_to_lds(acc, cred, wm, wn, l32, lh);
        if (FUSED) {
#pragma unroll
            for (int mi = 0; mi < 4; ++mi) {
                const float s0 = st[mi][0] + __shfl_xor(st[mi][0], 32, WAVE);
                const float s1 = st[mi][1] + __shfl_xor(st[mi][1], 32, WAVE);
                const float s2 = fmaxf(st[mi][2], __shfl_xor(st[mi][2], 32, WAVE));
                const float s3 = fminf(st[mi][3], __shfl_xor(st[mi][3], 32, WAVE));
                if (lh == 0) {
                    const int r = wm * 128 + mi * 32 + l32;
                    sred[(wn * 4 + 0) * BM + r] = s0;
                    sred[(wn * 4 + 1) * BM + r] = s1;
                    sred[(wn * 4 + 2) * BM + r] = s2;
                    sred[(wn * 4 + 3) * BM + r] = s3;
                }
            }
        }
        __syncthreads();
        const int gi = row0 + tid;
        float* rowpart = reinterpret_cast<float*>(g.rowpart);
        float* apart = reinterpret_cast<float*>(g.apart);
        float* rowpart2 = reinterpret_cast<float*>(g.rowpart2);
        st_agent(rowpart + (int64_t)bn * g.M + gi, red[tid] + red[BM + tid]);
        if (WSUM) st_agent(rowpart2 + (int64_t)bn * g.M + gi, red2[tid] + red2[BM + tid]);
        // column-sum partials are compared by a kernel of their own after this one: plain stores
        if (CSUM) reinterpret_cast<float*>(g.colpart)[(int64_t)bm * g.N + col0 + tid] = cred[tid] + cred[BN + tid];
        if (FUSED) {
            float* ap = apart + (int64_t)bn * 4 * g.M + gi;
            st_agent(ap, sred[0 * BM + tid] + sred[4 * BM + tid]);
            st_agent(ap + (int64_t)g.M, sred[1 * BM + tid] + sred[5 * BM + tid]);
            st_agent(ap + 2 * (int64_t)g.M, fmaxf(sred[2 * BM + tid], sred[6 * BM + tid]));
            st_agent(ap + 3 * (int64_t)g.M, fminf(sred[3 * BM + tid], sred[7 * BM + tid]));
        }
        // block-wise check: the partials are all this kernel leaves; a later kernel compares them per block
        const bool partials_only = MODE == 5 || (MODE == 2 && g.block_mode);
        if (partials_only) {
            __syncthreads();  // the store below reuses the LDS the reductions read
            gemm16_store_c<T, false>(g, acc, smem, row0, col0, lane, wm, wn, l32, lh);
            return;
        }
        // every thread's partials are performed (vmcnt(0)) before the workgroup takes this
        // tile-row's arrival ticket.  These round trips are short because no workgroup has issued
        // its C stores yet (all tiles finish together); behind the store burst they would each
        // cost several microseconds, which is why the check runs before the store and not in its
        // shadow.
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (tid == 0) *s_last = (atomicAdd(&g.tickets[bm], 1) == g.tiles_n - 1);
        __syncthreads();
        if (*s_last) {
            // Combine the tile-column partials in tile order.  The device-scope loads are issued
            // in batches of 16 tile-columns before anything is folded, so their latencies overlap.
            // every batch of 16 is folded as a tree and lands in one of four rotating accumulators, themselves
            // folded pairwise at the end: the rounding chain of a sum is log-like in the number of tile-columns
            float rs4[4] = {0.f, 0.f, 0.f, 0.f}, rs24[4] = {0.f, 0.f, 0.f, 0.f}, sum4[4] = {0.f, 0.f, 0.f, 0.f},
                  dot4[4] = {0.f, 0.f, 0.f, 0.f};
            float mx = -3.402823466e+38f, mn = 3.402823466e+38f;
            for (int t0 = 0; t0 < g.tiles_n; t0 += 16) {
                float v[16][5];
                float v2[16];
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const int t = t0 + j < g.tiles_n ? t0 + j : g.tiles_n - 1;  // clamped duplicates are not folded
                    v[j][0] = ld_agent(rowpart + (int64_t)t * g.M + gi);
                    if (WSUM) v2[j] = ld_agent(rowpart2 + (int64_t)t * g.M + gi);
                    if (FUSED) {
                        const float* ap = apart + (int64_t)t * 4 * g.M + gi;
                        v[j][1] = ld_agent(ap);
                        v[j][2] = ld_agent(ap + (int64_t)g.M);
                        v[j][3] = ld_agent(ap + 2 * (int64_t)g.M);
                        v[j][4] = ld_agent(ap + 3 * (int64_t)g.M);
                    }
                }
                // absent tile-columns count as the neutral element
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    if (!(t0 + j < g.tiles_n)) {
                        v[j][0] = 0.f;
                        if (WSUM) v2[j] = 0.f;
                        v[j][1] = 0.f;
                        v[j][2] = 0.f;
                        v[j][3] = -3.402823466e+38f;
                        v[j][4] = 3.402823466e+38f;
                    }
                float q[4], q2[4], qs[4], qd[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    q[j] = (v[4 * j][0] + v[4 * j + 1][0]) + (v[4 * j + 2][0] + v[4 * j + 3][0]);
                    if (WSUM) q2[j] = (v2[4 * j] + v2[4 * j + 1]) + (v2[4 * j + 2] + v2[4 * j + 3]);
                    if (FUSED) {
                        qs[j] = (v[4 * j][1] + v[4 * j + 1][1]) + (v[4 * j + 2][1] + v[4 * j + 3][1]);
                        qd[j] = (v[4 * j][2] + v[4 * j + 1][2]) + (v[4 * j + 2][2] + v[4 * j + 3][2]);
                        mx = fmaxf(mx, fmaxf(fmaxf(v[4 * j][3], v[4 * j + 1][3]), fmaxf(v[4 * j + 2][3], v[4 * j + 3][3])));
                        mn = fminf(mn, fminf(fminf(v[4 * j][4], v[4 * j + 1][4]), fminf(v[4 * j + 2][4], v[4 * j + 3][4])));
                    }
                }
                const int slot = (t0 >> 4) & 3;  // x + 0 is exact: the other three accumulators stay as they are
                const float b = (q[0] + q[1]) + (q[2] + q[3]);
                const float b2 = WSUM ? (q2[0] + q2[1]) + (q2[2] + q2[3]) : 0.f;
                const float bs = FUSED ? (qs[0] + qs[1]) + (qs[2] + qs[3]) : 0.f;
                const float bd = FUSED ? (qd[0] + qd[1]) + (qd[2] + qd[3]) : 0.f;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    rs4[k] += slot == k ? b : 0.f;
                    if (WSUM) rs24[k] += slot == k ? b2 : 0.f;
                    if (FUSED) {
                        sum4[k] += slot == k ? bs : 0.f;
                        dot4[k] += slot == k ? bd : 0.f;
                    }
                }
            }
            const float rs = (rs4[0] + rs4[1]) + (rs4[2] + rs4[3]), rs2 = (rs24[0] + rs24[1]) + (rs24[2] + rs24[3]);
            const float sum = (sum4[0] + sum4[1]) + (sum4[2] + sum4[3]), dot = (dot4[0] + dot4[1]) + (dot4[2] + dot4[3]);
            float expv, thr;
            if (FUSED) {
                const double mu = (double)sum / (double)g.K;
                double var = ((double)mx - mu) * (mu - (double)mn);
                var = var > 0 ? var : 0;
                const double* s_red = reinterpret_cast<const double*>(smem + S_RED_OFFSET);
                const double S1 = g.S ? g.S[0] : folded_s(s_red, 0), S2 = g.S ? g.S[1] : folded_s(s_red, 1),
                             S3 = g.S ? g.S[2] : folded_s(s_red, 2), dN = (double)g.N;
                const double t_det = dN * fabs(mu) * S1;
                const double t_var23 = g.c_sigma * sqrt(dN * mu * mu * S2 + dN * dN * var * S3);
                const double t_var4 = g.c_sigma * sqrt(dN) * sqrt(var) * sqrt(S2);
                expv = dot;
                thr = (float)(g.e_max * (t_det + t_var23 + t_var4));
                float* astat = reinterpret_cast<float*>(g.astat);
                astat[3 * (int64_t)gi + 0] = mx;
                astat[3 * (int64_t)gi + 1] = mn;
                astat[3 * (int64_t)gi + 2] = (float)mu;
                reinterpret_cast<float*>(const_cast<void*>(g.expected))[gi] = expv;
                reinterpret_cast<float*>(const_cast<void*>(g.T))[gi] = thr;
            } else {
                expv = reinterpret_cast<const float*>(g.expected)[gi];
                thr = reinterpret_cast<const float*>(g.T)[gi];
            }
            const float e = expv - rs;
            const int f = !(fabsf(e) <= thr);
            reinterpret_cast<float*>(g.rowsum)[gi] = rs;
            if (WSUM && g.rowsum2) reinterpret_cast<float*>(g.rowsum2)[gi] = rs2;
            reinterpret_cast<float*>(g.E)[gi] = e;
            g.flags[gi] = f;
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
        __syncthreads();  // the store below reuses the LDS the reductions read
    }
    gemm16_store_c<T, false>(g, acc, smem, row0, col0, lane, wm, wn, l32, lh);
}

template <typename T, int TRANSB, int MODE, bool FUSED>
__global__ __launch_bounds__(256) void gemm16_fast_kernel(const GemmArgs g) {
    using namespace g16f;
    constexpr bool VERIFY = MODE >= 1, INJECT = MODE == 2, WSUM = MODE == 2 || MODE == 3;
    constexpr bool CSUM = MODE == 2 || MODE == 4;
    static_assert(!FUSED || VERIFY, "fused statistics belong to the verified kernel");
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

    // ---- global -> LDS: each wavefront issues 8 + 8 loads of 1 KiB per k-tile -----------
    // Addresses are a wave-uniform 64-bit base (scalar registers) plus a 32-bit lane offset.
    // A (and N x K B): load i of a wavefront covers rows wave*64 + i*8 .. +7; lane l sits at row
    // l/8, chunk position l%8, and fetches chunk (l%8) ^ ((row>>1)&7) with
    // (row>>1)&7 = 4*(i&1) + l/16.  Two lane offsets (even / odd i) cover all loads.
    const uint32_t rk_e = ((lane & 7) ^ (lane >> 4)) << 4, rk_o = ((lane & 7) ^ (lane >> 4) ^ 4) << 4;
    const unsigned char* const a_base = A + (int64_t)(row0 + wave * 64) * g.lda * 2;
    const uint32_t a_lane_e = (uint32_t)(lane >> 3) * (uint32_t)g.lda * 2 + rk_e;
    const uint32_t a_lane_o = (uint32_t)(lane >> 3) * (uint32_t)g.lda * 2 + rk_o;
    const int64_t a_step = 8 * g.lda * 2;
    const unsigned char* b_base;
    uint32_t b_lane_e, b_lane_o;
    int64_t b_step;
    if (TRANSB) {
        b_base = B + (int64_t)(col0 + wave * 64) * g.ldb * 2;
        b_lane_e = (uint32_t)(lane >> 3) * (uint32_t)g.ldb * 2 + rk_e;
        b_lane_o = (uint32_t)(lane >> 3) * (uint32_t)g.ldb * 2 + rk_o;
        b_step = 8 * g.ldb * 2;
    } else {
        // K x N B: load i covers k rows wave*16 + 2*i, +1; lane l sits at row l/32, chunk position
        // l%32 and fetches chunk (l%32) ^ (4*(k&3)), k & 3 = (2*i + l/32) & 3.
        b_base = B + ((int64_t)(wave * 16) * g.ldb + col0) * 2;
        b_lane_e = (uint32_t)lh * (uint32_t)g.ldb * 2 + ((l32 ^ (4 * lh)) << 4);
        b_lane_o = (uint32_t)lh * (uint32_t)g.ldb * 2 + ((l32 ^ (4 * (2 + lh))) << 4);
        b_step = 2 * g.ldb * 2;
    }
    const int64_t b_ktile = TRANSB ? (int64_t)(BK * 2) : (int64_t)BK * g.ldb * 2;
    lds_u8* const a_dst = lds + wave * (64 * 128);
    lds_u8* const b_dst = lds + A_BYTES + (TRANSB ? wave * (64 * 128) : wave * (16 * 512));

    // load `l` (0..7: A, 8..15: B) of the tile whose uniform bases are (ap, bp), into stage LS
    auto issue_load = [&](auto ls_c, auto l_c, const unsigned char* ap, const unsigned char* bp) {
        constexpr int LS = decltype(ls_c)::value, l = decltype(l_c)::value;
        if constexpr (l < 8)
            g2l16(ap + l * a_step + ((l & 1) ? a_lane_o : a_lane_e), a_dst + LS * STAGE + l * 1024);
        else
            g2l16(bp + (l - 8) * b_step + ((l & 1) ? b_lane_o : b_lane_e), b_dst + LS * STAGE + (l - 8) * 1024);
    };

    // ---- LDS -> fragments: loop-invariant lane addresses, everything else is an immediate ----
    const int f_swz = (l32 >> 1) & 7;  // ((row >> 1) & 7) for row = 32*x + l32
    lds_u8* a_rd[2][4];                // [stage][k-step]
    lds_u8* b_rd[2][4];                // N x K B: [stage][k-step];  K x N B: [stage][ni]
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            a_rd[st][q] = lds + st * STAGE + (wm * 128 + l32) * 128 + (((q * 2 + lh) ^ f_swz) << 4);
            if (TRANSB) {
                b_rd[st][q] = lds + st * STAGE + A_BYTES + (wn * 128 + l32) * 128 + (((q * 2 + lh) ^ f_swz) << 4);
            } else {
                // 16-lane block b = lane/16 reads the 4(k) x 16(n) sub-tile at
                //   k = 8*(b/2) + s/4 (+4 for the second half), n = 16*(b%2) + 4*(s%4), s = lane%16
                const int t_s = lane & 15, t_b = lane >> 4;
                const int t_k = 8 * (t_b >> 1) + (t_s >> 2);
                const int t_n = wn * 128 + 16 * (t_b & 1) + 4 * (t_s & 3) + q * 32;
                b_rd[st][q] = lds + st * STAGE + A_BYTES + t_k * 512 + (((t_n >> 3) ^ (4 * (t_k & 3))) << 4) +
                              (t_n & 4) * 2;
            }
        }

    // One fragment read operation `op` of k-step KS from stage S into (af, bf).  A k-step needs
    // NRD operations: 4 ds_read_b128 for A, then 4 ds_read_b128 (N x K B) or 8 transposing
    // 8-byte reads (K x N B: low halves first, then high halves).
    constexpr int NRD = TRANSB ? 8 : 12;
    auto frag_op = [&](auto s_c, auto ks_c, auto op_c, raw16 (&af)[4], raw16 (&bf)[4]) {
        constexpr int S = decltype(s_c)::value, KS = decltype(ks_c)::value, op = decltype(op_c)::value;
        if constexpr (op < 4) {
            af[op] = lds_read16(a_rd[S][KS] + op * 4096);
        } else if constexpr (TRANSB != 0) {
            bf[op - 4] = lds_read16(b_rd[S][KS] + (op - 4) * 4096);
        } else {
            constexpr int ni = (op - 4) & 3, hi = (op - 4) >> 2;
            const uint64_t v = lds_read_tr16_b64<(KS * 16 + 4 * hi) * 512>(b_rd[S][ni]);
            bf[ni].w[2 * hi] = (uint32_t)v;
            bf[ni].w[2 * hi + 1] = (uint32_t)(v >> 32);
        }
    };

    // ---- fused A-side statistics (FUSED) ------------------------------------------------
    // Both wavefronts of a wm pair hold the same A fragments; wavefront wn takes elements
    // 4*wn .. 4*wn+3 of each 8-element fragment, so a lane accumulates, per mi, over
    // k = kbase + 8*(lane/32) + 4*wn + 0..3 of row wm*128 + mi*32 + lane%32.
    // st[mi] = (sum, dot with Be, max, min); bev[q] = the four Be values of k-step q of the body.
    float st[4][4];
    f32x4_t bev[2][4];  // [tile of the unit][k-step of the body]
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
        st[mi][0] = 0.f;
        st[mi][1] = 0.f;
        st[mi][2] = -3.402823466e+38f;
        st[mi][3] = 3.402823466e+38f;
    }
    const float* const Be = reinterpret_cast<const float*>(g.Be);
    // Be values of folded unit number j of this workgroup (unit u = bn + j*tiles_n, tiles 2u and
    // 2u+1), from the LDS cache filled in the prologue.  k-step q of body kb = 2u + t multiplies
    // step (kb-1, 3) for q = 0 and (kb, q-1) otherwise, i.e. k = 128u - 16 + 64t + 16q + ...
    auto load_bev = [&](int j) {
        const float* slot = reinterpret_cast<const float*>(smem + BE_CACHE_OFFSET) + j * 128 + 8 * lh + 4 * wn;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int q = 0; q < 4; ++q) bev[t][q] = *reinterpret_cast<const f32x4_t*>(slot + 64 * t + 16 * q);
    };
    uint32_t sd0 = 0, sd1 = 0;  // the two dwords of the current fragment that this wavefront folds
    // `skip` (wave-uniform) keeps the all-zero fragments of the very first pass out of max / min
    auto stats_elem = [&](const raw16 (&af)[4], auto t_c, auto q_c, auto slot_c, bool skip) {
        constexpr int t = decltype(t_c)::value, q = decltype(q_c)::value, slot = decltype(slot_c)::value;
        constexpr int mi = slot >> 2, e = slot & 3;
        if constexpr (e == 0) {
            // select by value (a conditional between the two array elements themselves would
            // become a pointer select and push the fragment arrays out of registers)
            const uint32_t lo0 = af[mi].w[0], lo1 = af[mi].w[1], hi0 = af[mi].w[2], hi1 = af[mi].w[3];
            sd0 = wn ? hi0 : lo0;
            sd1 = wn ? hi1 : lo1;
        }
        const float x = frag_elem<T>(sd0, sd1, e);
        st[mi][0] += x;
        st[mi][1] = fmaf(x, bev[t][q][e], st[mi][1]);
        if constexpr (q == 0 && t == 0) {
            st[mi][2] = fmaxf(st[mi][2], skip ? -3.402823466e+38f : x);
            st[mi][3] = fminf(st[mi][3], skip ? 3.402823466e+38f : x);
        } else {
            st[mi][2] = fmaxf(st[mi][2], x);
            st[mi][3] = fminf(st[mi][3], x);
        }
    };

    // One k-step = 16 slots of one MFMA.  Slot i also issues fragment read i of the NEXT k-step
    // (stage S, k-step KS, into the other register set) and, on odd slots when LBASE >= 0,
    // global -> LDS load LBASE + i/2 of the next tile into stage S^1; with STATS it also folds one
    // element per mi-slot of the fragments being multiplied into the A statistics.  Everything a
    // slot issues besides its MFMA should fit under that MFMA's 32 cycles; a scheduling barrier
    // closes every slot so the compiler keeps the interleaving.
    auto kstep = [&](auto s_c, auto ks_c, auto lbase_c, auto stats_c, auto q_c, const raw16 (&af)[4],
                     const raw16 (&bf)[4], raw16 (&naf)[4], raw16 (&nbf)[4], const unsigned char* ap,
                     const unsigned char* bp, bool skip) {
        constexpr int S = decltype(s_c)::value, LBASE = decltype(lbase_c)::value;
        constexpr bool STATS = decltype(stats_c)::value != 0;
        if (!TRANSB) wait_lgkmcnt0();  // the assembly reads of (af, bf) issued during the previous k-step
        static_for<0, 16>([&](auto slot_c) {
            constexpr int slot = decltype(slot_c)::value;
            constexpr int mi = slot >> 2, ni = slot & 3;
            acc[mi][ni] = Mfma16<T>::run(bf[ni], af[mi], acc[mi][ni]);
            __builtin_amdgcn_sched_barrier(0);  // MFMA first, the rest of the slot in its shadow
            if constexpr (slot < NRD) frag_op(s_c, ks_c, slot_c, naf, nbf);  // one read per slot, front-loaded
            if constexpr (LBASE >= 0 && (slot & 1))
                issue_load(std::integral_constant<int, S ^ 1>{}, std::integral_constant<int, LBASE + slot / 2>{}, ap,
                           bp);
            if constexpr (FUSED && STATS) stats_elem(af, s_c, q_c, slot_c, skip);
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    using I3 = std::integral_constant<int, 3>;
    using I8 = std::integral_constant<int, 8>;
    using IN = std::integral_constant<int, -1>;

    const int nk = g.K / BK;
    raw16 af0[4], bf0[4], af1[4], bf1[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) af1[i] = bf1[i] = raw16{{0u, 0u, 0u, 0u}};
    static_for<0, 16>([&](auto l_c) { issue_load(I0{}, l_c, a_base, b_base); });
    if (FUSED) {
        // cache the Be slices of every unit this tile-column folds (the host guarantees they fit)
        float* cache = reinterpret_cast<float*>(smem + BE_CACHE_OFFSET);
        const int nunits = nk >> 1;
        for (int j = 0, u = bn; u <= nunits && j < BE_CACHE_SLOTS; ++j, u += g.tiles_n) {
            if (tid < 128) {
                const int k = 128 * u - 16 + tid;
                cache[j * 128 + tid] = (k >= 0 && k < g.K) ? Be[k] : 0.f;
            }
        }
        // S1..S3 still in partials: every workgroup folds them here, under the latency of its first tile
        if (!g.S) fold_s_partials_to_lds(g.s_partial, g.s_nparts, tid, reinterpret_cast<double*>(smem + S_RED_OFFSET));
    }
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    // One body per k-tile, running from barrier to barrier.  Global k-step j = 4*kt + ks
    // multiplies register set j%2 and fetches the fragments of step j+1 into the other set.
    // The barrier that publishes tile kt sits BEFORE the last k-step of tile kt-1, so that
    // step's MFMAs cover the latency of the first fragment reads of tile kt (the very first
    // pass multiplies zeros).  The 16 loads of tile kt+1 (clamped at the last tile; the reload
    // is harmless) ride in the first two k-steps after the barrier; the stage they fill held
    // tile kt-1, whose last reads completed before that barrier.  The body is instantiated for
    // both stage parities so that every LDS offset is an instruction immediate, with and
    // without the statistics.  (The stage parity of tile kt is kt & 1 = its position in a unit.)
    auto tile_body = [&](auto s_c, auto st_c, int kt, bool skip) {
        const int ktn = kt + 1 < nk ? kt + 1 : nk - 1;
        const unsigned char* ap = a_base + (int64_t)ktn * (BK * 2);
        const unsigned char* bp = b_base + ktn * b_ktile;
        kstep(s_c, I0{}, I0{}, st_c, I0{}, af1, bf1, af0, bf0, ap, bp, skip);  // step (kt-1, 3)
        kstep(s_c, I1{}, I8{}, st_c, I1{}, af0, bf0, af1, bf1, ap, bp, false);  // step (kt, 0)
        kstep(s_c, I2{}, IN{}, st_c, I2{}, af1, bf1, af0, bf0, ap, bp, false);  // step (kt, 1)
        kstep(s_c, I3{}, IN{}, st_c, I3{}, af0, bf0, af1, bf1, ap, bp, false);  // step (kt, 2)
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
    };
    if (FUSED) {
        // Tiles are walked in units of two (so the stage parity stays a compile-time constant).
        // Tile-column bn folds the units u with u % tiles_n == bn into the statistics: plain
        // units run in a branch-free inner loop, the folded unit in straight-line code between
        // two such loops.  K is a multiple of 128 here (the host checks), so there is no odd tile.
        const int nunits = nk >> 1;
        int hu = bn, hj = 0;
        int u = 0;
        for (;;) {
            const int stop = hu < nunits ? hu : nunits;
            for (; u < stop; ++u) {
                tile_body(I0{}, I0{}, 2 * u, false);
                tile_body(I1{}, I0{}, 2 * u + 1, false);
            }
            if (u >= nunits) break;
            load_bev(hj);
            tile_body(I0{}, I1{}, 2 * u, u == 0);
            tile_body(I1{}, I1{}, 2 * u + 1, false);
            ++u;
            hu += g.tiles_n;
            ++hj;
        }
        // step (nk-1, 3) is the first k-step of the unit that would follow the last one
        if (!TRANSB) wait_lgkmcnt0();
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int ni = 0; ni < 4; ++ni) acc[mi][ni] = Mfma16<T>::run(bf1[ni], af1[mi], acc[mi][ni]);
        if (hu == nunits) {
            load_bev(hj);
            static_for<0, 16>([&](auto slot_c) { stats_elem(af1, I0{}, I0{}, slot_c, false); });
        }
    } else {
        int kt = 0;
        for (; kt + 1 < nk; kt += 2) {
            tile_body(I0{}, I0{}, kt, false);
            tile_body(I1{}, I0{}, kt + 1, false);
        }
        if (kt < nk) tile_body(I0{}, I0{}, kt, false);
        if (!TRANSB) wait_lgkmcnt0();
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int ni = 0; ni < 4; ++ni) acc[mi][ni] = Mfma16<T>::run(bf1[ni], af1[mi], acc[mi][ni]);
    }

    // ---- epilogue -------------------------------------------------------------------------
    gemm16_fast_epilogue<T, MODE, FUSED>(g, acc, st, smem, bm, bn, row0, col0, tid, lane, wm, wn, l32, lh);
}

template <typename T, int TRANSB>
static int gemm16_fast_launch_tb(const GemmArgs& a, int mode, hipStream_t st) {
    const dim3 grid(a.tiles_m * a.tiles_n), block(256);
    const int fused = a.fused_stats ? 1 : 0;
    const size_t lds = fused ? g16f::LDS_BYTES_FUSED : g16::LDS_BYTES;
#define VABFT_G16F_CASE(VF, FU)                                                                            \
    if (mode == VF && fused == FU) {                                                                       \
        auto kern = gemm16_fast_kernel<T, TRANSB, VF, FU != 0>;                                            \
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
    VABFT_G16F_CASE(0, 0)
    VABFT_G16F_CASE(1, 0)
    VABFT_G16F_CASE(2, 0)
    VABFT_G16F_CASE(3, 0)
    VABFT_G16F_CASE(4, 0)
    VABFT_G16F_CASE(5, 0)
    VABFT_G16F_CASE(1, 1)
    VABFT_G16F_CASE(2, 1)
#undef VABFT_G16F_CASE
    return VABFT_EINVAL;
}

}  // namespace vabft
