// Pieces shared by the whole-tile (unguarded) GEMM kernels, and the epilogue of the kernels whose accumulator
// tiles are 32 x 32 (the FP8 kernel): LDS / global -> LDS access helpers, device-scope publication of
// partials, the compare-and-flag step of a tile-row, and the 32 x 32-layout epilogue.
//
// Check-side work fused into the whole-tile kernels (MODE >= 1):
//   * row sums of the accumulator tile before quantisation (section 3.6 fused check);
//   * optionally (FUSED) the A-side of Algorithm 1 for the rows of A, split over the tile-columns of a tile-row;
//   * the compare-and-flag step: the last workgroup to finish a tile-row (an arrival ticket per
//     tile-row) combines that row block's partials in a fixed order, evaluates the threshold
//     in double precision, and writes rowsum, E, flags; the last row block writes nflag;
//   * (MODE 2, 3) the position-weighted row sums C r2 of section 2.2, through the same partials;
//   * (MODE 2, 4) the column sums c1 C of section 2.2, as per-tile-row partials for a later compare.
#pragma once
#include "gemm16.h"

namespace vabft {

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
// The order relied on is the hardware's, not the language's (a release fence at agent scope writes back the
// whole L2 on this chip and cost 27 us per launch):
//   1. an agent-scope atomic store is a write-through store: the issuing XCD's L2 keeps no dirty copy, the
//      value goes to the memory-side coherence point that all XCDs share;
//   2. s_waitcnt vmcnt(0) returns only when that point has acknowledged every outstanding store of the wavefront;
//   3. the workgroup barrier that follows puts all wavefronts' waits in front of the one thread's ticket
//      atomicAdd, itself executed at the same coherence point, so a workgroup that sees ticket == tiles_n - 1
//      comes after every other workgroup's partials there;
//   4. the last arriver reads the partials with agent-scope atomic loads, which are not served from its
//      XCD's L2 or the compute unit's vector cache.
// The s_waitcnt builtin and the barrier are also compiler barriers for these atomics (volatile-like side effects),
// so the compiler keeps the same order.  A back-to-back soak test on rotating inputs watches this protocol.
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

// Compare-and-flag step of a tile-row, run by every workgroup after it has published its partials: the
// workgroup takes the tile-row's arrival ticket, and the last one to arrive combines the partials of all
// tile-columns in a fixed order, evaluates Algorithm 1 in double precision (FUSED) and writes rowsum, E, flags
// (section 2.2, Eq. abft-check); the last row block writes nflag.  gi = the row this thread owns; s_red = the
// workgroup's fold of the S1..S3 partials in LDS (used when g.S is null).
template <bool WSUM, bool FUSED>
__device__ __forceinline__ void gemm_tile_row_check(const GemmArgs& g, unsigned char* smem, const double* s_red, int bm,
                                                    int gi, int tid) {
    using namespace g16f;
    int* s_last = reinterpret_cast<int*>(smem + 2048);
    float* rowpart = reinterpret_cast<float*>(g.rowpart);
    float* apart = reinterpret_cast<float*>(g.apart);
    float* rowpart2 = reinterpret_cast<float*>(g.rowpart2);
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
            const double S1 = g.S ? g.S[0] : folded_s(s_red, 0), S2 = g.S ? g.S[1] : folded_s(s_red, 1),
                         S3 = g.S ? g.S[2] : folded_s(s_red, 2), dN = (double)g.N;
            const double t_det = dN * fabs(mu) * S1;
            const double t_var23 = g.c_sigma * sqrt(dN * mu * mu * S2 + dN * dN * var * S3);
            const double t_var4 = g.c_sigma * sqrt(dN * var * S2);  // = c sqrt(N) sigma_A sqrt(S2), one root
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
}

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
        gemm_tile_row_check<WSUM, FUSED>(g, smem, reinterpret_cast<const double*>(smem + S_RED_OFFSET), bm, gi, tid);
        __syncthreads();  // the store below reuses the LDS the reductions read
    }
    gemm16_store_c<T, false>(g, acc, smem, row0, col0, lane, wm, wn, l32, lh);
}

}  // namespace vabft
