// BF16 / FP16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16) with the fused V-ABFT
// epilogue: row sums of the FP32 accumulator tile before output quantisation (paper section
// 3.6 "Online (Fused Kernel) ABFT"; section 2.2 C^{r1'} = C r1), and the accumulator bit-flip
// injector (section 6.1).
//
// Tile 256 x 256 x 64 per workgroup of 4 wavefronts (2 x 2), 128 x 128 per wavefront as
// 4 x 4 MFMA tiles.  Operands are staged in LDS as [row][64 k] with the eight 16-byte chunks
// of a row XOR-swizzled so that both the staging stores and the ds_read_b128 fragment loads
// are bank-conflict free.  The MFMA is issued with the roles of A and B swapped
// (D' = B^T A^T), which puts one C row in one lane: lane l of a tile owns row (l % 32) and the
// 16 registers run along 16 of the tile's 32 columns, the other 16 sit in lane l ^ 32.  A row
// sum is therefore 16 in-register adds per tile plus one cross-lane add.
#pragma once
#include "gemm_common.h"

namespace vabft {

template <typename T> struct Mfma16;
template <> struct Mfma16<bf16_t> {
    static __device__ __forceinline__ f32x16_t run(const raw16& a, const raw16& b, f32x16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b),
                                                       c, 0, 0, 0);
    }
};
template <> struct Mfma16<f16_t> {
    static __device__ __forceinline__ f32x16_t run(const raw16& a, const raw16& b, f32x16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c,
                                                      0, 0, 0);
    }
};

namespace g16 {
constexpr int BM = 256, BN = 256, BK = 64;
constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
constexpr int STAGE = A_BYTES + B_BYTES;
constexpr int LDS_BYTES = 2 * STAGE;  // double buffered: 128 KiB
// epilogue scratch (the operand stages are free by then): row-sum staging at 0, the C staging slabs
// from 4096, the fused A-statistics staging at 40960 and the weighted row sums behind it
constexpr int SRED_OFFSET = 40960;
constexpr int RED2_OFFSET = SRED_OFFSET + 2 * 4 * BM * 4;
constexpr int CRED_OFFSET = RED2_OFFSET + 2 * BM * 4;  // column sums, [2 wm][256 columns]

__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }
__device__ __forceinline__ int lds_pos(int row, int chunk) { return row * 128 + ((chunk ^ swz(row)) << 4); }
}  // namespace g16

// Pieces of the epilogue of the 16-bit GEMM kernels.  Accumulator element (mi, ni, r) of a
// wavefront is
//   C[row0 + wm*128 + mi*32 + lane%32][col0 + wn*128 + ni*32 + 8*(r/4) + 4*(lane/32) + r%4].

// Fault injector on the accumulator registers (paper section 6.1 "Error injection").
template <bool INJECT>
__device__ __forceinline__ void gemm16_inject(const GemmArgs& g, f32x16_t (&acc)[4][4], int row0, int col0, int wm,
                                              int wn, int l32, int lh) {
    using namespace g16;
    const int rl_base = wm * 128 + l32;
    const int cl_base = wn * 128 + 4 * lh;
    if (INJECT) {
        const InjectArgs& inj = g.inj;
        if (inj.mode == 1) {
            for (int e = 0; e < inj.n_list; ++e) {
                const int fr = inj.d_list[3 * e], fc = inj.d_list[3 * e + 1], fb = inj.d_list[3 * e + 2];
                if (fr < row0 || fr >= row0 + BM || fc < col0 || fc >= col0 + BN) continue;
                if (fr >= g.M || fc >= g.N || fb < 0 || fb > 31) continue;
                const int rl = fr - row0, cl = fc - col0;
                const bool own = (rl >> 7) == wm && (cl >> 7) == wn && (rl & 31) == l32 && ((cl >> 2) & 1) == lh;
                if (own) {
                    const int idx = ((rl >> 5) & 3) * 64 + ((cl >> 5) & 3) * 16 + ((cl & 31) >> 3) * 4 + (cl & 3);
                    float before = 0.f, after = 0.f;
                    static_for<0, 4>([&](auto mi_c) {
                        static_for<0, 4>([&](auto ni_c) {
                            static_for<0, 16>([&](auto r_c) {
                                constexpr int mi = decltype(mi_c)::value, ni = decltype(ni_c)::value,
                                              r = decltype(r_c)::value;
                                if (idx == mi * 64 + ni * 16 + r) {
                                    before = acc[mi][ni][r];
                                    after = flip_bit(before, fb);
                                    acc[mi][ni][r] = after;
                                }
                            });
                        });
                    });
                    log_fault(inj, fr, fc, fb, (double)before, (double)after);
                }
            }
        } else if (inj.mode == 2) {
            static_for<0, 4>([&](auto mi_c) {
                static_for<0, 4>([&](auto ni_c) {
                    static_for<0, 16>([&](auto r_c) {
                        constexpr int mi = decltype(mi_c)::value, ni = decltype(ni_c)::value, r = decltype(r_c)::value;
                        const int gi = row0 + rl_base + mi * 32;
                        const int gj = col0 + cl_base + ni * 32 + 8 * (r >> 2) + (r & 3);
                        if (gi < g.M && gj < g.N) {
                            const int bit = bernoulli_bit(inj, gi, gj, g.N);
                            if (bit >= 0) acc[mi][ni][r] = flip_and_log<float>(inj, acc[mi][ni][r], gi, gj, bit);
                        }
                    });
                });
            });
        }
    }

}

// Row sums of the wavefront's accumulator tile, taken before quantisation (section 2.2
// C^{r1'} = C r1 on the tile; section 3.6 fused check): 63 in-register adds per row, arranged
// pairwise, plus one cross-lane add.  Lanes 0..31 leave the sum of row (wm*128 + mi*32 + lane) over the
// wavefront's 128 columns in red[wn][row].
__device__ __forceinline__ void gemm16_rowsum_to_lds(const f32x16_t (&acc)[4][4], float* red, int wm, int wn, int l32,
                                                     int lh) {
    using namespace g16;
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
        // pairwise over the 16 registers of a tile, then pairwise over the 4 tiles: a short
        // rounding-error chain (depth 7 with the cross-lane add) instead of 64 sequential adds
        float t[4];
#pragma unroll
        for (int ni = 0; ni < 4; ++ni) {
            float q[4];
#pragma unroll
            for (int k = 0; k < 4; ++k)
                q[k] = (acc[mi][ni][4 * k] + acc[mi][ni][4 * k + 1]) + (acc[mi][ni][4 * k + 2] + acc[mi][ni][4 * k + 3]);
            t[ni] = (q[0] + q[1]) + (q[2] + q[3]);
        }
        float s = (t[0] + t[1]) + (t[2] + t[3]);
        s += __shfl_xor(s, 32, WAVE);
        if (lh == 0) red[wn * BM + wm * 128 + mi * 32 + l32] = s;
    }
}

// Position-weighted row sums of the wavefront's accumulator tile (section 2.2 C^{r2'} = C r2,
// r2 = [1..N]): sum_j (j + 1) acc[i][j].  Inside the tile the weights are small compile-time
// constants; the offset of the lane's first column is applied once to the plain partial sum.
// Lanes 0..31 leave the result over the wavefront's 128 columns in red2[wn][row].
__device__ __forceinline__ void gemm16_rowsum2_to_lds(const f32x16_t (&acc)[4][4], float* red2, int col0, int wm,
                                                      int wn, int l32, int lh) {
    using namespace g16;
    const float w0 = (float)(col0 + wn * 128 + 4 * lh + 1);  // weight of the lane's first column
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
        float t1[4], t2[4];
#pragma unroll
        for (int ni = 0; ni < 4; ++ni) {
            float a1 = 0.f, a2 = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                a1 += acc[mi][ni][r];
                a2 = fmaf((float)(ni * 32 + 8 * (r >> 2) + (r & 3)), acc[mi][ni][r], a2);
            }
            t1[ni] = a1;
            t2[ni] = a2;
        }
        float s = fmaf(w0, (t1[0] + t1[1]) + (t1[2] + t1[3]), (t2[0] + t2[1]) + (t2[2] + t2[3]));
        s += __shfl_xor(s, 32, WAVE);
        if (lh == 0) red2[wn * BM + wm * 128 + mi * 32 + l32] = s;
    }
}

// Column sums of the wavefront's accumulator tile (section 2.2 C^{c1'} = c1 C): the four row blocks in
// registers first (64 values per lane, index v = ni*16 + r), then a reduce-scatter butterfly over the 32
// lanes that hold the 32 rows of a block: in step s the lanes that differ in bit 4-s exchange the half of
// their values whose index bit 5-s belongs to the partner and add what they receive, so the number of
// values per lane halves in every step (62 exchanges instead of 320).  Lane l ends with the complete sums
// of values 2*(l%32) and 2*(l%32)+1 and stores them to cred[wm][column].
template <int NV> struct ColReduce {
    static __device__ __forceinline__ void run(const float (&cur)[NV], int l32, float (&out)[2]) {
        constexpr int H = NV / 2;
        // NV = 64, 32, 16, 8, 4 pairs with lane bit 4, 3, 2, 1, 0
        constexpr int BIT = NV == 64 ? 4 : NV == 32 ? 3 : NV == 16 ? 2 : NV == 8 ? 1 : 0;
        const bool up = (l32 >> BIT) & 1;
        float nxt[H];
#pragma unroll
        for (int i = 0; i < H; ++i) {
            const float lo = cur[i], hi = cur[i + H];
            const float keep = up ? hi : lo, send = up ? lo : hi;
            nxt[i] = keep + __shfl_xor(send, 1 << BIT, WAVE);
        }
        if constexpr (H == 2) {
            out[0] = nxt[0];
            out[1] = nxt[1];
        } else {
            ColReduce<H>::run(nxt, l32, out);
        }
    }
};

__device__ __forceinline__ void gemm16_colsum_to_lds(const f32x16_t (&acc)[4][4], float* cred, int wm, int wn, int l32,
                                                     int lh) {
    using namespace g16;
    float v[64];
#pragma unroll
    for (int ni = 0; ni < 4; ++ni)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            v[ni * 16 + r] = (acc[0][ni][r] + acc[1][ni][r]) + (acc[2][ni][r] + acc[3][ni][r]);
    float out[2];
    ColReduce<64>::run(v, l32, out);
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int idx = 2 * l32 + e, ni = idx >> 4, r = idx & 15;
        cred[wm * BN + wn * 128 + ni * 32 + 8 * (r >> 2) + 4 * lh + (r & 3)] = out[e];
    }
}

// Quantise and store the wavefront's tile of C.
template <typename T, bool EDGE>
__device__ __forceinline__ void gemm16_store_c(const GemmArgs& g, const f32x16_t (&acc)[4][4], unsigned char* smem,
                                               int row0, int col0, int lane, int wm, int wn, int l32, int lh) {
    using namespace g16;
    const int rl_base = wm * 128 + l32;
    const int cl_base = wn * 128 + 4 * lh;
    uint16_t* __restrict__ C = reinterpret_cast<uint16_t*>(g.C);
    if (!EDGE) {
        // Whole tiles: pass each 32 x 128 slab of the wavefront's tile through a private LDS
        // buffer so that global stores are 16 bytes per lane and 256 contiguous bytes per row
        // (a lane owns 4 consecutive columns of one row, which alone would give 8-byte pieces
        // scattered over 32 rows).  Row pitch 264 B keeps the ds_write_b64 conflict free.
        constexpr int PITCH = 264;
        unsigned char* stage = smem + 4096 + (wm * 2 + wn) * (32 * PITCH);
        const int srow = lane >> 4, schunk = lane & 15;
#pragma unroll
        for (int mi = 0; mi < 4; ++mi) {
#pragma unroll
            for (int ni = 0; ni < 4; ++ni)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    uint16_t h[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) h[e] = Elem<T>::from_acc(acc[mi][ni][4 * q + e]);
                    uint2 v;
                    v.x = (uint32_t)h[0] | ((uint32_t)h[1] << 16);
                    v.y = (uint32_t)h[2] | ((uint32_t)h[3] << 16);
                    *reinterpret_cast<uint2*>(stage + l32 * PITCH + ni * 64 + q * 16 + lh * 8) = v;
                }
            // LDS operations of one wavefront complete in order; only the compiler must not
            // move the reads above the writes (or the next slab's writes above these reads)
            asm volatile("" ::: "memory");
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const int r = srow + 4 * t;
                const raw16 v = *reinterpret_cast<const raw16*>(stage + r * PITCH + schunk * 16);
                const int gi = row0 + wm * 128 + mi * 32 + r;
                const int gj = col0 + wn * 128 + schunk * 8;
                // C is not read again by this kernel: non-temporal store (measured 1.3 % of kernel time)
                typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_st;
                __builtin_nontemporal_store(__builtin_bit_cast(u32x4_st, v),
                                            reinterpret_cast<u32x4_st*>(C + (int64_t)gi * g.ldc + gj));
            }
            asm volatile("" ::: "memory");
        }
    } else {
#pragma unroll
        for (int mi = 0; mi < 4; ++mi) {
            const int gi = row0 + rl_base + mi * 32;
#pragma unroll
            for (int ni = 0; ni < 4; ++ni)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int gj = col0 + cl_base + ni * 32 + 8 * q;
                    uint16_t h[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) h[e] = Elem<T>::from_acc(acc[mi][ni][4 * q + e]);
                    if (gi < g.M) {
                        if (g.c_vec_ok && gj + 4 <= g.N) {
                            uint2 v;
                            v.x = (uint32_t)h[0] | ((uint32_t)h[1] << 16);
                            v.y = (uint32_t)h[2] | ((uint32_t)h[3] << 16);
                            *reinterpret_cast<uint2*>(C + (int64_t)gi * g.ldc + gj) = v;
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (gj + e < g.N) C[(int64_t)gi * g.ldc + gj + e] = h[e];
                        }
                    }
                }
        }
    }
}

// Epilogue of the guarded kernel: injector, row sums -> rowpart[bn][row], store.
// `smem` must be free for reuse (all wavefronts past their last LDS read).
template <typename T, int MODE, bool EDGE>
__device__ __forceinline__ void gemm16_epilogue(const GemmArgs& g, f32x16_t (&acc)[4][4], unsigned char* smem,
                                                int row0, int col0, int bn, int tid, int lane, int wm, int wn,
                                                int l32, int lh) {
    using namespace g16;
    constexpr bool VERIFY = MODE >= 1, INJECT = MODE == 2, WSUM = MODE == 2 || MODE == 3;
    constexpr bool CSUM = MODE == 2 || MODE == 4;
    gemm16_inject<INJECT>(g, acc, row0, col0, wm, wn, l32, lh);
    if (VERIFY) {
        float* red = reinterpret_cast<float*>(smem);                       // [2][256]
        float* red2 = reinterpret_cast<float*>(smem + g16::RED2_OFFSET);  // [2][256]
        float* cred = reinterpret_cast<float*>(smem + g16::CRED_OFFSET);  // [2][256]
        gemm16_rowsum_to_lds(acc, red, wm, wn, l32, lh);
        if (WSUM) gemm16_rowsum2_to_lds(acc, red2, col0, wm, wn, l32, lh);
        if (CSUM) gemm16_colsum_to_lds(acc, cred, wm, wn, l32, lh);
        __syncthreads();
        const int gi = row0 + tid;
        if (gi < g.M) {
            reinterpret_cast<float*>(g.rowpart)[(int64_t)bn * g.M + gi] = red[tid] + red[BM + tid];
            if (WSUM) reinterpret_cast<float*>(g.rowpart2)[(int64_t)bn * g.M + gi] = red2[tid] + red2[BM + tid];
        }
        const int gj = col0 + tid;
        if (CSUM && gj < g.N) reinterpret_cast<float*>(g.colpart)[(int64_t)(row0 / BM) * g.N + gj] = cred[tid] + cred[BN + tid];
    }
    gemm16_store_c<T, EDGE>(g, acc, smem, row0, col0, lane, wm, wn, l32, lh);
}

// Eight FP8 elements of a row-major matrix, widened to FP16 (exact: every E4M3 and E5M2 value is an FP16 value),
// zero-filled outside [nr) x [nc).  FMT 1: E4M3, 2: E5M2.
template <int FMT>
__device__ __forceinline__ raw16 guarded_chunk8to16(const uint8_t* base, int r, int nr, int c, int nc, int64_t ld,
                                                    int vec_ok) {
    uint32_t w0 = 0u, w1 = 0u;
    if (r < nr && c < nc) {
        const uint8_t* p = base + (int64_t)r * ld + c;
        if (vec_ok && c + 8 <= nc) {  // rows are 16-byte aligned and c is a multiple of 8
            const uint2 v = *reinterpret_cast<const uint2*>(p);
            w0 = v.x;
            w1 = v.y;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (c + e < nc) (e < 4 ? w0 : w1) |= ((uint32_t)p[e]) << ((e & 3) * 8);
        }
    }
    auto widen = [](uint32_t w, int byte) -> uint32_t {
        float x;
        if constexpr (FMT == 1)
            x = byte == 0 ? __builtin_amdgcn_cvt_f32_fp8((int)w, 0) : byte == 1 ? __builtin_amdgcn_cvt_f32_fp8((int)w, 1)
              : byte == 2 ? __builtin_amdgcn_cvt_f32_fp8((int)w, 2) : __builtin_amdgcn_cvt_f32_fp8((int)w, 3);
        else
            x = byte == 0 ? __builtin_amdgcn_cvt_f32_bf8((int)w, 0) : byte == 1 ? __builtin_amdgcn_cvt_f32_bf8((int)w, 1)
              : byte == 2 ? __builtin_amdgcn_cvt_f32_bf8((int)w, 2) : __builtin_amdgcn_cvt_f32_bf8((int)w, 3);
        return (uint32_t)Elem<f16_t>::from_acc(x);
    };
    raw16 out;
    out.w[0] = widen(w0, 0) | (widen(w0, 1) << 16);
    out.w[1] = widen(w0, 2) | (widen(w0, 3) << 16);
    out.w[2] = widen(w1, 0) | (widen(w1, 1) << 16);
    out.w[3] = widen(w1, 2) | (widen(w1, 3) << 16);
    return out;
}

// MODE 0: plain GEMM; 1: fused row-sum check; 2: check plus the fault injector.
// IN8 (guarded kernel with T = f16_t only): A and B hold FP8 elements (1: E4M3, 2: E5M2) that are widened to
// FP16 on their way into LDS; the products and their FP32 accumulation are then exactly those of the FP8
// problem (section 3.6: FP8 inputs, FP32 accumulation, FP16 output), for any shape and either layout of B.
template <typename T, int TRANSB, int MODE, bool EDGE, int IN8 = 0>
__global__ __launch_bounds__(256) void gemm16_kernel(const GemmArgs g) {
    static_assert(IN8 == 0 || (EDGE && std::is_same<T, f16_t>::value), "FP8 inputs ride the guarded FP16 kernel");
    using namespace g16;
    constexpr bool VERIFY = MODE >= 1, INJECT = MODE == 2;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lh = lane >> 5;
    int bm, bn;
    tile_of_block(blockIdx.x, g.tiles_m, g.tiles_n, bm, bn);
    if (VERIFY && blockIdx.x == 0 && tid == 0) *g.d_nflag = 0;
    if (VERIFY && blockIdx.x == 0 && tid == 0 && g.block_mode) *g.d_nblockflag = 0;
    if ((MODE == 2 || MODE == 4) && blockIdx.x == 0 && tid == 0 && g.d_ncolflag) *g.d_ncolflag = 0;
    const int row0 = bm * BM, col0 = bn * BN;
    const uint16_t* __restrict__ A = reinterpret_cast<const uint16_t*>(g.A);
    const uint16_t* __restrict__ B = reinterpret_cast<const uint16_t*>(g.B);

    f32x16_t acc[4][4];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

    raw16 ra[8], rb[8];

    // ---- global -> registers ------------------------------------------------
    auto load_tiles = [&](int kt) {
        const int kbase = kt * BK;
        {
            const int c = tid & 7, r = tid >> 3;
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                const int gr = row0 + r + 32 * p, gk = kbase + c * 8;
                if constexpr (IN8 != 0)
                    ra[p] = guarded_chunk8to16<IN8>(reinterpret_cast<const uint8_t*>(g.A), gr, g.M, gk, g.K, g.lda,
                                                    g.a_vec_ok);
                else if (!EDGE)
                    ra[p] = ld16(A + (int64_t)gr * g.lda + gk);
                else
                    ra[p] = guarded_chunk2(A, gr, g.M, gk, g.K, g.lda, g.a_vec_ok);
            }
        }
        if (TRANSB) {
            const int c = tid & 7, r = tid >> 3;
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                const int gn = col0 + r + 32 * p, gk = kbase + c * 8;
                if constexpr (IN8 != 0)
                    rb[p] = guarded_chunk8to16<IN8>(reinterpret_cast<const uint8_t*>(g.B), gn, g.N, gk, g.K, g.ldb,
                                                    g.b_vec_ok);
                else if (!EDGE)
                    rb[p] = ld16(B + (int64_t)gn * g.ldb + gk);
                else
                    rb[p] = guarded_chunk2(B, gn, g.N, gk, g.K, g.ldb, g.b_vec_ok);
            }
        } else {
            const int nc = tid & 31, kb = tid >> 5;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int gk = kbase + kb * 8 + e, gn = col0 + nc * 8;
                if constexpr (IN8 != 0)
                    rb[e] = guarded_chunk8to16<IN8>(reinterpret_cast<const uint8_t*>(g.B), gk, g.K, gn, g.N, g.ldb,
                                                    g.b_vec_ok);
                else if (!EDGE)
                    rb[e] = ld16(B + (int64_t)gk * g.ldb + gn);
                else
                    rb[e] = guarded_chunk2(B, gk, g.K, gn, g.N, g.ldb, g.b_vec_ok);
            }
        }
    };

    // ---- registers -> LDS ---------------------------------------------------
    auto store_tiles = [&](int s) {
        unsigned char* As = smem + s * STAGE;
        unsigned char* Bs = As + A_BYTES;
        {
            const int c = tid & 7, r = tid >> 3;
#pragma unroll
            for (int p = 0; p < 8; ++p) *reinterpret_cast<raw16*>(As + lds_pos(r + 32 * p, c)) = ra[p];
        }
        if (TRANSB) {
            const int c = tid & 7, r = tid >> 3;
#pragma unroll
            for (int p = 0; p < 8; ++p) *reinterpret_cast<raw16*>(Bs + lds_pos(r + 32 * p, c)) = rb[p];
        } else {
            // 8 x 8 transpose of 16-bit elements: rb[e] holds k = kb*8+e, n = nc*8 .. +7
            const int nc = tid & 31, kb = tid >> 5;
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                raw16 o;
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const uint32_t lo = rb[2 * w].w[q >> 1], hi = rb[2 * w + 1].w[q >> 1];
                    o.w[w] = (q & 1) ? ((lo >> 16) | (hi & 0xffff0000u)) : ((lo & 0xffffu) | (hi << 16));
                }
                *reinterpret_cast<raw16*>(Bs + lds_pos(nc * 8 + q, kb)) = o;
            }
        }
    };

    // ---- LDS -> MFMA ----------------------------------------------------------
    auto compute = [&](int s) {
        const unsigned char* As = smem + s * STAGE;
        const unsigned char* Bs = As + A_BYTES;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            raw16 af[4], bf[4];
#pragma unroll
            for (int mi = 0; mi < 4; ++mi)
                af[mi] = *reinterpret_cast<const raw16*>(As + lds_pos(wm * 128 + mi * 32 + l32, ks * 2 + lh));
#pragma unroll
            for (int ni = 0; ni < 4; ++ni)
                bf[ni] = *reinterpret_cast<const raw16*>(Bs + lds_pos(wn * 128 + ni * 32 + l32, ks * 2 + lh));
#pragma unroll
            for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                for (int ni = 0; ni < 4; ++ni) acc[mi][ni] = Mfma16<T>::run(bf[ni], af[mi], acc[mi][ni]);
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

    gemm16_epilogue<T, MODE, EDGE>(g, acc, smem, row0, col0, bn, tid, lane, wm, wn, l32, lh);
}

// Launcher of the guarded (ragged-size) kernel.
template <typename T, int TRANSB, int IN8 = 0>
static int gemm16_edge_launch_tb(const GemmArgs& a, int mode, hipStream_t st) {
    const dim3 grid(a.tiles_m * a.tiles_n), block(256);
    const size_t lds = g16::LDS_BYTES;
#define VABFT_G16_CASE(VF)                                                                                 \
    if (mode == VF) {                                                                                      \
        auto kern = gemm16_kernel<T, TRANSB, VF, true, IN8>;                                               \
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
    VABFT_G16_CASE(0)
    VABFT_G16_CASE(1)
    VABFT_G16_CASE(2)
    VABFT_G16_CASE(3)
    VABFT_G16_CASE(4)
#undef VABFT_G16_CASE
    return VABFT_EINVAL;
}

}  // namespace vabft
