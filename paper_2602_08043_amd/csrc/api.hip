// C ABI of libvabft: argument validation, workspace layout, dispatch, and the compare-and-flag
// step (paper section 2.2 Eq. abft-check, E_i = C^{r1}[i] - C^{r1'}[i]).
#include <math.h>

#include <mutex>

#include "vabft_device.h"
#include "vabft_host.h"

namespace vabft {

// sum_t part[t][i] in a fixed order: batches of 16 folded as trees into four rotating accumulators, themselves
// folded pairwise at the end (the order the whole-tile kernels use for their partials)
template <typename acc_t>
__device__ __forceinline__ acc_t fold_partials(const acc_t* __restrict__ part, int nparts, int M, int i) {
    acc_t a4[4] = {0, 0, 0, 0};
    for (int t0 = 0; t0 < nparts; t0 += 16) {
        acc_t v[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) v[j] = part[(int64_t)(t0 + j < nparts ? t0 + j : nparts - 1) * M + i];
#pragma unroll
        for (int j = 0; j < 16; ++j)
            if (!(t0 + j < nparts)) v[j] = 0;
        acc_t q[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) q[j] = (v[4 * j] + v[4 * j + 1]) + (v[4 * j + 2] + v[4 * j + 3]);
        const acc_t b = (q[0] + q[1]) + (q[2] + q[3]);
        const int slot = (t0 >> 4) & 3;  // x + 0 is exact: the other three stay as they are
#pragma unroll
        for (int k = 0; k < 4; ++k) a4[k] += slot == k ? b : (acc_t)0;
    }
    return (a4[0] + a4[1]) + (a4[2] + a4[3]);
}

// rowsum[i] = sum_t rowpart[t][i] in a fixed order; E = expected - rowsum; flag = !(|E| <= T)
template <typename acc_t>
__global__ __launch_bounds__(256) void finalize_kernel(const acc_t* __restrict__ rowpart, int tiles_n, int M,
                                                       const acc_t* __restrict__ expected,
                                                       const acc_t* __restrict__ T, acc_t* __restrict__ rowsum,
                                                       acc_t* __restrict__ E, int32_t* __restrict__ flags,
                                                       int32_t* __restrict__ nflag,
                                                       const acc_t* __restrict__ rowpart2,
                                                       acc_t* __restrict__ rowsum2) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    int f = 0;
    if (i < M) {
        if (rowsum2) rowsum2[i] = fold_partials(rowpart2, tiles_n, M, i);  // position-weighted row sums C r2
        const acc_t s = fold_partials(rowpart, tiles_n, M, i);
        const acc_t e = expected[i] - s;
        f = !(fabs(e) <= T[i]);
        rowsum[i] = s;
        E[i] = e;
        flags[i] = f;
    }
    const int cnt = __syncthreads_count(f);
    if (threadIdx.x == 0 && cnt) atomicAdd(nflag, cnt);
}

__global__ void zero_int_kernel(int32_t* p) { *p = 0; }

// colsum[j] = sum over tile-rows of colpart[t][j] in a fixed order; E_col = expected_col - colsum;
// flag = !(|E_col| <= T_col)   (section 2.2, the column form of Eq. abft-check)
template <typename acc_t>
__global__ __launch_bounds__(256) void finalize_cols_kernel(const acc_t* __restrict__ colpart, int nparts, int N,
                                                            const acc_t* __restrict__ expected_col,
                                                            const acc_t* __restrict__ Tcol, acc_t* __restrict__ colsum,
                                                            acc_t* __restrict__ Ecol, int32_t* __restrict__ colflags,
                                                            int32_t* __restrict__ ncolflag) {
    const int j = blockIdx.x * 256 + threadIdx.x;
    int f = 0;
    if (j < N) {
        const acc_t s = fold_partials(colpart, nparts, N, j);
        const acc_t e = expected_col[j] - s;
        f = !(fabs(e) <= Tcol[j]);
        colsum[j] = s;
        Ecol[j] = e;
        colflags[j] = f;
    }
    const int cnt = __syncthreads_count(f);
    if (threadIdx.x == 0 && cnt) atomicAdd(ncolflag, cnt);
}

// one stored element of C, read and written in the accumulator type
template <typename T> struct CElem;
template <> struct CElem<bf16_t> {
    using store_t = uint16_t;
    static __device__ __forceinline__ float get(const store_t* p) { return Elem<bf16_t>::to_acc(*p); }
    static __device__ __forceinline__ void put(store_t* p, float v) { *p = Elem<bf16_t>::from_acc(v); }
};
template <> struct CElem<f16_t> {
    using store_t = uint16_t;
    static __device__ __forceinline__ float get(const store_t* p) { return Elem<f16_t>::to_acc(*p); }
    static __device__ __forceinline__ void put(store_t* p, float v) { *p = Elem<f16_t>::from_acc(v); }
};
template <> struct CElem<float> {
    using store_t = float;
    static __device__ __forceinline__ float get(const store_t* p) { return *p; }
    static __device__ __forceinline__ void put(store_t* p, float v) { *p = v; }
};
template <> struct CElem<double> {
    using store_t = double;
    static __device__ __forceinline__ double get(const store_t* p) { return *p; }
    static __device__ __forceinline__ void put(store_t* p, double v) { *p = v; }
};

// Localisation and correction under the single-error-per-row model (paper section 2.2 "Error
// localization and correction"): D1 = C^{r1'} - C^{r1}, D2 = C^{r2'} - C^{r2}, column
// j = D2 / D1 - 1 for the linear weights w(k) = k + 1, correction C[i][j] -= D1.
// loc[i]: -1 row not flagged; -2 flagged but the ratio is not finite, further than 0.25 from an
// integer or outside 0..N-1 (more than one error, or an error too close to the rounding noise of
// the weighted sums); else the column.  delta[i] = D1 for flagged rows, 0 otherwise.
template <typename T>
__global__ __launch_bounds__(256) void locate_correct_kernel(void* __restrict__ Cv, int M, int N, int64_t ldc,
                                                             const typename Elem<T>::acc_t* __restrict__ expected,
                                                             const typename Elem<T>::acc_t* __restrict__ expected2,
                                                             const typename Elem<T>::acc_t* __restrict__ rowsum,
                                                             const typename Elem<T>::acc_t* __restrict__ rowsum2,
                                                             const int32_t* __restrict__ flags, int correct,
                                                             int32_t* __restrict__ loc,
                                                             typename Elem<T>::acc_t* __restrict__ delta,
                                                             int32_t* __restrict__ ncorrected) {
    using acc_t = typename Elem<T>::acc_t;
    using store_t = typename CElem<T>::store_t;
    const int i = blockIdx.x * 256 + threadIdx.x;
    int done = 0;
    if (i < M) {
        int l = -1;
        acc_t d = 0;
        if (flags[i]) {
            l = -2;
            const double d1 = (double)rowsum[i] - (double)expected[i];
            const double d2 = (double)rowsum2[i] - (double)expected2[i];
            d = (acc_t)d1;
            if (d1 != 0.0 && isfinite(d1) && isfinite(d2)) {
                const double q = d2 / d1 - 1.0;
                const double j = rint(q);
                if (isfinite(q) && fabs(q - j) <= 0.25 && j >= 0.0 && j <= (double)(N - 1)) {
                    l = (int)j;
                    if (correct) {
                        store_t* c = reinterpret_cast<store_t*>(Cv) + (int64_t)i * ldc + l;
                        CElem<T>::put(c, CElem<T>::get(c) - d);
                        done = 1;
                    }
                }
            }
        }
        loc[i] = l;
        delta[i] = d;
    }
    const int cnt = __syncthreads_count(done);
    if (threadIdx.x == 0 && cnt) atomicAdd(ncorrected, cnt);
}

static inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

static bool problem_ok(const vabft_problem* p) {
    if (!p) return false;
    if (p->M <= 0 || p->N <= 0 || p->K <= 0) return false;
    if (p->dtype < VABFT_F64 || p->dtype > VABFT_F8E5M2) return false;
    if (p->transB != 0 && p->transB != 1) return false;
    if (p->lda < p->K || p->ldc < p->N) return false;
    if (p->ldb < (p->transB ? p->K : p->N)) return false;
    return true;
}

// bytes of an element of A / B, and of C (an FP8 problem stores FP16)
static inline bool is_fp8(int dtype) { return dtype == VABFT_F8E4M3 || dtype == VABFT_F8E5M2; }
static inline size_t elem_bytes(int dtype) {
    return dtype == VABFT_F64 ? 8 : dtype == VABFT_F32 ? 4 : is_fp8(dtype) ? 1 : 2;
}
static inline size_t out_bytes(int dtype) { return is_fp8(dtype) ? 2 : elem_bytes(dtype); }
// types that run on the 256 x 256 tile kernels with FP32 accumulation
static inline bool is_tile256(int dtype) { return dtype == VABFT_F16 || dtype == VABFT_BF16 || is_fp8(dtype); }
static inline size_t acc_bytes(int dtype) { return dtype == VABFT_F64 ? 8 : 4; }
static inline bool aligned_to(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// FP32 / FP64 problems with fewer than 128 tiles of 128 x 128 (half the compute units or fewer would work) run
// 64 x 64 tiles instead: 256^3 is 16 workgroups of 16 k-tiles then, not 4.  The block-wise route keeps the large
// tile: its column blocks are what one wavefront of that tile sums.
static bool small_wide_tiles(const vabft_problem* p) {
    if (is_tile256(p->dtype)) return false;
    return (((int64_t)p->M + 127) / 128) * (((int64_t)p->N + 127) / 128) < 128;
}
static void tile_shape(const vabft_problem* p, bool blockwise, int* bm, int* bn) {
    if (is_tile256(p->dtype)) {
        *bm = 256;
        *bn = 256;
    } else if (!blockwise && small_wide_tiles(p)) {
        *bm = 64;
        *bn = 64;
    } else {
        *bm = 128;
        *bn = 128;
    }
}

// Workspace layout: [S area][tickets][scratch].
// S area (its place and size depend on B's shape only, never on M, so an encode of B stays valid for GEMMs
// with any number of rows): three doubles at +0 (the fold of the partials, when a kernel of its own has to
// make it), the encode's arrival counter at +32, the per-workgroup partials of S1..S3 of the last encode at
// +64, rounded up to 256 B.
// Tickets: tiles_m int32 arrival counters + one 64-bit counter, in a region of fixed size (TICKETS_REGION).  They
// must be zero between launches: the kernels leave them zero, vabft_workspace_init zeroes them the first time.
// The scratch area holds, for the GEMM, in units of tiles_n * M accumulator words: 16-bit
// types rowpart [0,1), apart [1,5), rowpart2 [5,6); wide types (two row-sum partials per
// tile-column) rowpart [0,2), rowpart2 [2,4), apart [4,8); then the column-sum partials.  The
// encode of an N x K B keeps its column partials there; the calls are ordered on one stream,
// so they share it.
static size_t s_area_bytes(const vabft_problem* p) {
    return round_up(64 + (size_t)s_partial_count(p) * 3 * sizeof(double), 256);
}
static size_t tickets_offset(const vabft_problem* p) { return s_area_bytes(p); }
// bytes of arrival counters a problem uses: tiles_m int32 + the 64-bit done counter, rounded to 256 B
static size_t tickets_used_bytes(const vabft_problem* p) {
    int bm, bn;
    tile_shape(p, false, &bm, &bn);  // the smaller tile of the two routes: the larger count
    const size_t tiles_m = ((size_t)p->M + bm - 1) / bm;
    return round_up((tiles_m + 4) * sizeof(int32_t), 256);
}
// The counters' region has a fixed size (64 KiB: 16 380 tile-rows, a million rows of the smallest tile), so the
// scratch area behind it starts at a place that depends on B's shape only.  Otherwise a call that shares the
// workspace with a problem of more rows (an encode of B made through a problem with few rows, say) would put its
// transient partials where the larger problem keeps counters that must stay zero.  Problems with more tile-rows
// than that get a larger region; they only share a workspace with problems of the same M.
constexpr size_t TICKETS_REGION = 64u << 10;
// everything in front of the scratch area
static size_t tickets_bytes(const vabft_problem* p) {
    const size_t used = tickets_used_bytes(p);
    return tickets_offset(p) + (used > TICKETS_REGION ? used : TICKETS_REGION);
}
static double* s_folded(const vabft_problem*, void* ws) { return reinterpret_cast<double*>(ws); }
static double* s_partials(const vabft_problem*, void* ws) {
    return reinterpret_cast<double*>(reinterpret_cast<unsigned char*>(ws) + 64);
}

__global__ __launch_bounds__(256) void fold_s_kernel(const double* __restrict__ partial, int count,
                                                     double* __restrict__ S) {
    __shared__ double s_red[12];
    fold_s_partials_to_lds(partial, count, threadIdx.x, s_red);
    __syncthreads();
    if (threadIdx.x < 3) S[threadIdx.x] = folded_s(s_red, threadIdx.x);
}
void fold_s_launch(const double* s_partial, int count, double* S, hipStream_t st) {
    fold_s_kernel<<<1, 256, 0, st>>>(s_partial, count, S);
}

// the encode's arrival counter (in the S area's header)
static int32_t* encode_ticket(const vabft_problem*, void* ws) {
    return reinterpret_cast<int32_t*>(reinterpret_cast<unsigned char*>(ws) + 32);
}

size_t gemm_workspace_bytes(const vabft_problem* p) {
    int bm, bn;
    tile_shape(p, false, &bm, &bn);  // the smaller tile of the two routes: the larger need
    const size_t tiles_n = ((size_t)p->N + bn - 1) / bn;
    const bool is16 = is_tile256(p->dtype);
    // 16-bit: rowpart + 4 A-statistics partials + weighted rowpart per tile-column; wide types: two
    // row-sum partials per tile-column (one per wavefront column), plain and weighted, + 4 A-statistics partials
    const size_t tiles_m = ((size_t)p->M + bm - 1) / bm;
    // ... and the column-sum partials: one (16-bit) or two (wide) vectors of N per tile-row
    return (tiles_n * (size_t)p->M * (is16 ? 6 : 8) + tiles_m * (size_t)p->N * (is16 ? 1 : 2)) * acc_bytes(p->dtype);
}

__global__ void fill_zero_kernel(uint32_t* p, size_t n) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0u;
}

void workspace_init_launch(void* ws, size_t bytes, hipStream_t st) {
    const size_t n = bytes / 4;
    const int blocks = (int)((n + 255) / 256 < 1024 ? (n + 255) / 256 : 1024);
    fill_zero_kernel<<<blocks > 0 ? blocks : 1, 256, 0, st>>>(reinterpret_cast<uint32_t*>(ws), n);
}

int gemm_dispatch(const vabft_problem* p, const void* dA, const void* dB, void* dC, void* d_expected, void* d_T,
                  int verify, const FusedArgs* fused, const vabft_inject* inj, void* d_rowsum, void* d_rowsum2,
                  void* d_E, int32_t* d_flags, int32_t* d_nflag, vabft_inject_rec* d_injlog, int32_t* d_ninj,
                  void* ws, hipStream_t st, const ColArgs* cols, const BlockArgs* blocks) {
    GemmArgs a;
    a.A = dA;
    a.B = dB;
    a.C = dC;
    a.M = p->M;
    a.N = p->N;
    a.K = p->K;
    a.lda = p->lda;
    a.ldb = p->ldb;
    a.ldc = p->ldc;
    int bm, bn;
    tile_shape(p, blocks != nullptr, &bm, &bn);
    a.tiles_m = (p->M + bm - 1) / bm;
    a.tiles_n = (p->N + bn - 1) / bn;
    const size_t eb = elem_bytes(p->dtype), ab = acc_bytes(p->dtype);
    const bool is16 = is_tile256(p->dtype);
    a.a_vec_ok = aligned_to(dA, 16) && (p->lda * eb) % 16 == 0;
    a.b_vec_ok = aligned_to(dB, 16) && (p->ldb * eb) % 16 == 0;
    a.c_vec_ok = aligned_to(dC, 16) && (p->ldc * out_bytes(p->dtype)) % 16 == 0;
    unsigned char* wsb = reinterpret_cast<unsigned char*>(ws);
    a.tickets = ws ? reinterpret_cast<int32_t*>(wsb + tickets_offset(p)) : nullptr;
    a.rowpart = ws ? wsb + tickets_bytes(p) : nullptr;
    a.apart = ws ? wsb + tickets_bytes(p) + (size_t)a.tiles_n * p->M * ab * (is16 ? 1 : 4) : nullptr;
    // weighted partials: behind rowpart + apart (16-bit) resp. behind the two plain partials (wide)
    a.rowpart2 = ws ? wsb + tickets_bytes(p) + (size_t)a.tiles_n * p->M * ab * (is16 ? 5 : 2) : nullptr;
    a.rowsum2 = d_rowsum2;
    a.colpart = ws ? wsb + tickets_bytes(p) + (size_t)a.tiles_n * p->M * ab * (is16 ? 6 : 8) : nullptr;
    a.d_ncolflag = cols ? cols->d_ncolflag : nullptr;
    a.block_mode = blocks ? 1 : 0;
    a.d_nblockflag = blocks ? blocks->d_nblockflag : nullptr;
    a.kprefix = nullptr;
    a.kblock_tiles = 0;
    a.d_nflag = d_nflag;
    a.expected = d_expected;
    a.T = d_T;
    a.rowsum = d_rowsum;
    a.E = d_E;
    a.flags = d_flags;
    a.fused_stats = 0;
    a.Be = nullptr;
    a.S = nullptr;
    a.s_partial = nullptr;
    a.s_nparts = 0;
    a.e_max = 0;
    a.c_sigma = 0;
    a.astat = nullptr;
    a.inj.mode = 0;
    a.inj.bit_lo = 0;
    a.inj.bit_span = 1;
    a.inj.n_list = 0;
    a.inj.seed = 0;
    a.inj.hit_limit = 0;
    a.inj.d_list = nullptr;
    a.inj.log_capacity = 0;
    a.inj.d_log = d_injlog;
    a.inj.d_ninj = d_ninj;
    if (inj && inj->mode != 0) {
        a.inj.mode = inj->mode;
        a.inj.bit_lo = inj->bit_lo;
        a.inj.bit_span = inj->bit_hi - inj->bit_lo + 1;
        a.inj.n_list = inj->n_list;
        a.inj.seed = inj->seed;
        a.inj.hit_limit = (uint64_t)floor(inj->rate * 9007199254740992.0);
        a.inj.d_list = inj->d_list;
        a.inj.log_capacity = inj->log_capacity;
        zero_int_kernel<<<1, 1, 0, st>>>(d_ninj);
    }
    // the unguarded kernels need whole tiles and 16-byte aligned rows
    const int bk = is_fp8(p->dtype) ? 256 : (is16 ? 64 : 16);
    // (the whole-tile 16-bit kernels address a tile's rows with 32-bit byte offsets from a per-wavefront base)
    const bool wide_rows = is16 && (p->lda > (1 << 24) || p->ldb > (1 << 24));
    // (the whole-tile FP8 kernel exists for B stored N x K only; a K x N B takes the guarded kernel)
    const bool edge = (p->M % bm) || (p->N % bn) || (p->K % bk) || !a.a_vec_ok || !a.b_vec_ok || !a.c_vec_ok ||
                      wide_rows || (is_fp8(p->dtype) && !p->transB);
    // whole-tile kernels do the compare-and-flag step (and, if asked, the A-side pass) in-kernel
    const bool in_kernel_finalize = !edge;
    if (fused) {
        // the fused 16-bit kernel caches the checksum panel of the k-units a tile-column folds: at most 16
        // (units of 128 k, dealt round-robin to the tile-columns; the FP8 kernel: units of 256 k, 8 slots,
        // B stored N x K)
        const bool fits16 = is_fp8(p->dtype)
                                ? (a.tiles_n >= 2 && p->K % 256 == 0 && p->transB && (p->K / 256) / a.tiles_n + 2 <= 8)
                                : (p->K % 128 == 0 && (p->K / 128 + a.tiles_n - 1) / a.tiles_n <= 16);
        if (in_kernel_finalize && (!is16 || fits16)) {
            a.fused_stats = 1;
            a.Be = fused->d_Be;
            a.S = fused->d_S;
            a.s_partial = s_partials(p, ws);
            a.s_nparts = s_partial_count(p);
            a.e_max = fused->e_max;
            a.c_sigma = fused->c_sigma;
            a.astat = fused->d_astat;
        } else {
            const double* dS = fused->d_S;
            if (!dS) {  // the pass of its own needs S1..S3 folded
                fold_s_launch(s_partials(p, ws), s_partial_count(p), s_folded(p, ws), st);
                dS = s_folded(p, ws);
            }
            const int rc = threshold_dispatch(p, dA, fused->d_Be, nullptr, dS, fused->e_max, fused->c_sigma,
                                              fused->d_astat, d_expected, nullptr, d_T, st);
            if (rc != VABFT_OK) return rc;
        }
    }
    int rc;
    // injector runs form every kind of sum; otherwise one extra kind per launch
    int mode = !verify ? 0 : (a.inj.mode != 0 ? 2 : (cols ? 4 : (d_rowsum2 ? 3 : 1)));
    if (cols && d_rowsum2 && mode != 2) return VABFT_EUNSUPPORTED;
    if (blocks) {
        if (cols || d_rowsum2) return VABFT_EUNSUPPORTED;
        if (mode == 1 && in_kernel_finalize && is16) mode = 5;  // partials only, no in-kernel compare (the wide
                                                                // kernels read block_mode at run time)
        if (blocks->kblock > 0) {
            // K split as well: the 16-bit whole-tile kernel leaves a prefix of the row sums per K-block
            if ((p->dtype != VABFT_BF16 && p->dtype != VABFT_F16) || edge) return VABFT_EUNSUPPORTED;
            mode = a.inj.mode != 0 ? 7 : 6;
            a.kprefix = blocks->kprefix;
            a.kblock_tiles = blocks->kblock / 64;
        }
    }
    switch (p->dtype) {
        case VABFT_F8E4M3:
        case VABFT_F8E5M2:
            if (edge)
                rc = gemm16_launch_f8_edge(a, mode, p->dtype == VABFT_F8E5M2, p->transB, st);
            else
                rc = p->dtype == VABFT_F8E4M3 ? gemm8_launch_f8_nt(a, mode, st) : gemm8_launch_bf8_nt(a, mode, st);
            break;
        case VABFT_BF16:
            rc = p->transB ? gemm16_launch_bf16_nt(a, mode, edge, st) : gemm16_launch_bf16_nn(a, mode, edge, st);
            break;
        case VABFT_F16:
            rc = p->transB ? gemm16_launch_f16_nt(a, mode, edge, st) : gemm16_launch_f16_nn(a, mode, edge, st);
            break;
        case VABFT_F32: rc = gemmw_launch_f32(a, p->transB, mode, edge, bm / 2, st); break;
        case VABFT_F64: rc = gemmw_launch_f64(a, p->transB, mode, edge, bm / 2, st); break;
        default: return VABFT_EINVAL;
    }
    if (rc != VABFT_OK || !verify) return rc;
    if (blocks && blocks->kblock > 0)
        return finalize_blocks_k_dispatch(p, (p->K + blocks->kblock - 1) / blocks->kblock, blocks->kprefix,
                                          blocks->d_expected_blk, blocks->d_T_blk, blocks->d_rowsum_blk, blocks->d_E_blk,
                                          blocks->d_blockflags, d_E, d_flags, d_nflag, blocks->d_nblockflag, st);
    if (blocks)
        return finalize_blocks_dispatch(p, a.rowpart, blocks->d_expected_blk, blocks->d_T_blk, blocks->d_rowsum_blk,
                                        blocks->d_E_blk, blocks->d_blockflags, d_E, d_flags, d_nflag,
                                        blocks->d_nblockflag, st);
    if (cols) {
        const dim3 cgrid((p->N + 255) / 256), cblock(256);
        const int ncparts = is16 ? a.tiles_m : 2 * a.tiles_m;
        if (p->dtype == VABFT_F64)
            finalize_cols_kernel<double><<<cgrid, cblock, 0, st>>>(
                (const double*)a.colpart, ncparts, p->N, (const double*)cols->d_expected_col,
                (const double*)cols->d_Tcol, (double*)cols->d_colsum, (double*)cols->d_Ecol, cols->d_colflags,
                cols->d_ncolflag);
        else
            finalize_cols_kernel<float><<<cgrid, cblock, 0, st>>>(
                (const float*)a.colpart, ncparts, p->N, (const float*)cols->d_expected_col, (const float*)cols->d_Tcol,
                (float*)cols->d_colsum, (float*)cols->d_Ecol, cols->d_colflags, cols->d_ncolflag);
        if (hipGetLastError() != hipSuccess) return VABFT_EDEVICE;
    }
    if (in_kernel_finalize) return rc;
    const dim3 grid((p->M + 255) / 256), block(256);
    const int nparts = is16 ? a.tiles_n : 2 * a.tiles_n;
    if (p->dtype == VABFT_F64)
        finalize_kernel<double><<<grid, block, 0, st>>>((const double*)a.rowpart, nparts, p->M,
                                                        (const double*)d_expected, (const double*)d_T,
                                                        (double*)d_rowsum, (double*)d_E, d_flags, d_nflag,
                                                        (const double*)a.rowpart2, (double*)d_rowsum2);
    else
        finalize_kernel<float><<<grid, block, 0, st>>>((const float*)a.rowpart, nparts, p->M,
                                                       (const float*)d_expected, (const float*)d_T, (float*)d_rowsum,
                                                       (float*)d_E, d_flags, d_nflag, (const float*)a.rowpart2,
                                                       (float*)d_rowsum2);
    return hipGetLastError() == hipSuccess ? VABFT_OK : VABFT_EDEVICE;
}

// Scratch of the entry point that allocates nothing (vabft_gemm_verified_fused_static): device memory that
// lives in the library's code object, one copy per GPU, held until the process ends.  In host code the array's
// name is only a handle for hipGetSymbolAddress; kernels receive the address that call returns.
static __device__ __align__(256) unsigned char scratch[VABFT_STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[MAX_DEVICES] = {};

// address of the current device's copy of `scratch` (looked up once per device); null on failure
static void* static_scratch_of_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

}  // namespace vabft

using namespace vabft;

extern "C" {

const char* vabft_status_string(int status) {
    switch (status) {
        case VABFT_OK: return "ok";
        case VABFT_EINVAL: return "invalid argument";
        case VABFT_EUNSUPPORTED: return "unsupported dtype or layout";
        case VABFT_EWORKSPACE: return "workspace missing or too small";
        case VABFT_EDEVICE: return "HIP runtime error at launch";
    }
    return "unknown status";
}

size_t vabft_workspace_bytes(const vabft_problem* p) {
    if (!problem_ok(p)) return 0;
    const size_t a = encode_workspace_bytes(p), b = gemm_workspace_bytes(p), c = cols_workspace_bytes(p),
                 d = blocks_workspace_bytes(p);
    size_t m = a > b ? a : b;
    m = m > c ? m : c;
    m = m > d ? m : d;
    return tickets_bytes(p) + round_up(m + 256, 256);
}

int vabft_workspace_init(void* d_workspace, size_t workspace_bytes, void* stream) {
    if (!d_workspace || workspace_bytes < 4 || !aligned_to(d_workspace, 16)) return VABFT_EWORKSPACE;
    workspace_init_launch(d_workspace, workspace_bytes, (hipStream_t)stream);
    return hipGetLastError() == hipSuccess ? VABFT_OK : VABFT_EDEVICE;
}

double vabft_default_emax(int32_t dtype, int32_t K, int32_t N) {
    // The larger of (a) the paper's recommended GPU law (table "Recommended e_max across
    // platforms", H100 rows) and (b) a law measured on MI355X with these kernels by the paper's
    // calibration protocol (|N(1,1)| matrices, max |E| / |checksum| over trials, +20 %).  Measured over
    // n = 128 .. 8192, both layouts of B, 100 000 trials per size: the relative difference is 3.1 - 6.0 u for
    // BF16 / FP16 / FP32 and 4.4 - 4.5 u for FP64, flat in n (every sum is a tree), which is above (a) at
    // small n.  (b) lies at least 25 % above every +20 % value of that table, i.e. at least 50 % above every
    // observed maximum; tests/test_library_cpu.py holds it to that against the committed table.
    const double n = (double)(K > N ? K : N);
    double paper, measured;
    // FP8: the 32x32x64 matrix instruction does not carry full FP32 precision through its 64-term dot
    // product; measured by the same protocol (n = 256 .. 8192, B stored N x K, 25 000 - 100 000 trials per size) the
    // relative difference is 31 - 72 u_FP32 for E4M3 and 18 - 48 u_FP32 for E5M2, largest at small n: a constant
    // 25 % above the largest +20 % value (5.15e-6).
    if (is_fp8(dtype)) return 6.5e-6;
    if (dtype == VABFT_F64) {
        paper = 1.0e-17 * sqrt(n) + 2.5e-16;
        measured = 8.0e-18 * sqrt(n) + 7.0e-16;
    } else {
        paper = 5.0e-9 * sqrt(n) + 1.2e-7;
        measured = 3.0e-9 * sqrt(n) + 4.2e-7;
    }
    return paper > measured ? paper : measured;
}

double vabft_default_emax_offline(int32_t dtype, int32_t K, int32_t N) {
    // section 3.6 "Practical recommendations": a check made after a 16-bit write-back sees one
    // rounding of every element to the output type, e_max ~ 2 u_output
    if (dtype == VABFT_BF16) return 2.0 * 0.00390625;       // 2 * 2^-8
    if (dtype == VABFT_F16 || is_fp8(dtype)) return 2.0 * 0.00048828125;  // 2 * 2^-11 (FP16 output)
    return vabft_default_emax(dtype, K, N);
}

int vabft_check_offline(const vabft_problem* p, const void* dC, const void* d_expected, const void* d_T,
                        void* d_rowsum, void* d_E, int32_t* d_flags, int32_t* d_nflag, void* stream) {
    if (!problem_ok(p) || !dC || !d_expected || !d_T || !d_rowsum || !d_E || !d_flags || !d_nflag) return VABFT_EINVAL;
    const size_t ab = acc_bytes(p->dtype);
    if (!aligned_to(dC, out_bytes(p->dtype)) || !aligned_to(d_expected, ab) || !aligned_to(d_T, ab) ||
        !aligned_to(d_rowsum, ab) || !aligned_to(d_E, ab) || !aligned_to(d_flags, 4) || !aligned_to(d_nflag, 4))
        return VABFT_EINVAL;
    zero_int_kernel<<<1, 1, 0, (hipStream_t)stream>>>(d_nflag);
    return check_offline_dispatch(p, dC, d_expected, d_T, d_rowsum, d_E, d_flags, d_nflag, (hipStream_t)stream);
}

int vabft_encode(const vabft_problem* p, const void* dB, void* d_Be, void* d_bstat, double* d_S, void* d_workspace,
                 size_t workspace_bytes, void* stream) {
    if (!problem_ok(p) || !dB || !d_Be || !d_bstat) return VABFT_EINVAL;  // d_S may be null: deferred fold
    if (!aligned_to(dB, elem_bytes(p->dtype)) || !aligned_to(d_Be, acc_bytes(p->dtype)) ||
        !aligned_to(d_bstat, acc_bytes(p->dtype)) || !aligned_to(d_S, 8))
        return VABFT_EINVAL;
    const size_t need = encode_workspace_bytes(p);
    if (!d_workspace || workspace_bytes < tickets_bytes(p) + need || !aligned_to(d_workspace, 16))
        return VABFT_EWORKSPACE;
    void* scratch = reinterpret_cast<unsigned char*>(d_workspace) + tickets_bytes(p);
    return encode_dispatch(p, dB, d_Be, nullptr, d_bstat, d_S, s_partials(p, d_workspace), scratch,
                           encode_ticket(p, d_workspace), (hipStream_t)stream);
}

int vabft_encode_weighted(const vabft_problem* p, const void* dB, void* d_Be, void* d_Be2, void* d_bstat, double* d_S,
                          void* d_workspace, size_t workspace_bytes, void* stream) {
    if (!problem_ok(p) || !dB || !d_Be || !d_Be2 || !d_bstat || !d_S) return VABFT_EINVAL;
    if (!aligned_to(dB, elem_bytes(p->dtype)) || !aligned_to(d_Be, acc_bytes(p->dtype)) ||
        !aligned_to(d_Be2, acc_bytes(p->dtype)) || !aligned_to(d_bstat, acc_bytes(p->dtype)) || !aligned_to(d_S, 8))
        return VABFT_EINVAL;
    const size_t need = encode_workspace_bytes(p);
    if (!d_workspace || workspace_bytes < tickets_bytes(p) + need || !aligned_to(d_workspace, 16))
        return VABFT_EWORKSPACE;
    void* scratch = reinterpret_cast<unsigned char*>(d_workspace) + tickets_bytes(p);
    return encode_dispatch(p, dB, d_Be, d_Be2, d_bstat, d_S, s_partials(p, d_workspace), scratch,
                           encode_ticket(p, d_workspace), (hipStream_t)stream);
}

int vabft_threshold(const vabft_problem* p, const void* dA, const void* d_Be, const double* d_S, double e_max,
                    double c_sigma, void* d_astat, void* d_expected, void* d_T, void* stream) {
    if (!problem_ok(p) || !dA || !d_Be || !d_S || !d_astat || !d_expected || !d_T) return VABFT_EINVAL;
    if (!(e_max > 0.0) || !(c_sigma >= 0.0) || !isfinite(e_max) || !isfinite(c_sigma)) return VABFT_EINVAL;
    const size_t ab = acc_bytes(p->dtype);
    if (!aligned_to(dA, elem_bytes(p->dtype)) || !aligned_to(d_Be, ab) || !aligned_to(d_S, 8) ||
        !aligned_to(d_astat, ab) || !aligned_to(d_expected, ab) || !aligned_to(d_T, ab))
        return VABFT_EINVAL;
    return threshold_dispatch(p, dA, d_Be, nullptr, d_S, e_max, c_sigma, d_astat, d_expected, nullptr, d_T,
                              (hipStream_t)stream);
}

int vabft_threshold_weighted(const vabft_problem* p, const void* dA, const void* d_Be, const void* d_Be2,
                             const double* d_S, double e_max, double c_sigma, void* d_astat, void* d_expected,
                             void* d_expected2, void* d_T, void* stream) {
    if (!problem_ok(p) || !dA || !d_Be || !d_Be2 || !d_S || !d_astat || !d_expected || !d_expected2 || !d_T)
        return VABFT_EINVAL;
    if (!(e_max > 0.0) || !(c_sigma >= 0.0) || !isfinite(e_max) || !isfinite(c_sigma)) return VABFT_EINVAL;
    const size_t ab = acc_bytes(p->dtype);
    if (!aligned_to(dA, elem_bytes(p->dtype)) || !aligned_to(d_Be, ab) || !aligned_to(d_Be2, ab) ||
        !aligned_to(d_S, 8) || !aligned_to(d_astat, ab) || !aligned_to(d_expected, ab) ||
        !aligned_to(d_expected2, ab) || !aligned_to(d_T, ab))
        return VABFT_EINVAL;
    return threshold_dispatch(p, dA, d_Be, d_Be2, d_S, e_max, c_sigma, d_astat, d_expected, d_expected2, d_T,
                              (hipStream_t)stream);
}

static int check_gemm_args(const vabft_problem* p, const void* dA, const void* dB, void* dC, int verify,
                           const vabft_inject* inj, const void* d_expected, const void* d_T, void* d_rowsum,
                           void* d_E, int32_t* d_flags, int32_t* d_nflag, vabft_inject_rec* d_injlog, int32_t* d_ninj,
                           void* d_workspace, size_t workspace_bytes) {
    if (!problem_ok(p) || !dA || !dB || !dC) return VABFT_EINVAL;
    if (verify != 0 && verify != 1) return VABFT_EINVAL;
    const size_t eb = elem_bytes(p->dtype), ab = acc_bytes(p->dtype);
    if (!aligned_to(dA, eb) || !aligned_to(dB, eb) || !aligned_to(dC, out_bytes(p->dtype))) return VABFT_EINVAL;
    const bool inj_on = inj && inj->mode != 0;
    if (verify) {
        if (!d_expected || !d_T || !d_rowsum || !d_E || !d_flags || !d_nflag) return VABFT_EINVAL;
        if (!aligned_to(d_expected, ab) || !aligned_to(d_T, ab) || !aligned_to(d_rowsum, ab) || !aligned_to(d_E, ab) ||
            !aligned_to(d_flags, 4) || !aligned_to(d_nflag, 4))
            return VABFT_EINVAL;
        const size_t need = tickets_bytes(p) + gemm_workspace_bytes(p);
        if (!d_workspace || workspace_bytes < need || !aligned_to(d_workspace, 16)) return VABFT_EWORKSPACE;
    } else if (inj_on) {
        return VABFT_EINVAL;  // the injector lives in the verified kernel
    }
    if (inj_on) {
        const int bits = (int)ab * 8;
        if (inj->mode != 1 && inj->mode != 2) return VABFT_EINVAL;
        if (!d_ninj || inj->log_capacity < 0 || (inj->log_capacity > 0 && !d_injlog)) return VABFT_EINVAL;
        if (inj->mode == 1 && (inj->n_list < 0 || (inj->n_list > 0 && !inj->d_list))) return VABFT_EINVAL;
        if (inj->mode == 2) {
            if (!(inj->rate >= 0.0 && inj->rate <= 1.0)) return VABFT_EINVAL;
            if (inj->bit_lo < 0 || inj->bit_hi < inj->bit_lo || inj->bit_hi >= bits) return VABFT_EINVAL;
        }
    }
    return VABFT_OK;
}

int vabft_gemm_verified(const vabft_problem* p, const void* dA, const void* dB, void* dC, const void* d_expected,
                        const void* d_T, int32_t verify, const vabft_inject* inj, void* d_rowsum, void* d_E,
                        int32_t* d_flags, int32_t* d_nflag, vabft_inject_rec* d_injlog, int32_t* d_ninj,
                        void* d_workspace, size_t workspace_bytes, void* stream) {
    const int rc = check_gemm_args(p, dA, dB, dC, verify, inj, d_expected, d_T, d_rowsum, d_E, d_flags, d_nflag,
                                   d_injlog, d_ninj, d_workspace, workspace_bytes);
    if (rc != VABFT_OK) return rc;
    return gemm_dispatch(p, dA, dB, dC, const_cast<void*>(d_expected), const_cast<void*>(d_T), verify, nullptr, inj,
                         d_rowsum, nullptr, d_E, d_flags, d_nflag, d_injlog, d_ninj, d_workspace, (hipStream_t)stream);
}

int vabft_gemm_verified_weighted(const vabft_problem* p, const void* dA, const void* dB, void* dC,
                                 const void* d_expected, const void* d_T, const vabft_inject* inj, void* d_rowsum,
                                 void* d_rowsum2, void* d_E, int32_t* d_flags, int32_t* d_nflag,
                                 vabft_inject_rec* d_injlog, int32_t* d_ninj, void* d_workspace,
                                 size_t workspace_bytes, void* stream) {
    const int rc = check_gemm_args(p, dA, dB, dC, 1, inj, d_expected, d_T, d_rowsum, d_E, d_flags, d_nflag, d_injlog,
                                   d_ninj, d_workspace, workspace_bytes);
    if (rc != VABFT_OK) return rc;
    if (!d_rowsum2 || !aligned_to(d_rowsum2, acc_bytes(p->dtype))) return VABFT_EINVAL;
    return gemm_dispatch(p, dA, dB, dC, const_cast<void*>(d_expected), const_cast<void*>(d_T), 1, nullptr, inj,
                         d_rowsum, d_rowsum2, d_E, d_flags, d_nflag, d_injlog, d_ninj, d_workspace,
                         (hipStream_t)stream);
}

int vabft_encode_a(const vabft_problem* p, const void* dA, void* d_eA, void* d_acolstat, double* d_SA,
                   void* d_workspace, size_t workspace_bytes, void* stream) {
    if (!problem_ok(p) || !dA || !d_eA || !d_acolstat || !d_SA) return VABFT_EINVAL;
    const size_t ab = acc_bytes(p->dtype);
    if (!aligned_to(dA, elem_bytes(p->dtype)) || !aligned_to(d_eA, ab) || !aligned_to(d_acolstat, ab) ||
        !aligned_to(d_SA, 8))
        return VABFT_EINVAL;
    if (!d_workspace || workspace_bytes < tickets_bytes(p) + cols_workspace_bytes(p) || !aligned_to(d_workspace, 16))
        return VABFT_EWORKSPACE;
    void* scratch = reinterpret_cast<unsigned char*>(d_workspace) + tickets_bytes(p);
    return encode_a_dispatch(p, dA, d_eA, d_acolstat, d_SA, s_partials(p, d_workspace), scratch,
                             encode_ticket(p, d_workspace), (hipStream_t)stream);
}

int vabft_threshold_cols(const vabft_problem* p, const void* dB, const void* d_eA, const double* d_SA, double e_max,
                         double c_sigma, void* d_bcolstat, void* d_expected_col, void* d_Tcol, void* d_workspace,
                         size_t workspace_bytes, void* stream) {
    if (!problem_ok(p) || !dB || !d_eA || !d_SA || !d_bcolstat || !d_expected_col || !d_Tcol) return VABFT_EINVAL;
    if (!(e_max > 0.0) || !(c_sigma >= 0.0) || !isfinite(e_max) || !isfinite(c_sigma)) return VABFT_EINVAL;
    const size_t ab = acc_bytes(p->dtype);
    if (!aligned_to(dB, elem_bytes(p->dtype)) || !aligned_to(d_eA, ab) || !aligned_to(d_SA, 8) ||
        !aligned_to(d_bcolstat, ab) || !aligned_to(d_expected_col, ab) || !aligned_to(d_Tcol, ab))
        return VABFT_EINVAL;
    if (!d_workspace || workspace_bytes < tickets_bytes(p) + cols_workspace_bytes(p) || !aligned_to(d_workspace, 16))
        return VABFT_EWORKSPACE;
    void* scratch = reinterpret_cast<unsigned char*>(d_workspace) + tickets_bytes(p);
    return threshold_cols_dispatch(p, dB, d_eA, d_SA, e_max, c_sigma, d_bcolstat, d_expected_col, d_Tcol, scratch,
                                   (hipStream_t)stream);
}

int vabft_gemm_verified_rc(const vabft_problem* p, const void* dA, const void* dB, void* dC, const void* d_expected,
                           const void* d_T, const void* d_expected_col, const void* d_Tcol, const vabft_inject* inj,
                           void* d_rowsum, void* d_E, int32_t* d_flags, int32_t* d_nflag, void* d_colsum, void* d_Ecol,
                           int32_t* d_colflags, int32_t* d_ncolflag, vabft_inject_rec* d_injlog, int32_t* d_ninj,
                           void* d_workspace, size_t workspace_bytes, void* stream) {
    const int rc = check_gemm_args(p, dA, dB, dC, 1, inj, d_expected, d_T, d_rowsum, d_E, d_flags, d_nflag, d_injlog,
                                   d_ninj, d_workspace, workspace_bytes);
    if (rc != VABFT_OK) return rc;
    if (!d_expected_col || !d_Tcol || !d_colsum || !d_Ecol || !d_colflags || !d_ncolflag) return VABFT_EINVAL;
    const size_t ab = acc_bytes(p->dtype);
    if (!aligned_to(d_expected_col, ab) || !aligned_to(d_Tcol, ab) || !aligned_to(d_colsum, ab) ||
        !aligned_to(d_Ecol, ab) || !aligned_to(d_colflags, 4) || !aligned_to(d_ncolflag, 4))
        return VABFT_EINVAL;
    ColArgs c;
    c.d_expected_col = d_expected_col;
    c.d_Tcol = d_Tcol;
    c.d_colsum = d_colsum;
    c.d_Ecol = d_Ecol;
    c.d_colflags = d_colflags;
    c.d_ncolflag = d_ncolflag;
    return gemm_dispatch(p, dA, dB, dC, const_cast<void*>(d_expected), const_cast<void*>(d_T), 1, nullptr, inj,
                         d_rowsum, nullptr, d_E, d_flags, d_nflag, d_injlog, d_ninj, d_workspace, (hipStream_t)stream,
                         &c);
}

int32_t vabft_block_width(int32_t dtype) { return block_width(dtype); }

int vabft_encode_blocks(const vabft_problem* p, const void* dB, void* d_Be_blk, double* d_S_blk, void* d_workspace,
                        size_t workspace_bytes, void* stream) {
    if (!problem_ok(p) || !dB || !d_Be_blk || !d_S_blk) return VABFT_EINVAL;
    if (!aligned_to(dB, elem_bytes(p->dtype)) || !aligned_to(d_Be_blk, acc_bytes(p->dtype)) || !aligned_to(d_S_blk, 8))
        return VABFT_EINVAL;
    if (!d_workspace || workspace_bytes < tickets_bytes(p) + blocks_workspace_bytes(p) || !aligned_to(d_workspace, 16))
        return VABFT_EWORKSPACE;
    void* scratch = reinterpret_cast<unsigned char*>(d_workspace) + tickets_bytes(p);
    return encode_blocks_dispatch(p, dB, d_Be_blk, d_S_blk, scratch, (hipStream_t)stream);
}

int vabft_threshold_blocks(const vabft_problem* p, const void* dA, const void* d_Be_blk, const double* d_S_blk,
                           double e_max, double c_sigma, void* d_astat, void* d_expected_blk, void* d_T_blk,
                           void* stream) {
    if (!problem_ok(p) || !dA || !d_Be_blk || !d_S_blk || !d_astat || !d_expected_blk || !d_T_blk) return VABFT_EINVAL;
    if (!(e_max > 0.0) || !(c_sigma >= 0.0) || !isfinite(e_max) || !isfinite(c_sigma)) return VABFT_EINVAL;
    const size_t ab = acc_bytes(p->dtype);
    if (!aligned_to(dA, elem_bytes(p->dtype)) || !aligned_to(d_Be_blk, ab) || !aligned_to(d_S_blk, 8) ||
        !aligned_to(d_astat, ab) || !aligned_to(d_expected_blk, ab) || !aligned_to(d_T_blk, ab))
        return VABFT_EINVAL;
    return threshold_blocks_dispatch(p, dA, d_Be_blk, d_S_blk, e_max, c_sigma, d_astat, d_expected_blk, d_T_blk,
                                     (hipStream_t)stream);
}

int vabft_gemm_verified_blocks(const vabft_problem* p, const void* dA, const void* dB, void* dC,
                               const void* d_expected_blk, const void* d_T_blk, const vabft_inject* inj,
                               void* d_rowsum_blk, void* d_E_blk, int32_t* d_blockflags, int32_t* d_nblockflag,
                               void* d_E, int32_t* d_flags, int32_t* d_nflag, vabft_inject_rec* d_injlog,
                               int32_t* d_ninj, void* d_workspace, size_t workspace_bytes, void* stream) {
    // the row-level vectors of the plain check are not inputs here: pass the block vectors through the checker
    const int rc = check_gemm_args(p, dA, dB, dC, 1, inj, d_expected_blk, d_T_blk, d_rowsum_blk, d_E, d_flags, d_nflag,
                                   d_injlog, d_ninj, d_workspace, workspace_bytes);
    if (rc != VABFT_OK) return rc;
    if (!d_E_blk || !d_blockflags || !d_nblockflag) return VABFT_EINVAL;
    if (!aligned_to(d_E_blk, acc_bytes(p->dtype)) || !aligned_to(d_blockflags, 4) || !aligned_to(d_nblockflag, 4))
        return VABFT_EINVAL;
    BlockArgs b;
    b.d_expected_blk = d_expected_blk;
    b.d_T_blk = d_T_blk;
    b.d_rowsum_blk = d_rowsum_blk;
    b.d_E_blk = d_E_blk;
    b.d_blockflags = d_blockflags;
    b.d_nblockflag = d_nblockflag;
    return gemm_dispatch(p, dA, dB, dC, nullptr, nullptr, 1, nullptr, inj, nullptr, nullptr, d_E, d_flags, d_nflag,
                         d_injlog, d_ninj, d_workspace, (hipStream_t)stream, nullptr, &b);
}

// ---- block-wise verification with K split as well -----------------------------------------------------------
// The K-blocks of the encode and threshold passes are sub-problems of the column-block passes: K-block b is the
// problem (M, N, len_b) on A + b*kblock columns and on the K-block's rows (K x N layout) or columns (N x K layout)
// of B.  They run on a part of the workspace of their own, behind everything the whole problem uses, so that
// their scratch never lands where the whole problem keeps counters that must stay zero.
static bool kblock_ok(const vabft_problem* p, int32_t kblock) { return kblock > 0 && kblock % 128 == 0; }
static int kblock_count(const vabft_problem* p, int32_t kblock) { return (p->K + kblock - 1) / kblock; }
static vabft_problem kblock_problem(const vabft_problem* p, int32_t kblock, int b) {
    vabft_problem q = *p;
    q.K = (b + 1) * kblock <= p->K ? kblock : p->K - b * kblock;
    return q;
}
static size_t kprefix_bytes(const vabft_problem* p, int32_t kblock) {
    const size_t tiles_n = ((size_t)p->N + 255) / 256;
    return round_up((size_t)kblock_count(p, kblock) * 2 * tiles_n * (size_t)p->M * sizeof(double), 256);
}
// [ workspace of the whole problem | K-block prefixes | workspace of one K-block sub-problem ]
static size_t kblock_sub_offset(const vabft_problem* p, int32_t kblock) {
    return round_up(vabft_workspace_bytes(p), 256) + kprefix_bytes(p, kblock);
}

int32_t vabft_kblock_count(const vabft_problem* p, int32_t kblock) {
    return (problem_ok(p) && kblock_ok(p, kblock)) ? kblock_count(p, kblock) : 0;
}

size_t vabft_workspace_bytes_blocks_k(const vabft_problem* p, int32_t kblock) {
    if (!problem_ok(p) || !kblock_ok(p, kblock)) return 0;
    const vabft_problem q = kblock_problem(p, kblock, 0);  // the largest K-block
    return kblock_sub_offset(p, kblock) + vabft_workspace_bytes(&q);
}

int vabft_encode_blocks_k(const vabft_problem* p, int32_t kblock, const void* dB, void* d_Be_blk_k, double* d_S_blk_k,
                          void* d_workspace, size_t workspace_bytes, void* stream) {
    if (!problem_ok(p) || !kblock_ok(p, kblock) || !dB || !d_Be_blk_k || !d_S_blk_k) return VABFT_EINVAL;
    if (!d_workspace || workspace_bytes < vabft_workspace_bytes_blocks_k(p, kblock) || !aligned_to(d_workspace, 16))
        return VABFT_EWORKSPACE;
    const size_t eb = elem_bytes(p->dtype), ab = acc_bytes(p->dtype);
    const int W = block_width(p->dtype), nblocks = (p->N + W - 1) / W, nkb = kblock_count(p, kblock);
    unsigned char* sub = reinterpret_cast<unsigned char*>(d_workspace) + kblock_sub_offset(p, kblock);
    for (int b = 0; b < nkb; ++b) {
        const vabft_problem q = kblock_problem(p, kblock, b);
        const size_t k0 = (size_t)b * kblock;
        const unsigned char* Bb = reinterpret_cast<const unsigned char*>(dB) + (p->transB ? k0 : k0 * (size_t)p->ldb) * eb;
        void* be = reinterpret_cast<unsigned char*>(d_Be_blk_k) + (size_t)nblocks * k0 * ab;
        const int rc = vabft_encode_blocks(&q, Bb, be, d_S_blk_k + (size_t)b * nblocks * 3, sub,
                                           workspace_bytes - kblock_sub_offset(p, kblock), stream);
        if (rc != VABFT_OK) return rc;
    }
    return VABFT_OK;
}

int vabft_threshold_blocks_k(const vabft_problem* p, int32_t kblock, const void* dA, const void* d_Be_blk_k,
                             const double* d_S_blk_k, double e_max, double c_sigma, void* d_astat_k,
                             void* d_expected_blk_k, void* d_T_blk_k, void* stream) {
    if (!problem_ok(p) || !kblock_ok(p, kblock) || !dA || !d_Be_blk_k || !d_S_blk_k || !d_astat_k || !d_expected_blk_k ||
        !d_T_blk_k)
        return VABFT_EINVAL;
    const size_t eb = elem_bytes(p->dtype), ab = acc_bytes(p->dtype);
    const int W = block_width(p->dtype), nblocks = (p->N + W - 1) / W, nkb = kblock_count(p, kblock);
    for (int b = 0; b < nkb; ++b) {
        const vabft_problem q = kblock_problem(p, kblock, b);
        const size_t k0 = (size_t)b * kblock;
        const unsigned char* Ab = reinterpret_cast<const unsigned char*>(dA) + k0 * eb;
        const void* be = reinterpret_cast<const unsigned char*>(d_Be_blk_k) + (size_t)nblocks * k0 * ab;
        const size_t piece = (size_t)b * nblocks * (size_t)p->M * ab;
        // K-block b's share is what the running accumulator gained while it already held b blocks: the rounding of
        // that accumulation goes with the running magnitude, (b + 1) blocks deep, not with the block's own terms.
        // e_max, the relative rounding error per unit of checksum magnitude, is therefore taken (b + 1)-fold.
        const int rc = vabft_threshold_blocks(&q, Ab, be, d_S_blk_k + (size_t)b * nblocks * 3, e_max * (b + 1), c_sigma,
                                              reinterpret_cast<unsigned char*>(d_astat_k) + (size_t)b * 3 * p->M * ab,
                                              reinterpret_cast<unsigned char*>(d_expected_blk_k) + piece,
                                              reinterpret_cast<unsigned char*>(d_T_blk_k) + piece, stream);
        if (rc != VABFT_OK) return rc;
    }
    return VABFT_OK;
}

int vabft_gemm_verified_blocks_k(const vabft_problem* p, int32_t kblock, const void* dA, const void* dB, void* dC,
                                 const void* d_expected_blk_k, const void* d_T_blk_k, const vabft_inject* inj,
                                 void* d_rowsum_blk_k, void* d_E_blk_k, int32_t* d_blockflags_k, int32_t* d_nblockflag,
                                 void* d_E, int32_t* d_flags, int32_t* d_nflag, vabft_inject_rec* d_injlog,
                                 int32_t* d_ninj, void* d_workspace, size_t workspace_bytes, void* stream) {
    if (!problem_ok(p) || !kblock_ok(p, kblock)) return VABFT_EINVAL;
    const int rc = check_gemm_args(p, dA, dB, dC, 1, inj, d_expected_blk_k, d_T_blk_k, d_rowsum_blk_k, d_E, d_flags,
                                   d_nflag, d_injlog, d_ninj, d_workspace, workspace_bytes);
    if (rc != VABFT_OK) return rc;
    if (workspace_bytes < vabft_workspace_bytes_blocks_k(p, kblock)) return VABFT_EWORKSPACE;
    if (!d_E_blk_k || !d_blockflags_k || !d_nblockflag) return VABFT_EINVAL;
    if (!aligned_to(d_E_blk_k, acc_bytes(p->dtype)) || !aligned_to(d_blockflags_k, 4) || !aligned_to(d_nblockflag, 4))
        return VABFT_EINVAL;
    BlockArgs b;
    b.d_expected_blk = d_expected_blk_k;
    b.d_T_blk = d_T_blk_k;
    b.d_rowsum_blk = d_rowsum_blk_k;
    b.d_E_blk = d_E_blk_k;
    b.d_blockflags = d_blockflags_k;
    b.d_nblockflag = d_nblockflag;
    b.kblock = kblock;
    b.kprefix = reinterpret_cast<double*>(reinterpret_cast<unsigned char*>(d_workspace) +
                                          round_up(vabft_workspace_bytes(p), 256));
    return gemm_dispatch(p, dA, dB, dC, nullptr, nullptr, 1, nullptr, inj, nullptr, nullptr, d_E, d_flags, d_nflag,
                         d_injlog, d_ninj, d_workspace, (hipStream_t)stream, nullptr, &b);
}

int vabft_locate_correct(const vabft_problem* p, void* dC, const void* d_expected, const void* d_expected2,
                         const void* d_rowsum, const void* d_rowsum2, const int32_t* d_flags, int32_t correct,
                         int32_t* d_loc, void* d_delta, int32_t* d_ncorrected, void* stream) {
    if (!problem_ok(p) || !dC || !d_expected || !d_expected2 || !d_rowsum || !d_rowsum2 || !d_flags || !d_loc ||
        !d_delta || !d_ncorrected)
        return VABFT_EINVAL;
    if (correct != 0 && correct != 1) return VABFT_EINVAL;
    const size_t ab = acc_bytes(p->dtype);
    if (!aligned_to(dC, out_bytes(p->dtype)) || !aligned_to(d_expected, ab) || !aligned_to(d_expected2, ab) ||
        !aligned_to(d_rowsum, ab) || !aligned_to(d_rowsum2, ab) || !aligned_to(d_flags, 4) || !aligned_to(d_loc, 4) ||
        !aligned_to(d_delta, ab) || !aligned_to(d_ncorrected, 4))
        return VABFT_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid((p->M + 255) / 256), block(256);
    zero_int_kernel<<<1, 1, 0, st>>>(d_ncorrected);
#define VABFT_LOC_CASE(T, A)                                                                                     \
    locate_correct_kernel<T><<<grid, block, 0, st>>>(dC, p->M, p->N, p->ldc, (const A*)d_expected,               \
                                                     (const A*)d_expected2, (const A*)d_rowsum,                  \
                                                     (const A*)d_rowsum2, d_flags, correct, d_loc, (A*)d_delta,  \
                                                     d_ncorrected)
    switch (p->dtype) {
        case VABFT_F64: VABFT_LOC_CASE(double, double); break;
        case VABFT_F32: VABFT_LOC_CASE(float, float); break;
        case VABFT_F16: VABFT_LOC_CASE(f16_t, float); break;
        case VABFT_BF16: VABFT_LOC_CASE(bf16_t, float); break;
        case VABFT_F8E4M3:
        case VABFT_F8E5M2: VABFT_LOC_CASE(f16_t, float); break;  // C of an FP8 problem is FP16
        default: return VABFT_EINVAL;
    }
#undef VABFT_LOC_CASE
    return hipGetLastError() == hipSuccess ? VABFT_OK : VABFT_EDEVICE;
}

int vabft_gemm_verified_fused(const vabft_problem* p, const void* dA, const void* dB, void* dC, const void* d_Be,
                              const double* d_S, double e_max, double c_sigma, void* d_astat, void* d_expected,
                              void* d_T, const vabft_inject* inj, void* d_rowsum, void* d_E, int32_t* d_flags,
                              int32_t* d_nflag, vabft_inject_rec* d_injlog, int32_t* d_ninj, void* d_workspace,
                              size_t workspace_bytes, void* stream) {
    const int rc = check_gemm_args(p, dA, dB, dC, 1, inj, d_expected, d_T, d_rowsum, d_E, d_flags, d_nflag, d_injlog,
                                   d_ninj, d_workspace, workspace_bytes);
    if (rc != VABFT_OK) return rc;
    if (!d_Be || !d_astat) return VABFT_EINVAL;  // d_S may be null: S1..S3 are the partials of the last encode
    if (!(e_max > 0.0) || !(c_sigma >= 0.0) || !isfinite(e_max) || !isfinite(c_sigma)) return VABFT_EINVAL;
    const size_t ab = acc_bytes(p->dtype);
    if (!aligned_to(d_Be, ab) || !aligned_to(d_S, 8) || !aligned_to(d_astat, ab)) return VABFT_EINVAL;
    FusedArgs f;
    f.d_Be = d_Be;
    f.d_S = d_S;
    f.e_max = e_max;
    f.c_sigma = c_sigma;
    f.d_astat = d_astat;
    return gemm_dispatch(p, dA, dB, dC, d_expected, d_T, 1, &f, inj, d_rowsum, nullptr, d_E, d_flags, d_nflag,
                         d_injlog, d_ninj, d_workspace, (hipStream_t)stream);
}

size_t vabft_static_scratch_bytes(void) { return VABFT_STATIC_SCRATCH_BYTES; }

int vabft_gemm_verified_fused_static(const vabft_problem* p, const void* dA, const void* dB, void* dC, const void* d_Be,
                                     const double* d_S, double e_max, double c_sigma, void* d_astat, void* d_expected,
                                     void* d_T, const vabft_inject* inj, void* d_rowsum, void* d_E, int32_t* d_flags,
                                     int32_t* d_nflag, vabft_inject_rec* d_injlog, int32_t* d_ninj, void* stream) {
    if (!problem_ok(p)) return VABFT_EINVAL;
    if (!d_S) return VABFT_EINVAL;  // no encode runs on this scratch: S1..S3 must come folded
    const size_t need = tickets_bytes(p) + gemm_workspace_bytes(p);
    if (need > VABFT_STATIC_SCRATCH_BYTES) return VABFT_EWORKSPACE;
    void* ws = static_scratch_of_current_device();
    if (!ws) return VABFT_EDEVICE;
    const int rc = check_gemm_args(p, dA, dB, dC, 1, inj, d_expected, d_T, d_rowsum, d_E, d_flags, d_nflag, d_injlog,
                                   d_ninj, ws, VABFT_STATIC_SCRATCH_BYTES);
    if (rc != VABFT_OK) return rc;
    if (!d_Be || !d_astat) return VABFT_EINVAL;
    if (!(e_max > 0.0) || !(c_sigma >= 0.0) || !isfinite(e_max) || !isfinite(c_sigma)) return VABFT_EINVAL;
    const size_t ab = acc_bytes(p->dtype);
    if (!aligned_to(d_Be, ab) || !aligned_to(d_S, 8) || !aligned_to(d_astat, ab)) return VABFT_EINVAL;
    // every call on this GPU shares the array, which keeps the last call's contents: the arrival counters
    // must start at zero (a fill kernel, not a memset, so that the call can be captured into a graph)
    const size_t tb = tickets_used_bytes(p);
    fill_zero_kernel<<<1, 256, 0, (hipStream_t)stream>>>(
        reinterpret_cast<uint32_t*>(reinterpret_cast<unsigned char*>(ws) + tickets_offset(p)), tb / 4);
    if (hipGetLastError() != hipSuccess) return VABFT_EDEVICE;
    FusedArgs f;
    f.d_Be = d_Be;
    f.d_S = d_S;
    f.e_max = e_max;
    f.c_sigma = c_sigma;
    f.d_astat = d_astat;
    return gemm_dispatch(p, dA, dB, dC, d_expected, d_T, 1, &f, inj, d_rowsum, nullptr, d_E, d_flags, d_nflag,
                         d_injlog, d_ninj, ws, (hipStream_t)stream);
}

}  // extern "C"
