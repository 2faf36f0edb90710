// Block-wise V-ABFT (paper section 5.2 "Integration with Block-wise ABFT"): the product is verified in blocks
// of W columns -- the width one GEMM workgroup (256; 64 for the FP32 / FP64 kernels) sums before it writes a
// partial row sum.  The section's three steps, per block t = columns [tW, min(N, (t+1)W)):
//   1. row statistics of the block of B (the rows of A are whole, K is not split);
//   2. Algorithm 1 with those statistics and the block's width in place of N;
//   3. block checksums Be_t = B_t r1, expected_t = A Be_t, rowsum_t = C_t r1, compared per block; a row's
//      aggregate is the sum of its block differences, its flag the OR of its block flags.
#include <math.h>

#include "unpack.h"
#include "vabft_device.h"
#include "vabft_host.h"

namespace vabft {

// ---------------------------------------------------------------------------
// step 1 + block checksum of B.  part layout: [nblocks][3][K] (sum, max, min)
// ---------------------------------------------------------------------------

// B stored K x N: one wavefront per row k walks the blocks of that row
template <typename T>
__global__ __launch_bounds__(256) void encode_blocks_rows_kernel(const void* __restrict__ B, int K, int N, int64_t ldb,
                                                                 int W, typename Elem<T>::acc_t* __restrict__ part) {
    using acc_t = typename Elem<T>::acc_t;
    const int lane = threadIdx.x & 63;
    const int k = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (k >= K) return;
    const int nblocks = (N + W - 1) / W;
    for (int t = 0; t < nblocks; ++t) {
        const int n_end = min(N, (t + 1) * W);
        acc_t sum = 0, mx = -type_max<acc_t>(), mn = type_max<acc_t>();
        for (int n = t * W + lane; n < n_end; n += 64) {
            const acc_t x = Unpack<T>::one(B, (int64_t)k * ldb + n);
            sum += x;
            mx = fmax(mx, x);
            mn = fmin(mn, x);
        }
        sum = wave_sum(sum);
        mx = wave_max(mx);
        mn = wave_min(mn);
        if (lane == 0) {
            acc_t* q = part + (int64_t)t * 3 * K;
            q[k] = sum;
            q[(int64_t)K + k] = mx;
            q[2 * (int64_t)K + k] = mn;
        }
    }
}

// B stored K x N, rows 16-byte aligned, N a multiple of the chunk width: one wavefront per row k, 16-byte loads.
// A block of W columns is W / V chunks = 16 or 32 consecutive lanes of one load, so each lane folds its chunk
// and a butterfly over those lanes finishes the block; four loads are in flight per lane.
template <typename T>
__global__ __launch_bounds__(256) void encode_blocks_rows_vec_kernel(const void* __restrict__ B, int K, int N,
                                                                     int64_t ldb, int W,
                                                                     typename Elem<T>::acc_t* __restrict__ part) {
    using acc_t = typename Elem<T>::acc_t;
    constexpr int V = Elem<T>::vec;
    const int lane = threadIdx.x & 63;
    const int k = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (k >= K) return;
    const int cpb = W / V;  // chunks (lanes) per block: 16 or 32
    const int nchunks = N / V;
    const char* row = reinterpret_cast<const char*>(B) + (int64_t)k * ldb * Elem<T>::bytes;
    for (int c0 = 0; c0 < nchunks; c0 += 256) {
        raw16 r[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = c0 + 64 * u + lane;
            r[u] = ld16(row + (int64_t)(c < nchunks ? c : nchunks - 1) * 16);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = c0 + 64 * u + lane;
            const bool ok = c < nchunks;
            acc_t v[V];
            Unpack<T>::run(r[u], v);
            acc_t sum = 0, mx = -type_max<acc_t>(), mn = type_max<acc_t>();
            if (ok) {
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    sum += v[e];
                    mx = fmax(mx, v[e]);
                    mn = fmin(mn, v[e]);
                }
            }
            if (cpb == 32) {
                sum += __shfl_xor(sum, 16, WAVE);
                const acc_t a = __shfl_xor(mx, 16, WAVE), b = __shfl_xor(mn, 16, WAVE);
                mx = fmax(mx, a);
                mn = fmin(mn, b);
            }
#pragma unroll
            for (int off = 8; off >= 1; off >>= 1) {
                sum += __shfl_xor(sum, off, WAVE);
                const acc_t a = __shfl_xor(mx, off, WAVE), b = __shfl_xor(mn, off, WAVE);
                mx = fmax(mx, a);
                mn = fmin(mn, b);
            }
            if (ok && lane % cpb == 0) {
                acc_t* q = part + (int64_t)(c / cpb) * 3 * K;
                q[k] = sum;
                q[(int64_t)K + k] = mx;
                q[2 * (int64_t)K + k] = mn;
            }
        }
    }
}

// B stored N x K: one thread per (k, block) walks the block's rows n (consecutive threads read consecutive k)
template <typename T>
__global__ __launch_bounds__(256) void encode_blocks_cols_kernel(const void* __restrict__ Bt, int K, int N,
                                                                 int64_t ldb, int W,
                                                                 typename Elem<T>::acc_t* __restrict__ part) {
    using acc_t = typename Elem<T>::acc_t;
    const int k = blockIdx.x * 256 + threadIdx.x;
    const int t = blockIdx.y;
    if (k >= K) return;
    const int n_end = min(N, (t + 1) * W);
    acc_t s[4] = {0, 0, 0, 0}, mx = -type_max<acc_t>(), mn = type_max<acc_t>();
    int n = t * W;
    for (; n + 3 < n_end; n += 4) {
        acc_t x[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) x[u] = Unpack<T>::one(Bt, (int64_t)(n + u) * ldb + k);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            s[u] += x[u];
            mx = fmax(mx, x[u]);
            mn = fmin(mn, x[u]);
        }
    }
    for (; n < n_end; ++n) {
        const acc_t x = Unpack<T>::one(Bt, (int64_t)n * ldb + k);
        s[0] += x;
        mx = fmax(mx, x);
        mn = fmin(mn, x);
    }
    acc_t* q = part + (int64_t)t * 3 * K;
    q[k] = (s[0] + s[1]) + (s[2] + s[3]);
    q[(int64_t)K + k] = mx;
    q[2 * (int64_t)K + k] = mn;
}

// Be_blk[t][k] and S1, S2, S3 of block t (Algorithm 1, loop over k, with the block's width): one workgroup per block
template <typename acc_t>
__global__ __launch_bounds__(256) void blocks_aggregate_kernel(const acc_t* __restrict__ part, int K, int N, int W,
                                                               acc_t* __restrict__ Be_blk,
                                                               double* __restrict__ S_blk) {
    __shared__ double red[3][4];
    const int t = blockIdx.x, tid = threadIdx.x;
    const int width = min(N, (t + 1) * W) - t * W;
    const acc_t* q = part + (int64_t)t * 3 * K;
    double s1 = 0, s2 = 0, s3 = 0;
    for (int k = tid; k < K; k += 256) {
        const acc_t sum = q[k];
        Be_blk[(int64_t)t * K + k] = sum;
        const double mu = (double)sum / (double)width;
        double var = ((double)q[(int64_t)K + k] - mu) * (mu - (double)q[2 * (int64_t)K + k]);
        var = var > 0 ? var : 0;
        s1 += fabs(mu);
        s2 += var;
        s3 += mu * mu;
    }
    s1 = wave_sum(s1);
    s2 = wave_sum(s2);
    s3 = wave_sum(s3);
    if ((tid & 63) == 0) {
        red[0][tid >> 6] = s1;
        red[1][tid >> 6] = s2;
        red[2][tid >> 6] = s3;
    }
    __syncthreads();
    if (tid < 3) S_blk[3 * t + tid] = (red[tid][0] + red[tid][1]) + (red[tid][2] + red[tid][3]);
}

// ---------------------------------------------------------------------------
// steps 2 + 3 on the A side: row statistics of A, expected_t = A Be_t and T_t for every block.
// A workgroup takes 16 rows (4 per wavefront).  K is walked in chunks of 256; the Be_t slices of a chunk are
// staged in LDS for up to 16 blocks at a time and every slice read serves the wavefront's 4 rows.
// ---------------------------------------------------------------------------
constexpr int TB_RW = 1;  // rows per wavefront: small, so that many workgroups share a compute unit and hide latency
constexpr int TB_ROWS = 4 * TB_RW, TB_KC = 256, TB_T = 16;

template <typename T>
__global__ __launch_bounds__(256) void threshold_blocks_kernel(const void* __restrict__ A, int M, int K, int N, int W,
                                                               int64_t lda,
                                                               const typename Elem<T>::acc_t* __restrict__ Be_blk,
                                                               const double* __restrict__ S_blk, double e_max,
                                                               double c_sigma,
                                                               typename Elem<T>::acc_t* __restrict__ astat,
                                                               typename Elem<T>::acc_t* __restrict__ expected_blk,
                                                               typename Elem<T>::acc_t* __restrict__ T_blk) {
    using acc_t = typename Elem<T>::acc_t;
    __shared__ acc_t be[TB_T][TB_KC];
    __shared__ acc_t rstat[TB_ROWS][3];  // (sum, max, min) of the rows, from the first pass
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nblocks = (N + W - 1) / W;
    const int r0 = blockIdx.x * TB_ROWS + wave * TB_RW;  // the wavefront's first row
    for (int t0 = 0; t0 < nblocks; t0 += TB_T) {
        const int nt = min(TB_T, nblocks - t0);
        acc_t dot[TB_RW][TB_T];
#pragma unroll
        for (int r = 0; r < TB_RW; ++r)
#pragma unroll
            for (int t = 0; t < TB_T; ++t) dot[r][t] = 0;
        acc_t sum[TB_RW] = {}, mx[TB_RW], mn[TB_RW];
#pragma unroll
        for (int r = 0; r < TB_RW; ++r) {
            mx[r] = -type_max<acc_t>();
            mn[r] = type_max<acc_t>();
        }
        for (int kc = 0; kc < K; kc += TB_KC) {
            __syncthreads();  // the previous chunk's slices are no longer read
            {
                // thread tid stages element kk = tid of every block's slice: all loads first, then all stores
                static_assert(TB_KC == 256, "one element per thread and block");
                acc_t stage[TB_T];
#pragma unroll
                for (int t = 0; t < TB_T; ++t) {
                    const int tc = t < nt ? t : nt - 1, kq = kc + tid < K ? kc + tid : K - 1;  // clamped, masked below
                    stage[t] = Be_blk[(int64_t)(t0 + tc) * K + kq];
                }
#pragma unroll
                for (int t = 0; t < TB_T; ++t) be[t][tid] = (t < nt && kc + tid < K) ? stage[t] : (acc_t)0;
            }
            __syncthreads();
            // lane l takes k = kc + l + 64 j, j = 0..3; all 16 loads of the chunk are issued before any is used
            acc_t a[4][TB_RW];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int k = kc + lane + 64 * j;
#pragma unroll
                for (int r = 0; r < TB_RW; ++r)
                    a[j][r] = (k < K && r0 + r < M) ? Unpack<T>::one(A, (int64_t)(r0 + r) * lda + k) : (acc_t)0;
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int kk = lane + 64 * j, k = kc + kk;
                if (t0 == 0 && k < K) {
#pragma unroll
                    for (int r = 0; r < TB_RW; ++r) {
                        sum[r] += a[j][r];
                        mx[r] = fmax(mx[r], a[j][r]);
                        mn[r] = fmin(mn[r], a[j][r]);
                    }
                }
#pragma unroll
                for (int t = 0; t < TB_T; ++t) {
                    const acc_t b = be[t][kk];
#pragma unroll
                    for (int r = 0; r < TB_RW; ++r) dot[r][t] = fma(a[j][r], b, dot[r][t]);
                }
            }
        }
        if (t0 == 0) {
#pragma unroll
            for (int r = 0; r < TB_RW; ++r) {
                const acc_t s = wave_sum(sum[r]), hi = wave_max(mx[r]), lo = wave_min(mn[r]);
                if (lane == 0) {
                    rstat[wave * TB_RW + r][0] = s;
                    rstat[wave * TB_RW + r][1] = hi;
                    rstat[wave * TB_RW + r][2] = lo;
                    if (r0 + r < M) {
                        astat[3 * (int64_t)(r0 + r) + 0] = hi;
                        astat[3 * (int64_t)(r0 + r) + 1] = lo;
                        astat[3 * (int64_t)(r0 + r) + 2] = (acc_t)((double)s / (double)K);
                    }
                }
            }
        }
#pragma unroll
        for (int r = 0; r < TB_RW; ++r)
#pragma unroll
            for (int t = 0; t < TB_T; ++t) dot[r][t] = wave_sum(dot[r][t]);
        // lane (r, t) = (lane % TB_RW, lane / TB_RW) writes one (row, block) pair
        {
            const int r = lane % TB_RW, t = lane / TB_RW;  // t >= TB_T for the upper lanes when TB_RW < 4
            acc_t d = 0;
#pragma unroll
            for (int rr = 0; rr < TB_RW; ++rr)
#pragma unroll
                for (int tt = 0; tt < TB_T; ++tt)
                    if (rr == r && tt == t) d = dot[rr][tt];
            const int row = r0 + r;
            if (t < nt && row < M) {
                const int tb = t0 + t;
                const int width = min(N, (tb + 1) * W) - tb * W;
                const double mu = (double)rstat[wave * TB_RW + r][0] / (double)K;
                double var = ((double)rstat[wave * TB_RW + r][1] - mu) * (mu - (double)rstat[wave * TB_RW + r][2]);
                var = var > 0 ? var : 0;
                const double S1 = S_blk[3 * tb], S2 = S_blk[3 * tb + 1], S3 = S_blk[3 * tb + 2], dN = (double)width;
                const double t_det = dN * fabs(mu) * S1;
                const double t_var23 = c_sigma * sqrt(dN * mu * mu * S2 + dN * dN * var * S3);
                const double t_var4 = c_sigma * sqrt(dN) * sqrt(var) * sqrt(S2);
                expected_blk[(int64_t)tb * M + row] = d;
                T_blk[(int64_t)tb * M + row] = (acc_t)(e_max * (t_det + t_var23 + t_var4));
            }
        }
    }
}

// The same pass for 16-byte aligned rows of A with K a multiple of the chunk width: a lane takes CH 16-byte
// chunks (V consecutive k each) of each of the wavefront's R rows per step, a workgroup 4 R rows, and K is walked
// in steps of KC = 64 V CH.  The Be_t slices of a step sit in LDS as [block][chunk][piece][lane][16 bytes], so that
// the 16-byte reads of a wavefront are contiguous, and every slice read serves R rows.  The chunks of A and the
// slice values of the next step are fetched into registers before the current step is multiplied.
template <typename T, int R>
__global__ __launch_bounds__(256) void threshold_blocks_vec_kernel(const void* __restrict__ A, int M, int K, int N,
                                                                   int W, int64_t lda,
                                                                   const typename Elem<T>::acc_t* __restrict__ Be_blk,
                                                                   const double* __restrict__ S_blk, double e_max,
                                                                   double c_sigma,
                                                                   typename Elem<T>::acc_t* __restrict__ astat,
                                                                   typename Elem<T>::acc_t* __restrict__ expected_blk,
                                                                   typename Elem<T>::acc_t* __restrict__ T_blk) {
    using acc_t = typename Elem<T>::acc_t;
    constexpr int V = Elem<T>::vec;                   // elements per 16-byte chunk of A
    constexpr int E = 16 / (int)sizeof(acc_t);        // accumulator-typed values per 16 bytes of LDS
    constexpr int P = V / E;                          // 16-byte pieces of a slice per chunk
    constexpr int CH = V >= 8 ? 1 : 8 / V;            // chunks per lane and step
    constexpr int KC = 64 * V * CH;                   // k per step: 512 (1024 for 1-byte elements)
    constexpr int TT = 32768 / (KC * (int)sizeof(acc_t));  // blocks per pass: 32 KiB of slices
    constexpr int NJ = KC / 256;
    static_assert(R * TT <= 64, "one lane per (row, block) pair at the end");
    struct alignas(16) piece_t { acc_t v[E]; };
    __shared__ piece_t be[TT][CH][P][64];
    __shared__ acc_t rstat[4 * R][3];  // (sum, max, min) of the rows, from the first pass
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nblocks = (N + W - 1) / W;
    const int r0 = blockIdx.x * 4 * R + wave * R;  // the wavefront's first row
    const char* rowp[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int row = r0 + r < M ? r0 + r : M - 1;  // clamped; results of rows past M are not written
        rowp[r] = reinterpret_cast<const char*>(A) + (int64_t)row * lda * Elem<T>::bytes;
    }
    for (int t0 = 0; t0 < nblocks; t0 += TT) {
        const int nt = min(TT, nblocks - t0);
        acc_t dot[R][TT];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int t = 0; t < TT; ++t) dot[r][t] = 0;
        acc_t sum[R], mx[R], mn[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            sum[r] = 0;
            mx[r] = -type_max<acc_t>();
            mn[r] = type_max<acc_t>();
        }
        raw16 araw[R][CH];
        acc_t stage[TT][NJ];
        // thread tid fetches elements kk = tid + 256 j of every block's slice, lane l chunk c of every row
        auto prefetch = [&](int kc) {
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int c = 0; c < CH; ++c) {
                    const int k0 = kc + (c * 64 + lane) * V;
                    araw[r][c] = ld16(rowp[r] + (int64_t)(k0 < K ? k0 : 0) * Elem<T>::bytes);  // masked below
                }
#pragma unroll
            for (int t = 0; t < TT; ++t)
#pragma unroll
                for (int j = 0; j < NJ; ++j) {
                    const int tc = t < nt ? t : nt - 1, kq = kc + tid + 256 * j;  // clamped, masked below
                    stage[t][j] = Be_blk[(int64_t)(t0 + tc) * K + (kq < K ? kq : K - 1)];
                }
        };
        prefetch(0);
        for (int kc = 0; kc < K; kc += KC) {
            __syncthreads();  // the previous step's slices are no longer read
#pragma unroll
            for (int t = 0; t < TT; ++t)
#pragma unroll
                for (int j = 0; j < NJ; ++j) {
                    const int kk = tid + 256 * j;
                    const int c = kk / (64 * V), l = (kk / V) % 64, w = kk % V;
                    be[t][c][w / E][l].v[w % E] = (t < nt && kc + kk < K) ? stage[t][j] : (acc_t)0;
                }
            acc_t av[R][CH][V];
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int c = 0; c < CH; ++c) Unpack<T>::run(araw[r][c], av[r][c]);
            __syncthreads();
            if (kc + KC < K) prefetch(kc + KC);
            if (t0 == 0) {
#pragma unroll
                for (int c = 0; c < CH; ++c) {
                    if (kc + (c * 64 + lane) * V < K) {
#pragma unroll
                        for (int r = 0; r < R; ++r)
#pragma unroll
                            for (int e = 0; e < V; ++e) {
                                sum[r] += av[r][c][e];
                                mx[r] = fmax(mx[r], av[r][c][e]);
                                mn[r] = fmin(mn[r], av[r][c][e]);
                            }
                    }
                }
            }
#pragma unroll
            for (int t = 0; t < TT; ++t)
#pragma unroll
                for (int c = 0; c < CH; ++c)
#pragma unroll
                    for (int pc = 0; pc < P; ++pc) {
                        const piece_t b = be[t][c][pc][lane];
#pragma unroll
                        for (int e = 0; e < E; ++e)
#pragma unroll
                            for (int r = 0; r < R; ++r) dot[r][t] = fma(av[r][c][pc * E + e], b.v[e], dot[r][t]);
                    }
        }
        if (t0 == 0) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const acc_t s = wave_sum(sum[r]), hi = wave_max(mx[r]), lo = wave_min(mn[r]);
                if (lane == 0) {
                    rstat[wave * R + r][0] = s;
                    rstat[wave * R + r][1] = hi;
                    rstat[wave * R + r][2] = lo;
                    if (r0 + r < M) {
                        astat[3 * (int64_t)(r0 + r) + 0] = hi;
                        astat[3 * (int64_t)(r0 + r) + 1] = lo;
                        astat[3 * (int64_t)(r0 + r) + 2] = (acc_t)((double)s / (double)K);
                    }
                }
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int t = 0; t < TT; ++t) dot[r][t] = wave_sum(dot[r][t]);
        // lane r * TT + t writes one (row, block) pair; rstat was written by this wavefront's own lane 0
        {
            const int r = lane / TT, t = lane % TT;
            acc_t d = 0;
#pragma unroll
            for (int rr = 0; rr < R; ++rr)
#pragma unroll
                for (int tt = 0; tt < TT; ++tt)
                    if (rr == r && tt == t) d = dot[rr][tt];
            const int row = r0 + r;
            if (r < R && t < nt && row < M) {
                const int tb = t0 + t;
                const int width = min(N, (tb + 1) * W) - tb * W;
                const double mu = (double)rstat[wave * R + r][0] / (double)K;
                double var = ((double)rstat[wave * R + r][1] - mu) * (mu - (double)rstat[wave * R + r][2]);
                var = var > 0 ? var : 0;
                const double S1 = S_blk[3 * tb], S2 = S_blk[3 * tb + 1], S3 = S_blk[3 * tb + 2], dN = (double)width;
                const double t_det = dN * fabs(mu) * S1;
                const double t_var23 = c_sigma * sqrt(dN * mu * mu * S2 + dN * dN * var * S3);
                const double t_var4 = c_sigma * sqrt(dN) * sqrt(var) * sqrt(S2);
                expected_blk[(int64_t)tb * M + row] = d;
                T_blk[(int64_t)tb * M + row] = (acc_t)(e_max * (t_det + t_var23 + t_var4));
            }
        }
    }
}

// ---------------------------------------------------------------------------
// compare per block and aggregate per row.  rowpart holds `sub` partials per block (1 for the 256-wide
// kernels, whose workgroup sums a whole block; the wide kernels leave the block's value directly too)
// ---------------------------------------------------------------------------
template <typename acc_t>
__global__ __launch_bounds__(64) void finalize_blocks_kernel(const acc_t* __restrict__ rowpart, int nblocks, int M,
                                                             const acc_t* __restrict__ expected_blk,
                                                             const acc_t* __restrict__ T_blk,
                                                             acc_t* __restrict__ rowsum_blk, acc_t* __restrict__ E_blk,
                                                             int32_t* __restrict__ blockflags,
                                                             acc_t* __restrict__ E, int32_t* __restrict__ flags,
                                                             int32_t* __restrict__ nflag,
                                                             int32_t* __restrict__ nblockflag) {
    // one wavefront per 64 rows (many small workgroups: the pass is a few dependent round trips long), the
    // loads of eight blocks in flight at once, blocks folded in order
    const int i = blockIdx.x * 64 + threadIdx.x;
    int any = 0, nb = 0;
    if (i < M) {
        acc_t esum = 0;
        for (int t0 = 0; t0 < nblocks; t0 += 8) {
            acc_t s[8], x[8], thr[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int64_t idx = (int64_t)(t0 + u < nblocks ? t0 + u : nblocks - 1) * M + i;
                s[u] = rowpart[idx];
                x[u] = expected_blk[idx];
                thr[u] = T_blk[idx];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (t0 + u < nblocks) {
                    const int64_t idx = (int64_t)(t0 + u) * M + i;
                    const acc_t e = x[u] - s[u];
                    const int f = !(fabs(e) <= thr[u]);
                    rowsum_blk[idx] = s[u];
                    E_blk[idx] = e;
                    blockflags[idx] = f;
                    esum += e;
                    nb += f;
                }
            }
        }
        any = nb > 0;
        E[i] = esum;
        flags[i] = any;
    }
    int cnt = any, w = nb;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        cnt += __shfl_xor(cnt, off, WAVE);
        w += __shfl_xor(w, off, WAVE);
    }
    if (threadIdx.x == 0) {
        if (cnt) atomicAdd(nflag, cnt);
        if (w) atomicAdd(nblockflag, w);
    }
}

// ---------------------------------------------------------------------------
// K split as well (section 5.2): kprefix[b][2 t + w][i] is the row sum, in double, of what wavefront column w of
// tile-column t had accumulated when K-block b ended (b = last: the whole product).  The share of K-block b is
// the difference of consecutive prefixes; it is compared with the piece's own expected value and threshold.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void finalize_blocks_k_kernel(const double* __restrict__ kprefix, int nkb,
                                                                int nblocks, int M,
                                                                const float* __restrict__ expected_blk,
                                                                const float* __restrict__ T_blk,
                                                                float* __restrict__ rowsum_blk,
                                                                float* __restrict__ E_blk,
                                                                int32_t* __restrict__ blockflags, float* __restrict__ E,
                                                                int32_t* __restrict__ flags, int32_t* __restrict__ nflag,
                                                                int32_t* __restrict__ nblockflag) {
    // 32 rows per workgroup, eight threads per row: thread (r, tl) takes the column blocks t = tl, tl + 8, ...; the
    // eight partial aggregates of a row are added in the order of tl (a fixed order: results repeat bit for bit)
    __shared__ double s_e[8][32];
    __shared__ int s_n[8][32];
    const int r = threadIdx.x & 31, tl = threadIdx.x >> 5;
    const int i = blockIdx.x * 32 + r;
    double esum = 0;
    int nb = 0;
    if (i < M) {
        for (int t = tl; t < nblocks; t += 8) {
            double prev = 0;
            // the loads of eight K-blocks in flight at once (the pass is a few dependent round trips long)
            for (int b0 = 0; b0 < nkb; b0 += 8) {
                double c0[8], c1[8];
                float x[8], thr[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int b = b0 + u < nkb ? b0 + u : nkb - 1;
                    const double* q = kprefix + ((int64_t)b * (2 * nblocks) + 2 * t) * M + i;
                    const int64_t idx = ((int64_t)b * nblocks + t) * M + i;
                    c0[u] = q[0];
                    c1[u] = q[M];
                    x[u] = expected_blk[idx];
                    thr[u] = T_blk[idx];
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    if (b0 + u < nkb) {
                        const int64_t idx = ((int64_t)(b0 + u) * nblocks + t) * M + i;
                        const double cur = c0[u] + c1[u];
                        const double share = cur - prev;
                        prev = cur;
                        const double e = (double)x[u] - share;
                        const int f = !(fabs(e) <= (double)thr[u]);
                        rowsum_blk[idx] = (float)share;
                        E_blk[idx] = (float)e;
                        blockflags[idx] = f;
                        esum += e;
                        nb += f;
                    }
                }
            }
        }
    }
    s_e[tl][r] = esum;
    s_n[tl][r] = nb;
    __syncthreads();
    int any = 0, w = 0;
    if (tl == 0) {
        double e = 0;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            e += s_e[q][r];
            w += s_n[q][r];
        }
        if (i < M) {
            any = w > 0;
            E[i] = (float)e;
            flags[i] = any;
        } else {
            w = 0;
        }
    }
    // the counts sit in the threads with tl == 0, the first half of the first wavefront
    if (threadIdx.x < 64) {
        int cnt = any;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            cnt += __shfl_xor(cnt, off, WAVE);
            w += __shfl_xor(w, off, WAVE);
        }
        if (threadIdx.x == 0) {
            if (cnt) atomicAdd(nflag, cnt);
            if (w) atomicAdd(nblockflag, w);
        }
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
int block_width(int dtype) { return (dtype == VABFT_F64 || dtype == VABFT_F32) ? 64 : 256; }

size_t blocks_workspace_bytes(const vabft_problem* p) {
    const size_t W = block_width(p->dtype);
    const size_t nblocks = ((size_t)p->N + W - 1) / W;
    return nblocks * 3 * (size_t)p->K * (p->dtype == VABFT_F64 ? 8 : 4);
}

template <typename T>
static int encode_blocks_launch(const vabft_problem* p, const void* dB, void* d_Be_blk, double* d_S_blk, void* ws,
                                hipStream_t st) {
    using acc_t = typename Elem<T>::acc_t;
    const int W = block_width(p->dtype), nblocks = (p->N + W - 1) / W;
    acc_t* part = reinterpret_cast<acc_t*>(ws);
    constexpr int V = Elem<T>::vec;
    const bool vec = aligned16(dB) && (p->ldb * Elem<T>::bytes) % 16 == 0 && p->N % V == 0 && W % V == 0 &&
                     (W / V == 16 || W / V == 32);
    if (!p->transB && vec)
        encode_blocks_rows_vec_kernel<T><<<dim3((p->K + 3) / 4), dim3(256), 0, st>>>(dB, p->K, p->N, p->ldb, W, part);
    else if (!p->transB)
        encode_blocks_rows_kernel<T><<<dim3((p->K + 3) / 4), dim3(256), 0, st>>>(dB, p->K, p->N, p->ldb, W, part);
    else
        encode_blocks_cols_kernel<T><<<dim3((p->K + 255) / 256, nblocks), dim3(256), 0, st>>>(dB, p->K, p->N, p->ldb, W,
                                                                                              part);
    blocks_aggregate_kernel<acc_t><<<dim3(nblocks), dim3(256), 0, st>>>(part, p->K, p->N, W, (acc_t*)d_Be_blk, d_S_blk);
    return hipGetLastError() == hipSuccess ? VABFT_OK : VABFT_EDEVICE;
}

int encode_blocks_dispatch(const vabft_problem* p, const void* dB, void* d_Be_blk, double* d_S_blk, void* ws,
                           hipStream_t st) {
    switch (p->dtype) {
        case VABFT_F64: return encode_blocks_launch<double>(p, dB, d_Be_blk, d_S_blk, ws, st);
        case VABFT_F32: return encode_blocks_launch<float>(p, dB, d_Be_blk, d_S_blk, ws, st);
        case VABFT_F16: return encode_blocks_launch<f16_t>(p, dB, d_Be_blk, d_S_blk, ws, st);
        case VABFT_BF16: return encode_blocks_launch<bf16_t>(p, dB, d_Be_blk, d_S_blk, ws, st);
        case VABFT_F8E4M3: return encode_blocks_launch<f8_t>(p, dB, d_Be_blk, d_S_blk, ws, st);
        case VABFT_F8E5M2: return encode_blocks_launch<bf8_t>(p, dB, d_Be_blk, d_S_blk, ws, st);
    }
    return VABFT_EINVAL;
}

template <typename T>
static int threshold_blocks_launch(const vabft_problem* p, const void* dA, const void* d_Be_blk, const double* d_S_blk,
                                   double e_max, double c_sigma, void* d_astat, void* d_expected_blk, void* d_T_blk,
                                   hipStream_t st) {
    using acc_t = typename Elem<T>::acc_t;
    constexpr int V = Elem<T>::vec, R = 2;
    if (aligned16(dA) && (p->lda * Elem<T>::bytes) % 16 == 0 && p->K % V == 0)
        threshold_blocks_vec_kernel<T, R><<<dim3((p->M + 4 * R - 1) / (4 * R)), dim3(256), 0, st>>>(
            dA, p->M, p->K, p->N, block_width(p->dtype), p->lda, (const acc_t*)d_Be_blk, d_S_blk, e_max, c_sigma,
            (acc_t*)d_astat, (acc_t*)d_expected_blk, (acc_t*)d_T_blk);
    else
        threshold_blocks_kernel<T><<<dim3((p->M + TB_ROWS - 1) / TB_ROWS), dim3(256), 0, st>>>(
            dA, p->M, p->K, p->N, block_width(p->dtype), p->lda, (const acc_t*)d_Be_blk, d_S_blk, e_max, c_sigma,
            (acc_t*)d_astat, (acc_t*)d_expected_blk, (acc_t*)d_T_blk);
    return hipGetLastError() == hipSuccess ? VABFT_OK : VABFT_EDEVICE;
}

int threshold_blocks_dispatch(const vabft_problem* p, const void* dA, const void* d_Be_blk, const double* d_S_blk,
                              double e_max, double c_sigma, void* d_astat, void* d_expected_blk, void* d_T_blk,
                              hipStream_t st) {
#define VABFT_TB_CASE(T) \
    return threshold_blocks_launch<T>(p, dA, d_Be_blk, d_S_blk, e_max, c_sigma, d_astat, d_expected_blk, d_T_blk, st)
    switch (p->dtype) {
        case VABFT_F64: VABFT_TB_CASE(double);
        case VABFT_F32: VABFT_TB_CASE(float);
        case VABFT_F16: VABFT_TB_CASE(f16_t);
        case VABFT_BF16: VABFT_TB_CASE(bf16_t);
        case VABFT_F8E4M3: VABFT_TB_CASE(f8_t);
        case VABFT_F8E5M2: VABFT_TB_CASE(bf8_t);
    }
#undef VABFT_TB_CASE
    return VABFT_EINVAL;
}

int finalize_blocks_dispatch(const vabft_problem* p, const void* rowpart, const void* d_expected_blk,
                             const void* d_T_blk, void* d_rowsum_blk, void* d_E_blk, int32_t* d_blockflags, void* d_E,
                             int32_t* d_flags, int32_t* d_nflag, int32_t* d_nblockflag, hipStream_t st) {
    const int W = block_width(p->dtype), nblocks = (p->N + W - 1) / W;
    // d_nflag and d_nblockflag were zeroed by the GEMM kernel that produced the partials
    const dim3 grid((p->M + 63) / 64), block(64);
    if (p->dtype == VABFT_F64)
        finalize_blocks_kernel<double><<<grid, block, 0, st>>>(
            (const double*)rowpart, nblocks, p->M, (const double*)d_expected_blk, (const double*)d_T_blk,
            (double*)d_rowsum_blk, (double*)d_E_blk, d_blockflags, (double*)d_E, d_flags, d_nflag, d_nblockflag);
    else
        finalize_blocks_kernel<float><<<grid, block, 0, st>>>(
            (const float*)rowpart, nblocks, p->M, (const float*)d_expected_blk, (const float*)d_T_blk,
            (float*)d_rowsum_blk, (float*)d_E_blk, d_blockflags, (float*)d_E, d_flags, d_nflag, d_nblockflag);
    return hipGetLastError() == hipSuccess ? VABFT_OK : VABFT_EDEVICE;
}

// FP32-accumulated 16-bit types only (the kernels that leave K-block prefixes)
int finalize_blocks_k_dispatch(const vabft_problem* p, int nkb, const double* kprefix, const void* d_expected_blk,
                               const void* d_T_blk, void* d_rowsum_blk, void* d_E_blk, int32_t* d_blockflags,
                               void* d_E, int32_t* d_flags, int32_t* d_nflag, int32_t* d_nblockflag, hipStream_t st) {
    const int W = block_width(p->dtype), nblocks = (p->N + W - 1) / W;
    // d_nflag and d_nblockflag were zeroed by the GEMM kernel that produced the prefixes
    finalize_blocks_k_kernel<<<dim3((p->M + 31) / 32), dim3(256), 0, st>>>(
        kprefix, nkb, nblocks, p->M, (const float*)d_expected_blk, (const float*)d_T_blk, (float*)d_rowsum_blk,
        (float*)d_E_blk, d_blockflags, (float*)d_E, d_flags, d_nflag, d_nblockflag);
    return hipGetLastError() == hipSuccess ? VABFT_OK : VABFT_EDEVICE;
}

}  // namespace vabft
