// Checksum encode B*r1 with per-row (max, min, mean) statistics and the three B aggregates
// of Algorithm 1 (paper section 2.2 Eq. r1 / encoded matrices; section 3.5; Algorithm 1 k-loop),
// and the A-side pass: row statistics, expected checksum A*(B r1) and the threshold T_m
// (section 3.4 boxed formula).  Both are single streaming passes bound by HBM bandwidth.
#include "unpack.h"
#include "vabft_device.h"
#include "vabft_host.h"

namespace vabft {

// ---------------------------------------------------------------------------
// S1, S2, S3 without a launch of their own: every block publishes the three sums over its own
// rows k (Algorithm 1: S1 += |mu_Bk|, S2 += sigma_Bk^2, S3 += mu_Bk^2) and takes an arrival ticket;
// the last block folds all partials in block order.  Partials and ticket go through device-scope
// relaxed atomics (the blocks sit on XCDs with private L2s); the ticket is left at zero.
// s1..s3 need to be valid in thread 0 only.  Every thread of the block must call this.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void st_agent_f64(double* p, double v) {
    __hip_atomic_store(reinterpret_cast<uint64_t*>(p), (uint64_t)__double_as_longlong(v), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ double ld_agent_f64(const double* p) {
    return __longlong_as_double((long long)__hip_atomic_load(reinterpret_cast<const uint64_t*>(p), __ATOMIC_RELAXED,
                                                            __HIP_MEMORY_SCOPE_AGENT));
}

__device__ __forceinline__ void publish_and_fold_S(double s1, double s2, double s3, double* __restrict__ partial,
                                                   int32_t* __restrict__ ticket, double* __restrict__ S) {
    __shared__ int s_last;
    __shared__ double s_red[3][4];
    const int t = threadIdx.x, nblocks = gridDim.x;
    if (S == nullptr) {
        // deferred fold: the partials stay where they are (plain stores: the consumer is a later kernel
        // on the stream, which folds them in this same order)
        if (t == 0) {
            double* mine = partial + 3 * (int64_t)blockIdx.x;
            mine[0] = s1;
            mine[1] = s2;
            mine[2] = s3;
        }
        return;
    }
    if (t == 0) {
        double* mine = partial + 3 * (int64_t)blockIdx.x;
        st_agent_f64(mine, s1);
        st_agent_f64(mine + 1, s2);
        st_agent_f64(mine + 2, s3);
        __builtin_amdgcn_s_waitcnt(0);  // the partials are performed before the ticket is taken
        s_last = atomicAdd(ticket, 1) == nblocks - 1;
    }
    __syncthreads();
    if (!s_last) return;
    if (t < 256) {
        // thread t folds blocks t, t + 256, ... in increasing order; butterfly inside each of the
        // four wavefronts; the four results in order
        double a1 = 0, a2 = 0, a3 = 0;
        for (int b = t; b < nblocks; b += 256) {
            const double* q = partial + 3 * (int64_t)b;
            a1 += ld_agent_f64(q);
            a2 += ld_agent_f64(q + 1);
            a3 += ld_agent_f64(q + 2);
        }
        a1 = wave_sum(a1);
        a2 = wave_sum(a2);
        a3 = wave_sum(a3);
        if ((t & 63) == 0) {
            s_red[0][t >> 6] = a1;
            s_red[1][t >> 6] = a2;
            s_red[2][t >> 6] = a3;
        }
    }
    __syncthreads();
    if (t < 3) {
        const int nw = blockDim.x < 256 ? (blockDim.x + 63) / 64 : 4;
        double v = 0;
        for (int w = 0; w < nw; ++w) v += s_red[t][w];
        S[t] = v;
    }
    if (t == 0) __hip_atomic_store(ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// the three per-row terms of S1, S2, S3 from (row sum, max, min) of a row of N elements
template <typename acc_t>
__device__ __forceinline__ void row_terms(acc_t sum, acc_t mx, acc_t mn, int N, double& t1, double& t2, double& t3) {
    const double mu = (double)sum / (double)N;
    double var = ((double)mx - mu) * (mu - (double)mn);  // section 3.5: sigma^2 <= (max - mu)(mu - min)
    var = var > 0 ? var : 0;
    t1 = fabs(mu);
    t2 = var;
    t3 = mu * mu;
}

// ---------------------------------------------------------------------------
// B stored K x N: WAVES wavefronts per block reduce RPB rows k, WAVES / RPB wavefronts per row (each a
// contiguous segment of the row, combined in segment order).  RPB is WAVES when that gives enough
// blocks to fill the chip, else half of it, and so on down to 1.
// WAVES is 16 when the kernel folds S1..S3 itself (the fold's tail is one atomic per block on one address,
// about 11 ns each, so fewer and larger blocks are faster: 11.7 against 13.9 us at 4096 x 4096 BF16) and 8 when
// the fold is deferred (smaller blocks retire and refill sooner: 25.3 against 28.3 us at 8192 x 8192 FP16).
// ---------------------------------------------------------------------------

// W: also the position-weighted checksum B*r2, r2 = [1..N] (section 2.2): Be2[k] = sum_n (n+1) B[k,n].
template <typename T, bool W, int RPB, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void encode_rows_kernel(const void* __restrict__ B, int K, int N, int64_t ldb,
                                                           typename Elem<T>::acc_t* __restrict__ Be,
                                                           typename Elem<T>::acc_t* __restrict__ Be2,
                                                           typename Elem<T>::acc_t* __restrict__ bstat, int vec_ok,
                                                           double* __restrict__ s_partial,
                                                           int32_t* __restrict__ ticket, double* __restrict__ S) {
    using acc_t = typename Elem<T>::acc_t;
    constexpr int V = Elem<T>::vec;
    constexpr int WPR = WAVES / RPB;  // wavefronts per row
    __shared__ double terms[RPB][3];
    __shared__ acc_t seg[WAVES][4];  // (sum, weighted sum, max, min) of each wavefront's segment
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int k = blockIdx.x * RPB + wave / WPR, part = wave % WPR;
    acc_t sum = 0, sum2 = 0, mx = -type_max<acc_t>(), mn = type_max<acc_t>();
    if (k < K) {
        const char* row = reinterpret_cast<const char*>(B) + (int64_t)k * ldb * Elem<T>::bytes;
        int done = 0;
        if (vec_ok) {
            const int nchunks = N / V;
            // segment of this wavefront: a multiple of 64 chunks, the last one takes what is left
            const int per = ((nchunks + WPR - 1) / WPR + 63) / 64 * 64;
            const int c_end = part == WPR - 1 ? nchunks : min(nchunks, (part + 1) * per);
            int c = part * per + lane;
            for (; c + 192 < c_end; c += 256) {
                raw16 r0 = ld16(row + (int64_t)c * 16);
                raw16 r1 = ld16(row + (int64_t)(c + 64) * 16);
                raw16 r2 = ld16(row + (int64_t)(c + 128) * 16);
                raw16 r3 = ld16(row + (int64_t)(c + 192) * 16);
                acc_t v[4][V];
                Unpack<T>::run(r0, v[0]);
                Unpack<T>::run(r1, v[1]);
                Unpack<T>::run(r2, v[2]);
                Unpack<T>::run(r3, v[3]);
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int e = 0; e < V; ++e) {
                        sum += v[u][e];
                        if constexpr (W) sum2 = fma((acc_t)((c + 64 * u) * V + e + 1), v[u][e], sum2);
                        mx = fmax(mx, v[u][e]);
                        mn = fmin(mn, v[u][e]);
                    }
            }
            for (; c < c_end; c += 64) {
                raw16 r0 = ld16(row + (int64_t)c * 16);
                acc_t v[V];
                Unpack<T>::run(r0, v);
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    sum += v[e];
                    if constexpr (W) sum2 = fma((acc_t)(c * V + e + 1), v[e], sum2);
                    mx = fmax(mx, v[e]);
                    mn = fmin(mn, v[e]);
                }
            }
            done = nchunks * V;
        }
        // what the 16-byte pieces do not cover (everything, for unaligned rows): the last segment's wavefront
        if (part == WPR - 1) {
            for (int n = done + lane; n < N; n += 64) {
                acc_t x = Unpack<T>::one(row, n);
                sum += x;
                if constexpr (W) sum2 = fma((acc_t)(n + 1), x, sum2);
                mx = fmax(mx, x);
                mn = fmin(mn, x);
            }
        }
        sum = wave_sum(sum);
        mx = wave_max(mx);
        mn = wave_min(mn);
        if constexpr (W) sum2 = wave_sum(sum2);
    }
    if constexpr (WPR > 1) {
        if (lane == 0) {
            seg[wave][0] = sum;
            seg[wave][1] = sum2;
            seg[wave][2] = mx;
            seg[wave][3] = mn;
        }
        __syncthreads();
        if (part == 0 && lane == 0) {
            sum = seg[wave][0];
            sum2 = seg[wave][1];
            mx = seg[wave][2];
            mn = seg[wave][3];
#pragma unroll
            for (int q = 1; q < WPR; ++q) {  // segments in order
                sum += seg[wave + q][0];
                sum2 += seg[wave + q][1];
                mx = fmax(mx, seg[wave + q][2]);
                mn = fmin(mn, seg[wave + q][3]);
            }
        }
    }
    double t1 = 0, t2 = 0, t3 = 0;
    if (k < K && part == 0 && lane == 0) {
        if constexpr (W) Be2[k] = sum2;
        Be[k] = sum;
        bstat[3 * (int64_t)k + 0] = mx;
        bstat[3 * (int64_t)k + 1] = mn;
        bstat[3 * (int64_t)k + 2] = (acc_t)((double)sum / (double)N);
        row_terms(sum, mx, mn, N, t1, t2, t3);
    }
    if (part == 0 && lane == 0) {
        terms[wave / WPR][0] = t1;
        terms[wave / WPR][1] = t2;
        terms[wave / WPR][2] = t3;
    }
    __syncthreads();
    double s1 = 0, s2 = 0, s3 = 0;
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 0; w < RPB; ++w) {  // rows of the block in order
            s1 += terms[w][0];
            s2 += terms[w][1];
            s3 += terms[w][2];
        }
    }
    publish_and_fold_S(s1, s2, s3, s_partial, ticket, S);
}

// ---------------------------------------------------------------------------
// B stored N x K (weight layout): column reduction in two steps.
// Step 1: block (kx, ny) reduces rows [ny*rows_per_block, ...) of 64*V columns.
// part layout: [nsplit][4][K] (sum, max, min, weighted sum; the last only when W).
// The weight of row n is n + 1 (the vector r2), or wvec[n] when a weight vector is given (then the
// weighted sum is the dot product of every column with that vector).
// ---------------------------------------------------------------------------
template <typename T, bool W, int COLS_NL>
__global__ __launch_bounds__(256) void encode_cols_kernel(const void* __restrict__ Bt, int K, int N, int64_t ldb,
                                                          int rows_per_block,
                                                          typename Elem<T>::acc_t* __restrict__ part, int vec_ok,
                                                          const typename Elem<T>::acc_t* __restrict__ wvec) {
    using acc_t = typename Elem<T>::acc_t;
    constexpr int V = Elem<T>::vec;
    __shared__ acc_t red[3][W ? 4 : 3][65 * V];  // waves 1..3 park their partials here, [e][lane] with pitch 65
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int k0 = (blockIdx.x * 64 + lane) * V;
    const int n_begin = blockIdx.y * rows_per_block;
    const int n_end = min(N, n_begin + rows_per_block);
    acc_t sum[V], sum2[V], mx[V], mn[V];
#pragma unroll
    for (int e = 0; e < V; ++e) {
        sum[e] = 0;
        sum2[e] = 0;
        mx[e] = -type_max<acc_t>();
        mn[e] = type_max<acc_t>();
    }
    const bool full = vec_ok && (k0 + V <= K);
    if (full) {
        int n = n_begin + wave;
        // COLS_NL rows in flight per wavefront (a wavefront reads 1 KiB of every fourth row of the slab)
        for (; n + 4 * (COLS_NL - 1) < n_end; n += 4 * COLS_NL) {
            raw16 r[COLS_NL];
#pragma unroll
            for (int u = 0; u < COLS_NL; ++u)
                r[u] = ld16(reinterpret_cast<const char*>(Bt) + ((int64_t)(n + 4 * u) * ldb + k0) * Elem<T>::bytes);
#pragma unroll
            for (int u = 0; u < COLS_NL; ++u) {
                acc_t v[V];
                Unpack<T>::run(r[u], v);
                const acc_t w = !W ? (acc_t)0 : (wvec ? wvec[n + 4 * u] : (acc_t)(n + 4 * u + 1));
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    sum[e] += v[e];
                    if constexpr (W) sum2[e] = fma(w, v[e], sum2[e]);
                    mx[e] = fmax(mx[e], v[e]);
                    mn[e] = fmin(mn[e], v[e]);
                }
            }
        }
        for (; n < n_end; n += 4) {
            raw16 r0 = ld16(reinterpret_cast<const char*>(Bt) + ((int64_t)n * ldb + k0) * Elem<T>::bytes);
            acc_t v[V];
            Unpack<T>::run(r0, v);
            const acc_t w = !W ? (acc_t)0 : (wvec ? wvec[n] : (acc_t)(n + 1));
#pragma unroll
            for (int e = 0; e < V; ++e) {
                sum[e] += v[e];
                if constexpr (W) sum2[e] = fma(w, v[e], sum2[e]);
                mx[e] = fmax(mx[e], v[e]);
                mn[e] = fmin(mn[e], v[e]);
            }
        }
    } else {
        for (int n = n_begin + wave; n < n_end; n += 4) {
#pragma unroll
            for (int e = 0; e < V; ++e) {
                if (k0 + e < K) {
                    acc_t x = Unpack<T>::one(Bt, (int64_t)n * ldb + k0 + e);
                    sum[e] += x;
                    if constexpr (W) sum2[e] = fma(wvec ? wvec[n] : (acc_t)(n + 1), x, sum2[e]);
                    mx[e] = fmax(mx[e], x);
                    mn[e] = fmin(mn[e], x);
                }
            }
        }
    }
    // LDS layout [e][lane] with a pitch of 65: conflict free both for a wavefront writing one e at a time and for
    // consecutive threads reading consecutive columns (lane * V + e) afterwards
    constexpr int PITCH = 65;
    if (wave > 0) {
#pragma unroll
        for (int e = 0; e < V; ++e) {
            red[wave - 1][0][e * PITCH + lane] = sum[e];
            red[wave - 1][1][e * PITCH + lane] = mx[e];
            red[wave - 1][2][e * PITCH + lane] = mn[e];
            if constexpr (W) red[wave - 1][3][e * PITCH + lane] = sum2[e];
        }
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int w = 0; w < 3; ++w)
#pragma unroll
            for (int e = 0; e < V; ++e) {
                sum[e] += red[w][0][e * PITCH + lane];
                acc_t a = red[w][1][e * PITCH + lane], b = red[w][2][e * PITCH + lane];
                mx[e] = fmax(mx[e], a);
                mn[e] = fmin(mn[e], b);
                if constexpr (W) sum2[e] += red[w][3][e * PITCH + lane];
            }
        // the block's results go back through the first area so that the global stores are contiguous
        // (LDS operations of one wavefront complete in order: the reads above are done)
#pragma unroll
        for (int e = 0; e < V; ++e) {
            red[0][0][e * PITCH + lane] = sum[e];
            red[0][1][e * PITCH + lane] = mx[e];
            red[0][2][e * PITCH + lane] = mn[e];
            if constexpr (W) red[0][3][e * PITCH + lane] = sum2[e];
        }
    }
    __syncthreads();
    {
        acc_t* p = part + (int64_t)blockIdx.y * 4 * K;
        const int kbase = blockIdx.x * 64 * V;
#pragma unroll
        for (int j = 0; j < (64 * V + 255) / 256; ++j) {
            const int idx = threadIdx.x + 256 * j;  // column kbase + idx = lane idx / V, element idx % V
            if (idx < 64 * V && kbase + idx < K) {
                const int at = (idx % V) * PITCH + idx / V;
                p[kbase + idx] = red[0][0][at];
                p[(int64_t)K + kbase + idx] = red[0][1][at];
                p[2 * (int64_t)K + kbase + idx] = red[0][2][at];
                if constexpr (W) p[3 * (int64_t)K + kbase + idx] = red[0][3][at];
            }
        }
    }
}

// Step 2: combine the nsplit partials of column k in a fixed order: 16 columns per block,
// 16 groups of threads per column; group g folds splits g, g+16, ... in increasing order and
// the 16 group results are folded in group order.
template <typename acc_t, bool W>
__global__ __launch_bounds__(256) void encode_cols_combine_kernel(const acc_t* __restrict__ part, int nsplit, int K,
                                                                  int N, acc_t* __restrict__ Be,
                                                                  acc_t* __restrict__ Be2,
                                                                  acc_t* __restrict__ bstat,
                                                                  double* __restrict__ s_partial,
                                                                  int32_t* __restrict__ ticket,
                                                                  double* __restrict__ S) {
    __shared__ acc_t red[W ? 4 : 3][16][16];
    __shared__ double terms[16][3];
    const int kl = threadIdx.x & 15, grp = threadIdx.x >> 4;
    const int k = blockIdx.x * 16 + kl;
    acc_t sum = 0, sum2 = 0, mx = -type_max<acc_t>(), mn = type_max<acc_t>();
    if (k < K) {
        for (int s = grp; s < nsplit; s += 16) {
            const acc_t* p = part + (int64_t)s * 4 * K;
            sum += p[k];
            if constexpr (W) sum2 += p[3 * (int64_t)K + k];
            const acc_t a = p[(int64_t)K + k], b = p[2 * (int64_t)K + k];
            mx = fmax(mx, a);
            mn = fmin(mn, b);
        }
    }
    red[0][grp][kl] = sum;
    red[1][grp][kl] = mx;
    red[2][grp][kl] = mn;
    if constexpr (W) red[3][grp][kl] = sum2;
    __syncthreads();
    if (grp == 0 && k < K) {
        sum = red[0][0][kl];
        mx = red[1][0][kl];
        mn = red[2][0][kl];
        if constexpr (W) sum2 = red[3][0][kl];
#pragma unroll
        for (int g = 1; g < 16; ++g) {
            sum += red[0][g][kl];
            if constexpr (W) sum2 += red[3][g][kl];
            const acc_t a = red[1][g][kl], b = red[2][g][kl];
            mx = fmax(mx, a);
            mn = fmin(mn, b);
        }
        Be[k] = sum;
        if constexpr (W) Be2[k] = sum2;
        bstat[3 * (int64_t)k + 0] = mx;
        bstat[3 * (int64_t)k + 1] = mn;
        bstat[3 * (int64_t)k + 2] = (acc_t)((double)sum / (double)N);
    }
    // S1, S2, S3: the block's 16 columns in order, then across blocks
    if (grp == 0) {
        double t1 = 0, t2 = 0, t3 = 0;
        if (k < K) row_terms(sum, mx, mn, N, t1, t2, t3);
        terms[kl][0] = t1;
        terms[kl][1] = t2;
        terms[kl][2] = t3;
    }
    __syncthreads();
    double s1 = 0, s2 = 0, s3 = 0;
    if (threadIdx.x == 0) {
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            s1 += terms[c][0];
            s2 += terms[c][1];
            s3 += terms[c][2];
        }
    }
    publish_and_fold_S(s1, s2, s3, s_partial, ticket, S);
}

// ---------------------------------------------------------------------------
// A side: one wavefront per row m: (max, min, mean), dot with Be, threshold
// ---------------------------------------------------------------------------
// W: also the expected weighted checksum C^{r2} = A (B r2) (section 2.2).
// THR_NL: 16-byte pieces of the row in flight per lane.  Rows of 1024 pieces or more run 4 (30.0 against 31.8 us
// at 8192 x 8192 FP16), shorter ones 2 (8.8 against 9.5 us at 4096 x 4096 BF16).
template <typename T, bool W, int THR_NL>
__global__ __launch_bounds__(256) void threshold_rows_kernel(const void* __restrict__ A, int M, int K, int N,
                                                             int64_t lda,
                                                             const typename Elem<T>::acc_t* __restrict__ Be,
                                                             const typename Elem<T>::acc_t* __restrict__ Be2,
                                                             const double* __restrict__ S, double e_max,
                                                             double c_sigma,
                                                             typename Elem<T>::acc_t* __restrict__ astat,
                                                             typename Elem<T>::acc_t* __restrict__ expected,
                                                             typename Elem<T>::acc_t* __restrict__ expected2,
                                                             typename Elem<T>::acc_t* __restrict__ Tout, int vec_ok) {
    using acc_t = typename Elem<T>::acc_t;
    constexpr int V = Elem<T>::vec;
    const int lane = threadIdx.x & 63;
    const int m = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (m >= M) return;
    const char* row = reinterpret_cast<const char*>(A) + (int64_t)m * lda * Elem<T>::bytes;
    acc_t sum = 0, dot = 0, dot2 = 0, mx = -type_max<acc_t>(), mn = type_max<acc_t>();
    int done = 0;
    if (vec_ok) {
        const int nchunks = K / V;
        int c = lane;
        // THR_NL 16-byte pieces of the row in flight per lane; the matching pieces of Be come from the caches
        for (; c + 64 * (THR_NL - 1) < nchunks; c += 64 * THR_NL) {
            raw16 r[THR_NL];
#pragma unroll
            for (int u = 0; u < THR_NL; ++u) r[u] = ld16(row + (int64_t)(c + 64 * u) * 16);
#pragma unroll
            for (int u = 0; u < THR_NL; ++u) {
                acc_t v[V], b[V];
#pragma unroll
                for (int e = 0; e < V; ++e) b[e] = Be[(int64_t)(c + 64 * u) * V + e];
                Unpack<T>::run(r[u], v);
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    sum += v[e];
                    dot = fma(v[e], b[e], dot);
                    if constexpr (W) dot2 = fma(v[e], Be2[(int64_t)(c + 64 * u) * V + e], dot2);
                    mx = fmax(mx, v[e]);
                    mn = fmin(mn, v[e]);
                }
            }
        }
        for (; c < nchunks; c += 64) {
            raw16 r0 = ld16(row + (int64_t)c * 16);
            acc_t v0[V];
            Unpack<T>::run(r0, v0);
#pragma unroll
            for (int e = 0; e < V; ++e) {
                const acc_t b = Be[(int64_t)c * V + e];
                sum += v0[e];
                dot = fma(v0[e], b, dot);
                if constexpr (W) dot2 = fma(v0[e], Be2[(int64_t)c * V + e], dot2);
                mx = fmax(mx, v0[e]);
                mn = fmin(mn, v0[e]);
            }
        }
        done = nchunks * V;
    }
    for (int k = done + lane; k < K; k += 64) {
        acc_t x = Unpack<T>::one(row, k);
        sum += x;
        dot = fma(x, Be[k], dot);
        if constexpr (W) dot2 = fma(x, Be2[k], dot2);
        mx = fmax(mx, x);
        mn = fmin(mn, x);
    }
    sum = wave_sum(sum);
    dot = wave_sum(dot);
    if constexpr (W) {
        dot2 = wave_sum(dot2);
        if (lane == 0) expected2[m] = dot2;
    }
    mx = wave_max(mx);
    mn = wave_min(mn);
    if (lane == 0) {
        const double mu = (double)sum / (double)K;
        double var = ((double)mx - mu) * (mu - (double)mn);
        var = var > 0 ? var : 0;
        const double S1 = S[0], S2 = S[1], S3 = S[2];
        const double dN = (double)N;
        const double t_det = dN * fabs(mu) * S1;
        const double t_var23 = c_sigma * sqrt(dN * mu * mu * S2 + dN * dN * var * S3);
        const double t_var4 = c_sigma * sqrt(dN) * sqrt(var) * sqrt(S2);
        astat[3 * (int64_t)m + 0] = mx;
        astat[3 * (int64_t)m + 1] = mn;
        astat[3 * (int64_t)m + 2] = (acc_t)mu;
        expected[m] = dot;
        Tout[m] = (acc_t)(e_max * (t_det + t_var23 + t_var4));
    }
}

// ---------------------------------------------------------------------------
// Offline check (section 3.6 "Offline ABFT"): row sums of the product as it sits in memory after
// quantisation to the output type, compared with the expected checksum.  One wavefront per row.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void check_offline_kernel(const void* __restrict__ C, int M, int N, int64_t ldc,
                                                            const typename Elem<T>::acc_t* __restrict__ expected,
                                                            const typename Elem<T>::acc_t* __restrict__ Tthr,
                                                            typename Elem<T>::acc_t* __restrict__ rowsum,
                                                            typename Elem<T>::acc_t* __restrict__ E,
                                                            int32_t* __restrict__ flags, int32_t* __restrict__ nflag,
                                                            int vec_ok) {
    using acc_t = typename Elem<T>::acc_t;
    constexpr int V = Elem<T>::vec;
    const int lane = threadIdx.x & 63;
    const int m = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (m >= M) return;
    const char* row = reinterpret_cast<const char*>(C) + (int64_t)m * ldc * Elem<T>::bytes;
    acc_t part[4] = {0, 0, 0, 0};
    int done = 0;
    if (vec_ok) {
        const int nchunks = N / V;
        int c = lane;
        for (; c + 192 < nchunks; c += 256) {
            raw16 r[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) r[u] = ld16(row + (int64_t)(c + 64 * u) * 16);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                acc_t v[V];
                Unpack<T>::run(r[u], v);
                acc_t cs = 0;
#pragma unroll
                for (int e = 0; e < V; ++e) cs += v[e];
                part[u] += cs;
            }
        }
        for (; c < nchunks; c += 64) {
            acc_t v[V];
            Unpack<T>::run(ld16(row + (int64_t)c * 16), v);
#pragma unroll
            for (int e = 0; e < V; ++e) part[0] += v[e];
        }
        done = nchunks * V;
    }
    for (int n = done + lane; n < N; n += 64) part[1] += Unpack<T>::one(row, n);
    const acc_t s = wave_sum((part[0] + part[1]) + (part[2] + part[3]));
    if (lane == 0) {
        const acc_t e = expected[m] - s;
        const int f = !(fabs(e) <= Tthr[m]);
        rowsum[m] = s;
        E[m] = e;
        flags[m] = f;
        if (f) atomicAdd(nflag, 1);
    }
}

// ---------------------------------------------------------------------------
// host launchers
// ---------------------------------------------------------------------------

// Rows per block of the column reduction over a (rows x cols) row-major matrix: 128 or 64.  Smaller slabs put more
// loads in flight, and every halving doubles the slab partials the finishing kernel folds.  Measured (two launches,
// N x K layouts): 8192 x 8192 FP16 42.2 us with 128-row slabs, 33.3 with 64-row slabs and eight rows in flight per
// wavefront; 4096 x 4096 FP32 23.3 -> 17.2; 11008 x 4096 BF16 (172 slabs of 64 rows) 23.0 -> 28.2, hence the
// limit on the row count; below 64 rows the fold costs more than the slabs bring.
static int col_rows_per_block(int dtype, int64_t rows, int64_t cols) {
    const int64_t v = dtype == VABFT_F64 ? 2 : dtype == VABFT_F32 ? 4 : (dtype == VABFT_F8E4M3 || dtype == VABFT_F8E5M2) ? 16 : 8;
    const int64_t xblocks = (cols + 64 * v - 1) / (64 * v);
    const int64_t blocks128 = xblocks * ((rows + 127) / 128);
    return (blocks128 < 512 || (blocks128 < 2048 && rows <= 8192)) ? 64 : 128;
}

// Rows k per block of the finishing kernel: 16, or fewer (K x N layout) when 16 would leave most of the
// chip's 256 compute units without a block
static int encode_rows_per_block(const vabft_problem* p, int waves) {
    if (p->transB) return 16;
    int rpb = waves;
    while (rpb > 1 && (p->K + rpb - 1) / rpb < 256) rpb >>= 1;
    return rpb;
}
constexpr int ENC_WAVES_OWN_FOLD = 16, ENC_WAVES_DEFERRED = 8;
// Wavefronts per workgroup of the row walk.  The smaller workgroup is only used when both sizes give one
// wavefront per row (K >= 4096): with several wavefronts per row the split of a row into segments (and with it
// the rounding of Be) would depend on the workgroup size, and both routes must produce the same bits.
static int encode_rows_waves(const vabft_problem* p, bool deferred) {
    if (deferred && encode_rows_per_block(p, ENC_WAVES_OWN_FOLD) == ENC_WAVES_OWN_FOLD) return ENC_WAVES_DEFERRED;
    return ENC_WAVES_OWN_FOLD;
}
// Per-block partials of (S1, S2, S3), [blocks][3] doubles: the number an encode with the fold deferred leaves
// (what the fused GEMM folds, and what the workspace reserves; an encode that folds them itself leaves no more)
int s_partial_count(const vabft_problem* p) {
    const int rpb = encode_rows_per_block(p, encode_rows_waves(p, true));
    return (p->K + rpb - 1) / rpb;
}

size_t encode_workspace_bytes(const vabft_problem* p) {
    size_t bytes = 0;
    if (p->transB) {
        const size_t acc_bytes = p->dtype == VABFT_F64 ? 8 : 4;
        const size_t rpb = col_rows_per_block(p->dtype, p->N, p->K);
        const size_t nsplit = ((size_t)p->N + rpb - 1) / rpb;
        bytes += nsplit * 4 * (size_t)p->K * acc_bytes;  // (sum, max, min, weighted sum) per slab
    }
    return bytes;
}

template <typename T, bool W>
static int encode_launch(const vabft_problem* p, const void* dB, void* d_Be, void* d_Be2, void* d_bstat, double* d_S,
                         double* s_partial, void* ws, int32_t* ticket, hipStream_t st) {
    using acc_t = typename Elem<T>::acc_t;
    const int vec_ok = aligned16(dB) && ((p->ldb * Elem<T>::bytes) % 16 == 0);
    if (!p->transB) {
        const int waves = encode_rows_waves(p, d_S == nullptr);
        const int rpb = encode_rows_per_block(p, waves);
        const int kblocks = (p->K + rpb - 1) / rpb;
#define VABFT_ENC_ROWS(R, WV)                                                                                    \
    if constexpr (R <= WV)                                                                                       \
        encode_rows_kernel<T, W, R, WV><<<dim3(kblocks), dim3(64 * WV), 0, st>>>(                                \
            dB, p->K, p->N, p->ldb, (acc_t*)d_Be, (acc_t*)d_Be2, (acc_t*)d_bstat, vec_ok, s_partial, ticket, d_S)
#define VABFT_ENC_ROWS_SWITCH(WV)                 \
    switch (rpb) {                                \
        case 16: VABFT_ENC_ROWS(16, WV); break;   \
        case 8: VABFT_ENC_ROWS(8, WV); break;     \
        case 4: VABFT_ENC_ROWS(4, WV); break;     \
        case 2: VABFT_ENC_ROWS(2, WV); break;     \
        default: VABFT_ENC_ROWS(1, WV); break;    \
    }
        if (waves == ENC_WAVES_OWN_FOLD) {
            VABFT_ENC_ROWS_SWITCH(ENC_WAVES_OWN_FOLD)
        } else {
            VABFT_ENC_ROWS_SWITCH(ENC_WAVES_DEFERRED)
        }
#undef VABFT_ENC_ROWS_SWITCH
#undef VABFT_ENC_ROWS
    } else {
        constexpr int V = Elem<T>::vec;
        const int rpb = col_rows_per_block(p->dtype, p->N, p->K);
        const int nsplit = (p->N + rpb - 1) / rpb;
        acc_t* part = reinterpret_cast<acc_t*>(ws);
        dim3 grid((p->K + 64 * V - 1) / (64 * V), nsplit);
        if (rpb == 64)
            encode_cols_kernel<T, W, 8><<<grid, dim3(256), 0, st>>>(dB, p->K, p->N, p->ldb, rpb, part, vec_ok, nullptr);
        else
            encode_cols_kernel<T, W, 4><<<grid, dim3(256), 0, st>>>(dB, p->K, p->N, p->ldb, rpb, part, vec_ok, nullptr);
        const int kblocks = s_partial_count(p);
        encode_cols_combine_kernel<acc_t, W><<<dim3(kblocks), dim3(256), 0, st>>>(
            part, nsplit, p->K, p->N, (acc_t*)d_Be, (acc_t*)d_Be2, (acc_t*)d_bstat, s_partial, ticket, d_S);
    }
    return hipGetLastError() == hipSuccess ? VABFT_OK : VABFT_EDEVICE;
}

// d_Be2 == nullptr: plain encode; otherwise the weighted checksum is produced in the same pass
// d_S == nullptr: S1..S3 stay as the s_partial_count() per-workgroup partials in s_partial
// ws: scratch of encode_workspace_bytes(); ticket: one int32 that is zero between launches
int encode_dispatch(const vabft_problem* p, const void* dB, void* d_Be, void* d_Be2, void* d_bstat, double* d_S,
                    double* s_partial, void* ws, int32_t* ticket, hipStream_t st) {
#define VABFT_ENC_CASE(T)                                                                               \
    return d_Be2 ? encode_launch<T, true>(p, dB, d_Be, d_Be2, d_bstat, d_S, s_partial, ws, ticket, st) \
                 : encode_launch<T, false>(p, dB, d_Be, nullptr, d_bstat, d_S, s_partial, ws, ticket, st)
    switch (p->dtype) {
        case VABFT_F64: VABFT_ENC_CASE(double);
        case VABFT_F32: VABFT_ENC_CASE(float);
        case VABFT_F16: VABFT_ENC_CASE(f16_t);
        case VABFT_BF16: VABFT_ENC_CASE(bf16_t);
        case VABFT_F8E4M3: VABFT_ENC_CASE(f8_t);
        case VABFT_F8E5M2: VABFT_ENC_CASE(bf8_t);
    }
#undef VABFT_ENC_CASE
    return VABFT_EINVAL;
}

template <typename T, bool W>
static int threshold_launch(const vabft_problem* p, const void* dA, const void* d_Be, const void* d_Be2,
                            const double* d_S, double e_max, double c_sigma, void* d_astat, void* d_expected,
                            void* d_expected2, void* d_T, hipStream_t st) {
    using acc_t = typename Elem<T>::acc_t;
    const int vec_ok = aligned16(dA) && ((p->lda * Elem<T>::bytes) % 16 == 0);
    if (p->K / Elem<T>::vec >= 1024)
        threshold_rows_kernel<T, W, 4><<<dim3((p->M + 3) / 4), dim3(256), 0, st>>>(
            dA, p->M, p->K, p->N, p->lda, (const acc_t*)d_Be, (const acc_t*)d_Be2, d_S, e_max, c_sigma,
            (acc_t*)d_astat, (acc_t*)d_expected, (acc_t*)d_expected2, (acc_t*)d_T, vec_ok);
    else
        threshold_rows_kernel<T, W, 2><<<dim3((p->M + 3) / 4), dim3(256), 0, st>>>(
            dA, p->M, p->K, p->N, p->lda, (const acc_t*)d_Be, (const acc_t*)d_Be2, d_S, e_max, c_sigma,
            (acc_t*)d_astat, (acc_t*)d_expected, (acc_t*)d_expected2, (acc_t*)d_T, vec_ok);
    return hipGetLastError() == hipSuccess ? VABFT_OK : VABFT_EDEVICE;
}

// d_Be2 / d_expected2 == nullptr: plain pass; otherwise A (B r2) rides in the same read of A
int threshold_dispatch(const vabft_problem* p, const void* dA, const void* d_Be, const void* d_Be2, const double* d_S,
                       double e_max, double c_sigma, void* d_astat, void* d_expected, void* d_expected2, void* d_T,
                       hipStream_t st) {
#define VABFT_THR_CASE(T)                                                                                          \
    return d_Be2 ? threshold_launch<T, true>(p, dA, d_Be, d_Be2, d_S, e_max, c_sigma, d_astat, d_expected,        \
                                             d_expected2, d_T, st)                                                 \
                 : threshold_launch<T, false>(p, dA, d_Be, nullptr, d_S, e_max, c_sigma, d_astat, d_expected,      \
                                              nullptr, d_T, st)
    switch (p->dtype) {
        case VABFT_F64: VABFT_THR_CASE(double);
        case VABFT_F32: VABFT_THR_CASE(float);
        case VABFT_F16: VABFT_THR_CASE(f16_t);
        case VABFT_BF16: VABFT_THR_CASE(bf16_t);
        case VABFT_F8E4M3: VABFT_THR_CASE(f8_t);
        case VABFT_F8E5M2: VABFT_THR_CASE(bf8_t);
    }
#undef VABFT_THR_CASE
    return VABFT_EINVAL;
}

// ---------------------------------------------------------------------------
// Column checksums (section 2.2: c1 = [1 .. 1], A^c = [A; c1 A], C^{c1} = c1 A B).  By the symmetry
// C^T = B^T A^T the column check is Algorithm 1 with the roles exchanged: column j of B (K entries) plays
// the row of A, column k of A (M entries) plays the row of B, and M replaces N.
// ---------------------------------------------------------------------------

// Per column n of a K x N row-major B: fold the row-slab partials (sum, max, min, dot with c1 A) in slab
// order and evaluate the column threshold.
template <typename acc_t>
__global__ __launch_bounds__(256) void threshold_cols_finish_kernel(const acc_t* __restrict__ part, int nsplit,
                                                                    int N, int K, int M, const double* __restrict__ SA,
                                                                    double e_max, double c_sigma,
                                                                    acc_t* __restrict__ colstat,
                                                                    acc_t* __restrict__ expected_col,
                                                                    acc_t* __restrict__ Tcol) {
    const int n = blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    acc_t sum = 0, dot = 0, mx = -type_max<acc_t>(), mn = type_max<acc_t>();
    for (int s0 = 0; s0 < nsplit; s0 += 8) {
        // eight slabs' loads in flight at once; folded in slab order
        acc_t v[8][4];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int sc = s0 + u < nsplit ? s0 + u : nsplit - 1;
            const acc_t* q = part + (int64_t)sc * 4 * N;
#pragma unroll
            for (int c = 0; c < 4; ++c) v[u][c] = q[c * (int64_t)N + n];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (s0 + u < nsplit) {
                sum += v[u][0];
                mx = fmax(mx, v[u][1]);
                mn = fmin(mn, v[u][2]);
                dot += v[u][3];
            }
    }
    const double mu = (double)sum / (double)K;
    double var = ((double)mx - mu) * (mu - (double)mn);
    var = var > 0 ? var : 0;
    const double S1 = SA[0], S2 = SA[1], S3 = SA[2], dM = (double)M;
    const double t_det = dM * fabs(mu) * S1;
    const double t_var23 = c_sigma * sqrt(dM * mu * mu * S2 + dM * dM * var * S3);
    const double t_var4 = c_sigma * sqrt(dM) * sqrt(var) * sqrt(S2);
    colstat[3 * (int64_t)n + 0] = mx;
    colstat[3 * (int64_t)n + 1] = mn;
    colstat[3 * (int64_t)n + 2] = (acc_t)mu;
    expected_col[n] = dot;
    Tcol[n] = (acc_t)(e_max * (t_det + t_var23 + t_var4));
}

static vabft_problem swapped_problem(const vabft_problem* p, int32_t M, int32_t N, int32_t transB, int64_t lda,
                                     int64_t ldb) {
    vabft_problem q = *p;
    q.M = M;
    q.N = N;
    q.transB = transB;
    q.lda = lda;
    q.ldb = ldb;
    return q;
}

// scratch of the two column-side passes: encode of A as an (M rows) x (K columns) "weight layout" matrix, and
// the slab partials of the column reduction over a K x N B
size_t cols_workspace_bytes(const vabft_problem* p) {
    const vabft_problem qa = swapped_problem(p, p->M, p->M, 1, p->lda, p->lda);
    const size_t a = encode_workspace_bytes(&qa);
    const size_t acc_bytes = p->dtype == VABFT_F64 ? 8 : 4;
    const size_t rpb = col_rows_per_block(p->dtype, p->K, p->N);
    const size_t nsplit = ((size_t)p->K + rpb - 1) / rpb;
    const size_t b = p->transB ? 0 : nsplit * 4 * (size_t)p->N * acc_bytes;
    return a > b ? a : b;
}

// c1 A, column statistics of A and their aggregates: the encode of the N x K layout applied to A (M x K)
int encode_a_dispatch(const vabft_problem* p, const void* dA, void* d_eA, void* d_acolstat, double* d_SA,
                      double* s_partial, void* ws, int32_t* ticket, hipStream_t st) {
    const vabft_problem q = swapped_problem(p, p->M, p->M, 1, p->lda, p->lda);
    return encode_dispatch(&q, dA, d_eA, nullptr, d_acolstat, d_SA, s_partial, ws, ticket, st);
}

template <typename T>
static int threshold_cols_launch(const vabft_problem* p, const void* dB, const void* d_eA, const double* d_SA,
                                 double e_max, double c_sigma, void* d_bcolstat, void* d_expected_col, void* d_Tcol,
                                 void* ws, hipStream_t st) {
    using acc_t = typename Elem<T>::acc_t;
    constexpr int V = Elem<T>::vec;
    const int vec_ok = aligned16(dB) && ((p->ldb * Elem<T>::bytes) % 16 == 0);
    const int rpb = col_rows_per_block(p->dtype, p->K, p->N);
    const int nsplit = (p->K + rpb - 1) / rpb;
    acc_t* part = reinterpret_cast<acc_t*>(ws);
    dim3 grid((p->N + 64 * V - 1) / (64 * V), nsplit);
    // rows of the reduction = k (K of them), columns = n (N of them), weight of row k = (c1 A)[k]
    encode_cols_kernel<T, true, 4><<<grid, dim3(256), 0, st>>>(dB, p->N, p->K, p->ldb, rpb, part, vec_ok,
                                                            (const acc_t*)d_eA);
    threshold_cols_finish_kernel<acc_t><<<dim3((p->N + 255) / 256), dim3(256), 0, st>>>(
        part, nsplit, p->N, p->K, p->M, d_SA, e_max, c_sigma, (acc_t*)d_bcolstat, (acc_t*)d_expected_col,
        (acc_t*)d_Tcol);
    return hipGetLastError() == hipSuccess ? VABFT_OK : VABFT_EDEVICE;
}

int threshold_cols_dispatch(const vabft_problem* p, const void* dB, const void* d_eA, const double* d_SA, double e_max,
                            double c_sigma, void* d_bcolstat, void* d_expected_col, void* d_Tcol, void* ws,
                            hipStream_t st) {
    if (p->transB) {
        // B stored N x K: its rows are the columns of the logical B, so this is the row pass with M := N, N := M
        const vabft_problem q = swapped_problem(p, p->N, p->M, 0, p->ldb, p->ldb);
        return threshold_dispatch(&q, dB, d_eA, nullptr, d_SA, e_max, c_sigma, d_bcolstat, d_expected_col, nullptr,
                                  d_Tcol, st);
    }
    switch (p->dtype) {
        case VABFT_F64:
            return threshold_cols_launch<double>(p, dB, d_eA, d_SA, e_max, c_sigma, d_bcolstat, d_expected_col, d_Tcol,
                                                 ws, st);
        case VABFT_F32:
            return threshold_cols_launch<float>(p, dB, d_eA, d_SA, e_max, c_sigma, d_bcolstat, d_expected_col, d_Tcol,
                                                ws, st);
        case VABFT_F16:
            return threshold_cols_launch<f16_t>(p, dB, d_eA, d_SA, e_max, c_sigma, d_bcolstat, d_expected_col, d_Tcol,
                                                ws, st);
        case VABFT_BF16:
            return threshold_cols_launch<bf16_t>(p, dB, d_eA, d_SA, e_max, c_sigma, d_bcolstat, d_expected_col, d_Tcol,
                                                 ws, st);
        case VABFT_F8E4M3:
            return threshold_cols_launch<f8_t>(p, dB, d_eA, d_SA, e_max, c_sigma, d_bcolstat, d_expected_col, d_Tcol,
                                               ws, st);
        case VABFT_F8E5M2:
            return threshold_cols_launch<bf8_t>(p, dB, d_eA, d_SA, e_max, c_sigma, d_bcolstat, d_expected_col, d_Tcol,
                                                ws, st);
    }
    return VABFT_EINVAL;
}

int check_offline_dispatch(const vabft_problem* p, const void* dC, const void* d_expected, const void* d_T,
                           void* d_rowsum, void* d_E, int32_t* d_flags, int32_t* d_nflag, hipStream_t st) {
    const dim3 grid((p->M + 3) / 4), block(256);
#define VABFT_OFF_CASE(T)                                                                                           \
    {                                                                                                               \
        using acc_t = typename Elem<T>::acc_t;                                                                      \
        const int vec_ok = aligned16(dC) && ((p->ldc * Elem<T>::bytes) % 16 == 0);                                  \
        check_offline_kernel<T><<<grid, block, 0, st>>>(dC, p->M, p->N, p->ldc, (const acc_t*)d_expected,           \
                                                        (const acc_t*)d_T, (acc_t*)d_rowsum, (acc_t*)d_E, d_flags,  \
                                                        d_nflag, vec_ok);                                           \
        break;                                                                                                      \
    }
    switch (p->dtype) {
        case VABFT_F64: VABFT_OFF_CASE(double)
        case VABFT_F32: VABFT_OFF_CASE(float)
        case VABFT_F16: VABFT_OFF_CASE(f16_t)
        case VABFT_F8E4M3:
        case VABFT_F8E5M2: VABFT_OFF_CASE(f16_t)  // the stored product of an FP8 problem is FP16
        case VABFT_BF16: VABFT_OFF_CASE(bf16_t)
        default: return VABFT_EINVAL;
    }
#undef VABFT_OFF_CASE
    return hipGetLastError() == hipSuccess ? VABFT_OK : VABFT_EDEVICE;
}

}  // namespace vabft
