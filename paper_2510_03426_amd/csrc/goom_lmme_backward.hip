// Backward pass of C' = LMME(A', B') (paper Section 3.2, with the derivatives of Section 3.1 in the limit eps -> 0).
//
// With C = A B over reals and G_ik the gradient of a loss with respect to the log-magnitude of C_ik,
//     dL / d Re A'_ij = A_ij sum_k (G_ik / C_ik) B_jk,        dL / d Re B'_jk = B_jk sum_i A_ij (G_ik / C_ik):
// two more matrix products, taken over GOOMs by the forward LMME itself on operands prepared here.
//
// A float log-magnitude near 1000 is only good to 6e-5, and W = G / C is as small as C is large, so the products do
// not run on A', B' and W' as given but with the row maxima r_i of A' and the column maxima c_k of B', rounded to
// whole numbers, taken out: A~ = A e^(-r_i), B~ = B e^(-c_k), W~_ik = G_ik / (C_ik e^(-r_i - c_k)).  Subtracting a
// whole number near a log-magnitude is exact in the component type, all three have log-magnitudes of ordinary size,
// and the shifts cancel in the results:  A_ij sum_k W_ik B_jk = A~_ij sum_k W~_ik B~_jk, likewise for B.
//
//   prepare  r_i = rint(max_j Re A'_ij), c_k = rint(max_j Re B'_jk)                (0 for an all-zero row / column)
//            A~'^T [d, n];  B~'^T [m, d]  (found and taken out by the transposing kernels);  W~' [n, m]
//   LMME     X~' = LMME(W~', B~'^T) [n, d];  Y~' = LMME(A~'^T, W~') [d, m]         (the forward kernels)
//   finish   grad_A_ij = +- exp(Re A~'_ij + Re X~'_ij),  grad_B_jk = +- exp(Re B~'_jk + Re Y~'_jk)
// For n = d = m = 128 the product kernel reads its operand transposed, takes the shift out and forms the gradient in its store
// pass itself: only the shifts and W~' are prepared here.
#include "goom_internal.h"

namespace {

constexpr double kInvPi = 0.318309886183790671538;
constexpr int kTile = 32;

template <typename R> struct C2;
template <> struct C2<float> { typedef float2 type; };
template <> struct C2<double> { typedef double2 type; };

template <typename R> __device__ inline R neg_inf() { return sizeof(R) == 4 ? (R)-__builtin_huge_valf() : (R)-__builtin_huge_val(); }
template <typename R> __device__ inline R pi_of() { return sizeof(R) == 4 ? (R)3.14159274101257324219f : (R)3.14159265358979311600; }
template <typename R> __device__ inline bool odd_phase(R im)
{
    const int k = (int)__builtin_rint((double)im * kInvPi);
    return (k & 1) != 0;
}
template <typename R> __device__ inline R whole_shift(R top)
{
    const bool finite = top > neg_inf<R>() && top < -neg_inf<R>();
    return finite ? (R)__builtin_rint((double)top) : (R)0;
}
template <typename R> __device__ inline double exp_for(double s)
{
    if (sizeof(R) == 4) return (double)__builtin_amdgcn_exp2f((float)(s * 1.44269504088896340736));
    return exp(s);
}

// dst[b, c, r] = src[b, r, c] with a whole-number shift taken from the log-magnitude: the maximum of the row (BY_ROW) or of the
// column, rounded, which the kernel finds itself and also writes to shift[b, r] or shift[b, c].  One workgroup per strip of 32 rows
// (BY_ROW; all columns) or 32 columns (all rows) of one batch item: a first pass over the strip for the maxima, a second one, out
// of L2, in 32 x 32 tiles through LDS so that both the reads and the writes are contiguous.  Grid: b * strips + strip.
template <typename R, bool BY_ROW> __global__ __launch_bounds__(256) void transpose_shift_kernel(const typename C2<R>::type *__restrict__ src,
                                                                                                R *__restrict__ shift,
                                                                                                typename C2<R>::type *__restrict__ dst, int rows, int cols)
{
    typedef typename C2<R>::type c2;
    __shared__ c2 tile[kTile][kTile + 1];
    __shared__ R red[8][kTile];
    __shared__ R sh[kTile];
    const int strips = ((BY_ROW ? rows : cols) + kTile - 1) / kTile;
    const size_t b = blockIdx.x / strips;
    const int s0 = (int)(blockIdx.x - b * strips) * kTile;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5; // 8 rows of 32 per pass
    const c2 *item = src + b * rows * (size_t)cols;
    if (BY_ROW) { // wave w: rows s0 + 8 w .. s0 + 8 w + 7, lanes along the row
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        R top[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            top[q] = neg_inf<R>();
            const int r = s0 + wave * 8 + q;
            if (r < rows)
                for (int j = lane; j < cols; j += 64) {
                    const R v = item[(size_t)r * cols + j].x;
                    top[q] = v > top[q] ? v : top[q];
                }
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            for (int sft = 32; sft > 0; sft >>= 1) {
                const R o = __shfl_xor(top[q], sft, 64);
                top[q] = o > top[q] ? o : top[q];
            }
            if (lane == 0) sh[wave * 8 + q] = whole_shift<R>(top[q]);
        }
    } else { // thread (tx, ty): column s0 + tx, rows ty, ty + 8, ...
        R top = neg_inf<R>();
        if (s0 + tx < cols)
            for (int r = ty; r < rows; r += 8) {
                const R v = item[(size_t)r * cols + s0 + tx].x;
                top = v > top ? v : top;
            }
        red[ty][tx] = top;
        __syncthreads();
        if (ty == 0) {
            for (int q = 1; q < 8; ++q) top = red[q][tx] > top ? red[q][tx] : top;
            sh[tx] = whole_shift<R>(top);
        }
    }
    __syncthreads();
    if (threadIdx.x < kTile && s0 + (int)threadIdx.x < (BY_ROW ? rows : cols)) shift[b * (size_t)(BY_ROW ? rows : cols) + s0 + threadIdx.x] = sh[threadIdx.x];
    const int span = BY_ROW ? cols : rows; // the tiles of the strip
    for (int t0 = 0; t0 < span; t0 += kTile) {
        const int r0 = BY_ROW ? s0 : t0, c0 = BY_ROW ? t0 : s0;
        for (int q = ty; q < kTile; q += 8) {
            const int r = r0 + q, c = c0 + tx;
            if (r < rows && c < cols) {
                c2 v = item[(size_t)r * cols + c];
                v.x = (R)((double)v.x - (double)sh[BY_ROW ? q : tx]);
                tile[q][tx] = v;
            }
        }
        __syncthreads();
        for (int q = ty; q < kTile; q += 8) {
            const int c = c0 + q, r = r0 + tx;
            if (r < rows && c < cols) dst[(b * cols + c) * (size_t)rows + r] = tile[tx][q];
        }
        __syncthreads();
    }
}

// The shifts alone, for products that take them out of their operands themselves: r[b, i] = rint(max_j Re A[b, i, j]), sixteen lanes a
// row; c[b, k] = rint(max_j Re B[b, j, k]), one thread per column (neighbouring threads read neighbouring columns).
template <typename R> __global__ __launch_bounds__(256) void row_shift_kernel(const typename C2<R>::type *__restrict__ A, R *__restrict__ r, long long rows,
                                                                              int cols)
{
    // sixteen lanes a row, four rows a wave
    const int lane = threadIdx.x & 63, sub = lane & 15;
    const long long row = ((long long)blockIdx.x * 4 + (threadIdx.x >> 6)) * 4 + (lane >> 4);
    R top = neg_inf<R>();
    if (row < rows) {
        const typename C2<R>::type *src = A + (size_t)row * cols;
        for (int j = sub; j < cols; j += 16) {
            const R v = src[j].x;
            top = v > top ? v : top;
        }
    }
    for (int s = 8; s > 0; s >>= 1) {
        const R o = __shfl_xor(top, s, 64);
        top = o > top ? o : top;
    }
    if (sub == 0 && row < rows) r[row] = whole_shift<R>(top);
}

template <typename R> __global__ __launch_bounds__(256) void col_shift_kernel(const typename C2<R>::type *__restrict__ B, R *__restrict__ c, int rows,
                                                                              int cols)
{
    __shared__ R red[8][32];
    const int per = (cols + 31) / 32; // workgroups per batch item: 32 columns each, 8 threads a column
    const size_t b = blockIdx.x / per;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int k = (int)(blockIdx.x - b * per) * 32 + tx;
    R top = neg_inf<R>();
    if (k < cols)
        for (int j = ty; j < rows; j += 8) {
            const R v = B[(b * rows + j) * (size_t)cols + k].x;
            top = v > top ? v : top;
        }
    red[ty][tx] = top;
    __syncthreads();
    if (ty == 0 && k < cols) {
        for (int q = 1; q < 8; ++q) top = red[q][tx] > top ? red[q][tx] : top;
        c[b * cols + k] = whole_shift<R>(top);
    }
}

constexpr int kPerGroup = 1024; // elements of one batch item per workgroup of the elementwise kernels

template <typename R> __device__ inline double log_for(double g)
{
    if (sizeof(R) == 4) return (double)__builtin_logf((float)g);
    return log(g);
}

// W~'[b, i, k] = GOOM(G[b, i, k]) - (C'[b, i, k] - r[b, i] - c[b, k]); zero where G is zero or C is zero.
// Grid: b * groups + group, a group being 1024 consecutive entries of one batch item (n m <= 2^20: 32-bit index arithmetic).
template <typename R> __global__ __launch_bounds__(256) void ratio_kernel(const R *__restrict__ G, const typename C2<R>::type *__restrict__ Cm,
                                                                          const R *__restrict__ r, const R *__restrict__ c,
                                                                          typename C2<R>::type *__restrict__ W, int n, int m)
{
    typedef typename C2<R>::type c2;
    const unsigned per_item = (unsigned)n * (unsigned)m, groups = (per_item + kPerGroup - 1) / kPerGroup;
    const size_t b = blockIdx.x / groups;
    const unsigned o0 = (unsigned)(blockIdx.x - b * groups) * kPerGroup + threadIdx.x;
    const size_t base = b * per_item;
#pragma unroll
    for (int u = 0; u < kPerGroup / 256; ++u) {
        const unsigned o = o0 + u * 256;
        if (o < per_item) {
            const unsigned i = o / (unsigned)m, k = o - i * (unsigned)m;
            const double g = (double)G[base + o];
            const c2 cv = Cm[base + o];
            const bool neg = (g < 0.0) != odd_phase<R>(cv.y);
            c2 w;
            if (g == 0.0 || cv.x == neg_inf<R>())
                w = c2{neg_inf<R>(), (R)0};
            else
                w = c2{(R)(log_for<R>(__builtin_fabs(g)) - ((double)cv.x - (double)r[b * n + i] - (double)c[b * m + k])), neg ? pi_of<R>() : (R)0};
            W[base + o] = w;
        }
    }
}

// grad[b, p, q] = +- exp((Re Z'[b, p, q] - shift) + Re X'[b, p, q]), shift = s[b, p] (BY_ROW) or s[b, q]; same grid as above
template <typename R, bool BY_ROW> __global__ __launch_bounds__(256) void finish_kernel(const typename C2<R>::type *__restrict__ Z,
                                                                                       const typename C2<R>::type *__restrict__ X,
                                                                                       const R *__restrict__ s, R *__restrict__ grad, int rows, int cols)
{
    typedef typename C2<R>::type c2;
    const unsigned per_item = (unsigned)rows * (unsigned)cols, groups = (per_item + kPerGroup - 1) / kPerGroup;
    const size_t b = blockIdx.x / groups;
    const unsigned o0 = (unsigned)(blockIdx.x - b * groups) * kPerGroup + threadIdx.x;
    const size_t base = b * per_item;
#pragma unroll
    for (int u = 0; u < kPerGroup / 256; ++u) {
        const unsigned o = o0 + u * 256;
        if (o < per_item) {
            const unsigned p = o / (unsigned)cols, q = o - p * (unsigned)cols;
            const c2 z = Z[base + o], x = X[base + o];
            double v = 0.0;
            if (z.x != neg_inf<R>() && x.x != neg_inf<R>()) v = exp_for<R>(((double)z.x - (double)s[BY_ROW ? b * rows + p : b * cols + q]) + (double)x.x);
            grad[base + o] = (R)(odd_phase<R>(z.y) != odd_phase<R>(x.y) ? -v : v);
        }
    }
}

unsigned groups_for(long long batch, int rows, int cols) { return (unsigned)(batch * (((long long)rows * cols + kPerGroup - 1) / kPerGroup)); }

template <typename R> int prepare_t(goom_ctx *ctx, const void *A, const void *B, const void *Cm, const void *G, void *r, void *c, void *W, void *At, void *Bt,
                                    long long batch, int n, int d, int m)
{
    typedef typename C2<R>::type c2;
    goom::prof_begin(ctx, "lmme_backward_prepare");
    hipLaunchKernelGGL((transpose_shift_kernel<R, true>), dim3((unsigned)(batch * ((n + kTile - 1) / kTile))), dim3(256), 0, ctx->stream,
                       static_cast<const c2 *>(A), static_cast<R *>(r), static_cast<c2 *>(At), n, d);
    hipLaunchKernelGGL((transpose_shift_kernel<R, false>), dim3((unsigned)(batch * ((m + kTile - 1) / kTile))), dim3(256), 0, ctx->stream,
                       static_cast<const c2 *>(B), static_cast<R *>(c), static_cast<c2 *>(Bt), d, m);
    hipLaunchKernelGGL(ratio_kernel<R>, dim3(groups_for(batch, n, m)), dim3(256), 0, ctx->stream, static_cast<const R *>(G), static_cast<const c2 *>(Cm),
                       static_cast<const R *>(r), static_cast<const R *>(c), static_cast<c2 *>(W), n, m);
    goom::prof_end(ctx);
    return goom::check_hip(ctx, hipGetLastError(), "launch lmme_backward_prepare");
}

template <typename R> int prepare128_t(goom_ctx *ctx, const void *A, const void *B, const void *Cm, const void *G, void *r, void *c, void *W, long long batch)
{
    typedef typename C2<R>::type c2;
    const int n = 128;
    goom::prof_begin(ctx, "lmme_backward_prepare");
    hipLaunchKernelGGL(row_shift_kernel<R>, dim3((unsigned)((batch * n + 15) / 16)), dim3(256), 0, ctx->stream, static_cast<const c2 *>(A), static_cast<R *>(r),
                       batch * n, n);
    hipLaunchKernelGGL(col_shift_kernel<R>, dim3((unsigned)(batch * ((n + 31) / 32))), dim3(256), 0, ctx->stream, static_cast<const c2 *>(B), static_cast<R *>(c), n,
                       n);
    hipLaunchKernelGGL(ratio_kernel<R>, dim3(groups_for(batch, n, n)), dim3(256), 0, ctx->stream, static_cast<const R *>(G), static_cast<const c2 *>(Cm),
                       static_cast<const R *>(r), static_cast<const R *>(c), static_cast<c2 *>(W), n, n);
    goom::prof_end(ctx);
    return goom::check_hip(ctx, hipGetLastError(), "launch lmme_backward_prepare");
}

template <typename R> int finish_t(goom_ctx *ctx, const void *A, const void *B, const void *X, const void *Y, const void *r, const void *c, void *gA, void *gB,
                                   long long batch, int n, int d, int m)
{
    typedef typename C2<R>::type c2;
    goom::prof_begin(ctx, "lmme_backward_finish");
    hipLaunchKernelGGL((finish_kernel<R, true>), dim3(groups_for(batch, n, d)), dim3(256), 0, ctx->stream, static_cast<const c2 *>(A), static_cast<const c2 *>(X),
                       static_cast<const R *>(r), static_cast<R *>(gA), n, d);
    hipLaunchKernelGGL((finish_kernel<R, false>), dim3(groups_for(batch, d, m)), dim3(256), 0, ctx->stream, static_cast<const c2 *>(B), static_cast<const c2 *>(Y),
                       static_cast<const R *>(c), static_cast<R *>(gB), d, m);
    goom::prof_end(ctx);
    return goom::check_hip(ctx, hipGetLastError(), "launch lmme_backward_finish");
}

} // namespace

namespace goom {

int launch_lmme_backward_prepare(goom_ctx *ctx, const void *A, const void *B, const void *Cm, const void *G, void *r, void *c, void *W, void *At, void *Bt,
                                 long long batch, int n, int d, int m, int dtype)
{
    return dtype == GOOM_C64 ? prepare_t<float>(ctx, A, B, Cm, G, r, c, W, At, Bt, batch, n, d, m)
                             : prepare_t<double>(ctx, A, B, Cm, G, r, c, W, At, Bt, batch, n, d, m);
}

int launch_lmme_backward_prepare128(goom_ctx *ctx, const void *A, const void *B, const void *Cm, const void *G, void *r, void *c, void *W, long long batch,
                                    int dtype)
{
    return dtype == GOOM_C64 ? prepare128_t<float>(ctx, A, B, Cm, G, r, c, W, batch) : prepare128_t<double>(ctx, A, B, Cm, G, r, c, W, batch);
}

int launch_lmme_backward_finish(goom_ctx *ctx, const void *A, const void *B, const void *X, const void *Y, const void *r, const void *c, void *gA, void *gB,
                                long long batch, int n, int d, int m, int dtype)
{
    return dtype == GOOM_C64 ? finish_t<float>(ctx, A, B, X, Y, r, c, gA, gB, batch, n, d, m) : finish_t<double>(ctx, A, B, X, Y, r, c, gA, gB, batch, n, d, m);
}

} // namespace goom
