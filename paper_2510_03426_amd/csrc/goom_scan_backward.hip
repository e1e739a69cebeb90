// Backward pass of the prefix scan P_t = M_t P_{t-1} over GOOMs (paper Section 4.1, with the derivatives of
// Section 3.1 in the limit eps -> 0).  P_{-1} is the initial state S0 (d x m) or, without one, the identity.
//
// With G_t the gradient of a loss with respect to the log-magnitudes of P_t, the adjoints of the values are d x m
// matrices that run backwards through the transposed factors:  Lam_t = G_t / P_t + M_{t+1}^T Lam_{t+1}.  Stacked on
// an identity, [Lam_t; I] = [[M_{t+1}^T, G_t / P_t], [0, I]] [Lam_{t+1}; I]: a prefix scan of (d + m) x (d + m)
// matrices in reverse time with the initial state [0; I], which the forward scan runs as it stands.  Then
//     dL / d Re M'_t[i, j] = M_t[i, j] sum_k Lam_t[i, k] P_{t-1}[j, k]           (one LMME per step, batched),
//     dL / d Re S0'[j, k] = S0[j, k] (M_0^T Lam_0)[j, k]                          (one more step of the same scan).
//
// The adjoints shrink as fast as the states grow and a float log-magnitude near 1000 is only good to 6e-5, so the
// scan runs on Lamhat_t = Lam_t e^(c_t), c_t the whole number nearest the largest log-magnitude of P_t:
//     Lamhat_t = G_t / (P_t e^(-c_t)) + (e^(c_t - c_{t+1}) M_{t+1}^T) Lamhat_{t+1},
// whose operands have log-magnitudes of ordinary size (P'_t - c_t is exact in the component type), and the
// gradients are formed from Lamhat_t, P_{t-1} e^(-c_{t-1}) and the whole number c_{t-1} - c_t.
//
// Kernels here (the scan and the LMME are the library's own):
//   scales     c[b, t + 1] for t = -1 .. T - 1                                            one wave per state
//   factors    F[b, s] = [[Nhat, Ghat], [0, I]] for s = T - 1 - t (and s = T: the step onto S0)  one workgroup per step
//   operands   Lamhat_t (the top d rows of the scan's state s = T - 1 - t) and (P'_{t-1} - c_{t-1})^T, contiguous
//   gradients  +- exp(M'_t + (c_{t-1} - c_t) + X'_t), X'_t = LMME(Lamhat'_t, Phat'^T_{t-1});  S0' + Lamhat'_{-1} - c_{-1}
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
template <typename R> __device__ inline double exp_for(double s)
{
    if (sizeof(R) == 4) return (double)__builtin_amdgcn_exp2f((float)(s * 1.44269504088896340736));
    return exp(s);
}
template <typename R> __device__ inline double log_for(double g)
{
    if (sizeof(R) == 4) return (double)__builtin_logf((float)g);
    return log(g);
}

// c[b, u], u = t + 1: the whole number nearest the largest log-magnitude of P_t (u = 0: of S0, or 0 for the identity);
// 0 for a state that is all zeros or not finite.  One wave per state.
template <typename R> __global__ __launch_bounds__(256) void scales_kernel(const typename C2<R>::type *__restrict__ P, const typename C2<R>::type *__restrict__ S0,
                                                                           R *__restrict__ c, long long T, int dm, long long total)
{
    const int lane = threadIdx.x & 63;
    const long long w = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (w >= total) return; // whole wave
    const long long b = w / (T + 1), u = w - b * (T + 1);
    const typename C2<R>::type *src = u == 0 ? (S0 ? S0 + (size_t)b * dm : nullptr) : P + (size_t)(b * T + u - 1) * dm;
    R top = neg_inf<R>();
    if (src)
        for (int e = lane; e < dm; e += 64) {
            const R v = src[e].x;
            top = v > top ? v : top;
        }
    for (int s = 32; s > 0; s >>= 1) {
        const R o = __shfl_xor(top, s, 64);
        top = o > top ? o : top;
    }
    const bool finite = top > neg_inf<R>() && top < -neg_inf<R>();
    if (lane == 0) c[w] = finite ? (R)__builtin_rint((double)top) : (R)0;
}

// dst[r][c] (row stride ldd) = src[c][r] (row stride lds) + delta on the log-magnitude, for r < rows, c < cols of dst;
// the whole workgroup (256 threads), 32 x 32 tiles through LDS
template <typename R> __device__ inline void transpose_add(const typename C2<R>::type *__restrict__ src, int lds, typename C2<R>::type *__restrict__ dst, int ldd,
                                                           int rows, int cols, double delta, typename C2<R>::type (*tile)[kTile + 1])
{
    typedef typename C2<R>::type c2;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int r0 = 0; r0 < rows; r0 += kTile)
        for (int c0 = 0; c0 < cols; c0 += kTile) {
            for (int q = ty; q < kTile; q += 8) { // source rows c0 + q, source columns r0 + tx
                const int sr = c0 + q, sc = r0 + tx;
                if (sr < cols && sc < rows) {
                    c2 v = src[(size_t)sr * lds + sc];
                    v.x = (R)((double)v.x + delta);
                    tile[q][tx] = v;
                }
            }
            __syncthreads();
            for (int q = ty; q < kTile; q += 8) {
                const int r = r0 + q, c = c0 + tx;
                if (r < rows && c < cols) dst[(size_t)r * ldd + c] = tile[tx][q];
            }
            __syncthreads();
        }
}

// One workgroup per (b, s): the factor of step s of the stacked reverse scan, (d + m) x (d + m); s = T exists only with S0.
// Workgroup 0 of every batch item also writes the initial state [0; I], (d + m) x m.
template <typename R> __global__ __launch_bounds__(256) void factors_kernel(const typename C2<R>::type *__restrict__ M, const typename C2<R>::type *__restrict__ P,
                                                                            const R *__restrict__ G, const R *__restrict__ c,
                                                                            typename C2<R>::type *__restrict__ F, typename C2<R>::type *__restrict__ init,
                                                                            long long T, long long nsteps, int d, int m)
{
    typedef typename C2<R>::type c2;
    __shared__ c2 tile[kTile][kTile + 1];
    const int D = d + m;
    const long long b = blockIdx.x / nsteps, s = blockIdx.x - b * nsteps, t = T - 1 - s; // t = -1 for s = T
    c2 *f = F + (size_t)blockIdx.x * D * D;
    const c2 zero = c2{neg_inf<R>(), (R)0}, one = c2{(R)0, (R)0};
    const R *cb = c + b * (T + 1);
    // the lower m rows: [0, I]
    for (int e = threadIdx.x; e < m * D; e += 256) {
        const int r = e / D, col = e - r * D;
        f[(size_t)(d + r) * D + col] = col == d + r ? one : zero;
    }
    if (s == 0)
        for (int e = threadIdx.x; e < D * m; e += 256) {
            const int r = e / m, col = e - r * m;
            init[(size_t)b * D * m + e] = r == d + col ? one : zero;
        }
    // upper right: G_t / (P_t e^(-c_t)), zero where G is zero or the state is zero (and for the step onto S0)
    const double ct = (double)cb[t + 1];
    for (int e = threadIdx.x; e < d * m; e += 256) {
        const int r = e / m, col = e - r * m;
        c2 w = zero;
        if (t >= 0) {
            const size_t at = (size_t)(b * T + t) * d * m + e;
            const double g = (double)G[at];
            const c2 pv = P[at];
            if (g != 0.0 && pv.x != neg_inf<R>())
                w = c2{(R)(log_for<R>(__builtin_fabs(g)) - ((double)pv.x - ct)), (g < 0.0) != odd_phase<R>(pv.y) ? pi_of<R>() : (R)0};
        }
        f[(size_t)r * D + d + col] = w;
    }
    // upper left: e^(c_t - c_{t+1}) M_{t+1}^T; the zero matrix at s = 0 (nothing follows the last step)
    if (s == 0) {
        for (int e = threadIdx.x; e < d * d; e += 256) f[(size_t)(e / d) * D + e % d] = zero;
    } else {
        transpose_add<R>(M + (size_t)(b * T + t + 1) * d * d, d, f, D, d, d, ct - (double)cb[t + 2], tile);
    }
}

// One workgroup per (b, t): Lam[b, t] = the top d rows of state s = T - 1 - t; Pt[b, t] = (P'_{t-1} - c_{t-1})^T, m x d
// (t = 0: S0, or the identity).
template <typename R> __global__ __launch_bounds__(256) void operands_kernel(const typename C2<R>::type *__restrict__ states, const typename C2<R>::type *__restrict__ P,
                                                                             const typename C2<R>::type *__restrict__ S0, const R *__restrict__ c,
                                                                             typename C2<R>::type *__restrict__ Lam, typename C2<R>::type *__restrict__ Pt,
                                                                             long long T, long long nsteps, int d, int m)
{
    typedef typename C2<R>::type c2;
    __shared__ c2 tile[kTile][kTile + 1];
    const int D = d + m;
    const long long b = blockIdx.x / T, t = blockIdx.x - b * T;
    const c2 *st = states + (size_t)(b * nsteps + (T - 1 - t)) * D * m;
    c2 *lam = Lam + (size_t)blockIdx.x * d * m;
    for (int e = threadIdx.x; e < d * m; e += 256) lam[e] = st[e];
    c2 *pt = Pt + (size_t)blockIdx.x * m * d;
    const c2 *prev = t > 0 ? P + (size_t)(b * T + t - 1) * d * m : (S0 ? S0 + (size_t)b * d * m : nullptr);
    if (prev) {
        transpose_add<R>(prev, m, pt, d, m, d, -(double)c[b * (T + 1) + t], tile);
    } else {
        const c2 zero = c2{neg_inf<R>(), (R)0}, one = c2{(R)0, (R)0};
        for (int e = threadIdx.x; e < m * d; e += 256) pt[e] = e / d == e % d ? one : zero;
    }
}

// One workgroup per (b, t): grad_M[b, t, i, j] = +- exp(Re M'_t[i, j] + (c_{t-1} - c_t) + Re X'_t[i, j])
template <typename R> __global__ __launch_bounds__(256) void factor_grad_kernel(const typename C2<R>::type *__restrict__ M, const typename C2<R>::type *__restrict__ X,
                                                                                const R *__restrict__ c, R *__restrict__ gM, long long T, int dd)
{
    typedef typename C2<R>::type c2;
    const long long b = blockIdx.x / T, t = blockIdx.x - b * T;
    const double shift = (double)c[b * (T + 1) + t] - (double)c[b * (T + 1) + t + 1];
    const size_t base = (size_t)blockIdx.x * dd;
    for (int e = threadIdx.x; e < dd; e += 256) {
        const c2 a = M[base + e], x = X[base + e];
        double v = 0.0;
        if (a.x != neg_inf<R>() && x.x != neg_inf<R>()) v = exp_for<R>(((double)a.x + shift) + (double)x.x);
        gM[base + e] = (R)(odd_phase<R>(a.y) != odd_phase<R>(x.y) ? -v : v);
    }
}

// grad_S0[b, j, k] = +- exp(Re S0'[j, k] - c_{-1} + Re Lamhat'_{-1}[j, k]), Lamhat_{-1} the top d rows of state s = T
template <typename R> __global__ __launch_bounds__(256) void init_grad_kernel(const typename C2<R>::type *__restrict__ S0, const typename C2<R>::type *__restrict__ states,
                                                                              const R *__restrict__ c, R *__restrict__ gS0, long long T, long long nsteps, int d, int m)
{
    typedef typename C2<R>::type c2;
    const long long b = blockIdx.x;
    const c2 *lam = states + (size_t)(b * nsteps + T) * (d + m) * m;
    const double c0 = (double)c[b * (T + 1)];
    for (int e = threadIdx.x; e < d * m; e += 256) {
        const c2 a = S0[(size_t)b * d * m + e], x = lam[e];
        double v = 0.0;
        if (a.x != neg_inf<R>() && x.x != neg_inf<R>()) v = exp_for<R>(((double)a.x - c0) + (double)x.x);
        gS0[(size_t)b * d * m + e] = (R)(odd_phase<R>(a.y) != odd_phase<R>(x.y) ? -v : v);
    }
}

template <typename R> int prepare_t(goom_ctx *ctx, const void *M, const void *S0, const void *P, const void *G, void *c, void *F, void *init, long long T, int d,
                                    int m, long long batch)
{
    typedef typename C2<R>::type c2;
    const long long nsteps = T + (S0 ? 1 : 0), states = batch * (T + 1);
    goom::prof_begin(ctx, "scan_backward_prepare");
    hipLaunchKernelGGL(scales_kernel<R>, dim3((unsigned)((states + 3) / 4)), dim3(256), 0, ctx->stream, static_cast<const c2 *>(P), static_cast<const c2 *>(S0),
                       static_cast<R *>(c), T, d * m, states);
    hipLaunchKernelGGL(factors_kernel<R>, dim3((unsigned)(batch * nsteps)), dim3(256), 0, ctx->stream, static_cast<const c2 *>(M), static_cast<const c2 *>(P),
                       static_cast<const R *>(G), static_cast<const R *>(c), static_cast<c2 *>(F), static_cast<c2 *>(init), T, nsteps, d, m);
    goom::prof_end(ctx);
    return goom::check_hip(ctx, hipGetLastError(), "launch scan_backward_prepare");
}

template <typename R> int operands_t(goom_ctx *ctx, const void *states, const void *P, const void *S0, const void *c, void *Lam, void *Pt, long long T, int d,
                                     int m, long long batch)
{
    typedef typename C2<R>::type c2;
    goom::prof_begin(ctx, "scan_backward_operands");
    hipLaunchKernelGGL(operands_kernel<R>, dim3((unsigned)(batch * T)), dim3(256), 0, ctx->stream, static_cast<const c2 *>(states), static_cast<const c2 *>(P),
                       static_cast<const c2 *>(S0), static_cast<const R *>(c), static_cast<c2 *>(Lam), static_cast<c2 *>(Pt), T, T + (S0 ? 1 : 0), d, m);
    goom::prof_end(ctx);
    return goom::check_hip(ctx, hipGetLastError(), "launch scan_backward_operands");
}

template <typename R> int gradients_t(goom_ctx *ctx, const void *M, const void *S0, const void *X, const void *states, const void *c, void *gM, void *gS0,
                                      long long T, int d, int m, long long batch)
{
    typedef typename C2<R>::type c2;
    goom::prof_begin(ctx, "scan_backward_gradients");
    hipLaunchKernelGGL(factor_grad_kernel<R>, dim3((unsigned)(batch * T)), dim3(256), 0, ctx->stream, static_cast<const c2 *>(M), static_cast<const c2 *>(X),
                       static_cast<const R *>(c), static_cast<R *>(gM), T, d * d);
    if (gS0)
        hipLaunchKernelGGL(init_grad_kernel<R>, dim3((unsigned)batch), dim3(256), 0, ctx->stream, static_cast<const c2 *>(S0), static_cast<const c2 *>(states),
                           static_cast<const R *>(c), static_cast<R *>(gS0), T, T + 1, d, m);
    goom::prof_end(ctx);
    return goom::check_hip(ctx, hipGetLastError(), "launch scan_backward_gradients");
}

} // namespace

namespace goom {

int launch_scan_backward_prepare(goom_ctx *ctx, const void *M, const void *S0, const void *P, const void *G, void *c, void *F, void *init, long long T, int d,
                                 int m, long long batch, int dtype)
{
    return dtype == GOOM_C64 ? prepare_t<float>(ctx, M, S0, P, G, c, F, init, T, d, m, batch) : prepare_t<double>(ctx, M, S0, P, G, c, F, init, T, d, m, batch);
}

int launch_scan_backward_operands(goom_ctx *ctx, const void *states, const void *P, const void *S0, const void *c, void *Lam, void *Pt, long long T, int d, int m,
                                  long long batch, int dtype)
{
    return dtype == GOOM_C64 ? operands_t<float>(ctx, states, P, S0, c, Lam, Pt, T, d, m, batch) : operands_t<double>(ctx, states, P, S0, c, Lam, Pt, T, d, m, batch);
}

int launch_scan_backward_gradients(goom_ctx *ctx, const void *M, const void *S0, const void *X, const void *states, const void *c, void *gM, void *gS0, long long T,
                                   int d, int m, long long batch, int dtype)
{
    return dtype == GOOM_C64 ? gradients_t<float>(ctx, M, S0, X, states, c, gM, gS0, T, d, m, batch)
                             : gradients_t<double>(ctx, M, S0, X, states, c, gM, gS0, T, d, m, batch);
}

} // namespace goom
