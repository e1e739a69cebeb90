// Backward passes (paper Section 3.1: the redefined finite derivatives of the real absolute value, the real
// logarithm and the complex exponential; Section 4.3: the recurrence h_t = A_t h_{t-1} + b_t over GOOMs).
//
// Codecs.  The log-magnitude of a GOOM is log(abs(x)) with d abs / dx := +-1 (+1 at zero, never 0) and
// d log(u) / du := 1 / (u + eps); the real value of a GOOM is Re exp(x') with d exp(x') / dx' := exp(x') +- eps.
// Both are one multiply per element around the forward value.
//
// Recurrence.  With G_t[i] the gradient of a loss with respect to the log-magnitude of h_t[i], the adjoint of the
// value h_t[i] is lam_t = G_t / h_t + A_{t+1}^T lam_{t+1}: the same kind of recurrence in reverse time over the
// transposed matrices, so it runs through the forward scan itself on operands prepared here (matrices transposed
// and reversed in time, bias G_t / h_t as GOOMs: the adjoints shrink as fast as the states grow, and only their
// products with states and matrix entries return to ordinary magnitudes).  The gradients with respect to
// log-magnitudes are lam_t[i] A_t[i, j] h_{t-1}[j] and lam_t[i] b_t[i].
//
// A float log-magnitude near 1000 is only good to 6e-5, and the adjoints are signed sums with cancellation, so the
// adjoint recurrence is not run on the adjoints themselves but on lamhat_t = lam_t e^(c_t), c_t the whole number
// nearest the largest log-magnitude of h_t: lamhat_t = G_t / (h_t e^(-c_t)) + (e^(c_t - c_{t+1}) A_{t+1}^T) lamhat_{t+1},
// whose operands all have log-magnitudes of ordinary size (h'_t - c_t is exact in the component type; the matrices
// move by the whole number c_t - c_{t+1}).  The shift is undone, in double, where the gradients are formed.
#include "goom_internal.h"

namespace {

constexpr double kInvPi = 0.318309886183790671538;

template <typename R> struct C2;
template <> struct C2<float> { typedef float2 type; };
template <> struct C2<double> { typedef double2 type; };

template <typename R> __device__ inline bool odd_phase(R im)
{
    const int k = (int)__builtin_rint((double)im * kInvPi);
    return (k & 1) != 0;
}
// e^s for a double sum of log-magnitudes, to the accuracy of the result type: float results take the hardware
// exponential on the rounded argument (its error, |s| 2^-24, is far inside a gradient's tolerance)
template <typename R> __device__ inline double exp_for(double s)
{
    if (sizeof(R) == 4) return (double)__builtin_amdgcn_exp2f((float)(s * 1.44269504088896340736));
    return exp(s);
}
// log of a positive real to the accuracy of the result type
template <typename R> __device__ inline double log_for(double g)
{
    if (sizeof(R) == 4) return (double)__builtin_logf((float)g);
    return log(g);
}
template <typename R> __device__ inline R pi_of() { return sizeof(R) == 4 ? (R)3.14159274101257324219f : (R)3.14159265358979311600; }

// ---- codecs -----------------------------------------------------------------------------------------------
template <typename R> __global__ __launch_bounds__(256) void to_goom_backward_kernel(const R *__restrict__ x, const R *__restrict__ g,
                                                                                     R *__restrict__ gx, size_t n, double eps)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const double v = (double)x[i];
        const double s = v < 0.0 ? -1.0 : 1.0; // zero counts as non-negative
        gx[i] = (R)((double)g[i] * s / (__builtin_fabs(v) + eps));
    }
}

template <typename R> __global__ __launch_bounds__(256) void from_goom_backward_kernel(const typename C2<R>::type *__restrict__ y,
                                                                                       const R *__restrict__ gx, R *__restrict__ g, size_t n, double eps)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const typename C2<R>::type z = y[i];
        const double mag = exp((double)z.x);
        const double v = odd_phase<R>(z.y) ? -mag : mag;
        g[i] = (R)((double)gx[i] * (v + (v < 0.0 ? -eps : eps)));
    }
}

// scaled exponentiation (Section 4.3): the log-scaling constant takes no gradient, so the gradient with respect to the
// log-magnitude is the scaled value times the gradient with respect to it
template <typename R> __global__ __launch_bounds__(256) void scaled_exp_backward_kernel(const R *__restrict__ scaled, const R *__restrict__ g, R *__restrict__ gre,
                                                                                        size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) gre[i] = scaled[i] * g[i];
}

// ---- recurrence -------------------------------------------------------------------------------------------
// Operands of the adjoint recurrence, indexed by s = T - 1 - t:
//   At[b, s] = A[b, T - s]^T for s >= 1 (the matrix for s = 0 multiplies the zero initial adjoint: written as zeros),
//   gt[b, s, i] = GOOM(G[b, T - 1 - s, i]) - H[b, T - 1 - s, i]   (zero where G is zero or the state is zero).
// One workgroup per (b, s); the matrix passes through LDS so that both its read and its write are contiguous.
// c_t: the whole number nearest the largest log-magnitude of h_t (0 for a zero state), the same in every lane of the wave
template <typename R> __device__ inline R state_scale(const typename C2<R>::type *h, int d)
{
    const R ninf = sizeof(R) == 4 ? (R)-__builtin_huge_valf() : (R)-__builtin_huge_val();
    R top = ninf;
    for (int i = threadIdx.x & 63; i < d; i += 64) {
        const R v = h[i].x;
        top = v > top ? v : top;
    }
    for (int sft = 32; sft > 0; sft >>= 1) {
        const R o = __shfl_xor(top, sft, 64);
        top = o > top ? o : top;
    }
    const bool finite = top > ninf && top < -ninf;
    return finite ? (R)__builtin_rint((double)top) : (R)0;
}

// One wave per (b, s), no workgroup barrier: the matrix passes through LDS words of the wave's own so that both its
// read and its write are contiguous.
template <typename R, int NW> __global__ __launch_bounds__(NW * 64) void bwd_prepare_kernel(const typename C2<R>::type *__restrict__ A,
                                                                                            const typename C2<R>::type *__restrict__ H,
                                                                                            const R *__restrict__ G, typename C2<R>::type *__restrict__ At,
                                                                                            typename C2<R>::type *__restrict__ gt, long long T, int d,
                                                                                            long long nsteps, int direct)
{
    typedef typename C2<R>::type c2;
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long long step = (long long)blockIdx.x * NW + wave;
    if (step >= nsteps) return; // whole wave
    c2 *tile = reinterpret_cast<c2 *>(smem) + (size_t)wave * d * (d + 1); // [d][d + 1]
    const long long b = step / T, s = step % T;
    const R ninf = sizeof(R) == 4 ? (R)-__builtin_huge_valf() : (R)-__builtin_huge_val();
    const long long t = T - 1 - s;
    const R ct = state_scale<R>(H + (size_t)(b * T + t) * d, d);
    c2 *dst = At + (size_t)(b * T + s) * d * d;
    const int nn = d * d;
    if (s == 0) {
        for (int e = lane; e < nn; e += 64) dst[e] = c2{ninf, (R)0};
    } else {
        const R delta = ct - state_scale<R>(H + (size_t)(b * T + t + 1) * d, d); // c_t - c_{t+1}, a whole number
        const c2 *src = A + (size_t)(b * T + (T - s)) * d * d;
        if (direct) { // a matrix too large for LDS (complex128 above 96 x 96): strided reads
            for (int e = lane; e < nn; e += 64) {
                c2 v = src[(e % d) * d + e / d];
                v.x += delta;
                dst[e] = v;
            }
        } else if (sizeof(R) == 4 && (d & 1) == 0) {
            const float4 *src4 = reinterpret_cast<const float4 *>(src);
            for (int q = lane; q < nn / 2; q += 64) {
                const float4 w = src4[q];
                const int i = (2 * q) / d, j = (2 * q) - i * d;
                tile[i * (d + 1) + j] = c2{(R)w.x, (R)w.y};
                tile[i * (d + 1) + j + 1] = c2{(R)w.z, (R)w.w};
            }
        } else {
            for (int e = lane; e < nn; e += 64) tile[(e / d) * (d + 1) + e % d] = src[e];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        if (direct) {
        } else if (sizeof(R) == 4 && (d & 1) == 0) {
            float4 *dst4 = reinterpret_cast<float4 *>(dst);
            for (int q = lane; q < nn / 2; q += 64) {
                const int i = (2 * q) / d, j = (2 * q) - i * d; // entries (i, j) and (i, j + 1) of the transpose
                const c2 u = tile[j * (d + 1) + i], v = tile[(j + 1) * (d + 1) + i];
                dst4[q] = float4{(float)u.x + (float)delta, (float)u.y, (float)v.x + (float)delta, (float)v.y}; // -inf stays -inf
            }
        } else {
            for (int e = lane; e < nn; e += 64) {
                c2 v = tile[(e % d) * (d + 1) + e / d];
                v.x += delta;
                dst[e] = v;
            }
        }
    }
    for (int i = lane; i < d; i += 64) {
        const R gv = G[(size_t)(b * T + t) * d + i];
        const c2 h = H[(size_t)(b * T + t) * d + i];
        c2 o;
        const bool live = gv != (R)0 && h.x > ninf;
        o.x = live ? (R)(log(__builtin_fabs((double)gv)) - ((double)h.x - (double)ct)) : ninf;
        o.y = (live && ((gv < (R)0) != odd_phase<R>(h.y))) ? pi_of<R>() : (R)0;
        gt[(size_t)(b * T + s) * d + i] = o;
    }
}

// The same without the copy of the matrices, for the scan kernels that read A transposed and in reverse order
// themselves: only the shift of step s's log-magnitudes, shift[b, s] = c_t - c_{t+1} (-inf for s = 0: the zero
// matrix), and gt.  A group of lanes per (b, s), so that a wave serves two to eight steps of short vectors.
template <typename R> __global__ __launch_bounds__(256) void bwd_shift_kernel(const typename C2<R>::type *__restrict__ H, const R *__restrict__ G,
                                                                             float *__restrict__ shift, typename C2<R>::type *__restrict__ gt,
                                                                             long long T, int d, long long nsteps, int group, int absolute)
{
    // absolute: shift[b, s] = c_t itself (for a scan that rescales its bias and its stored states by it, its factors unchanged)
    // a group of `group` lanes (8, 16, 32 or 64: the power of two that holds d, or the whole wave) per (b, s)
    typedef typename C2<R>::type c2;
    const int lane = threadIdx.x & 63, sub = lane % group;
    const long long step = ((long long)blockIdx.x * 256 + threadIdx.x) / group;
    const bool active = step < nsteps;
    const long long b = active ? step / T : 0, s = active ? step % T : 0;
    const R ninf = sizeof(R) == 4 ? (R)-__builtin_huge_valf() : (R)-__builtin_huge_val();
    const long long t = T - 1 - s;
    // c_t and c_{t+1}: the whole numbers nearest the largest log-magnitudes of h_t and h_{t+1} (0 for a zero state)
    auto scale_of = [&](long long tt) {
        R top = ninf;
        if (active && tt < T)
            for (int i = sub; i < d; i += group) {
                const R v = H[(size_t)(b * T + tt) * d + i].x;
                top = v > top ? v : top;
            }
        for (int sft = group >> 1; sft > 0; sft >>= 1) {
            const R o = __shfl_xor(top, sft, 64);
            top = o > top ? o : top;
        }
        const bool finite = top > ninf && top < -ninf;
        return finite ? (R)__builtin_rint((double)top) : (R)0;
    };
    const R ct = scale_of(t);
    const R cnext = absolute ? (R)0 : scale_of(t + 1); // (uniform: a kernel argument)
    if (!active) return;
    if (sub == 0) shift[b * T + s] = absolute ? (float)ct : s == 0 ? (float)ninf : (float)(ct - cnext);
    for (int i = sub; i < d; i += group) {
        const R gv = G[(size_t)(b * T + t) * d + i];
        const c2 h = H[(size_t)(b * T + t) * d + i];
        c2 o;
        const bool live = gv != (R)0 && h.x > ninf;
        o.x = live ? (R)(log_for<R>(__builtin_fabs((double)gv)) - ((double)h.x - (double)ct)) : ninf;
        o.y = (live && ((gv < (R)0) != odd_phase<R>(h.y))) ? pi_of<R>() : (R)0;
        gt[(size_t)(b * T + s) * d + i] = o;
    }
}

// Gradients from the scaled adjoints mu[b, s] = lam[b, T - 1 - s] e^(c_{T-1-s}) (GOOMs), one wave per (b, t), no
// workgroup barrier:
//   gA[b, t, i, j] = lam_t[i] A_t[i, j] h_{t-1}[j],   gb[b, t, i] = lam_t[i] b_t[i].
// Sums of three log-magnitudes are formed in double (the adjoint and the state are large and opposite); the wave
// keeps the adjoint's and the previous state's log-magnitudes and signs in LDS words of its own.
constexpr int kGradWaves = 4;

template <typename R> __global__ __launch_bounds__(kGradWaves * 64) void bwd_grad_kernel(const typename C2<R>::type *__restrict__ A,
                                                                                         const typename C2<R>::type *__restrict__ bias,
                                                                                         const typename C2<R>::type *__restrict__ h0,
                                                                                         const typename C2<R>::type *__restrict__ H,
                                                                                         const typename C2<R>::type *__restrict__ mu, R *__restrict__ gA,
                                                                                         R *__restrict__ gb, long long T, int d, long long nsteps)
{
    typedef typename C2<R>::type c2;
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long long step = (long long)blockIdx.x * kGradWaves + wave;
    if (step >= nsteps) return; // whole wave
    const long long b = step / T, t = step % T;
    // this wave's words: lre[d], pre[d] (double), signs packed with them as separate int arrays
    double *lre = reinterpret_cast<double *>(smem) + (size_t)wave * 2 * d;
    double *pre = lre + d;
    int *lneg = reinterpret_cast<int *>(reinterpret_cast<double *>(smem) + (size_t)kGradWaves * 2 * d) + (size_t)wave * 2 * d;
    int *pneg = lneg + d;
    const double ninf = -__builtin_huge_val();
    // c_t: the whole number nearest the largest log-magnitude of h_t
    const c2 *ht = H + (size_t)(b * T + t) * d;
    R top = sizeof(R) == 4 ? (R)-__builtin_huge_valf() : (R)-__builtin_huge_val();
    for (int i = lane; i < d; i += 64) {
        const R v = ht[i].x;
        top = v > top ? v : top;
    }
    for (int sft = 32; sft > 0; sft >>= 1) {
        const R o = __shfl_xor(top, sft, 64);
        top = o > top ? o : top;
    }
    const bool finite = (double)top > ninf && (double)top < -ninf;
    const double ct = finite ? __builtin_rint((double)top) : 0.0;
    for (int i = lane; i < d; i += 64) {
        const c2 l = mu[(size_t)(b * T + (T - 1 - t)) * d + i];
        lre[i] = (double)l.x - ct; // -inf stays -inf
        lneg[i] = odd_phase<R>(l.y) ? 1 : 0;
        c2 p = c2{(R)ninf, (R)0};
        if (t > 0) p = H[(size_t)(b * T + t - 1) * d + i];
        else if (h0) p = h0[(size_t)b * d + i];
        pre[i] = (double)p.x;
        pneg[i] = odd_phase<R>(p.y) ? 1 : 0;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const c2 *ap = A + (size_t)(b * T + t) * d * d;
    R *op = gA + (size_t)(b * T + t) * d * d;
    auto one = [&](int e, c2 a) {
        const int i = e / d, j = e - i * d;
        const double s = lre[i] + (double)a.x + pre[j];
        const bool live = lre[i] > ninf && (double)a.x > ninf && pre[j] > ninf;
        const double v = live ? exp_for<R>(s) : 0.0;
        const bool neg = (lneg[i] ^ pneg[j] ^ (odd_phase<R>(a.y) ? 1 : 0)) != 0;
        return (R)(neg ? -v : v);
    };
    const int nn = d * d;
    if (sizeof(R) == 4 && (nn & 1) == 0) {
        // two adjacent entries per lane and pass: one 16-byte load, one 8-byte store
        const float4 *ap4 = reinterpret_cast<const float4 *>(ap);
        float2 *op2 = reinterpret_cast<float2 *>(op);
        for (int q = lane; q < nn / 2; q += 64) {
            const float4 w = ap4[q];
            float2 o;
            o.x = (float)one(2 * q, c2{(R)w.x, (R)w.y});
            o.y = (float)one(2 * q + 1, c2{(R)w.z, (R)w.w});
            op2[q] = o;
        }
    } else {
        for (int e = lane; e < nn; e += 64) op[e] = one(e, ap[e]);
    }
    if (gb) {
        for (int i = lane; i < d; i += 64) {
            const c2 bb = bias[(size_t)(b * T + t) * d + i];
            const bool live = lre[i] > ninf && (double)bb.x > ninf;
            const double v = live ? exp_for<R>(lre[i] + (double)bb.x) : 0.0;
            const bool neg = (lneg[i] ^ (odd_phase<R>(bb.y) ? 1 : 0)) != 0;
            gb[(size_t)(b * T + t) * d + i] = (R)(neg ? -v : v);
        }
    }
}

// gh0[b, j] = sum_i gA[b, 0, i, j]   (= h_{-1}[j] sum_i lam_0[i] A_0[i, j]), summed in a fixed order
template <typename R> __global__ __launch_bounds__(128) void bwd_h0_kernel(const R *__restrict__ gA, R *__restrict__ gh0, long long T, int d)
{
    const long long b = blockIdx.x;
    for (int j = threadIdx.x; j < d; j += 128) {
        double acc = 0.0;
        for (int i = 0; i < d; ++i) acc += (double)gA[((size_t)b * T * d + i) * d + j];
        gh0[(size_t)b * d + j] = (R)acc;
    }
}

// One matrix for all steps: its gradient is A[i, j] sum_t lam_t[i] h_{t-1}[j].  partial[b, q] = sum over the steps of span q of
// u_t v_t^T, DP x DP doubles (rows and columns beyond d are zero), with u_t[i] = lam_t[i] e^r and v_t[j] = h_{t-1}[j] e^(-r), r the
// largest log-magnitude of h_{t-1} (|v| <= 1; u is of the size of the gradient's terms).  Eight steps at a time: each of the four
// waves forms u and v of two steps in LDS (side by side in its two halves when d <= 32) (and writes those steps' bias gradients lam_t[i] b_t[i]), then every thread adds the
// eight products to its DP * DP / 256 neighbouring entries of one row.  u and v of step 0 are kept for the initial state's gradient.
constexpr int kOuterSteps = 8;

template <typename R, int DP> __global__ __launch_bounds__(256) void bwd_outer_kernel(const typename C2<R>::type *__restrict__ bias,
                                                                                     const typename C2<R>::type *__restrict__ h0,
                                                                                     const typename C2<R>::type *__restrict__ H,
                                                                                     const typename C2<R>::type *__restrict__ mu, R *__restrict__ gb,
                                                                                     double *__restrict__ partial, double *__restrict__ uv0, long long T, int d,
                                                                                     int nsplit)
{
    typedef typename C2<R>::type c2;
    constexpr int EPT = DP * DP / 256;
    constexpr int GROUP = DP <= 32 ? 32 : 64; // lanes that serve one step: short vectors share a wave two by two
    constexpr int SPW = 64 / GROUP;
    __shared__ double u[kOuterSteps][DP], v[kOuterSteps][DP];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, sub = lane % GROUP;
    const long long b = blockIdx.x / nsplit;
    const int q = (int)(blockIdx.x - b * nsplit);
    const long long per = (T + nsplit - 1) / nsplit, t0 = q * per, t1 = t0 + per < T ? t0 + per : T;
    const int e0 = threadIdx.x * EPT, row = e0 / DP, j0 = e0 - row * DP;
    const double ninf = -__builtin_huge_val();
    double acc[EPT];
#pragma unroll
    for (int k = 0; k < EPT; ++k) acc[k] = 0.0;
    for (long long tb = t0; tb < t1; tb += kOuterSteps) {
        for (int kb0 = wave * SPW; kb0 < kOuterSteps; kb0 += 4 * SPW) {
            const int kb = kb0 + lane / GROUP;
            const long long t = tb + kb;
            const bool in = t < t1; // the same in all lanes of a group
            // c_t: the whole number nearest the largest log-magnitude of h_t; r: the largest log-magnitude of h_{t-1}
            double top = ninf, r = ninf;
            const c2 *prev = !in ? nullptr : t > 0 ? H + (size_t)(b * T + t - 1) * d : h0 ? h0 + (size_t)b * d : nullptr;
            for (int i = sub; i < d && in; i += GROUP) {
                const double hv = (double)H[(size_t)(b * T + t) * d + i].x;
                top = hv > top ? hv : top;
                if (prev) {
                    const double pv = (double)prev[i].x;
                    r = pv > r ? pv : r;
                }
            }
            for (int sft = GROUP / 2; sft > 0; sft >>= 1) {
                const double o1 = __shfl_xor(top, sft, 64), o2 = __shfl_xor(r, sft, 64);
                top = o1 > top ? o1 : top;
                r = o2 > r ? o2 : r;
            }
            const double ct = (top > ninf && top < -ninf) ? __builtin_rint(top) : 0.0;
            const bool any = r > ninf && r < -ninf;
            for (int i = sub; i < DP; i += GROUP) {
                double uu = 0.0, vv = 0.0;
                if (in && i < d) {
                    const c2 l = mu[(size_t)(b * T + (T - 1 - t)) * d + i];
                    const double lre = (double)l.x - ct; // log-magnitude of lam_t[i]; -inf stays -inf
                    const bool lneg = odd_phase<R>(l.y);
                    if (any && lre > ninf) uu = exp_for<R>(lre + r); // (float GOOMs: the hardware exponential of the small double sum)
                    if (lneg) uu = -uu;
                    if (prev) {
                        const c2 p = prev[i];
                        if (any && (double)p.x > ninf) vv = exp_for<R>((double)p.x - r);
                        if (odd_phase<R>(p.y)) vv = -vv;
                    }
                    if (gb) {
                        const c2 bb = bias[(size_t)(b * T + t) * d + i];
                        const bool live = lre > ninf && (double)bb.x > ninf;
                        const double g = live ? exp_for<R>(lre + (double)bb.x) : 0.0;
                        gb[(size_t)(b * T + t) * d + i] = (R)(lneg != odd_phase<R>(bb.y) ? -g : g);
                    }
                    if (t == 0) {
                        uv0[((size_t)b * 2) * d + i] = uu;
                        uv0[((size_t)b * 2 + 1) * d + i] = vv;
                    }
                }
                u[kb][i] = uu;
                v[kb][i] = vv;
            }
        }
        __syncthreads();
#pragma unroll
        for (int kb = 0; kb < kOuterSteps; ++kb) {
            const double ui = u[kb][row];
#pragma unroll
            for (int k = 0; k < EPT; ++k) acc[k] += ui * v[kb][j0 + k];
        }
        __syncthreads();
    }
    double *out = partial + (size_t)blockIdx.x * DP * DP + e0;
#pragma unroll
    for (int k = 0; k < EPT; ++k) out[k] = acc[k];
}

// gA[b, i, j] = A[b, i, j] sum_q partial[b, q, i, j] (in the order of q);  gh0[b, j] = v_0[j] sum_i u_0[i] A[b, i, j]  (uv0[b] = u_0, v_0)
template <typename R> __global__ __launch_bounds__(256) void bwd_outer_finish_kernel(const typename C2<R>::type *__restrict__ A, const double *__restrict__ partial,
                                                                                     const double *__restrict__ uv0, R *__restrict__ gA,
                                                                                     R *__restrict__ gh0, int d, int dp, int nsplit)
{
    typedef typename C2<R>::type c2;
    const long long b = blockIdx.x;
    const double ninf = -__builtin_huge_val();
    for (int e = threadIdx.x; e < d * d; e += 256) {
        const int i = e / d, j = e - i * d;
        double acc = 0.0;
        for (int q = 0; q < nsplit; ++q) acc += partial[((size_t)b * nsplit + q) * dp * dp + (size_t)i * dp + j];
        const c2 a = A[(size_t)b * d * d + e];
        // (through the logarithm of the sum: the entry alone may lie outside the range of a double)
        const double mag = (acc != 0.0 && (double)a.x > ninf) ? exp((double)a.x + log(__builtin_fabs(acc))) : 0.0;
        gA[(size_t)b * d * d + e] = (R)((acc < 0.0) != odd_phase<R>(a.y) ? -mag : mag);
    }
    if (gh0)
        for (int j = threadIdx.x; j < d; j += 256) {
            double acc = 0.0;
            for (int i = 0; i < d; ++i) {
                const c2 a = A[(size_t)b * d * d + (size_t)i * d + j];
                const double ui = uv0[((size_t)b * 2) * d + i];
                const double mag = (ui != 0.0 && (double)a.x > ninf) ? exp((double)a.x + log(__builtin_fabs(ui))) : 0.0;
                acc += (ui < 0.0) != odd_phase<R>(a.y) ? -mag : mag;
            }
            gh0[(size_t)b * d + j] = (R)(acc * uv0[((size_t)b * 2 + 1) * d + j]);
        }
}

unsigned blocks_for(size_t n)
{
    const size_t b = (n + 255) / 256;
    return (unsigned)(b < 65536 * 16 ? (b ? b : 1) : 65536 * 16);
}

} // namespace

namespace goom {

int launch_to_goom_backward(goom_ctx *ctx, const void *x, const void *g, void *gx, size_t n, int dtype, double eps)
{
    if (n == 0) return GOOM_OK;
    prof_begin(ctx, "to_goom_backward");
    if (dtype == GOOM_C64)
        hipLaunchKernelGGL(to_goom_backward_kernel<float>, dim3(blocks_for(n)), dim3(256), 0, ctx->stream, static_cast<const float *>(x),
                           static_cast<const float *>(g), static_cast<float *>(gx), n, eps);
    else
        hipLaunchKernelGGL(to_goom_backward_kernel<double>, dim3(blocks_for(n)), dim3(256), 0, ctx->stream, static_cast<const double *>(x),
                           static_cast<const double *>(g), static_cast<double *>(gx), n, eps);
    prof_end(ctx);
    return check_hip(ctx, hipGetLastError(), "launch to_goom_backward");
}

int launch_scaled_exp_backward(goom_ctx *ctx, const void *scaled, const void *g, void *gre, size_t n, int dtype)
{
    if (n == 0) return GOOM_OK;
    prof_begin(ctx, "scaled_exp_backward");
    if (dtype == GOOM_C64)
        hipLaunchKernelGGL(scaled_exp_backward_kernel<float>, dim3(blocks_for(n)), dim3(256), 0, ctx->stream, static_cast<const float *>(scaled),
                           static_cast<const float *>(g), static_cast<float *>(gre), n);
    else
        hipLaunchKernelGGL(scaled_exp_backward_kernel<double>, dim3(blocks_for(n)), dim3(256), 0, ctx->stream, static_cast<const double *>(scaled),
                           static_cast<const double *>(g), static_cast<double *>(gre), n);
    prof_end(ctx);
    return check_hip(ctx, hipGetLastError(), "launch scaled_exp_backward");
}

int launch_from_goom_backward(goom_ctx *ctx, const void *y, const void *gx, void *g, size_t n, int dtype, double eps)
{
    if (n == 0) return GOOM_OK;
    prof_begin(ctx, "from_goom_backward");
    if (dtype == GOOM_C64)
        hipLaunchKernelGGL(from_goom_backward_kernel<float>, dim3(blocks_for(n)), dim3(256), 0, ctx->stream, static_cast<const float2 *>(y),
                           static_cast<const float *>(gx), static_cast<float *>(g), n, eps);
    else
        hipLaunchKernelGGL(from_goom_backward_kernel<double>, dim3(blocks_for(n)), dim3(256), 0, ctx->stream, static_cast<const double2 *>(y),
                           static_cast<const double *>(gx), static_cast<double *>(g), n, eps);
    prof_end(ctx);
    return check_hip(ctx, hipGetLastError(), "launch from_goom_backward");
}

template <typename R, int NW> static int bwd_prepare_launch(goom_ctx *ctx, const void *A, const void *H, const void *G, void *At, void *gt, long long T, int d,
                                                           long long batch)
{
    typedef typename C2<R>::type c2;
    const size_t tile_bytes = (size_t)d * (d + 1) * sizeof(c2);
    const int direct = tile_bytes > 150 * 1024 ? 1 : 0;
    const size_t lds = direct ? 0 : (size_t)NW * tile_bytes;
    auto kern = bwd_prepare_kernel<R, NW>;
    if (lds > 48 * 1024) {
        if (int s = check_hip(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds), "hipFuncSetAttribute(bwd_prepare)")) return s;
    }
    const long long nsteps = batch * T;
    prof_begin(ctx, "affine_backward_prepare_operands");
    hipLaunchKernelGGL(kern, dim3((unsigned)((nsteps + NW - 1) / NW)), dim3(NW * 64), lds, ctx->stream, static_cast<const c2 *>(A), static_cast<const c2 *>(H),
                       static_cast<const R *>(G), static_cast<c2 *>(At), static_cast<c2 *>(gt), T, d, nsteps, direct);
    prof_end(ctx);
    return check_hip(ctx, hipGetLastError(), "launch bwd_prepare_kernel");
}

// waves (steps) per workgroup: as many as the matrices' LDS tiles allow
template <typename R> static int bwd_prepare_t(goom_ctx *ctx, const void *A, const void *H, const void *G, void *At, void *gt, long long T, int d, long long batch)
{
    const size_t tile = (size_t)d * (d + 1) * 2 * sizeof(R);
    if (4 * tile <= 64 * 1024) return bwd_prepare_launch<R, 4>(ctx, A, H, G, At, gt, T, d, batch);
    if (2 * tile <= 96 * 1024) return bwd_prepare_launch<R, 2>(ctx, A, H, G, At, gt, T, d, batch);
    return bwd_prepare_launch<R, 1>(ctx, A, H, G, At, gt, T, d, batch);
}

// At[b] = A[b]^T, d x d (one matrix per batch item)
template <typename R> __global__ __launch_bounds__(256) void bwd_transpose_kernel(const typename C2<R>::type *__restrict__ A, typename C2<R>::type *__restrict__ At, int d)
{
    const size_t base = (size_t)blockIdx.x * d * d;
    for (int e = threadIdx.x; e < d * d; e += 256) At[base + e] = A[base + (size_t)(e % d) * d + e / d];
}

template <typename R> static int bwd_shift_t(goom_ctx *ctx, const void *H, const void *G, float *shift, void *gt, long long T, int d, long long batch,
                                             const void *A = nullptr, void *At = nullptr)
{
    typedef typename C2<R>::type c2;
    const long long nsteps = batch * T;
    prof_begin(ctx, "affine_backward_prepare_operands");
    const int group = d <= 8 ? 8 : d <= 16 ? 16 : d <= 32 ? 32 : 64;
    const long long per_block = 256 / group;
    hipLaunchKernelGGL(bwd_shift_kernel<R>, dim3((unsigned)((nsteps + per_block - 1) / per_block)), dim3(256), 0, ctx->stream, static_cast<const c2 *>(H),
                       static_cast<const R *>(G), shift, static_cast<c2 *>(gt), T, d, nsteps, group, At ? 1 : 0);
    if (At) hipLaunchKernelGGL(bwd_transpose_kernel<R>, dim3((unsigned)batch), dim3(256), 0, ctx->stream, static_cast<const c2 *>(A), static_cast<c2 *>(At), d);
    prof_end(ctx);
    return check_hip(ctx, hipGetLastError(), "launch bwd_shift_kernel");
}

// At: the transposed, reversed, rescaled copy of A; or NULL, and then shift receives the shifts alone
int launch_affine_backward_prepare(goom_ctx *ctx, const void *A, const void *H, const void *G, void *At, float *shift, void *gt, long long T, int d,
                                   long long batch, int dtype)
{
    if (batch * T > 0x7fffffffLL) return fail(ctx, GOOM_EUNSUPPORTED, "too many steps for one launch");
    if (!At) return dtype == GOOM_C64 ? bwd_shift_t<float>(ctx, H, G, shift, gt, T, d, batch) : bwd_shift_t<double>(ctx, H, G, shift, gt, T, d, batch);
    return dtype == GOOM_C64 ? bwd_prepare_t<float>(ctx, A, H, G, At, gt, T, d, batch) : bwd_prepare_t<double>(ctx, A, H, G, At, gt, T, d, batch);
}

// One matrix for all steps, scan over the matrix itself: At [batch, d, d] = A^T, shift[b, s] = c_t, gt as above
int launch_affine_backward_prepare_one_matrix(goom_ctx *ctx, const void *A, const void *H, const void *G, void *At, float *shift, void *gt, long long T, int d,
                                              long long batch, int dtype)
{
    if (batch * T > 0x7fffffffLL) return fail(ctx, GOOM_EUNSUPPORTED, "too many steps for one launch");
    return dtype == GOOM_C64 ? bwd_shift_t<float>(ctx, H, G, shift, gt, T, d, batch, A, At) : bwd_shift_t<double>(ctx, H, G, shift, gt, T, d, batch, A, At);
}

template <typename R> static int bwd_grad_t(goom_ctx *ctx, const void *A, const void *bias, const void *h0, const void *H, const void *mu, void *gA,
                                            void *gb, void *gh0, long long T, int d, long long batch)
{
    typedef typename C2<R>::type c2;
    const size_t lds = (size_t)kGradWaves * d * (2 * sizeof(double) + 2 * sizeof(int));
    const long long nsteps = batch * T;
    prof_begin(ctx, "affine_backward_gradients");
    hipLaunchKernelGGL(bwd_grad_kernel<R>, dim3((unsigned)((nsteps + kGradWaves - 1) / kGradWaves)), dim3(kGradWaves * 64), lds, ctx->stream,
                       static_cast<const c2 *>(A), static_cast<const c2 *>(bias), static_cast<const c2 *>(h0), static_cast<const c2 *>(H),
                       static_cast<const c2 *>(mu), static_cast<R *>(gA), static_cast<R *>(gb), T, d, nsteps);
    if (gh0) hipLaunchKernelGGL(bwd_h0_kernel<R>, dim3((unsigned)batch), dim3(128), 0, ctx->stream, static_cast<const R *>(gA), static_cast<R *>(gh0), T, d);
    prof_end(ctx);
    return check_hip(ctx, hipGetLastError(), "launch bwd_grad_kernel");
}

int launch_affine_backward_gradients(goom_ctx *ctx, const void *A, const void *bias, const void *h0, const void *H, const void *mu, void *gA,
                                     void *gb, void *gh0, long long T, int d, long long batch, int dtype)
{
    if (batch * T > 0x7fffffffLL) return fail(ctx, GOOM_EUNSUPPORTED, "too many steps for one launch");
    return dtype == GOOM_C64 ? bwd_grad_t<float>(ctx, A, bias, h0, H, mu, gA, gb, gh0, T, d, batch)
                             : bwd_grad_t<double>(ctx, A, bias, h0, H, mu, gA, gb, gh0, T, d, batch);
}

// One matrix for all steps.  partial: [batch, nsplit, dp, dp] doubles (dp: d padded to 16, 32, 64 or 128); uv0: [batch, 2, d] doubles
template <typename R> static int bwd_grad_ti_t(goom_ctx *ctx, const void *A, const void *bias, const void *h0, const void *H, const void *mu, void *gA, void *gb,
                                               void *gh0, double *uv0, double *partial, int nsplit, long long T, int d, long long batch)
{
    typedef typename C2<R>::type c2;
    const int dp = d <= 16 ? 16 : d <= 32 ? 32 : d <= 64 ? 64 : 128;
    prof_begin(ctx, "affine_backward_gradients");
    const dim3 grid((unsigned)(batch * nsplit));
    const c2 *bp = static_cast<const c2 *>(bias), *hp = static_cast<const c2 *>(h0), *Hp = static_cast<const c2 *>(H), *mp = static_cast<const c2 *>(mu);
    R *gbp = static_cast<R *>(gb);
    if (dp == 16) hipLaunchKernelGGL((bwd_outer_kernel<R, 16>), grid, dim3(256), 0, ctx->stream, bp, hp, Hp, mp, gbp, partial, uv0, T, d, nsplit);
    else if (dp == 32) hipLaunchKernelGGL((bwd_outer_kernel<R, 32>), grid, dim3(256), 0, ctx->stream, bp, hp, Hp, mp, gbp, partial, uv0, T, d, nsplit);
    else if (dp == 64) hipLaunchKernelGGL((bwd_outer_kernel<R, 64>), grid, dim3(256), 0, ctx->stream, bp, hp, Hp, mp, gbp, partial, uv0, T, d, nsplit);
    else hipLaunchKernelGGL((bwd_outer_kernel<R, 128>), grid, dim3(256), 0, ctx->stream, bp, hp, Hp, mp, gbp, partial, uv0, T, d, nsplit);
    hipLaunchKernelGGL(bwd_outer_finish_kernel<R>, dim3((unsigned)batch), dim3(256), 0, ctx->stream, static_cast<const c2 *>(A), partial, uv0, static_cast<R *>(gA),
                       static_cast<R *>(gh0), d, dp, nsplit);
    prof_end(ctx);
    return check_hip(ctx, hipGetLastError(), "launch bwd_outer_kernel");
}

int launch_affine_backward_gradients_one_matrix(goom_ctx *ctx, const void *A, const void *bias, const void *h0, const void *H, const void *mu, void *gA,
                                                void *gb, void *gh0, void *uv0, void *partial, int nsplit, long long T, int d, long long batch, int dtype)
{
    if (batch * T > 0x7fffffffLL || batch * nsplit > 0x7fffffffLL) return fail(ctx, GOOM_EUNSUPPORTED, "too many steps for one launch");
    return dtype == GOOM_C64 ? bwd_grad_ti_t<float>(ctx, A, bias, h0, H, mu, gA, gb, gh0, static_cast<double *>(uv0), static_cast<double *>(partial), nsplit, T, d, batch)
                             : bwd_grad_ti_t<double>(ctx, A, bias, h0, H, mu, gA, gb, gh0, static_cast<double *>(uv0), static_cast<double *>(partial), nsplit, T, d,
                                                     batch);
}

} // namespace goom
