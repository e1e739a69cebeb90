// Codec kernels: real floats <-> GOOMs (paper Section 3.1).  Pure streaming: 4 or 8
// bytes in and 8 or 16 bytes out per element (or the reverse), so HBM bandwidth binds;
// the logarithm / exponential is evaluated in double and rounded once to the component
// type.  For float components that evaluation is a short series of its own (the library's
// double routines made these kernels compute bound).
#include "goom_internal.h"
#include "goom_codec_tables.h"

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));

// 2 log(smallest normal): the finite stand-in for log 0 (paper Section 3.1, footnote)
constexpr double kFloorF32 = -174.67308950110621797; // 2 ln(2^-126)
constexpr double kFloorF64 = -1416.7928370645282124; // 2 ln(2^-1022)
constexpr float kPiF = 3.14159274101257324219f;
constexpr double kPiD = 3.14159265358979311600;
constexpr double kInvPi = 0.318309886183790671538;

// ln|x| in double for a finite non-zero x: x = m 2^k with m in [sqrt(1/2), sqrt(2)), ln m = 2 atanh(s),
// s = (m - 1) / (m + 1), |s| < 0.1716, as its series to s^21 (remainder below 1e-17 relative; near x = 1
// the result is the series alone, so it keeps its relative accuracy there).  About a third of the
// instructions of the library routine, which made the float encoder compute bound.
// k ln 2 + 2 atanh(num / den), the common tail of the logarithms below: |num / den| < 0.1716
__device__ inline double ln_from_ratio(double num, double den, double k)
{
    double r = (double)__builtin_amdgcn_rcpf((float)den);
    r = r * (2.0 - den * r);
    r = r * (2.0 - den * r);
    double s = num * r;
    s = __builtin_fma(__builtin_fma(-s, den, num), r, s); // s = num / den to rounding
    const double z = s * s;
    double p = 1.0 / 21.0;
    p = __builtin_fma(p, z, 1.0 / 19.0);
    p = __builtin_fma(p, z, 1.0 / 17.0);
    p = __builtin_fma(p, z, 1.0 / 15.0);
    p = __builtin_fma(p, z, 1.0 / 13.0);
    p = __builtin_fma(p, z, 1.0 / 11.0);
    p = __builtin_fma(p, z, 1.0 / 9.0);
    p = __builtin_fma(p, z, 1.0 / 7.0);
    p = __builtin_fma(p, z, 1.0 / 5.0);
    p = __builtin_fma(p, z, 1.0 / 3.0);
    p = __builtin_fma(p, z * s, s); // s + s^3 (1/3 + ...)
    // k ln 2 with ln 2 in two parts: the high part has 32 significant bits, so k times it is exact
    const double kLn2Hi = 0.693147180369123816490, kLn2Lo = 1.90821492927058770002e-10;
    return __builtin_fma(k, kLn2Hi, __builtin_fma(k, kLn2Lo, p + p));
}

// x = m 2^k with m in [sqrt(1/2), sqrt(2)): the ratio (m - 1) / (m + 1) and k for the tail above
__device__ inline void ln_reduce(double x, double &num, double &den, double &kd)
{
    int k;
    double m = __builtin_frexp(__builtin_fabs(x), &k); // [1/2, 1)
    const bool low = m < 0.70710678118654752440;
    m = low ? m + m : m;
    k = low ? k - 1 : k;
    num = m - 1.0;
    den = m + 1.0;
    kd = (double)k;
}

__device__ inline double ln_abs_f64(double x)
{
    double num, den, kd;
    ln_reduce(x, num, den, kd);
    return ln_from_ratio(num, den, kd);
}

// e^x in double: k = round(x / ln 2), r = x - k ln 2 with ln 2 in two parts (exact for a float x), e^r as
// its series to r^13 (|r| < 0.35: remainder below 1e-17), scaled by 2^k.  Also returns, for k = 0, the
// series of e^r - 1 with its relative accuracy (r times the series without its last step).
// (straight-line: out-of-range arguments are clamped for the series and their results selected at the end)
__device__ inline double exp_series(double x0, double *expm1_small = nullptr, bool *k_is_zero = nullptr)
{
    const double x = __builtin_fmin(__builtin_fmax(x0, -800.0), 800.0); // NaN -> -800 here, restored below
    const double k = __builtin_rint(x * 1.44269504088896340736);
    const double kLn2Hi = 0.693147180369123816490, kLn2Lo = 1.90821492927058770002e-10;
    const double r = __builtin_fma(-k, kLn2Lo, __builtin_fma(-k, kLn2Hi, x));
    double p = 1.0 / 6227020800.0;
    p = __builtin_fma(p, r, 1.0 / 479001600.0);
    p = __builtin_fma(p, r, 1.0 / 39916800.0);
    p = __builtin_fma(p, r, 1.0 / 3628800.0);
    p = __builtin_fma(p, r, 1.0 / 362880.0);
    p = __builtin_fma(p, r, 1.0 / 40320.0);
    p = __builtin_fma(p, r, 1.0 / 5040.0);
    p = __builtin_fma(p, r, 1.0 / 720.0);
    p = __builtin_fma(p, r, 1.0 / 120.0);
    p = __builtin_fma(p, r, 1.0 / 24.0);
    p = __builtin_fma(p, r, 1.0 / 6.0);
    p = __builtin_fma(p, r, 0.5);
    p = __builtin_fma(p, r, 1.0);
    if (expm1_small) *expm1_small = p * r;
    if (k_is_zero) *k_is_zero = k == 0.0;
    p = __builtin_fma(p, r, 1.0);
    double y = __builtin_ldexp(p, (int)k);
    y = x0 > -800.0 ? y : 0.0;                    // -inf and everything that underflows even in double
    y = x0 < 800.0 ? y : __builtin_huge_val();    // overflows float by far
    return x0 == x0 ? y : x0;                     // NaN stays
}

// ---- double-double arithmetic for the complex128 codecs --------------------------------------------------
// The paper's codecs are the real logarithm and exponential (Section 3.1); "rounded once" for double
// components needs more than double inside, so these two are evaluated as unevaluated sums hi + lo of two
// doubles (about 100 significant bits), and the result is hi after the last renormalisation, i.e. the
// double nearest the exact value except when that value lies within 2^-45 ulp or so of a rounding boundary.
struct dd {
    double hi, lo;
};
__device__ inline dd two_sum(double a, double b)
{
#pragma clang fp contract(off) // the error-free sums and products below need every operation rounded as written
    const double s = a + b, bb = s - a;
    return dd{s, (a - (s - bb)) + (b - bb)};
}
__device__ inline dd fast_two_sum(double a, double b) // |a| >= |b|
{
#pragma clang fp contract(off) // the error-free sums and products below need every operation rounded as written
    const double s = a + b;
    return dd{s, b - (s - a)};
}
__device__ inline dd two_prod(double a, double b)
{
#pragma clang fp contract(off) // the error-free sums and products below need every operation rounded as written
    const double p = a * b;
    return dd{p, __builtin_fma(a, b, -p)};
}
__device__ inline dd dd_add(dd x, dd y)
{
#pragma clang fp contract(off) // the error-free sums and products below need every operation rounded as written
    dd s = two_sum(x.hi, y.hi);
    const dd t = two_sum(x.lo, y.lo);
    s.lo += t.hi;
    s = fast_two_sum(s.hi, s.lo);
    s.lo += t.lo;
    return fast_two_sum(s.hi, s.lo);
}
__device__ inline dd dd_add_d(dd x, double y)
{
#pragma clang fp contract(off) // the error-free sums and products below need every operation rounded as written
    dd s = two_sum(x.hi, y);
    s.lo += x.lo;
    return fast_two_sum(s.hi, s.lo);
}
__device__ inline dd dd_mul(dd x, dd y)
{
#pragma clang fp contract(off) // the error-free sums and products below need every operation rounded as written
    dd p = two_prod(x.hi, y.hi);
    p.lo = __builtin_fma(x.hi, y.lo, __builtin_fma(x.lo, y.hi, p.lo));
    return fast_two_sum(p.hi, p.lo);
}
__device__ inline dd dd_mul_d(dd x, double y)
{
#pragma clang fp contract(off) // the error-free sums and products below need every operation rounded as written
    dd p = two_prod(x.hi, y);
    p.lo = __builtin_fma(x.lo, y, p.lo);
    return fast_two_sum(p.hi, p.lo);
}

// ln|x| for a finite non-zero double x, as a double-double.  x = m 2^k with m in [sqrt(1/2), sqrt(2));
// m = c (1 + r) with 1 / c a 24-bit table value near 1 / m (so m / c - 1 is formed exactly, |r| < 0.0056, and
// c = 1 for m next to 1, where the result keeps its relative accuracy); ln(1 + r) = 2 atanh(s), s = r / (2 + r),
// |s| < 2^-8.4: s + s^3 / 3 + ... to s^15 (remainder 2^-140 relative), the leading terms in double-double.
__device__ inline dd ln_abs_dd(double x)
{
#pragma clang fp contract(off) // the error-free sums and products below need every operation rounded as written
    using namespace goom_codec_tables;
    int k;
    double m = __builtin_frexp(__builtin_fabs(x), &k); // [1/2, 1)
    const bool low = m < 0.70710678118654752440;
    m = low ? m + m : m;
    k = low ? k - 1 : k;
    const int i = (int)__builtin_rint((m - 1.0) * 128.0);
    const double *tab = kLogTab[i - kLogIndexMin];
    const dd p = two_prod(m, tab[0]);
    dd r = fast_two_sum(p.hi - 1.0, p.lo); // exact: p.hi is within 2^-7 of 1
    // s = r / (2 + r)
    dd den = two_sum(2.0, r.hi);
    den.lo += r.lo;
    double inv = (double)__builtin_amdgcn_rcpf((float)den.hi);
    inv = inv * (2.0 - den.hi * inv);
    inv = inv * (2.0 - den.hi * inv);
    const double q1 = r.hi * inv;
    // remainder r - q1 den, exactly enough: q1 den.hi as a product pair
    const dd qd = two_prod(q1, den.hi);
    const double rem = ((r.hi - qd.hi) - qd.lo) + (r.lo - q1 * den.lo);
    const dd s = fast_two_sum(q1, rem * inv);
    const dd z = dd_mul(s, s);
    // s^2 (1/3 + z/5 + z^2/7 + z^3/9 + ...): the tail from z^3/9 on in double
    double tail = 1.0 / 15.0;
    tail = __builtin_fma(tail, z.hi, 1.0 / 13.0);
    tail = __builtin_fma(tail, z.hi, 1.0 / 11.0);
    tail = __builtin_fma(tail, z.hi, 1.0 / 9.0);
    dd poly = dd_add(dd_mul_d(z, tail), dd{kInv7Hi, kInv7Lo});
    poly = dd_add(dd_mul(poly, z), dd{kInv5Hi, kInv5Lo});
    poly = dd_add(dd_mul(poly, z), dd{kInv3Hi, kInv3Lo});
    dd lg = dd_mul(dd_mul(poly, z), s); // s^3 (1/3 + ...)
    lg = dd_add(s, lg);
    lg.hi *= 2.0;
    lg.lo *= 2.0;
    // + ln c + k ln 2, largest parts first (k ln 2 in three parts, the first exact)
    const double kd = (double)k;
    dd acc = two_prod(kd, kLn2B);
    acc = dd_add_d(acc, kd * kLn2C);
    acc = dd_add(dd{kd * kLn2A, 0.0}, acc);
    acc = dd_add(acc, dd{tab[1], tab[2]});
    return dd_add(acc, lg);
}

// e^x for |x| < 746 as a double-double times 2^k: x = (64 k + j) ln2 / 64 + r, |r| < 0.0055 (the step in three
// parts, the first with 32 significant bits so that its multiple is exact); e^r = 1 + r + r^2 (1/2 + r/6 + ...) to
// r^12, the leading terms in double-double; times the table value 2^(j / 64).
__device__ inline dd exp_dd(double x, int &k)
{
#pragma clang fp contract(off) // the error-free sums and products below need every operation rounded as written
    using namespace goom_codec_tables;
    const double nd = __builtin_rint(x * kExpInvStep);
    const int n = (int)nd;
    k = n >> 6;
    const int j = n & 63;
    const double r1 = __builtin_fma(-nd, kExpStepA, x); // exact
    const dd pb = two_prod(nd, kExpStepB);
    dd r = two_sum(r1, -pb.hi);
    r.lo -= pb.lo + nd * kExpStepC;
    r = fast_two_sum(r.hi, r.lo);
    double tail = 1.0 / 479001600.0;
    tail = __builtin_fma(tail, r.hi, 1.0 / 39916800.0);
    tail = __builtin_fma(tail, r.hi, 1.0 / 3628800.0);
    tail = __builtin_fma(tail, r.hi, 1.0 / 362880.0);
    tail = __builtin_fma(tail, r.hi, 1.0 / 40320.0);
    tail = __builtin_fma(tail, r.hi, 1.0 / 5040.0);
    tail = __builtin_fma(tail, r.hi, 1.0 / 720.0);
    dd poly = dd_add(dd_mul_d(r, tail), dd{kInvF120Hi, kInvF120Lo});
    poly = dd_add(dd_mul(poly, r), dd{kInvF24Hi, kInvF24Lo});
    poly = dd_add(dd_mul(poly, r), dd{kInvF6Hi, kInvF6Lo});
    poly = dd_add_d(dd_mul(poly, r), 0.5);
    dd q = dd_mul(dd_mul(poly, r), r); // r^2 (1/2 + ...)
    q = dd_add(r, q);                  // e^r - 1
    const dd t = dd{kExpTab[j][0], kExpTab[j][1]};
    return dd_add(t, dd_mul(t, q));
}

// exp of a double log-magnitude, rounded once (also into the subnormal range)
__device__ inline double exp_rounded_once(double x)
{
#pragma clang fp contract(off) // the error-free sums and products below need every operation rounded as written
    if (!(x == x)) return x;
    if (x > 709.79) return __builtin_huge_val();
    if (x < -745.14) return 0.0;
    int k;
    const dd y = exp_dd(x, k); // value (y.hi + y.lo) 2^k, y.hi in [1, 2)
    if (k > -1022) { // normal result: a power-of-two scaling of an already rounded hi (1024 cannot happen below 709.79)
        return __builtin_ldexp(y.hi, k);
    }
    // subnormal result: the value in units of 2^-1074 is w = (y.hi + y.lo) 2^(k + 1074) < 2^52; adding 2^52 rounds
    // w's high part to a whole number, and what that addition and y.lo leave decides the last unit
    const double whi = __builtin_ldexp(y.hi, k + 1074), wlo = __builtin_ldexp(y.lo, k + 1074);
    const double big = 4503599627370496.0; // 2^52
    const double sh = big + whi;
    double nint = sh - big;
    const double left = (whi - nint) + wlo; // exact difference plus the low part
    if (left > 0.5 || (left == 0.5 && __builtin_fmod(nint, 2.0) != 0.0)) nint += 1.0;
    if (left < -0.5 || (left == -0.5 && __builtin_fmod(nint, 2.0) != 0.0)) nint -= 1.0;
    return __builtin_ldexp(nint, -1074);
}

__device__ inline double exp_of_f32(float xf) { return exp_series((double)xf); }

// (straight-line: the series runs on every input, zeros, infinities and NaN included, and the special results
// are selected afterwards; with the special cases as branches the four elements of a thread serialised)
__device__ inline float enc_re_f32(float v, bool zero_floor)
{
    const float av = __builtin_fabsf(v);
    float r = (float)ln_abs_f64((double)av);
    r = av < __builtin_huge_valf() ? r : av; // infinities and NaN pass through
    return v == 0.0f ? (zero_floor ? (float)kFloorF32 : -__builtin_huge_valf()) : r;
}

__global__ __launch_bounds__(256) void to_goom_f32_kernel(const float *__restrict__ x, float *__restrict__ y,
                                                          size_t n, int zero_floor)
{
    const size_t nvec = n / 4;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += stride) {
        f4 v = reinterpret_cast<const f4 *>(x)[i];
        f4 lo, hi;
        lo[0] = enc_re_f32(v[0], zero_floor); lo[1] = v[0] < 0.0f ? kPiF : 0.0f;
        lo[2] = enc_re_f32(v[1], zero_floor); lo[3] = v[1] < 0.0f ? kPiF : 0.0f;
        hi[0] = enc_re_f32(v[2], zero_floor); hi[1] = v[2] < 0.0f ? kPiF : 0.0f;
        hi[2] = enc_re_f32(v[3], zero_floor); hi[3] = v[3] < 0.0f ? kPiF : 0.0f;
        reinterpret_cast<f4 *>(y)[2 * i] = lo;
        reinterpret_cast<f4 *>(y)[2 * i + 1] = hi;
    }
    // ragged tail (n not a multiple of 4)
    const size_t tail0 = nvec * 4;
    const size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid < n - tail0) {
        float v = x[tail0 + gid];
        y[2 * (tail0 + gid)] = enc_re_f32(v, zero_floor);
        y[2 * (tail0 + gid) + 1] = v < 0.0f ? kPiF : 0.0f;
    }
}

__global__ __launch_bounds__(256) void to_goom_f64_kernel(const double *__restrict__ x, double *__restrict__ y,
                                                          size_t n, int zero_floor)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        double v = x[i];
        const double av = __builtin_fabs(v);
        double re = ln_abs_dd(av < __builtin_huge_val() ? (av > 0.0 ? av : 1.0) : 1.0).hi;
        re = av < __builtin_huge_val() ? re : av; // infinities and NaN pass through
        re = (v == 0.0) ? (zero_floor ? kFloorF64 : -__builtin_huge_val()) : re;
        double2 o;
        o.x = re;
        o.y = v < 0.0 ? kPiD : 0.0;
        reinterpret_cast<double2 *>(y)[i] = o;
    }
}

// (through a 32-bit integer: one conversion instruction where a 64-bit one is a dozen; a phase beyond
// 2^31 pi carries no parity in a double product with 1 / pi anyway)
__device__ inline bool odd_multiple_of_pi(double im)
{
    const int k = (int)__builtin_rint(im * kInvPi);
    return (k & 1) != 0;
}

__global__ __launch_bounds__(256) void from_goom_f32_kernel(const float *__restrict__ y, float *__restrict__ x, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        float2 z = reinterpret_cast<const float2 *>(y)[i];
        float mag = (float)exp_of_f32(z.x);
        x[i] = odd_multiple_of_pi((double)z.y) ? -mag : mag;
    }
}

__global__ __launch_bounds__(256) void from_goom_f64_kernel(const double *__restrict__ y, double *__restrict__ x, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        double2 z = reinterpret_cast<const double2 *>(y)[i];
        double mag = exp_rounded_once(z.x);
        x[i] = odd_multiple_of_pi(z.y) ? -mag : mag;
    }
}

// Scaled exponentiation of GOOM vectors (paper Section 4.3, eq. 27): per vector of length d,
// c = max of the log-magnitudes, scaled_i = (+-) exp(re_i - c + 2).  A group of G = 2^k >= d
// lanes (at most 64) owns a vector when d <= 64, so the maximum is a few lane exchanges;
// longer vectors take a whole wave and several elements per lane.  Evaluated in double and
// rounded once, like the codecs.
template <typename R, typename R2> __global__ __launch_bounds__(256) void scaled_exp_kernel(const R2 *__restrict__ z, R *__restrict__ out,
                                                                                            R *__restrict__ cout, size_t nvec, int d, int group)
{
    const int lane = threadIdx.x & 63;
    const size_t wave = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const size_t nwaves = ((size_t)gridDim.x * blockDim.x) >> 6;
    const int per_wave = 64 / group; // vectors a wave handles at a time
    const int sub = lane / group, el = lane % group;
    const int reps = (d + group - 1) / group; // > 1 only when d > 64
    if (sizeof(R) == 4 && reps == 1) {
        // float vectors of at most 64 elements, one element per lane: several rounds of vectors per iteration, so
        // that as many loads per lane are in flight
        constexpr int U = 2; // (four are no faster: the series in double then bounds the kernel)
        const R ninf = (R)-__builtin_huge_valf();
        const size_t round = nwaves * per_wave;
        for (size_t v0 = wave * per_wave; v0 < nvec; v0 += U * round) {
            R2 e[U];
            R m[U];
            bool live[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const size_t v = v0 + sub + u * round;
                live[u] = v < nvec && el < d;
                e[u].x = ninf;
                e[u].y = (R)0;
                if (live[u]) e[u] = z[v * d + el];
            }
#pragma unroll
            for (int u = 0; u < U; ++u) m[u] = e[u].x;
            for (int sft = 1; sft < group; sft <<= 1) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const R o = __shfl_xor(m[u], sft, 64);
                    m[u] = o > m[u] ? o : m[u];
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const size_t v = v0 + sub + u * round;
                double x = exp_series((double)e[u].x - (double)m[u] + 2.0);
                x = m[u] > ninf ? x : 0.0;
                if (odd_multiple_of_pi((double)e[u].y)) x = -x;
                if (live[u]) out[v * d + el] = (R)x;
                if (cout && live[u] && el == 0) cout[v] = m[u];
            }
        }
        return;
    }
    for (size_t v0 = wave * per_wave; v0 < nvec; v0 += nwaves * per_wave) {
        const size_t v = v0 + sub;
        const bool live = v < nvec;
        // (the maximum in the component type: exact, and for floats half the lane exchanges of a double)
        R mr = sizeof(R) == 4 ? (R)-__builtin_huge_valf() : (R)-__builtin_huge_val();
        R2 first;
        first.x = mr;
        first.y = (R)0;
        if (live && el < d) first = z[v * d + el];
        mr = first.x;
        for (int r = 1; r < reps; ++r) {
            const int i = el + r * group;
            if (live && i < d) {
                const R t = z[v * d + i].x;
                mr = t > mr ? t : mr;
            }
        }
        for (int sft = 1; sft < group; sft <<= 1) {
            const R o = __shfl_xor(mr, sft, 64);
            mr = o > mr ? o : mr;
        }
        const double m = (double)mr;
        for (int r = 0; r < reps; ++r) {
            const int i = el + r * group;
            if (live && i < d) {
                // (floats keep the first element in its register; doubles are faster reading it again from cache)
                const R2 e = (sizeof(R) == 4 && r == 0) ? first : z[v * d + i];
                const double arg = (double)e.x - m + 2.0;
                // float results: the short series (good to 1e-13 for such arguments); double results: the library's
                double x = sizeof(R) == 4 ? exp_series(arg) : exp(arg);
                x = m > -__builtin_huge_val() ? x : 0.0;
                if (odd_multiple_of_pi((double)e.y)) x = -x;
                out[v * d + i] = (R)x;
            }
        }
        if (cout && live && el == 0) cout[v] = (R)m;
    }
}

// Signed log-add of two GOOM arrays: the GOOM of exp(x') + exp(y') (paper Section 2, Example 2; the
// step that adds the input term in the recurrence over GOOMs, Section 4.3, eq. 26).  In double, rounded once: with m the larger log-magnitude and delta the gap,
// m + log1p(exp(-delta)) for equal signs, m + log(-expm1(-delta)) for opposite ones.
// Float components: the same in straight-line code on the short series.  With a the larger log-magnitude,
// delta = a - b >= 0 and e = exp(-delta): equal signs give a + ln(1 + e), where the ratio for the atanh series is
// formed from e itself (e / (2 + e), or (e - 1) / (e + 3) plus ln 2 above sqrt(2) - 1), so a tiny e keeps its
// relative accuracy; opposite signs give a + ln(1 - e), with 1 - e taken from the series of e^r - 1 when
// delta < (ln 2) / 2, where the subtraction would cancel.
__global__ __launch_bounds__(256) void log_add_exp_f32_kernel(const float2 *__restrict__ x, const float2 *__restrict__ y,
                                                              float2 *__restrict__ out, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    const double ninf = -__builtin_huge_val();
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const float2 p = x[i], q = y[i];
        const bool sp = odd_multiple_of_pi((double)p.y), sq = odd_multiple_of_pi((double)q.y);
        // the larger magnitude first; of two equal ones the non-negative
        const bool swap = q.x > p.x || (q.x == p.x && !sq && sp);
        const double a = swap ? (double)q.x : (double)p.x, b = swap ? (double)p.x : (double)q.x;
        const bool sa = swap ? sq : sp, sb = swap ? sp : sq;
        const bool same = sa == sb;
        const double delta = b > ninf ? a - b : 800.0; // (a = b = -inf would give NaN: selected away below)
        double em1;
        bool k0;
        const double e = exp_series(-delta, &em1, &k0); // in (0, 1]
        // 1 - e without cancellation
        const double u = k0 ? -em1 : 1.0 - e;
        double num_d, den_d, k_d;
        ln_reduce(u, num_d, den_d, k_d); // garbage for u = 0, selected away below
        const bool big = e > 0.41421356237309504880;
        const double num = same ? (big ? e - 1.0 : e) : num_d;
        const double den = same ? (big ? e + 3.0 : e + 2.0) : den_d;
        const double kd = same ? (big ? 1.0 : 0.0) : k_d;
        double re = a + ln_from_ratio(num, den, kd);
        bool neg = sa;
        const bool cancel = !same && delta == 0.0;
        re = cancel ? ninf : re;
        neg = cancel ? false : neg;
        re = b > ninf ? re : a;          // a zero second operand: the first one as it is
        const bool zero = !(a > ninf);   // both zero (a is the larger)
        re = zero ? ninf : re;
        neg = zero ? false : neg;
        re = a < __builtin_huge_val() ? re : a; // +inf stays
        re = (a == a && b == b) ? re : a + b;   // NaN stays
        float2 o;
        o.x = (float)re;
        o.y = neg ? kPiF : 0.0f;
        out[i] = o;
    }
}

template <typename R, typename R2> __global__ __launch_bounds__(256) void log_add_exp_kernel(const R2 *__restrict__ x, const R2 *__restrict__ y,
                                                                                             R2 *__restrict__ out, size_t n, R pi)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const R2 p = x[i], q = y[i];
        double a = (double)p.x, b = (double)q.x;
        bool sa = odd_multiple_of_pi((double)p.y), sb = odd_multiple_of_pi((double)q.y);
        if (b > a || (b == a && !sb && sa)) {
            const double t = a; a = b; b = t;
            const bool u = sa; sa = sb; sb = u;
        }
        double re;
        bool neg = sa;
        const double ninf = -__builtin_huge_val();
        if (!(a > ninf)) {
            re = ninf;
            neg = false;
        } else if (!(b > ninf)) {
            re = a;
        } else {
            const double delta = a - b;
            if (sa == sb) {
                re = a + log1p(exp(-delta));
            } else if (delta == 0.0) {
                re = ninf;
                neg = false;
            } else {
                re = a + log(-expm1(-delta));
            }
        }
        R2 o;
        o.x = (R)re;
        o.y = neg ? pi : (R)0;
        out[i] = o;
    }
}

unsigned grid_for(size_t work_items)
{
    size_t blocks = (work_items + 255) / 256;
    const size_t cap = 256 * 32; // enough workgroups to fill 256 CUs several times over
    if (blocks > cap) blocks = cap;
    if (blocks == 0) blocks = 1;
    return (unsigned)blocks;
}

} // namespace

namespace goom {

int launch_to_goom(goom_ctx *ctx, const void *x, void *y, size_t n, int dtype, uint32_t flags)
{
    if (n == 0) return GOOM_OK;
    const int zf = (flags & GOOM_ZERO_FLOOR) ? 1 : 0;
    prof_begin(ctx, "to_goom");
    if (dtype == GOOM_C64) {
        hipLaunchKernelGGL(to_goom_f32_kernel, dim3(grid_for(n / 4 + 4)), dim3(256), 0, ctx->stream,
                           static_cast<const float *>(x), static_cast<float *>(y), n, zf);
    } else {
        hipLaunchKernelGGL(to_goom_f64_kernel, dim3(grid_for(n)), dim3(256), 0, ctx->stream,
                           static_cast<const double *>(x), static_cast<double *>(y), n, zf);
    }
    prof_end(ctx);
    return check_hip(ctx, hipGetLastError(), "launch to_goom");
}

int launch_scaled_exp(goom_ctx *ctx, const void *z, void *scaled, void *logscale, size_t nvec, int d, int dtype)
{
    if (nvec == 0) return GOOM_OK;
    int group = 1;
    while (group < d && group < 64) group <<= 1;
    const size_t lanes = (nvec + (64 / group) - 1) / (64 / group) * 64;
    prof_begin(ctx, "scaled_exp");
    if (dtype == GOOM_C64)
        hipLaunchKernelGGL((scaled_exp_kernel<float, float2>), dim3(grid_for(lanes)), dim3(256), 0, ctx->stream,
                           static_cast<const float2 *>(z), static_cast<float *>(scaled), static_cast<float *>(logscale), nvec, d, group);
    else
        hipLaunchKernelGGL((scaled_exp_kernel<double, double2>), dim3(grid_for(lanes)), dim3(256), 0, ctx->stream,
                           static_cast<const double2 *>(z), static_cast<double *>(scaled), static_cast<double *>(logscale), nvec, d, group);
    prof_end(ctx);
    return check_hip(ctx, hipGetLastError(), "launch scaled_exp");
}

// complex64 GOOMs as complex128 GOOMs (the log-magnitude widened exactly; the phase as 0 or the double pi)
__global__ __launch_bounds__(256) void widen_goom_kernel(const float2 *z, double2 *w, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const float2 v = z[i];
        const int k = (int)__builtin_rintf(v.y * 0.318309886183790671538f);
        w[i] = double2{(double)v.x, (k & 1) ? 3.14159265358979311600 : 0.0};
    }
}

int launch_widen_goom(goom_ctx *ctx, const void *z64, void *z128, size_t n)
{
    if (n == 0) return GOOM_OK;
    const size_t blocks = (n + 255) / 256;
    hipLaunchKernelGGL(widen_goom_kernel, dim3((unsigned)(blocks < 4096 ? blocks : 4096)), dim3(256), 0, ctx->stream,
                       static_cast<const float2 *>(z64), static_cast<double2 *>(z128), n);
    return check_hip(ctx, hipGetLastError(), "launch widen_goom");
}

// Entries of a GOOM array whose log-magnitude is +inf or NaN (-inf is the GOOM of zero and counts as finite): the
// paper's one failure notion, a chain that ends in "catastrophic numerical error" (Section 4.1).  Per-wave counts
// are added to the caller's counter with integer atomics (the sum does not depend on their order).
template <typename R2> __global__ __launch_bounds__(256) void count_nonfinite_kernel(const R2 *__restrict__ z, size_t n, unsigned long long *count)
{
    unsigned long long mine = 0;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const auto re = z[i].x;
        mine += (re != re || re == (decltype(re))__builtin_huge_val()) ? 1ull : 0ull; // NaN or +inf
    }
    for (int sft = 32; sft > 0; sft >>= 1) mine += __shfl_xor(mine, sft, 64);
    if ((threadIdx.x & 63) == 0 && mine) atomicAdd(count, mine);
}

__global__ void zero_counter_kernel(unsigned long long *count) { *count = 0ull; }

int launch_count_nonfinite(goom_ctx *ctx, const void *z, size_t n, int dtype, unsigned long long *count)
{
    hipLaunchKernelGGL(zero_counter_kernel, dim3(1), dim3(1), 0, ctx->stream, count);
    if (n == 0) return check_hip(ctx, hipGetLastError(), "launch zero_counter");
    prof_begin(ctx, "count_nonfinite");
    if (dtype == GOOM_C64)
        hipLaunchKernelGGL(count_nonfinite_kernel<float2>, dim3(grid_for(n)), dim3(256), 0, ctx->stream, static_cast<const float2 *>(z), n, count);
    else
        hipLaunchKernelGGL(count_nonfinite_kernel<double2>, dim3(grid_for(n)), dim3(256), 0, ctx->stream, static_cast<const double2 *>(z), n, count);
    prof_end(ctx);
    return check_hip(ctx, hipGetLastError(), "launch count_nonfinite");
}

int launch_log_add_exp(goom_ctx *ctx, const void *x, const void *y, void *out, size_t n, int dtype)
{
    if (n == 0) return GOOM_OK;
    prof_begin(ctx, "log_add_exp");
    if (dtype == GOOM_C64)
        hipLaunchKernelGGL(log_add_exp_f32_kernel, dim3(grid_for(n)), dim3(256), 0, ctx->stream, static_cast<const float2 *>(x),
                           static_cast<const float2 *>(y), static_cast<float2 *>(out), n);
    else
        hipLaunchKernelGGL((log_add_exp_kernel<double, double2>), dim3(grid_for(n)), dim3(256), 0, ctx->stream, static_cast<const double2 *>(x),
                           static_cast<const double2 *>(y), static_cast<double2 *>(out), n, 3.14159265358979311600);
    prof_end(ctx);
    return check_hip(ctx, hipGetLastError(), "launch log_add_exp");
}

int launch_from_goom(goom_ctx *ctx, const void *y, void *x, size_t n, int dtype)
{
    if (n == 0) return GOOM_OK;
    prof_begin(ctx, "from_goom");
    if (dtype == GOOM_C64) {
        hipLaunchKernelGGL(from_goom_f32_kernel, dim3(grid_for(n)), dim3(256), 0, ctx->stream,
                           static_cast<const float *>(y), static_cast<float *>(x), n);
    } else {
        hipLaunchKernelGGL(from_goom_f64_kernel, dim3(grid_for(n)), dim3(256), 0, ctx->stream,
                           static_cast<const double *>(y), static_cast<double *>(x), n);
    }
    prof_end(ctx);
    return check_hip(ctx, hipGetLastError(), "launch from_goom");
}


// ---- streaming probes: every workgroup walks a contiguous span, eight 16-byte accesses per thread in flight
namespace {
typedef float pf4 __attribute__((ext_vector_type(4)));
template <int MODE> __global__ __launch_bounds__(256) void probe_kernel(const pf4 *__restrict__ a, pf4 *__restrict__ b, size_t n)
{
    const size_t per = (n + gridDim.x - 1) / gridDim.x;
    const size_t lo = per * blockIdx.x;
    size_t hi = lo + per;
    if (hi > n) hi = n;
    pf4 acc = {0.f, 0.f, 0.f, 0.f};
    for (size_t i = lo + threadIdx.x; i < hi; i += 8 * 256) {
        pf4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = (MODE != 1 && i + u * 256 < hi) ? a[i + u * 256] : pf4{1.f, 2.f, 3.f, 4.f};
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (MODE == 0) acc += v[u];
            else if (i + u * 256 < hi) b[i + u * 256] = v[u];
        }
    }
    if (MODE == 0 && acc[0] + acc[1] + acc[2] + acc[3] == 1.2345f) reinterpret_cast<float *>(b)[0] = 1.0f;
}
} // namespace

// ---- matrix-unit probe: nothing but 16 x 16 x 4 matrix instructions on eight independent accumulators
namespace {
typedef double pd4 __attribute__((ext_vector_type(4)));
// (second launch bound, double only: at two waves per SIMD the compiler keeps the accumulators in ordinary
// registers; with the whole register file to itself it parks them in the accumulation registers and copies all
// of them back and forth in every iteration, which costs the double-precision loop a third of its rate; the
// float loop is 3 % faster the other way round)
template <typename R, typename V> __global__ __launch_bounds__(256, sizeof(R) == 8 ? 2 : 1) void matrix_probe_kernel(float *sink, long long iters)
{
    V acc[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc[u] = V{0, 0, 0, 0};
    const R x = (R)(threadIdx.x & 3) * (R)0.25, y = (R)(threadIdx.x & 7) * (R)0.125;
    for (long long i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if constexpr (sizeof(R) == 4) acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(x, y, acc[u], 0, 0, 0);
            else acc[u] = __builtin_amdgcn_mfma_f64_16x16x4f64(x, y, acc[u], 0, 0, 0);
        }
    }
    R t = 0;
#pragma unroll
    for (int u = 0; u < 8; ++u) t += acc[u][0] + acc[u][1] + acc[u][2] + acc[u][3];
    if (t == (R)-1.2345) sink[0] = 1.0f; // never true: the sums are non-negative
}
} // namespace

int launch_matrix_probe(goom_ctx *ctx, void *sink, long long iters, int dtype)
{
    // 2048 workgroups of four waves: two waves on every SIMD of the chip
    if (dtype == GOOM_C64) hipLaunchKernelGGL((matrix_probe_kernel<float, pf4>), dim3(2048), dim3(256), 0, ctx->stream, static_cast<float *>(sink), iters);
    else hipLaunchKernelGGL((matrix_probe_kernel<double, pd4>), dim3(2048), dim3(256), 0, ctx->stream, static_cast<float *>(sink), iters);
    return check_hip(ctx, hipGetLastError(), "launch matrix_probe_kernel");
}

int launch_probe(goom_ctx *ctx, const void *a, void *b, size_t bytes, int mode)
{
    const size_t n = bytes / 16;
    const pf4 *pa = static_cast<const pf4 *>(a);
    pf4 *pb = static_cast<pf4 *>(b);
    const unsigned grid = 4096;
    if (mode == 0) hipLaunchKernelGGL(probe_kernel<0>, dim3(grid), dim3(256), 0, ctx->stream, pa, pb, n);
    else if (mode == 1) hipLaunchKernelGGL(probe_kernel<1>, dim3(grid), dim3(256), 0, ctx->stream, pa, pb, n);
    else hipLaunchKernelGGL(probe_kernel<2>, dim3(grid), dim3(256), 0, ctx->stream, pa, pb, n);
    return check_hip(ctx, hipGetLastError(), "launch probe_kernel");
}

} // namespace goom
