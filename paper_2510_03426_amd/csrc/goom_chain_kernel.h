// Chain kernel: walks a sequence of left factors M_1, M_2, ... and keeps the running
// product S <- M_t S on chip.  It is the combine of the prefix scan (paper Section 4.1,
// eq. 14: S'_t = LMME(A'_t, S'_{t-1})) and, with one step, LMME itself (Section 3.2).
//
// Each step is the paper's scaled real product (Section 3.2, eq. 10) with two changes that
// keep what the scaling identity (eq. 12) allows:
//   * all shifts are whole powers of two, so scaling never rounds;
//   * the running product is not turned back into logarithms between steps.  It stays a
//     matrix of real mantissas W with one exponent per column, S[:, k] = W[:, k] 2^e_k
//     (left multiplication acts on every column independently, so a per-column scale
//     commutes with the product).  Logarithms are taken only for values that are stored.
//
// Work decomposition (wave64, v_mfma_*_16x16x4): a workgroup owns one chain; wave w owns
// the 16-column slab w of the state for all rows.  The 16x16 accumulator tile of the
// matrix instruction puts four rows of column lane % 16 in one lane (rows 4g+v for float,
// 4v+g for double; g = lane / 16, v = register), and the B operand wants one row per
// lane group g of that column: so the accumulators of one step are, register for
// register, the B operands of the next, with the contraction index visited in the
// order the accumulator rows come in.  The left factor is exponentiated by all
// waves into a padded LDS tile (double buffered), from which A operands are read as
// 16-byte vectors.
#pragma once
#include "goom_internal.h"

namespace goom_chain {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef double d4 __attribute__((ext_vector_type(4)));
typedef unsigned int u2 __attribute__((ext_vector_type(2)));

constexpr double kLog2e = 1.44269504088896340736;
constexpr double kLn2 = 0.693147180559945309417;
constexpr double kNegBig = -1.0e300; // stands for "log2 of zero" in exponent arithmetic

struct ChainArgs {
    const unsigned char *left;
    long long left_batch_stride, left_step_stride;
    long long steps, chunk_len, chunks_per_item, chunks_launched;
    int n, d, m, nslabs; // left factors are n x d, the state is d x m, outputs are n x m
    int init_mode;
    const unsigned char *init;
    long long init_stride;
    unsigned char *out_goom;
    int out_goom_last_only;
    unsigned char *out_fact_steps;
    unsigned char *out_fact_final;
    int final_common_exponent;
    long long fact_stride;
    int fact_cols;      // padded columns of factored states written / read
    int left_fact_cols; // padded columns of factored left factors
    int bias_mode; // 0 none, 1 GOOM vectors [batch, steps, d], 2 column d of the factored left factor
    int bias_col;  // state column that receives the bias
    long long init_group;   // > 0: factored initial states come from a grouped carry array, (init_group + 1)
    long long init_ngroups; //      entries per group of init_group chunks, init_ngroups groups per batch item
    const unsigned char *bias;
    // linear recurrence with bias, matrix-vector walk only: states in scaled floating-point form
    // (paper Section 4.3, eq. 27) instead of, or besides, GOOMs
    int left_real;       // 1: the left factors are real matrices (component type), not GOOMs (hot float kernel only)
    float *out_scaled;   // NULL or [batch, steps, d]
    float *out_logscale; // NULL or [batch, steps]
    // float kernels of the recurrence working beside double chunk products and carries:
    int fact_f64;        // 1: the factored matrices read (init_mode 1) and written (out_fact_final) have double mantissas
    int acc_f64;         // 1: chunk products [A* | b*] with the running product in double (d = 16, 32)
    // adjoint recurrence (backward pass of the recurrence), the double chunk products and the matrix-vector walk only:
    // NULL, or [batch, steps] floats; the factor of step s is then the transpose of matrix steps - s of the array
    // `left` (any matrix for s = 0) with left_shift[s] added to every log-magnitude (-inf: a zero matrix)
    const float *left_shift;
    // the matrix-vector walk over one matrix for all steps and the general kernel with GOOM bias vectors: NULL, or [batch, steps] floats
    // (whole numbers); the bias of step s
    // is then bias[s] e^(-io_shift[s]) and the state written for step s is h_s e^(+io_shift[s]): values far from 1 pass
    // through GOOM arrays of float components with log-magnitudes of ordinary size
    const float *io_shift;
};

template <typename R> struct Comp;
template <> struct Comp<float> {
    typedef f4 vec4;
    static constexpr int kPad = 4; // LDS row padding in elements
    __device__ static float pi() { return 3.14159274101257324219f; }
    __device__ static f4 mfma(float a, float b, f4 c) { return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0); }
    __device__ static float exp2_frac(float f) { return __builtin_amdgcn_exp2f(f); }
    __device__ static float log2_abs(float x) { return ::log2f(__builtin_fabsf(x)); }
    __device__ static float ldexp_(float x, int e) { return __builtin_ldexpf(x, e); }
    __device__ static int frexp_exp(float x) { int e; (void)__builtin_frexpf(x, &e); return e; }
    __device__ static float abs_(float x) { return __builtin_fabsf(x); }
    __device__ static float ceil_(float x) { return __builtin_ceilf(x); }
    __device__ static float neg_inf() { return -__builtin_huge_valf(); }
    __device__ static float max_(float a, float b) { return a > b ? a : b; }
    // Cross-lane maxima run on integer keys (a monotone map of the float bits), so that
    // each step is one integer max with a lane-permuted operand on the vector ALU: quad
    // permutes, half-row and row mirrors, then 16- and 32-lane row swaps.  No LDS traffic.
    __device__ static int key_of(float x)
    {
        const int b = __builtin_bit_cast(int, x);
        return b ^ ((b >> 31) & 0x7fffffff);
    }
    __device__ static float of_key(int k) { return __builtin_bit_cast(float, k ^ ((k >> 31) & 0x7fffffff)); }
    __device__ static int imax(int a, int b) { return a > b ? a : b; }
    template <int CTRL> __device__ static int dpp(int v) { return __builtin_amdgcn_mov_dpp(v, CTRL, 0xF, 0xF, true); }
    __device__ static int xor16_imax(int v)
    {
        const u2 r = __builtin_amdgcn_permlane16_swap((unsigned)v, (unsigned)v, false, false);
        return imax((int)r[0], (int)r[1]);
    }
    __device__ static int xor32_imax(int v)
    {
        const u2 r = __builtin_amdgcn_permlane32_swap((unsigned)v, (unsigned)v, false, false);
        return imax((int)r[0], (int)r[1]);
    }
    // max over lane l and lane l ^ 16 / l ^ 32
    __device__ static float xor16_max(float v) { return of_key(xor16_imax(key_of(v))); }
    __device__ static float xor32_max(float v) { return of_key(xor32_imax(key_of(v))); }
    __device__ static float xor16_32_max(float v) { return of_key(xor32_imax(xor16_imax(key_of(v)))); }
    // max of a and b over aligned groups of LANES lanes, result in every lane
    template <int LANES> __device__ static float group_allmax(float a, float b)
    {
        int v = imax(key_of(a), key_of(b));
        v = imax(v, dpp<0xB1>(v));                   // quad_perm [1,0,3,2]
        v = imax(v, dpp<0x4E>(v));                   // quad_perm [2,3,0,1]
        if (LANES >= 8) v = imax(v, dpp<0x141>(v));  // row_half_mirror
        if (LANES >= 16) v = imax(v, dpp<0x140>(v)); // row_mirror
        if (LANES >= 32) v = xor16_imax(v);
        if (LANES >= 64) v = xor32_imax(v);
        return of_key(v);
    }
    // accumulator register v of lane group g holds row 4 g + v of the 16 x 16 tile
    __device__ static int row_of(int g, int v) { return 4 * g + v; }
    // position of logical index j inside LDS rows / the row-shift array
    __device__ static int phys(int j) { return j; }
    // negative iff im is an odd multiple of pi
    __device__ static bool is_negative(float im)
    {
        int k = (int)__builtin_rintf(im * 0.318309886183790671538f);
        return (k & 1) != 0;
    }
    // x with its sign flipped when im is an odd multiple of pi: the parity bit of
    // round(im / pi) is moved onto the sign bit
    __device__ static float apply_sign(float x, float im)
    {
        const int k = (int)__builtin_rintf(im * 0.318309886183790671538f);
        return __builtin_bit_cast(float, __builtin_bit_cast(int, x) ^ (k << 31));
    }
    // binary exponent of x in the frexp convention (|x| = m 2^e, 1/2 <= m < 1), as a float;
    // zero counts as 2^-126 (it only has to lose every comparison that matters)
    __device__ static float exponent_of(float x)
    {
        const unsigned b = __builtin_bit_cast(unsigned, x);
        return (float)(int)((b >> 23) & 0xffu) - 126.0f;
    }
    __device__ static float clamp_shift(float sh) { return __builtin_amdgcn_fmed3f(sh, -4000.0f, 4000.0f); }
    // row shift for a row whose largest log-magnitude is r: a whole number near r log2(e)
    __device__ static float row_shift(float r) { return r > neg_inf() ? __builtin_ceilf(r * 1.44269504088896340736f) : 0.0f; }
    // 2^(re log2(e) - n) for a whole number n >= re log2(e) (about): the product with
    // log2(e) is carried in two floats, the whole part of the exponent is applied with
    // ldexp, so the result is good to a few units in the last place for any shift.
    __device__ static float exp2_shifted(float re, float n)
    {
#pragma clang fp contract(off) // p_hi must stay a rounded product: p_lo is its rounding error
        const float kHi = 1.44269502162933349609375f;  // float nearest log2(e)
        const float kLo = 1.925963033500011e-8f;       // log2(e) - kHi
        const float kLn2 = 0.693147182464599609375f;
        const float p_hi = re * kHi;
        float p_lo = __builtin_fmaf(re, kHi, -p_hi);
        p_lo = __builtin_fmaf(re, kLo, p_lo);
        const float t_hi = p_hi - n;                    // exact where it matters (like magnitudes)
        const float y = __builtin_amdgcn_exp2f(t_hi);   // hardware 2^x on an exactly represented argument
        const float yc = __builtin_fmaf(y, p_lo * kLn2, y); // 2^(t_hi + p_lo) = 2^t_hi (1 + p_lo ln 2 + O(p_lo^2)), |p_lo| < 2^-17
        return t_hi > -150.0f ? yc : 0.0f; // false for -inf and NaN as well: they become zero
    }
    // log-magnitude (natural log) of x 2^(n + e), rounded to the component type; x = 0 -> -inf
    // same with the exponents already summed: log-magnitude of x 2^s
    __device__ static float out_re_f(float x, float s)
    {
#pragma clang fp contract(off)
        const float kLn2Hi = 0.693147182464599609375f;
        const float kLn2Lo = -1.90465429995776806e-9f;
        const float l2 = __builtin_amdgcn_logf(__builtin_fabsf(x) * 4294967296.0f) - 32.0f;
        return __builtin_fmaf(s, kLn2Hi, __builtin_fmaf(s, kLn2Lo, l2 * kLn2Hi));
    }
    __device__ static float out_re(float x, float n, double e)
    {
#pragma clang fp contract(off)
        const float kLn2Hi = 0.693147182464599609375f; // float nearest ln 2
        const float kLn2Lo = -1.90465429995776806e-9f; // ln 2 - kLn2Hi
        // scaling by 2^32 keeps subnormal x inside the hardware logarithm's domain
        float l2 = __builtin_amdgcn_logf(__builtin_fabsf(x) * 4294967296.0f) - 32.0f;
        float s = n + (float)e;
        return __builtin_fmaf(s, kLn2Hi, __builtin_fmaf(s, kLn2Lo, l2 * kLn2Hi));
    }
};
template <> struct Comp<double> {
    typedef d4 vec4;
    static constexpr int kPad = 2;
    __device__ static double pi() { return 3.14159265358979311600; }
    __device__ static d4 mfma(double a, double b, d4 c) { return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0); }
    __device__ static double exp2_frac(double f) { return ::exp2(f); }
    __device__ static double log2_abs(double x) { return ::log2(__builtin_fabs(x)); }
    __device__ static double ldexp_(double x, int e) { return __builtin_ldexp(x, e); }
    __device__ static int frexp_exp(double x) { int e; (void)__builtin_frexp(x, &e); return e; }
    __device__ static double abs_(double x) { return __builtin_fabs(x); }
    __device__ static double ceil_(double x) { return __builtin_ceil(x); }
    __device__ static double neg_inf() { return -__builtin_huge_val(); }
    __device__ static double max_(double a, double b) { return a > b ? a : b; }
    __device__ static double xor16_max(double v) { return max_(v, __shfl_xor(v, 16, 64)); }
    __device__ static double xor32_max(double v) { return max_(v, __shfl_xor(v, 32, 64)); }
    __device__ static double xor16_32_max(double v) { return xor32_max(xor16_max(v)); }
    template <int LANES> __device__ static double group_allmax(double a, double b)
    {
        double v = max_(a, b);
#pragma unroll
        for (int s = 1; s < LANES; s <<= 1) v = max_(v, __shfl_xor(v, s, 64));
        return v;
    }
    // the double-precision instruction interleaves rows: register v of lane group g holds row 4 v + g
    __device__ static int row_of(int g, int v) { return 4 * v + g; }
    // ... so contraction index 16 kt + 4 v + g is stored at position 16 kt + 4 g + v, which
    // keeps the four values a lane needs contiguous
    __device__ static int phys(int j) { return (j & ~15) | ((j & 3) << 2) | ((j >> 2) & 3); }
    // (the multiple of pi goes through a 32-bit integer: one conversion instruction, where a 64-bit one is a
    // dozen; phases beyond 2^31 pi carry no parity in a double product with 1 / pi anyway)
    __device__ static bool is_negative(double im)
    {
        const int k = (int)__builtin_rint(im * 0.318309886183790671538);
        return (k & 1) != 0;
    }
    __device__ static double apply_sign(double x, double im) { return is_negative(im) ? -x : x; }
    __device__ static double exponent_of(double x) { return x != 0.0 ? (double)frexp_exp(x) : -1022.0; }
    __device__ static double clamp_shift(double sh) { return sh > -4000.0 ? (sh < 4000.0 ? sh : 4000.0) : -4000.0; }
    __device__ static double row_shift(double r) { return r > neg_inf() ? __builtin_ceil(r * kLog2e) : 0.0; }
    // 2^f for |f| <= 1/2: the exponential series in f ln 2 to degree 13 (remainder below 2e-16),
    // evaluated by Horner's rule; about a third of the instructions of the library routine, which
    // matters because double-precision vector instructions issue at half rate
    __device__ static double exp2_small(double f)
    {
        const double x = f * kLn2;
        double p = 1.6059043836821613e-10; // 1 / 13!
        p = __builtin_fma(p, x, 2.08767569878681e-09);  // 1 / 12!
        p = __builtin_fma(p, x, 2.505210838544172e-08); // 1 / 11!
        p = __builtin_fma(p, x, 2.755731922398589e-07); // 1 / 10!
        p = __builtin_fma(p, x, 2.7557319223985893e-06);
        p = __builtin_fma(p, x, 2.48015873015873e-05);
        p = __builtin_fma(p, x, 0.0001984126984126984);
        p = __builtin_fma(p, x, 0.001388888888888889);
        p = __builtin_fma(p, x, 0.008333333333333333);
        p = __builtin_fma(p, x, 0.041666666666666664);
        p = __builtin_fma(p, x, 0.16666666666666666);
        p = __builtin_fma(p, x, 0.5);
        p = __builtin_fma(p, x, 1.0);
        return __builtin_fma(p, x, 1.0);
    }
    // natural logarithm of |x|, x finite and non-zero: x = m 2^k with m in [sqrt(1/2), sqrt(2)), and
    // ln m = 2 atanh(s), s = (m - 1) / (m + 1), |s| < 0.1716, as its series to s^21 (remainder below 1e-17)
    __device__ static double ln_abs(double x)
    {
        int k;
        double m = __builtin_frexp(__builtin_fabs(x), &k); // [1/2, 1)
        const bool low = m < 0.70710678118654752440;
        m = low ? m + m : m;
        k = low ? k - 1 : k;
        const double den = m + 1.0;
        double r = (double)__builtin_amdgcn_rcpf((float)den);
        r = r * (2.0 - den * r);
        r = r * (2.0 - den * r);
        const double num = m - 1.0;
        double s = num * r;
        s = __builtin_fma(__builtin_fma(-s, den, num), r, s); // one correction step: s = num / den to rounding
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
        return __builtin_fma((double)k, kLn2, p + p);
    }
    __device__ static double exp2_shifted(double re, double n)
    {
        double t = __builtin_fma(re, kLog2e, -n);
        double k = __builtin_rint(t);
        double y = __builtin_ldexp(exp2_small(t - k), (int)(k > -4000.0 ? k : -4000.0));
        return t > -1200.0 ? y : 0.0;
    }
    __device__ static double out_re(double x, double n, double e)
    {
        const double l = __builtin_fma(n + e, kLn2, ln_abs(x)); // evaluated for zero as well, then discarded: no branch
        return x != 0.0 ? l : neg_inf();
    }
};

// 2^t for a double exponent t (t = -inf allowed), used off the hot path (initial states,
// bias terms): whole and fractional part are split in double, so the fraction is exact.
template <typename R> __device__ inline R exp2_of(double t)
{
    t = t > -4000.0 ? t : -4000.0; // also maps -inf and NaN to "underflows to zero"
    t = t < 4000.0 ? t : 4000.0;
    double k = __builtin_rint(t);
    R f = (R)(t - k);
    return Comp<R>::ldexp_(Comp<R>::exp2_frac(f), (int)k);
}

template <typename R> __device__ inline R wave_xor_max(R v, int mask)
{
    R o = __shfl_xor(v, mask, 64);
    return o > v ? o : v;
}

__device__ inline double shfl_xor_double(double v, int mask) { return __shfl_xor(v, mask, 64); }

// One item of the producer: two horizontally adjacent elements of the left factor.
template <typename R> struct Item {
    R re0, im0, re1, im1;
};

// Register budget: waves per SIMD the compiler must leave room for.  The 64 x 64 float
// kernel keeps 16 state + 16 accumulator + 32 prefetch registers per lane and fits in a
// quarter of the register file, so four workgroups share a compute unit.
constexpr int waves_per_simd(int comp_bytes, int dp, int nw)
{
    return (comp_bytes == 4 && dp <= 64) ? 2 : (comp_bytes == 8 && dp == 64 && nw == 4) ? 2 : 1;
}

// FAST: the factor fills the padded tile exactly (n = d = DP), the state has whole
// 16-column slabs and there is no bias column, so every bounds test and the bias path
// compile away and the step is straight-line code.
// IO: component type of the GOOM arrays in memory (left factors, initial state, bias, outputs).  It differs
// from R in one combination only, IO = float with R = double: complex64 data walked with a double running
// product (every load widened, every output rounded once when it is stored).
template <typename R, int DP, int NW, int LEFT_FACT, bool FAST, typename IO = R>
__global__ __launch_bounds__(NW * 64, waves_per_simd(sizeof(R), DP, NW)) void chain_kernel(ChainArgs a)
{
    constexpr int KT = DP / 16;
    constexpr int LPR = DP / 2; // producer lanes per row
    constexpr int NT = NW * 64;
    constexpr int LDA = DP + Comp<R>::kPad;
    constexpr int NITEMS = DP * LPR;
    constexpr int Q = (NITEMS + NT - 1) / NT;  // items per thread
    constexpr bool PREFETCH = Q <= 16 && !(sizeof(R) == 8 && DP >= 128); // items of the next factor wait in registers during the product
    constexpr int QB = PREFETCH ? Q : 8;       // items per batch
    typedef typename Comp<R>::vec4 vec4;

    extern __shared__ __align__(16) unsigned char smem[];
    constexpr size_t kTileBytes = (size_t)DP * LDA * sizeof(R);
    constexpr size_t kBufBytes = kTileBytes + (size_t)DP * sizeof(double);
    constexpr int NBUF = (2 * kBufBytes + 128 <= 160 * 1024) ? 2 : 1; // double buffer when it fits in LDS
    // buffer b: tile at smem + b * kBufBytes, row shifts after the tile
    auto tile_of = [&](int b) { return reinterpret_cast<R *>(smem + (size_t)b * kBufBytes); };
    auto nsh_of = [&](int b) { return reinterpret_cast<R *>(smem + (size_t)b * kBufBytes + kTileBytes); };
    double *wave_red = reinterpret_cast<double *>(smem + NBUF * kBufBytes); // NW doubles

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6); // wave-uniform, kept in a scalar register
    const int g = lane >> 4;
    const int c = lane & 15;
    const int n_rows = a.n, d = a.d, m = a.m;
    const int col = wave * 16 + c;
    const bool slab_active = FAST || wave < a.nslabs; // FAST: every wave owns a slab
    const R kNegInf = Comp<R>::neg_inf();

    const long long chain = blockIdx.x;
    const long long item = chain / a.chunks_launched;
    const long long chunk = chain % a.chunks_launched;
    const long long t0 = chunk * a.chunk_len;
    long long len = a.steps - t0;
    if (len > a.chunk_len) len = a.chunk_len;
    const long long chain_global = item * a.chunks_per_item + chunk; // index into per-chain arrays

    const unsigned char *left0 = a.left + item * a.left_batch_stride + t0 * a.left_step_stride;
    const bool vec_ok = (d % 2) == 0;

    // ------------------------------------------------------------------ producer
    // Left factor number t is turned into an LDS tile
    //   tile[i][j] = (+-) 2^(log2|A_ij| - n_i),  n_i = a whole number near max_j log2|A_ij|
    // (0 for a zero row), with n_i recorded beside it.  Rows and columns beyond the
    // factor's size are zero.  load_items reads batch q0 of the factor into registers,
    // convert_items exponentiates it into the tile.
    auto load_items = [&](long long t, int q0, Item<R> (&it)[QB]) {
        const unsigned char *src = left0 + t * a.left_step_stride;
        // row strides: the template's size where it is known, else opaque to the optimiser, so that the
        // items' offsets are not carried in registers across the chain's loop
        int ld = FAST ? DP : d, lfc = a.left_fact_cols;
        if (!FAST) asm volatile("" : "+s"(ld));
        asm volatile("" : "+s"(lfc));
#pragma unroll
        for (int q = 0; q < QB; ++q) {
            const int p = tid + (q0 + q) * NT;
            const int row = p / LPR, cj = 2 * (p % LPR);
            const bool v0 = FAST || ((p < NITEMS) && row < n_rows && cj < d);
            const bool v1 = FAST || (v0 && (cj + 1 < d));
            if (LEFT_FACT) {
                // factored left factor: mantissas [DP][left_fact_cols], leading columns on one exponent
                const R *mp = reinterpret_cast<const R *>(src) + (size_t)(row * lfc + cj);
                it[q].re0 = v0 ? mp[0] : (R)0;
                it[q].re1 = v1 ? mp[1] : (R)0;
                it[q].im0 = it[q].im1 = (R)0;
            } else {
                const IO *gp = reinterpret_cast<const IO *>(src) + (size_t)(row * ld + cj) * 2;
                if (FAST || (v1 && vec_ok)) {
                    if (sizeof(IO) == 4) {
                        const f4 w = *reinterpret_cast<const f4 *>(gp);
                        it[q].re0 = w[0]; it[q].im0 = w[1]; it[q].re1 = w[2]; it[q].im1 = w[3];
                    } else {
                        const d4 w = *reinterpret_cast<const d4 *>(gp);
                        it[q].re0 = w[0]; it[q].im0 = w[1]; it[q].re1 = w[2]; it[q].im1 = w[3];
                    }
                } else {
                    it[q].re0 = v0 ? gp[0] : kNegInf; it[q].im0 = v0 ? gp[1] : (R)0;
                    it[q].re1 = v1 ? gp[2] : kNegInf; it[q].im1 = v1 ? gp[3] : (R)0;
                }
            }
        }
    };
    auto convert_items = [&](long long t, int q0, const Item<R> (&it)[QB], int buf) {
        R *tile = tile_of(buf);
        R *nsh = nsh_of(buf);
        R common = (R)0;
        if (LEFT_FACT) {
            const unsigned char *src = left0 + t * a.left_step_stride;
            common = (R) * reinterpret_cast<const double *>(src + (size_t)DP * a.left_fact_cols * sizeof(R));
        }
#pragma unroll
        for (int q = 0; q < QB; ++q) {
            const int p = tid + (q0 + q) * NT;
            const int row = p / LPR, cj = 2 * (p % LPR);
            R x0, x1, n;
            if (LEFT_FACT) {
                const R a0 = Comp<R>::abs_(it[q].re0), a1 = Comp<R>::abs_(it[q].re1);
                const R r = Comp<R>::template group_allmax<LPR>(a0, a1);
                const int e = (r > (R)0 && r < -kNegInf) ? Comp<R>::frexp_exp(r) : 0;
                x0 = Comp<R>::ldexp_(it[q].re0, -e);
                x1 = Comp<R>::ldexp_(it[q].re1, -e);
                n = (R)e + common;
            } else {
                const R r = Comp<R>::template group_allmax<LPR>(it[q].re0, it[q].re1);
                n = Comp<R>::row_shift(r);
                x0 = Comp<R>::apply_sign(Comp<R>::exp2_shifted(it[q].re0, n), it[q].im0);
                x1 = Comp<R>::apply_sign(Comp<R>::exp2_shifted(it[q].re1, n), it[q].im1);
            }
            if (FAST || p < NITEMS) {
                tile[row * LDA + Comp<R>::phys(cj)] = x0;
                tile[row * LDA + Comp<R>::phys(cj + 1)] = x1;
                nsh[Comp<R>::phys(row)] = n; // every lane of the row writes the same value
            }
        }
    };
    // whole factor, no registers kept (start-up, and factors too large to prefetch)
    auto produce_now = [&](long long t, int buf) __attribute__((always_inline)) {
#pragma unroll 1
        for (int q0 = 0; q0 < Q; q0 += QB) {
            Item<R> it[QB];
            load_items(t, q0, it);
            convert_items(t, q0, it, buf);
        }
    };

    // ------------------------------------------------------------------ initial state
    R st[KT][4]; // st[kt][v] = W[16 kt + row_of(g, v)][col]
    double ecol = 0.0;
    const size_t fact_mant_bytes = (size_t)DP * a.fact_cols * sizeof(R);
    if (a.init_mode == 0 || a.init_mode == 3) { // identity / zero
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = 16 * kt + Comp<R>::row_of(g, v);
                st[kt][v] = (a.init_mode == 0 && row == col && row < d && col < m) ? (R)1 : (R)0;
            }
    } else if (a.init_mode == 1) {
        long long iidx = chain_global;
        if (a.init_group > 0) { // chunk c sits in group min(c / S, G - 1) at offset c - group * S
            long long grp = chunk / a.init_group;
            if (grp >= a.init_ngroups) grp = a.init_ngroups - 1;
            iidx = (item * a.init_ngroups + grp) * (a.init_group + 1) + (chunk - grp * a.init_group);
        }
        const unsigned char *ip = a.init + iidx * a.init_stride;
        const R *mp = reinterpret_cast<const R *>(ip);
        const double *ep = reinterpret_cast<const double *>(ip + fact_mant_bytes);
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                st[kt][v] = slab_active ? mp[(size_t)(16 * kt + Comp<R>::row_of(g, v)) * a.fact_cols + col] : (R)0;
        ecol = slab_active ? ep[col] : 0.0;
    } else {
        // GOOM initial state [d, m]: column shift e = ceil(max_i log2|x_ik|), W = +-2^(log2|x| - e)
        const IO *gp = reinterpret_cast<const IO *>(a.init + item * a.init_stride);
        R cmax = kNegInf;
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = 16 * kt + Comp<R>::row_of(g, v);
                const bool ok = slab_active && row < d && col < m;
                const R re = ok ? gp[((size_t)row * m + col) * 2] : kNegInf;
                cmax = re > cmax ? re : cmax;
            }
        cmax = wave_xor_max<R>(cmax, 16);
        cmax = wave_xor_max<R>(cmax, 32);
        ecol = (cmax > kNegInf) ? __builtin_ceil((double)cmax * kLog2e) : 0.0;
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = 16 * kt + Comp<R>::row_of(g, v);
                const bool ok = slab_active && row < d && col < m;
                const R re = ok ? gp[((size_t)row * m + col) * 2] : kNegInf;
                const R im = ok ? gp[((size_t)row * m + col) * 2 + 1] : (R)0;
                const R x = exp2_of<R>(__builtin_fma((double)re, kLog2e, -ecol));
                st[kt][v] = Comp<R>::is_negative(im) ? -x : x;
            }
    }

    auto store_fact = [&](unsigned char *dst, bool common_exponent) {
        // dst: mantissas [DP][fact_cols] then exponents [fact_cols] (double)
        R *mp = reinterpret_cast<R *>(dst);
        double *ep = reinterpret_cast<double *>(dst + fact_mant_bytes);
        double e_out = ecol;
        int shift = 0;
        if (common_exponent) {
            // one exponent for the leading columns (< d when a bias column exists, all otherwise)
            R cm = (R)0;
#pragma unroll
            for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    R av = Comp<R>::abs_(st[kt][v]);
                    cm = av > cm ? av : cm;
                }
            cm = wave_xor_max<R>(cm, 16);
            cm = wave_xor_max<R>(cm, 32);
            const int ncommon = a.bias_mode ? d : m;
            double ev = (slab_active && col < ncommon && cm > (R)0) ? ecol : kNegBig;
#pragma unroll
            for (int s = 1; s < 16; s <<= 1) {
                double o = shfl_xor_double(ev, s);
                ev = o > ev ? o : ev;
            }
            __syncthreads();
            if (lane == 0) wave_red[wave] = ev;
            __syncthreads();
            double emax = kNegBig;
            for (int w = 0; w < NW; ++w) emax = wave_red[w] > emax ? wave_red[w] : emax;
            if (emax == kNegBig) emax = 0.0;
            if (col < ncommon) {
                double dsh = ecol - emax;
                dsh = dsh > -4000.0 ? dsh : -4000.0;
                shift = (cm > (R)0) ? (int)dsh : 0;
                e_out = emax;
            }
        }
        if (slab_active) {
            // the row stride goes through an empty asm so that the DP / 4 offsets of a lane's entries are
            // worked out here, where they are used, and not kept in (spilled) registers across the chain's loop
            int fc = a.fact_cols;
            asm volatile("" : "+s"(fc));
#pragma unroll
            for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    mp[(size_t)((16 * kt + Comp<R>::row_of(g, v)) * fc + col)] = Comp<R>::ldexp_(st[kt][v], shift);
            if (g == 0) ep[col] = e_out;
        }
    };

    unsigned char *fact_steps = a.out_fact_steps ? a.out_fact_steps + (chain_global * (a.chunk_len + 1)) * a.fact_stride : nullptr;

    Item<R> pre[QB]; // the next left factor, on its way from memory while the current product runs
    if (len > 0) produce_now(0, 0);
    if (PREFETCH && len > 1) load_items(1, 0, pre);
    __syncthreads();

    for (long long t = 0; t < len; ++t) {
        const int cur = NBUF == 2 ? (int)(t & 1) : 0;
        const R *tile = tile_of(cur);
        const R *nsh = nsh_of(cur);

        if (fact_steps) store_fact(fact_steps + t * a.fact_stride, false);

        // ------------------------------------------------------------ product on the matrix cores
        vec4 acc[KT];
#pragma unroll
        for (int mt = 0; mt < KT; ++mt) acc[mt] = vec4{0, 0, 0, 0};
        if (FAST) {
            // Straight-line step: the product of this step and the exponentiation of the
            // next factor (already in registers) are independent, so they sit in one
            // scheduling region and the matrix instructions are interleaved with the
            // vector work.  Past the end of the chain the last factor is converted and
            // loaded again (clamped index) instead of branching; nobody reads the result.
            const long long tn = t + 1 < len ? t + 1 : len - 1;
            const long long tl = t + 2 < len ? t + 2 : len - 1;
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) {
                vec4 av[KT];
#pragma unroll
                for (int mt = 0; mt < KT; ++mt)
                    av[mt] = *reinterpret_cast<const vec4 *>(&tile[(16 * mt + c) * LDA + 16 * kt + 4 * g]);
#pragma unroll
                for (int v = 0; v < 4; ++v)
#pragma unroll
                    for (int mt = 0; mt < KT; ++mt) acc[mt] = Comp<R>::mfma(av[mt][v], st[kt][v], acc[mt]);
            }
            if (PREFETCH && NBUF == 2) {
                convert_items(tn, 0, pre, cur ^ 1);
                load_items(tl, 0, pre);
            }
        } else if (slab_active) {
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) {
                vec4 av[KT];
#pragma unroll
                for (int mt = 0; mt < KT; ++mt)
                    av[mt] = *reinterpret_cast<const vec4 *>(&tile[(16 * mt + c) * LDA + 16 * kt + 4 * g]);
#pragma unroll
                for (int v = 0; v < 4; ++v)
#pragma unroll
                    for (int mt = 0; mt < KT; ++mt) acc[mt] = Comp<R>::mfma(av[mt][v], st[kt][v], acc[mt]);
            }
        }

        // ------------------------------------------------------------ epilogue
        // acc[mt][v] is entry (i = 16 mt + row_of(g, v), col) of the scaled product; the
        // true value is acc * 2^(n_i + ecol).  Exponent arithmetic runs in the component
        // type on whole numbers: differences that matter are between numbers of like size
        // and therefore exact; a reference exponent that is a few units off only moves the
        // mantissas' scale, never the represented value.
        //
        // bias column (linear recurrence with bias): b_i, given as a GOOM or as a column
        // of the factored left factor, is added to entry (i, bias_col) in the log2 domain.
        const bool bias_lane = !FAST && a.bias_mode != 0 && slab_active && col == a.bias_col;
        // bias and stored states rescaled by e^(-+io_shift[s]) (see ChainArgs): the shift joins the column's exponent, in double
        const double ios = (!FAST && a.io_shift) ? (double)a.io_shift[item * a.steps + t0 + t] * kLog2e : 0.0;
        auto bias_term = [&](int i, double &blog, bool &bneg) { // blog = log2|b_i| - ecol
            blog = kNegBig;
            bneg = false;
            if (i >= n_rows) return;
            if (a.bias_mode == 1) {
                const IO *bp = reinterpret_cast<const IO *>(a.bias) + ((size_t)(item * a.steps + t0 + t) * n_rows + i) * 2;
                R br = bp[0];
                if (br > kNegInf) blog = (double)br * kLog2e - ecol - ios; // (ios: the step's io_shift in powers of two, else 0)
                bneg = Comp<R>::is_negative(bp[1]);
            } else {
                const unsigned char *src = left0 + t * a.left_step_stride;
                const R *mp = reinterpret_cast<const R *>(src);
                const double *ex = reinterpret_cast<const double *>(src + (size_t)DP * a.left_fact_cols * sizeof(R));
                int lfc = a.left_fact_cols; // opaque, as in load_items
                asm volatile("" : "+s"(lfc));
                R bv = mp[(size_t)(i * lfc + d)];
                if (bv != (R)0) blog = (double)Comp<R>::log2_abs(bv) + ex[d] - ecol;
                bneg = bv < (R)0;
            }
        };

        // column reference: cm = max_i of (binary exponent of the entry) + n_i
        R cm = kNegInf;
#pragma unroll
        for (int mt = 0; mt < KT; ++mt) {
            const vec4 nv = *reinterpret_cast<const vec4 *>(&nsh[16 * mt + 4 * g]);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const R x = acc[mt][v];
                const R lg = Comp<R>::exponent_of(x) + nv[v];
                cm = Comp<R>::max_(lg, cm);
            }
        }
        if (bias_lane) {
#pragma unroll
            for (int mt = 0; mt < KT; ++mt)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    double blog;
                    bool bneg;
                    bias_term(16 * mt + Comp<R>::row_of(g, v), blog, bneg);
                    const R lb = blog > kNegBig ? (R)__builtin_ceil(blog) : kNegInf;
                    cm = lb > cm ? lb : cm;
                }
        }
        cm = Comp<R>::xor16_32_max(cm);
        if (bias_lane) cm += (R)2; // room for the sum of two terms
        const bool col_nonzero = cm > kNegInf;
        const R cms = col_nonzero ? cm : (R)0;

        const bool want_out = a.out_goom && slab_active && (FAST || col < m) && (!a.out_goom_last_only || t == len - 1);
        // (in FAST kernels every term above is wave-uniform)
        IO *outp = nullptr;
        if (want_out) {
            long long o_idx = a.out_goom_last_only ? chain_global : (item * a.steps + t0 + t);
            // (FAST: the sizes are the template's, so the offsets of a lane's entries are constants and
            // need no registers across the loop)
            outp = reinterpret_cast<IO *>(a.out_goom) + (FAST ? (size_t)o_idx * (DP * 16 * NW) : (size_t)o_idx * n_rows * m) * 2;
        }

        // (the row stride is made opaque here so that the offsets of a lane's entries are not kept in
        // registers, which would be spilled, across the loop)
        int mo = m;
        if (!FAST) asm volatile("" : "+s"(mo));

        // rescale: entry <- entry 2^(n_i - cm), exact; the state's exponent takes cm
        auto rescale = [&](R x, R n_i) {
            return Comp<R>::ldexp_(x, (int)Comp<R>::clamp_shift(n_i - cms));
        };
        if (FAST) {
            if (want_out) { // wave-uniform: one branch around all of this step's stores
                // the lane's first entry; the others lie at constant distances from it (row_of is linear)
                IO *ob = outp + (Comp<R>::row_of(g, 0) * (16 * NW) + col) * 2;
#pragma unroll
                for (int mt = 0; mt < KT; ++mt) {
                    const vec4 nv = *reinterpret_cast<const vec4 *>(&nsh[16 * mt + 4 * g]);
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const R x = acc[mt][v];
                        const R re = Comp<R>::out_re(x, nv[v], ecol);
                        const IO im = x < (R)0 ? Comp<IO>::pi() : (IO)0;
                        IO *o = ob + ((16 * mt + Comp<R>::row_of(0, v)) * (16 * NW)) * 2;
                        if (sizeof(IO) == 4) {
                            *reinterpret_cast<float2 *>(o) = float2{(float)re, (float)im};
                        } else {
                            *reinterpret_cast<double2 *>(o) = double2{(double)re, (double)im};
                        }
                        st[mt][v] = rescale(x, nv[v]);
                    }
                }
            } else {
#pragma unroll
                for (int mt = 0; mt < KT; ++mt) {
                    const vec4 nv = *reinterpret_cast<const vec4 *>(&nsh[16 * mt + 4 * g]);
#pragma unroll
                    for (int v = 0; v < 4; ++v) st[mt][v] = rescale(acc[mt][v], nv[v]);
                }
            }
        } else if (!bias_lane) {
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) {
                const vec4 nv = *reinterpret_cast<const vec4 *>(&nsh[16 * mt + 4 * g]);
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int i = 16 * mt + Comp<R>::row_of(g, v);
                    const R x = acc[mt][v];
                    if (want_out && i < n_rows) {
                        const R re = Comp<R>::out_re(x, nv[v], ecol + ios);
                        const IO im = x < (R)0 ? Comp<IO>::pi() : (IO)0;
                        IO *o = outp + (size_t)(i * mo + col) * 2;
                        if (sizeof(IO) == 4) {
                            *reinterpret_cast<float2 *>(o) = float2{(float)re, (float)im};
                        } else {
                            *reinterpret_cast<double2 *>(o) = double2{(double)re, (double)im};
                        }
                    }
                    st[mt][v] = rescale(x, nv[v]);
                }
            }
        } else {
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) {
                const vec4 nv = *reinterpret_cast<const vec4 *>(&nsh[16 * mt + 4 * g]);
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int i = 16 * mt + Comp<R>::row_of(g, v);
                    const R x = acc[mt][v];
                    double blog;
                    bool bneg;
                    bias_term(i, blog, bneg);
                    // entry = x 2^(n_i - cm) + (+-) 2^(blog - cm), in units of 2^(ecol + cm)
                    const R xa = rescale(x, nv[v]);
                    const R xb = (col_nonzero && blog > kNegBig) ? exp2_of<R>(blog - (double)cm) : (R)0;
                    const R xs = xa + (bneg ? -xb : xb);
                    if (want_out && i < n_rows) {
                        const R re = Comp<R>::out_re(xs, cms, ecol + ios);
                        const IO im = xs < (R)0 ? Comp<IO>::pi() : (IO)0;
                        IO *o = outp + (size_t)(i * mo + col) * 2;
                        o[0] = (IO)re;
                        o[1] = im;
                    }
                    st[mt][v] = xs;
                }
            }
        }
        if (col_nonzero) ecol += (double)cm;

        // ------------------------------------------------------------ next left factor
        if (NBUF == 1) __syncthreads(); // every wave is done reading the only tile
        if (FAST && PREFETCH && NBUF == 2) {
            // the next factor was converted beside the product above
        } else if (t + 1 < len) {
            const int nxt = NBUF == 2 ? (cur ^ 1) : 0;
            if (PREFETCH) {
                convert_items(t + 1, 0, pre, nxt);
                if (t + 2 < len) load_items(t + 2, 0, pre);
            } else {
                produce_now(t + 1, nxt);
            }
        }
        __syncthreads();
    }

    if (fact_steps) store_fact(fact_steps + len * a.fact_stride, false);
    if (a.out_fact_final) store_fact(a.out_fact_final + chain_global * a.fact_stride, a.final_common_exponent != 0);
}

template <typename R, int DP, int NW, int LEFT_FACT, bool FAST, typename IO = R> int launch_one(goom_ctx *ctx, const ChainArgs &args, long long grid, const char *label)
{
    constexpr int LDA = DP + Comp<R>::kPad;
    const size_t buf = (size_t)DP * LDA * sizeof(R) + (size_t)DP * sizeof(double);
    const int nbuf = (2 * buf + 128 <= 160 * 1024) ? 2 : 1;
    size_t lds = nbuf * buf + 128;
    auto kern = chain_kernel<R, DP, NW, LEFT_FACT, FAST, IO>;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return goom::check_hip(ctx, e, "hipFuncSetAttribute(chain_kernel)");
    }
    if (grid <= 0) return GOOM_OK;
    if (grid > 0x7fffffffLL) return goom::fail(ctx, GOOM_EUNSUPPORTED, "too many chains for one launch (%lld)", grid);
    goom::prof_begin(ctx, label);
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(NW * 64), lds, ctx->stream, args);
    goom::prof_end(ctx);
    return goom::check_hip(ctx, hipGetLastError(), "launch chain_kernel");
}

template <typename R, int LEFT_FACT, typename IO = R> int dispatch(goom_ctx *ctx, const ChainArgs &args, int dp, int nw, long long grid, const char *label)
{
    const bool fast = args.n == dp && args.d == dp && args.m == 16 * nw && args.bias_mode == 0;
#define GOOM_CASE(DPV, NWV)                                                                           \
    if (dp == DPV && nw == NWV)                                                                       \
        return fast ? launch_one<R, DPV, NWV, LEFT_FACT, true, IO>(ctx, args, grid, label)            \
                    : launch_one<R, DPV, NWV, LEFT_FACT, false, IO>(ctx, args, grid, label);
    GOOM_CASE(16, 1)
    GOOM_CASE(16, 2)
    GOOM_CASE(32, 1)
    GOOM_CASE(32, 2)
    GOOM_CASE(32, 3)
    GOOM_CASE(64, 1)
    GOOM_CASE(64, 4)
    GOOM_CASE(64, 5)
    GOOM_CASE(128, 1)
    GOOM_CASE(128, 8)
    GOOM_CASE(128, 9)
#undef GOOM_CASE
    return goom::fail(ctx, GOOM_EUNSUPPORTED, "no kernel for padded size %d with %d waves", dp, nw);
}


// one explicit instantiation per translation unit (they compile in parallel)
int dispatch_f32_goom(goom_ctx *ctx, const ChainArgs &args, int dp, int nw, long long grid, const char *label);
int dispatch_f32_fact(goom_ctx *ctx, const ChainArgs &args, int dp, int nw, long long grid, const char *label);
int dispatch_f64_goom(goom_ctx *ctx, const ChainArgs &args, int dp, int nw, long long grid, const char *label);
int dispatch_f64_fact(goom_ctx *ctx, const ChainArgs &args, int dp, int nw, long long grid, const char *label);
// double running product over complex64 GOOMs (left factors, initial state, bias, outputs)
int dispatch_f64_goom_io32(goom_ctx *ctx, const ChainArgs &args, int dp, int nw, long long grid, const char *label);

} // namespace goom_chain
