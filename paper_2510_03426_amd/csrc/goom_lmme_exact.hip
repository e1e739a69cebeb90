// Repair pass of LMME (paper Section 3.2): recompute, by the definition
//     C'_ik = LSE_j(A'_ij + B'_jk)                                   (eq. 6)
// every output whose scaled real product (eq. 7, computed by the chain kernel) may have lost
// terms to underflow.  The paper itself calls the scaled product a compromise in precision;
// when the logarithms of the operands spread over hundreds of units, almost every term sits
// below the component format's range after the row/column shifts and the product comes out
// as zero although the true value is finite.
//
// Certificate.  With row shifts n_i and column shifts e_k (whole powers of two, largest entry
// of the row / column scaled to at most 1), a term that is dropped is smaller than the
// smallest normal number 2^-E of the format, so the dropped mass of one output is below
// d 2^-E.  An output whose scaled magnitude log2|C~_ik| = Re(C'_ik) log2(e) - n_i - e_k is
// at least -E + log2(d) + 20 is therefore right to about 2^-20 relative and is kept; all
// others are recomputed term by term on the vector ALUs, in two passes over j (maximum, then
// signed sum of exponentials), which never leaves the representable range.
//
// One workgroup handles a 16 x 16 block of outputs of one batch item; the rows of A and the
// columns of B it needs are staged in LDS, up to 128 inner indices at a time.  A block whose
// outputs are all certified returns after the first sweep.
#include "goom_internal.h"

namespace {

constexpr int kTile = 16;
constexpr int kThreads = kTile * kTile;

struct ExactArgs {
    const void *A, *B;
    void *C;
    long long batch;
    int n, d, m;
};

template <typename R> struct Num;
template <> struct Num<float> {
    static constexpr float kLog2e = 1.44269504088896340736f;
    static constexpr float kLn2 = 0.693147180559945309417f;
    static constexpr float kMargin = -126.0f + 20.0f;
    __device__ static float neg_inf() { return -__builtin_huge_valf(); }
    __device__ static float pi() { return 3.14159274101257324219f; }
    __device__ static float exp2_(float x) { return __builtin_amdgcn_exp2f(x); }
    __device__ static float log2_(float x) { return ::log2f(x); }
    __device__ static int parity(float im) { return (int)__builtin_rintf(im * 0.318309886183790671538f) & 1; }
};
template <> struct Num<double> {
    static constexpr double kLog2e = 1.44269504088896340736;
    static constexpr double kLn2 = 0.693147180559945309417;
    static constexpr double kMargin = -1022.0 + 40.0;
    __device__ static double neg_inf() { return -__builtin_huge_val(); }
    __device__ static double pi() { return 3.14159265358979311600; }
    __device__ static double exp2_(double x) { return ::exp2(x); }
    __device__ static double log2_(double x) { return ::log2(x); }
    __device__ static int parity(double im) { return (int)((long long)__builtin_rint(im * 0.318309886183790671538) & 1LL); }
};

constexpr int kJBlock = 128; // inner indices staged in LDS at a time

template <typename R> __global__ __launch_bounds__(kThreads) void lmme_exact_kernel(ExactArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int n = a.n, d = a.d, m = a.m;
    const int jb = d < kJBlock ? d : kJBlock;
    // LDS: log-magnitudes of 16 rows of A [16][jb], 16 columns of B [jb][16], then their signs as bytes
    R *are = reinterpret_cast<R *>(smem);
    R *bre = are + (size_t)kTile * jb;
    unsigned char *asg = reinterpret_cast<unsigned char *>(bre + (size_t)jb * kTile);
    unsigned char *bsg = asg + (size_t)kTile * jb;

    const int tid = threadIdx.x;
    const int ti = tid / kTile, tk = tid % kTile;
    const int blocks_k = (m + kTile - 1) / kTile, blocks_i = (n + kTile - 1) / kTile;
    const long long bid = blockIdx.x;
    const long long b = bid / ((long long)blocks_i * blocks_k);
    const int rem = (int)(bid % ((long long)blocks_i * blocks_k));
    const int i0 = (rem / blocks_k) * kTile, k0 = (rem % blocks_k) * kTile;
    const R *Ab = static_cast<const R *>(a.A) + (size_t)b * n * d * 2;
    const R *Bb = static_cast<const R *>(a.B) + (size_t)b * d * m * 2;
    R *Cb = static_cast<R *>(a.C) + (size_t)b * n * m * 2;

    // stage inner indices [j0, j0 + len) of the 16 rows of A and the 16 columns of B
    auto stage = [&](int j0, int len) {
        __syncthreads();
        for (int e = tid; e < kTile * len; e += kThreads) {
            const int r = e / len, j = e % len;
            const bool ok = i0 + r < n;
            are[r * jb + j] = ok ? Ab[((size_t)(i0 + r) * d + j0 + j) * 2] : Num<R>::neg_inf();
            asg[r * jb + j] = ok ? (unsigned char)Num<R>::parity(Ab[((size_t)(i0 + r) * d + j0 + j) * 2 + 1]) : 0;
        }
        for (int e = tid; e < len * kTile; e += kThreads) {
            const int j = e / kTile, c = e % kTile;
            const bool ok = k0 + c < m;
            bre[j * kTile + c] = ok ? Bb[((size_t)(j0 + j) * m + k0 + c) * 2] : Num<R>::neg_inf();
            bsg[j * kTile + c] = ok ? (unsigned char)Num<R>::parity(Bb[((size_t)(j0 + j) * m + k0 + c) * 2 + 1]) : 0;
        }
        __syncthreads();
    };

    const int i = i0 + ti, k = k0 + tk;
    const bool live = i < n && k < m;
    // first sweep over j: the shifts of the scaled product, as its kernels choose them (to within one
    // unit), and the largest pairwise sum
    R amax = Num<R>::neg_inf(), bmax = Num<R>::neg_inf(), mx = Num<R>::neg_inf();
    for (int j0 = 0; j0 < d; j0 += jb) {
        const int len = d - j0 < jb ? d - j0 : jb;
        stage(j0, len);
        for (int j = 0; j < len; ++j) {
            const R x = are[ti * jb + j], y = bre[j * kTile + tk];
            amax = x > amax ? x : amax;
            bmax = y > bmax ? y : bmax;
            const R z = x + y;
            mx = z > mx ? z : mx;
        }
    }
    bool need = false;
    if (live) {
        const R cre = Cb[((size_t)i * m + k) * 2];
        if (amax > Num<R>::neg_inf() && bmax > Num<R>::neg_inf()) {
            const R ni = __builtin_ceil((double)amax * 1.44269504088896340736);
            const R ek = __builtin_ceil((double)bmax * 1.44269504088896340736);
            const R scaled = cre * Num<R>::kLog2e - ni - ek; // log2 of the scaled product's magnitude
            R log2d = 0;
            for (int s = 1; s < d; s <<= 1) log2d += 1;
            need = !(scaled >= Num<R>::kMargin + log2d + 1); // also true for -inf and NaN
        }
        // a zero row or column gives an exact zero either way
    }
    if (!__syncthreads_or(need ? 1 : 0)) return;

    // second sweep: signed sum of exponentials relative to the largest pairwise sum (every thread of the
    // block stages; only the uncertified outputs are rewritten)
    R sum = 0;
    for (int j0 = 0; j0 < d; j0 += jb) {
        const int len = d - j0 < jb ? d - j0 : jb;
        if (d > jb) stage(j0, len); // a single block of j is still in LDS
        if (need && mx > Num<R>::neg_inf()) {
            for (int j = 0; j < len; ++j) {
                const R z = are[ti * jb + j] + bre[j * kTile + tk];
                const R t = Num<R>::exp2_((z - mx) * Num<R>::kLog2e);
                sum += ((asg[ti * jb + j] ^ bsg[j * kTile + tk]) & 1) ? -t : t;
            }
        }
    }
    if (!need) return;
    R re_out = Num<R>::neg_inf(), im_out = 0;
    if (mx > Num<R>::neg_inf() && sum != 0) {
        re_out = mx + Num<R>::log2_(sum < 0 ? -sum : sum) * Num<R>::kLn2;
        im_out = sum < 0 ? Num<R>::pi() : (R)0;
    }
    Cb[((size_t)i * m + k) * 2] = re_out;
    Cb[((size_t)i * m + k) * 2 + 1] = im_out;
}

} // namespace

namespace goom {

int launch_lmme_exact(goom_ctx *ctx, const void *A, const void *B, void *C, long long batch, int n, int d, int m, int dtype)
{
    ExactArgs a;
    a.A = A;
    a.B = B;
    a.C = C;
    a.batch = batch;
    a.n = n;
    a.d = d;
    a.m = m;
    const long long grid = batch * ((n + kTile - 1) / kTile) * ((m + kTile - 1) / kTile);
    if (grid > 0x7fffffffLL) return fail(ctx, GOOM_EUNSUPPORTED, "too many output blocks for one launch");
    const size_t comp = dtype == GOOM_C64 ? 4 : 8;
    const int jb = d < kJBlock ? d : kJBlock;
    const size_t lds = 2 * (size_t)kTile * jb * comp + 2 * (size_t)kTile * jb;
    prof_begin(ctx, "lmme_exact_repair");
    if (dtype == GOOM_C64)
        hipLaunchKernelGGL(lmme_exact_kernel<float>, dim3((unsigned)grid), dim3(kThreads), lds, ctx->stream, a);
    else
        hipLaunchKernelGGL(lmme_exact_kernel<double>, dim3((unsigned)grid), dim3(kThreads), lds, ctx->stream, a);
    prof_end(ctx);
    return check_hip(ctx, hipGetLastError(), "launch lmme_exact_kernel");
}

} // namespace goom
