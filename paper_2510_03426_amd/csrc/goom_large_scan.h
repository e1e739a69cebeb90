// Scans of matrices above 128 x 128 (paper Section 4.1 runs chains up to 1024 x 1024), for float and double
// components.  The running product of a chain is kept TRANSPOSED, St[column of the state][row], as mantissas
// of the component type with one power-of-two exponent per state column (double), so that one step,
//     St <- St A~^T,  then every row of St rescaled (the row shifts of A~ folded in),
// is an "NT" GEMM plus two light passes, and closes under iteration.  All chains of a launch (batch items x
// chunks) advance together, one step per round of launches.  The kernels and the driver are templates over
// the component type R; what differs between the formats (the GEMM kernel, the conversion of an initial
// state, the register-resident chains of 256 x 256 float matrices) comes in through the Ops parameter.
#pragma once
#include <cmath>

#include "goom_chain_kernel.h"

namespace goom_large {

using goom_chain::Comp;
using goom_chain::kLog2e;

template <typename R> struct Pair;
template <> struct Pair<float> { typedef float2 type; };
template <> struct Pair<double> { typedef double2 type; };

__device__ inline float vmaxr(float a, float b) { return fmaxf(a, b); }
__device__ inline double vmaxr(double a, double b) { return fmax(a, b); }

template <typename R> __device__ inline R signed_scaled(R re, R im, R shift)
{
    return Comp<R>::apply_sign(Comp<R>::exp2_shifted(re, shift), im);
}

inline int pad_to(int v, int a) { return (v + a - 1) / a * a; }

struct ChainGeom {
    long long T, L;           // chain length, chunk length
    long long chunks;         // chunks per batch item the launch covers (chain = item * chunks + chunk)
    int d, dp;                // matrix size, padded to 128
};

// rows of M[b][chunk * L + s], scaled; a chain whose chunk has fewer than s + 1 steps gets the identity.
// One wave per row (a row is at most 1024 entries: 16 per lane), four rows per workgroup:
// grid (dp / 4, chains), 256 threads.
template <typename R>
__global__ __launch_bounds__(256) void chain_convert_left_kernel(const typename Pair<R>::type *__restrict__ M, R *__restrict__ X,
                                                                 double *__restrict__ shifts, ChainGeom q, long long s)
{
    typedef typename Pair<R>::type R2;
    const R kNegInf = Comp<R>::neg_inf();
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    const long long chain = blockIdx.y, item = chain / q.chunks, chunk = chain % q.chunks;
    const long long t = chunk * q.L + s;
    const bool active = s < q.L && t < q.T;
    R *xrow = X + ((size_t)chain * q.dp + row) * q.dp;
    if (!active || row >= q.d) {
        for (int j = lane; j < q.dp; j += 64) xrow[j] = (!active && j == row && row < q.d) ? (R)1 : (R)0;
        if (lane == 0) shifts[(size_t)chain * q.dp + row] = 0.0;
        return;
    }
    const R2 *arow = M + (((size_t)item * q.T + t) * q.d + row) * q.d;
    R2 e[16];
    R mx = kNegInf;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int j = lane + 64 * r;
        e[r].x = kNegInf;
        e[r].y = (R)0;
        if (j < q.d) e[r] = arow[j];
        mx = vmaxr(mx, e[r].x);
    }
#pragma unroll
    for (int sft = 32; sft >= 1; sft >>= 1) mx = vmaxr(mx, (R)__shfl_xor(mx, sft, 64));
    const bool zero_row = !(mx > kNegInf);
    const R sh = zero_row ? (R)0 : Comp<R>::ceil_(mx * (R)kLog2e);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int j = lane + 64 * r;
        if (j < q.dp) xrow[j] = (j < q.d && !zero_row) ? signed_scaled<R>(e[r].x, e[r].y, sh) : (R)0;
    }
    if (lane == 0) shifts[(size_t)chain * q.dp + row] = (double)sh;
}

// Row n of the product (state column n): out[n][i] = in[n][i] 2^(shift_i - s_n) with s_n the largest
// exponent of in[n][i] 2^shift_i, and the column's exponent grows by s_n.  shifts: [.][len] doubles with
// stride shift_stride per chain (0: the same vector for all), or NULL for none.  One wave per row
// (len <= 1024), four rows per workgroup: grid (rows / 4, chains), 256 threads; in and out may be the
// same buffer.
template <typename R>
__global__ __launch_bounds__(256) void rescale_rows_kernel(const R *in, R *out, const double *__restrict__ shifts, long long shift_stride,
                                                           double *__restrict__ expo, int rows_padded, int len)
{
    const int lane = threadIdx.x & 63;
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
    const long long chain = blockIdx.y;
    const R *src = in + ((size_t)chain * rows_padded + n) * len;
    R *dst = out + ((size_t)chain * rows_padded + n) * len;
    const double *sh = shifts ? shifts + (size_t)chain * shift_stride : nullptr;
    // shifts relative to their largest, so that they fit the component type next to the entries' exponents
    double smax = sh ? -1.0e300 : 0.0;
    if (sh)
        for (int i = lane; i < len; i += 64) smax = fmax(smax, sh[i]);
#pragma unroll
    for (int sft = 32; sft >= 1; sft >>= 1) smax = fmax(smax, __shfl_xor(smax, sft, 64));
    R v[16], rel[16];
    R mx = (R)-1.0e30;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int i = lane + 64 * r;
        v[r] = (R)0;
        rel[r] = (R)0;
        if (i < len) {
            v[r] = src[i];
            const double dr = sh ? sh[i] - smax : 0.0;
            rel[r] = dr > -4000.0 ? (R)dr : (R)-4000.0;
            if (v[r] != (R)0) mx = vmaxr(mx, Comp<R>::exponent_of(v[r]) + rel[r]);
        }
    }
#pragma unroll
    for (int sft = 32; sft >= 1; sft >>= 1) mx = vmaxr(mx, (R)__shfl_xor(mx, sft, 64));
    const bool all_zero = !(mx > (R)-1.0e29);
    const R sn = all_zero ? (R)0 : mx;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int i = lane + 64 * r;
        if (i < len) dst[i] = Comp<R>::ldexp_(v[r], (int)Comp<R>::clamp_shift(rel[r] - sn));
    }
    if (lane == 0) {
        double &e = expo[(size_t)chain * rows_padded + n];
        e = all_zero ? 0.0 : e + smax + (double)sn;
    }
}

// The carry phase's pass between two products: from the raw product in[n][i] (state column n, exponent
// ein[n]) it writes (B) the state itself, rows normalised, where the scan wants it kept, and / or (A) the
// state with the exponents of the next left factor's columns folded onto its rows (shifts[i]), ready to be
// multiplied.  One wave per row, four rows per workgroup: grid (rows / 4, batch), 256 threads.
template <typename R> struct CarryPass {
    const R *in; const double *ein; long long in_stride, ein_stride;
    R *outA; double *eA; long long outA_stride, eA_stride; const double *shifts; long long shift_stride;
    R *outB; double *eB; long long outB_stride, eB_stride;
    int rows_padded, len;
};
template <typename R> __global__ __launch_bounds__(256) void carry_pass_kernel(CarryPass<R> p)
{
    const int lane = threadIdx.x & 63;
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
    const long long b = blockIdx.y;
    const R *src = p.in + b * p.in_stride + (size_t)n * p.len;
    const double e0 = p.ein[b * p.ein_stride + n];
    R v[16];
    R mxB = (R)-1.0e30;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int i = lane + 64 * r;
        v[r] = i < p.len ? src[i] : (R)0;
        if (v[r] != (R)0) mxB = vmaxr(mxB, Comp<R>::exponent_of(v[r]));
    }
#pragma unroll
    for (int sft = 32; sft >= 1; sft >>= 1) mxB = vmaxr(mxB, (R)__shfl_xor(mxB, sft, 64));
    const bool all_zero = !(mxB > (R)-1.0e29);
    if (p.outB) {
        R *dst = p.outB + b * p.outB_stride + (size_t)n * p.len;
        const int sh = all_zero ? 0 : -(int)mxB;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int i = lane + 64 * r;
            if (i < p.len) dst[i] = Comp<R>::ldexp_(v[r], sh);
        }
        if (lane == 0) p.eB[b * p.eB_stride + n] = all_zero ? 0.0 : e0 + (double)mxB;
    }
    if (p.outA) {
        const double *sh = p.shifts + b * p.shift_stride;
        double smax = -1.0e300;
        for (int i = lane; i < p.len; i += 64) smax = fmax(smax, sh[i]);
#pragma unroll
        for (int sft = 32; sft >= 1; sft >>= 1) smax = fmax(smax, __shfl_xor(smax, sft, 64));
        R rel[16];
        R mxA = (R)-1.0e30;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int i = lane + 64 * r;
            rel[r] = (R)0;
            if (i < p.len) {
                const double dr = sh[i] - smax;
                rel[r] = dr > -4000.0 ? (R)dr : (R)-4000.0;
                if (v[r] != (R)0) mxA = vmaxr(mxA, Comp<R>::exponent_of(v[r]) + rel[r]);
            }
        }
#pragma unroll
        for (int sft = 32; sft >= 1; sft >>= 1) mxA = vmaxr(mxA, (R)__shfl_xor(mxA, sft, 64));
        const bool zeroA = !(mxA > (R)-1.0e29);
        const R sn = zeroA ? (R)0 : mxA;
        R *dst = p.outA + b * p.outA_stride + (size_t)n * p.len;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int i = lane + 64 * r;
            if (i < p.len) dst[i] = Comp<R>::ldexp_(v[r], (int)Comp<R>::clamp_shift(rel[r] - sn));
        }
        if (lane == 0) p.eA[b * p.eA_stride + n] = zeroA ? 0.0 : e0 + smax + (double)sn;
    }
}

// St = identity (first d rows and columns), exponents 0.  grid (rows_padded, chains), 256 threads.
template <typename R> __global__ __launch_bounds__(256) void state_identity_kernel(R *St, double *expo, int rows_padded, int len, int d)
{
    const int n = blockIdx.x;
    const long long chain = blockIdx.y;
    R *row = St + ((size_t)chain * rows_padded + n) * len;
    for (int i = threadIdx.x; i < len; i += 256) row[i] = (i == n && n < d) ? (R)1 : (R)0;
    if (threadIdx.x == 0) expo[(size_t)chain * rows_padded + n] = 0.0;
}

// out[b][j][i] = in[b][i][j], square dp x dp.  grid (dp / 32, dp / 32, batch), block 32 x 8.
template <typename R>
__global__ __launch_bounds__(256) void transpose_kernel(const R *__restrict__ in, long long in_stride, R *__restrict__ out, long long out_stride, int dp)
{
    __shared__ R tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int i0 = blockIdx.x * 32, j0 = blockIdx.y * 32;
    const long long b = blockIdx.z;
#pragma unroll
    for (int r = 0; r < 4; ++r) tile[ty + 8 * r][tx] = in[b * in_stride + (size_t)(i0 + ty + 8 * r) * dp + j0 + tx];
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 4; ++r) out[b * out_stride + (size_t)(j0 + ty + 8 * r) * dp + i0 + tx] = tile[tx][ty + 8 * r];
}

// P[b][t][i][n] = GOOM of St[chain][n][i] 2^(expo[chain][n]), t = chunk * L + s (or slot `fixed_slot`
// of a [b][slots] array when fixed_slot >= 0); chains without that step store nothing.
// grid (ceil(d / 32), ceil(m / 32), chains), block 32 x 8.
template <typename R>
__global__ __launch_bounds__(256) void chain_store_kernel(const R *__restrict__ St, const double *__restrict__ expo,
                                                          typename Pair<R>::type *__restrict__ P, ChainGeom q, long long s, int m, int rows_padded,
                                                          long long slots, long long fixed_slot)
{
    __shared__ R tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int i0 = blockIdx.x * 32, n0 = blockIdx.y * 32;
    const long long chain = blockIdx.z, item = chain / q.chunks, chunk = chain % q.chunks;
    const long long t = chunk * q.L + s;
    if (fixed_slot < 0 && !(s < q.L && t < q.T)) return;
    const long long slot = fixed_slot >= 0 ? fixed_slot : t;
#pragma unroll
    for (int r = 0; r < 4; ++r) tile[ty + 8 * r][tx] = St[((size_t)chain * rows_padded + n0 + ty + 8 * r) * q.dp + i0 + tx]; // [n][i]
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int i = i0 + ty + 8 * r, n = n0 + tx;
        if (i < q.d && n < m) {
            const R x = tile[tx][ty + 8 * r];
            typename Pair<R>::type o;
            o.x = x != (R)0 ? Comp<R>::out_re(x, (R)0, expo[(size_t)chain * rows_padded + n]) : Comp<R>::neg_inf();
            o.y = x < (R)0 ? Comp<R>::pi() : (R)0;
            P[(((size_t)item * slots + slot) * q.d + i) * m + n] = o;
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Scan / reduction driver: the three phases of the chunked scan, every phase advancing all of its
// chains by one step per round of launches.
// ------------------------------------------------------------------------------------------------
struct LargePlan {
    long long L, C, C1; // chunk length, chunks per item, chunks whose products phase 1 forms
    int dp, mp;
    size_t off_atil, off_na, off_s1, off_e1, off_s3, off_e3, off_cbuf, off_yt, off_ey, off_trow, off_nrow, off_x2, off_ey2, total;
    bool resident; // 128 < d <= 256 and m <= 256, float components: the chains run with register-resident states
};

// cb: bytes per component; may_be_resident: the format has the register-resident kernel
inline LargePlan plan_large(long long T, int d, int m, long long batch, long long requested, bool final_only, size_t cb, bool may_be_resident)
{
    LargePlan p;
    p.dp = pad_to(d, 128);
    p.mp = pad_to(m, 128);
    const long long tiles = (long long)(p.dp / 128) * (p.dp / 128);
    const size_t per_chain = ((size_t)4 * p.dp * p.dp + (size_t)2 * p.mp * p.dp) * cb;
    long long c;
    if (requested > 0) {
        c = (T + requested - 1) / requested;
    } else {
        const long long c_par = (512 + batch * tiles - 1) / (batch * tiles); // enough tiles to fill the chip
        const long long c_depth = (long long)std::ceil(std::sqrt(2.0 * (double)T));
        c = c_par < c_depth ? c_par : c_depth;
        const long long c_mem = (long long)((size_t)8 << 30) / (long long)(per_chain * (size_t)batch);
        if (c > c_mem) c = c_mem;
    }
    if (c < 1) c = 1;
    p.L = (T + c - 1) / c;
    p.C = (T + p.L - 1) / p.L;
    p.C1 = p.C <= 1 ? 0 : (final_only ? p.C : p.C - 1);
    const size_t chains = (size_t)batch * p.C;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += goom::align_up(bytes, 256); return o; };
    p.off_atil = take(chains * p.dp * p.dp * cb);
    p.off_na = take(chains * p.dp * 8);
    p.off_s1 = take((size_t)batch * p.C1 * p.dp * p.dp * cb);
    p.off_e1 = take((size_t)batch * p.C1 * p.dp * 8);
    p.off_s3 = take(final_only ? 0 : chains * p.mp * p.dp * cb);
    p.off_e3 = take(final_only ? 0 : chains * p.mp * 8);
    p.off_cbuf = take(chains * (size_t)(p.mp > p.dp ? p.mp : p.dp) * p.dp * cb);
    p.off_yt = take((size_t)batch * p.mp * p.dp * cb);
    p.off_ey = take((size_t)batch * p.mp * 8);
    p.off_trow = take((size_t)batch * (p.C1 > 0 ? p.C1 : 1) * p.dp * p.dp * cb); // chunk products, transposed back
    p.off_x2 = take((size_t)batch * p.mp * p.dp * cb); // carry phase: the operand of the next product and its exponents
    p.off_ey2 = take((size_t)batch * p.mp * 8);
    p.resident = may_be_resident && p.dp == 256 && p.mp <= 256;
    p.off_nrow = take(p.resident ? (size_t)batch * T * 256 * 4 : 0);
    p.total = off;
    return p;
}

// Ops supplies, for the component type R:
//   static constexpr bool kResident;
//   static int prepare(goom_ctx *);                                     once per call, before any launch
//   static void gemm(hipStream_t, const R *X, const R *Y, R *C, unsigned gx, unsigned gy, unsigned gz, int M, int N, int K,
//                    long long sx, long long sy, long long sc);         C[b] = X[b] Y[b]^T, 128 x 128 tiles
//   static void init_state(hipStream_t, const void *init, double *ey, R *yt, int d, int m, int mp, int dp, unsigned batch);
//   static int row_shifts(...), chains(...);                            the register-resident kernels (kResident only)
template <typename R, typename Ops>
int run_scan_large_t(goom_ctx *ctx, const void *M, const void *init, void *P, long long T, int d, int m, long long batch,
                     long long requested_chunk, void *ws, bool final_only)
{
    using goom::check_hip;
    using goom::fail;
    using goom::prof_begin;
    using goom::prof_end;
    typedef typename Pair<R>::type R2;
    const LargePlan p = plan_large(T, d, m, batch, requested_chunk, final_only, sizeof(R), Ops::kResident);
    const long long chains_all = batch * p.C;
    if (chains_all > 65535) return fail(ctx, GOOM_EUNSUPPORTED, "too many chains (%lld) for matrices above %d", chains_all, GOOM_MAX_DIM);
    if (int e = Ops::prepare(ctx)) return e;
    unsigned char *w = static_cast<unsigned char *>(ws);
    R *atil = reinterpret_cast<R *>(w + p.off_atil);
    double *na = reinterpret_cast<double *>(w + p.off_na);
    R *s1 = reinterpret_cast<R *>(w + p.off_s1);
    double *e1 = reinterpret_cast<double *>(w + p.off_e1);
    R *s3 = reinterpret_cast<R *>(w + p.off_s3);
    double *e3 = reinterpret_cast<double *>(w + p.off_e3);
    R *cbuf = reinterpret_cast<R *>(w + p.off_cbuf);
    R *yt = reinterpret_cast<R *>(w + p.off_yt);
    double *ey = reinterpret_cast<double *>(w + p.off_ey);
    R *trow = reinterpret_cast<R *>(w + p.off_trow);
    R *cbuf2 = reinterpret_cast<R *>(w + p.off_x2);
    double *ey2 = reinterpret_cast<double *>(w + p.off_ey2);
    const R2 *Mg = static_cast<const R2 *>(M);
    const int dp = p.dp, mp = p.mp;
    hipStream_t st = ctx->stream;
    auto ok = [&](const char *what) { return check_hip(ctx, hipGetLastError(), what); };

    // one step of all chains of a launch: state[chain] (rows x dp) <- state A~^T, rescaled
    auto advance = [&](R *state, double *expo, int rows, const ChainGeom &q, long long chains, long long s) {
        hipLaunchKernelGGL(chain_convert_left_kernel<R>, dim3(dp / 4, (unsigned)chains), dim3(256), 0, st, Mg, atil, na, q, s);
        Ops::gemm(st, state, atil, cbuf, dp / 128, rows / 128, (unsigned)chains, rows, dp, dp, (long long)rows * dp, (long long)dp * dp,
                  (long long)rows * dp);
        hipLaunchKernelGGL(rescale_rows_kernel<R>, dim3(rows / 4, (unsigned)chains), dim3(256), 0, st, cbuf, state, na, (long long)dp, expo, rows, dp);
    };

    float *nrow = reinterpret_cast<float *>(w + p.off_nrow);
    if constexpr (Ops::kResident) {
        if (p.resident) {
            prof_begin(ctx, "scan_large_row_shifts");
            const int e = Ops::row_shifts(ctx, M, nrow, d, batch * T);
            prof_end(ctx);
            if (e) return e;
        }
    }

    // ---- phase 1: chunk products
    if (p.C1 > 0) {
        ChainGeom q{T, p.L, p.C1, d, dp};
        const long long chains = batch * p.C1;
        prof_begin(ctx, "scan_large_phase1_chunk_products");
        bool done = false;
        if constexpr (Ops::kResident) {
            if (p.resident) {
                if (int e = Ops::chains(ctx, M, nrow, T, p.L, p.C1, batch, d, d, nullptr, nullptr, s1, e1, nullptr)) return e;
                done = true;
            }
        }
        if (!done) {
            hipLaunchKernelGGL(state_identity_kernel<R>, dim3(dp, (unsigned)chains), dim3(256), 0, st, s1, e1, dp, dp, d);
            for (long long s = 0; s < p.L; ++s) advance(s1, e1, dp, q, chains, s);
        }
        prof_end(ctx);
        if (int e = ok("scan_large phase 1")) return e;
    }

    // ---- phase 2: prefixes at the chunk boundaries (and, for a reduction, the final product)
    prof_begin(ctx, "scan_large_phase2_carries");
    if (init)
        Ops::init_state(st, init, ey, yt, d, m, mp, dp, (unsigned)batch);
    else
        hipLaunchKernelGGL(state_identity_kernel<R>, dim3(mp, (unsigned)batch), dim3(256), 0, st, yt, ey, mp, dp, d);
    // Y <- T_c Y for c = 0, 1, ...: the exponents of T_c's columns go onto Y's rows, T_c (held transposed, as a
    // state) is turned K-contiguous again; two launches per chunk.  The scan keeps every Y (the carry into chunk c).
    if (p.C1 > 0)
        hipLaunchKernelGGL(transpose_kernel<R>, dim3(dp / 32, dp / 32, (unsigned)(batch * p.C1)), dim3(256), 0, st, s1, (long long)dp * dp, trow,
                           (long long)dp * dp, dp);
    auto pass = [&](const R *in, const double *ein, long long c_next) {
        // from `in`: the carry into chunk c_next (kept, for a scan) and the operand of the product with T_c_next
        CarryPass<R> cp;
        cp.in = in; cp.ein = ein; cp.in_stride = (long long)mp * dp; cp.ein_stride = (long long)mp;
        const bool more = c_next < p.C1;
        cp.outA = more ? cbuf2 : nullptr; cp.eA = ey2; cp.outA_stride = (long long)mp * dp; cp.eA_stride = (long long)mp;
        cp.shifts = more ? e1 + (size_t)c_next * dp : nullptr; cp.shift_stride = (long long)p.C1 * dp;
        const bool keep = !final_only;
        cp.outB = keep ? s3 + (size_t)c_next * mp * dp : (more ? nullptr : yt);
        cp.eB = keep ? e3 + (size_t)c_next * mp : ey;
        cp.outB_stride = keep ? (long long)p.C * mp * dp : (long long)mp * dp;
        cp.eB_stride = keep ? (long long)p.C * mp : (long long)mp;
        cp.rows_padded = mp; cp.len = dp;
        if (cp.outA || cp.outB) hipLaunchKernelGGL(carry_pass_kernel<R>, dim3(mp / 4, (unsigned)batch), dim3(256), 0, st, cp);
    };
    pass(yt, ey, 0);
    for (long long c = 0; c < p.C1; ++c) {
        Ops::gemm(st, cbuf2, trow + (size_t)c * dp * dp, cbuf, dp / 128, mp / 128, (unsigned)batch, mp, dp, dp, (long long)mp * dp,
                  (long long)p.C1 * dp * dp, (long long)mp * dp);
        pass(cbuf, ey2, c + 1);
    }
    if (final_only && p.C1 > 0) {
        ChainGeom q{T, p.L, 1, d, dp};
        hipLaunchKernelGGL(chain_store_kernel<R>, dim3((d + 31) / 32, (m + 31) / 32, (unsigned)batch), dim3(256), 0, st, yt, ey, static_cast<R2 *>(P), q,
                           0LL, m, mp, 1LL, 0LL);
    }
    prof_end(ctx);
    if (int e = ok("scan_large phase 2")) return e;
    if (final_only && p.C1 > 0) return GOOM_OK;

    // ---- phase 3: every chunk from its incoming prefix, all prefixes stored (a single chunk runs only this)
    {
        ChainGeom q{T, p.L, p.C, d, dp};
        R *state = final_only ? yt : s3; // a reduction of a single chunk walks it here
        double *expo = final_only ? ey : e3;
        prof_begin(ctx, final_only ? "scan_large_single_chunk" : "scan_large_phase3_outputs");
        bool done = false;
        if constexpr (Ops::kResident) {
            if (p.resident) {
                // (a reduction of a single chunk leaves its product in the state, stored below)
                const int e = final_only ? Ops::chains(ctx, M, nrow, T, p.L, p.C, batch, d, m, state, expo, state, expo, nullptr)
                                         : Ops::chains(ctx, M, nrow, T, p.L, p.C, batch, d, m, state, expo, nullptr, nullptr, P);
                if (e) return e;
                done = true;
            }
        }
        for (long long s = 0; s < (done ? 0 : p.L); ++s) {
            advance(state, expo, mp, q, chains_all, s);
            if (!final_only)
                hipLaunchKernelGGL(chain_store_kernel<R>, dim3((d + 31) / 32, (m + 31) / 32, (unsigned)chains_all), dim3(256), 0, st, state, expo,
                                   static_cast<R2 *>(P), q, s, m, mp, T, -1LL);
        }
        if (final_only) {
            ChainGeom q1{T, p.L, 1, d, dp};
            hipLaunchKernelGGL(chain_store_kernel<R>, dim3((d + 31) / 32, (m + 31) / 32, (unsigned)batch), dim3(256), 0, st, state, expo,
                               static_cast<R2 *>(P), q1, 0LL, m, mp, 1LL, 0LL);
        }
        prof_end(ctx);
    }
    return ok("scan_large phase 3");
}

} // namespace goom_large
