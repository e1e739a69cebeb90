// LMME for shapes beyond the register-resident kernels (any of n, d, m above 128, up to 1024; float
// components): the same scaled real product (paper Section 3.2, eqs. 7-9; shifts by eq. 10), but as
// separate passes, because a d x d state no longer fits one workgroup and the product is a large
// dense GEMM that dominates everything else:
//   1. rows of A' -> reals scaled by the row's power of two (K-contiguous, zero padded);
//   2. columns of B' -> reals scaled by the column's power of two, written TRANSPOSED, so that
//      both GEMM operands are K-contiguous;
//   3. C~^T = B~^T A~^T on the matrix unit: an "NT" GEMM, 128 x 128 tile per workgroup,
//      64 x 64 per wave, K in steps of 16 through double-buffered LDS;
//   4. signed logarithm, shifts re-added, transposed back on the way out.
// All intermediates live in the caller's workspace, padded to the tile sizes, so the GEMM has no
// edge cases.
#include <cmath>

#include "goom_chain_kernel.h"

namespace {

using goom_chain::Comp;
using goom_chain::f4;
typedef Comp<float> CF;

constexpr float kLog2eF = 1.44269504088896340736f;

__device__ inline float signed_scaled(float re, float im, float shift)
{
    return CF::apply_sign(CF::exp2_shifted(re, shift), im);
}

// ---- 1. rows of the left operand.  grid (rows_padded, batch), 256 threads.
__global__ __launch_bounds__(256) void convert_left_kernel(const float2 *__restrict__ A, float *__restrict__ X, float *__restrict__ shifts,
                                                           int n, int d, int rows_padded, int k_padded)
{
    __shared__ float red[4];
    const int row = blockIdx.x;
    const long long b = blockIdx.y;
    const int tid = threadIdx.x;
    float *xrow = X + ((size_t)b * rows_padded + row) * k_padded;
    if (row >= n) { // padding rows
        for (int j = tid; j < k_padded; j += 256) xrow[j] = 0.0f;
        if (tid == 0) shifts[(size_t)b * rows_padded + row] = 0.0f;
        return;
    }
    const float2 *arow = A + ((size_t)b * n + row) * d;
    float mx = -__builtin_huge_valf();
    for (int j = tid; j < d; j += 256) mx = fmaxf(mx, arow[j].x);
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) mx = fmaxf(mx, __shfl_xor(mx, s, 64));
    if ((tid & 63) == 0) red[tid >> 6] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    const bool zero_row = !(mx > -__builtin_huge_valf());
    const float sh = zero_row ? 0.0f : ceilf(mx * kLog2eF);
    for (int j = tid; j < k_padded; j += 256) {
        float v = 0.0f;
        if (j < d && !zero_row) {
            const float2 e = arow[j];
            v = signed_scaled(e.x, e.y, sh);
        }
        xrow[j] = v;
    }
    if (tid == 0) shifts[(size_t)b * rows_padded + row] = sh;
}

// ---- 2a. column maxima of the right operand.  grid (ceil(m / 64), batch), block 64 x 4.
template <typename S>
__global__ __launch_bounds__(256) void column_shift_kernel(const float2 *__restrict__ B, S *__restrict__ shifts, int d, int m, int cols_padded)
{
    __shared__ float red[4][64];
    const int cx = threadIdx.x & 63, ry = threadIdx.x >> 6;
    const int col = blockIdx.x * 64 + cx;
    const long long b = blockIdx.y;
    float mx = -__builtin_huge_valf();
    if (col < m) {
        // eight independent loads in flight per thread: the loop is bound by memory latency otherwise
        float part[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) part[u] = -__builtin_huge_valf();
        const float2 *base = B + (size_t)b * d * m + col;
        int j = ry;
        for (; j + 28 < d; j += 32) {
#pragma unroll
            for (int u = 0; u < 8; ++u) part[u] = fmaxf(part[u], base[(size_t)(j + 4 * u) * m].x);
        }
        for (; j < d; j += 4) part[0] = fmaxf(part[0], base[(size_t)j * m].x);
#pragma unroll
        for (int u = 0; u < 8; ++u) mx = fmaxf(mx, part[u]);
    }
    red[ry][cx] = mx;
    __syncthreads();
    if (ry == 0 && col < cols_padded) {
        mx = fmaxf(fmaxf(red[0][cx], red[1][cx]), fmaxf(red[2][cx], red[3][cx]));
        shifts[(size_t)b * cols_padded + col] = (col < m && mx > -__builtin_huge_valf()) ? (S)ceilf(mx * kLog2eF) : (S)0;
    }
}

// ---- 2b. right operand scaled and transposed: Y[b][col][j] = (+-) 2^(log2|B_j,col| - shift_col).
// grid (cols_padded / 32, k_padded / 32 rounded up, batch), block 32 x 8.
template <typename S>
__global__ __launch_bounds__(256) void convert_right_kernel(const float2 *__restrict__ B, const S *__restrict__ shifts, float *__restrict__ Y,
                                                            int d, int m, int cols_padded, int k_padded)
{
    __shared__ float tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int c0 = blockIdx.x * 32, j0 = blockIdx.y * 32;
    const long long b = blockIdx.z;
    const int col = c0 + tx;
    const float sh = col < cols_padded ? (float)shifts[(size_t)b * cols_padded + col] : 0.0f;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int j = j0 + ty + 8 * r;
        float v = 0.0f;
        if (j < d && col < m) {
            const float2 e = B[((size_t)b * d + j) * m + col];
            v = signed_scaled(e.x, e.y, sh);
        }
        tile[ty + 8 * r][tx] = v; // [j][col]
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int cc = c0 + ty + 8 * r, j = j0 + tx;
        if (cc < cols_padded && j < k_padded) Y[((size_t)b * cols_padded + cc) * k_padded + j] = tile[tx][ty + 8 * r];
    }
}

// ---- 3. C[b][M][N] = X[b][M][K] Y[b][N][K]^T, all row-major; M, N multiples of 128, K of 16.
// grid (N / 128, M / 128, batch), 256 threads = 2 x 2 waves of 64 x 64.
constexpr int BM = 128, BN = 128, BK = 16, LDK = BK + 4;

__global__ __launch_bounds__(256, 2) void gemm_nt_kernel(const float *__restrict__ X, const float *__restrict__ Y, float *__restrict__ Cout, int M,
                                                          int N, int K, long long sx, long long sy, long long sc)
{
    __shared__ __align__(16) float xs[2][BM * LDK];
    __shared__ __align__(16) float ys[2][BN * LDK];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 4, c = lane & 15;
    const int wm = wave >> 1, wn = wave & 1;
    // Workgroups are handed to the eight XCDs in turn, each with its own L2: renumber them so that one
    // XCD works on a contiguous range of tiles, whose operand panels it then shares in its L2.
    const unsigned tiles_x = gridDim.x, tiles_y = gridDim.y;
    const unsigned long long nwg = (unsigned long long)tiles_x * tiles_y * gridDim.z;
    unsigned long long lin = ((unsigned long long)blockIdx.z * tiles_y + blockIdx.y) * tiles_x + blockIdx.x;
    if (nwg % 8 == 0) lin = (lin % 8) * (nwg / 8) + lin / 8;
    const unsigned bx = (unsigned)(lin % tiles_x), by = (unsigned)((lin / tiles_x) % tiles_y);
    const long long b = (long long)(lin / ((unsigned long long)tiles_x * tiles_y));
    const float *Xb = X + b * sx + (size_t)by * BM * K;
    const float *Yb = Y + b * sy + (size_t)bx * BN * K;
    // global -> registers: the 128 x 16 tile is 512 pieces of four floats; a thread takes two
    const int r0 = tid >> 2, r1 = r0 + 64, kq = (tid & 3) * 4;
    f4 xr0, xr1, yr0, yr1;
    auto load_tiles = [&](int k0) {
        xr0 = *reinterpret_cast<const f4 *>(Xb + (size_t)r0 * K + k0 + kq);
        xr1 = *reinterpret_cast<const f4 *>(Xb + (size_t)r1 * K + k0 + kq);
        yr0 = *reinterpret_cast<const f4 *>(Yb + (size_t)r0 * K + k0 + kq);
        yr1 = *reinterpret_cast<const f4 *>(Yb + (size_t)r1 * K + k0 + kq);
    };
    auto store_tiles = [&](int buf) {
        *reinterpret_cast<f4 *>(&xs[buf][r0 * LDK + kq]) = xr0;
        *reinterpret_cast<f4 *>(&xs[buf][r1 * LDK + kq]) = xr1;
        *reinterpret_cast<f4 *>(&ys[buf][r0 * LDK + kq]) = yr0;
        *reinterpret_cast<f4 *>(&ys[buf][r1 * LDK + kq]) = yr1;
    };
    f4 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = f4{0.f, 0.f, 0.f, 0.f};
    const int nk = K / BK;
    load_tiles(0);
    store_tiles(0);
    __syncthreads();
    int buf = 0;
    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk) load_tiles((kt + 1) * BK);
        f4 av[4], bv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            av[i] = *reinterpret_cast<const f4 *>(&xs[buf][(wm * 64 + 16 * i + c) * LDK + 4 * g]);
            bv[i] = *reinterpret_cast<const f4 *>(&ys[buf][(wn * 64 + 16 * i + c) * LDK + 4 * g]);
        }
#pragma unroll
        for (int v = 0; v < 4; ++v)
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = CF::mfma(av[i][v], bv[j][v], acc[i][j]);
        if (kt + 1 < nk) store_tiles(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }
    float *Cb = Cout + b * sc + ((size_t)by * BM + wm * 64) * N + (size_t)bx * BN + wn * 64;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) Cb[(size_t)(16 * i + 4 * g + v) * N + 16 * j + c] = acc[i][j][v];
}

// ---- 4. C'[b][i][k] = GOOM of Ct[b][k][i] 2^(row_shift_i + col_shift_k).
// grid (ceil(n / 32), ceil(m / 32), batch), block 32 x 8.
__global__ __launch_bounds__(256) void lmme_store_kernel(const float *__restrict__ Ct, const float *__restrict__ row_shift,
                                                         const float *__restrict__ col_shift, float2 *__restrict__ Cg, int n, int m,
                                                         int rows_padded, int cols_padded)
{
    __shared__ float tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int i0 = blockIdx.x * 32, k0 = blockIdx.y * 32;
    const long long b = blockIdx.z;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int k = k0 + ty + 8 * r, i = i0 + tx; // k < cols_padded and i < rows_padded always (multiples of 128)
        tile[ty + 8 * r][tx] = Ct[((size_t)b * cols_padded + k) * rows_padded + i];
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int i = i0 + ty + 8 * r, k = k0 + tx;
        if (i < n && k < m) {
            const float x = tile[tx][ty + 8 * r];
            const float s = row_shift[(size_t)b * rows_padded + i] + col_shift[(size_t)b * cols_padded + k];
            float2 o;
            o.x = x != 0.0f ? CF::out_re_f(x, s) : -__builtin_huge_valf();
            o.y = x < 0.0f ? CF::pi() : 0.0f;
            Cg[((size_t)b * n + i) * m + k] = o;
        }
    }
}


// =====================================================================================
// Scans of matrices above 128 x 128 (paper Section 4.1 runs chains up to 1024 x 1024).  The running
// product of a chain is kept TRANSPOSED, St[column of the state][row], as float mantissas with one
// power-of-two exponent per state column (double), so that one step,
//     St <- St A~^T,  then every row of St rescaled (the row shifts of A~ folded in),
// is the same NT GEMM plus two light passes, and closes under iteration.  All chains of a launch
// (batch items x chunks) advance together, one step per round of launches.
// =====================================================================================

struct ChainGeom {
    long long T, L;           // chain length, chunk length
    long long chunks;         // chunks per batch item the launch covers (chain = item * chunks + chunk)
    int d, dp;                // matrix size, padded to 128
};

// rows of M[b][chunk * L + s], scaled; a chain whose chunk has fewer than s + 1 steps gets the identity.
// One wave per row (a row is at most 1024 entries: 16 per lane), four rows per workgroup:
// grid (dp / 4, chains), 256 threads.
__global__ __launch_bounds__(256) void chain_convert_left_kernel(const float2 *__restrict__ M, float *__restrict__ X, double *__restrict__ shifts,
                                                                 ChainGeom q, long long s)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    const long long chain = blockIdx.y, item = chain / q.chunks, chunk = chain % q.chunks;
    const long long t = chunk * q.L + s;
    const bool active = s < q.L && t < q.T;
    float *xrow = X + ((size_t)chain * q.dp + row) * q.dp;
    if (!active || row >= q.d) {
        for (int j = lane; j < q.dp; j += 64) xrow[j] = (!active && j == row && row < q.d) ? 1.0f : 0.0f;
        if (lane == 0) shifts[(size_t)chain * q.dp + row] = 0.0;
        return;
    }
    const float2 *arow = M + (((size_t)item * q.T + t) * q.d + row) * q.d;
    float2 e[16];
    float mx = -__builtin_huge_valf();
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int j = lane + 64 * r;
        e[r] = float2{-__builtin_huge_valf(), 0.0f};
        if (j < q.d) e[r] = arow[j];
        mx = fmaxf(mx, e[r].x);
    }
#pragma unroll
    for (int sft = 32; sft >= 1; sft >>= 1) mx = fmaxf(mx, __shfl_xor(mx, sft, 64));
    const bool zero_row = !(mx > -__builtin_huge_valf());
    const float sh = zero_row ? 0.0f : ceilf(mx * kLog2eF);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int j = lane + 64 * r;
        if (j < q.dp) xrow[j] = (j < q.d && !zero_row) ? signed_scaled(e[r].x, e[r].y, sh) : 0.0f;
    }
    if (lane == 0) shifts[(size_t)chain * q.dp + row] = (double)sh;
}

// Row n of the product (state column n): out[n][i] = in[n][i] 2^(shift_i - s_n) with s_n the largest
// exponent of in[n][i] 2^shift_i, and the column's exponent grows by s_n.  shifts: [.][len] doubles with
// stride shift_stride per chain (0: the same vector for all), or NULL for none.  One wave per row
// (len <= 1024), four rows per workgroup: grid (rows / 4, chains), 256 threads; in and out may be the
// same buffer.
__global__ __launch_bounds__(256) void rescale_rows_kernel(const float *in, float *out, const double *__restrict__ shifts, long long shift_stride,
                                                           double *__restrict__ expo, int rows_padded, int len)
{
    const int lane = threadIdx.x & 63;
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
    const long long chain = blockIdx.y;
    const float *src = in + ((size_t)chain * rows_padded + n) * len;
    float *dst = out + ((size_t)chain * rows_padded + n) * len;
    const double *sh = shifts ? shifts + (size_t)chain * shift_stride : nullptr;
    // shifts relative to their largest, so that they fit float arithmetic next to the entries' exponents
    double smax = sh ? -1.0e300 : 0.0;
    if (sh)
        for (int i = lane; i < len; i += 64) smax = fmax(smax, sh[i]);
#pragma unroll
    for (int sft = 32; sft >= 1; sft >>= 1) smax = fmax(smax, __shfl_xor(smax, sft, 64));
    float v[16], rel[16];
    float mx = -1.0e30f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int i = lane + 64 * r;
        v[r] = 0.0f;
        rel[r] = 0.0f;
        if (i < len) {
            v[r] = src[i];
            const double dr = sh ? sh[i] - smax : 0.0;
            rel[r] = dr > -4000.0 ? (float)dr : -4000.0f;
            if (v[r] != 0.0f) mx = fmaxf(mx, CF::exponent_of(v[r]) + rel[r]);
        }
    }
#pragma unroll
    for (int sft = 32; sft >= 1; sft >>= 1) mx = fmaxf(mx, __shfl_xor(mx, sft, 64));
    const bool all_zero = !(mx > -1.0e29f);
    const float sn = all_zero ? 0.0f : mx;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int i = lane + 64 * r;
        if (i < len) dst[i] = __builtin_ldexpf(v[r], (int)CF::clamp_shift(rel[r] - sn));
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
struct CarryPass {
    const float *in; const double *ein; long long in_stride, ein_stride;
    float *outA; double *eA; long long outA_stride, eA_stride; const double *shifts; long long shift_stride;
    float *outB; double *eB; long long outB_stride, eB_stride;
    int rows_padded, len;
};
__global__ __launch_bounds__(256) void carry_pass_kernel(CarryPass p)
{
    const int lane = threadIdx.x & 63;
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
    const long long b = blockIdx.y;
    const float *src = p.in + b * p.in_stride + (size_t)n * p.len;
    const double e0 = p.ein[b * p.ein_stride + n];
    float v[16];
    float mxB = -1.0e30f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int i = lane + 64 * r;
        v[r] = i < p.len ? src[i] : 0.0f;
        if (v[r] != 0.0f) mxB = fmaxf(mxB, CF::exponent_of(v[r]));
    }
#pragma unroll
    for (int sft = 32; sft >= 1; sft >>= 1) mxB = fmaxf(mxB, __shfl_xor(mxB, sft, 64));
    const bool all_zero = !(mxB > -1.0e29f);
    if (p.outB) {
        float *dst = p.outB + b * p.outB_stride + (size_t)n * p.len;
        const int sh = all_zero ? 0 : -(int)mxB;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int i = lane + 64 * r;
            if (i < p.len) dst[i] = __builtin_ldexpf(v[r], sh);
        }
        if (lane == 0) p.eB[b * p.eB_stride + n] = all_zero ? 0.0 : e0 + (double)mxB;
    }
    if (p.outA) {
        const double *sh = p.shifts + b * p.shift_stride;
        double smax = -1.0e300;
        for (int i = lane; i < p.len; i += 64) smax = fmax(smax, sh[i]);
#pragma unroll
        for (int sft = 32; sft >= 1; sft >>= 1) smax = fmax(smax, __shfl_xor(smax, sft, 64));
        float rel[16];
        float mxA = -1.0e30f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int i = lane + 64 * r;
            rel[r] = 0.0f;
            if (i < p.len) {
                const double dr = sh[i] - smax;
                rel[r] = dr > -4000.0 ? (float)dr : -4000.0f;
                if (v[r] != 0.0f) mxA = fmaxf(mxA, CF::exponent_of(v[r]) + rel[r]);
            }
        }
#pragma unroll
        for (int sft = 32; sft >= 1; sft >>= 1) mxA = fmaxf(mxA, __shfl_xor(mxA, sft, 64));
        const bool zeroA = !(mxA > -1.0e29f);
        const float sn = zeroA ? 0.0f : mxA;
        float *dst = p.outA + b * p.outA_stride + (size_t)n * p.len;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int i = lane + 64 * r;
            if (i < p.len) dst[i] = __builtin_ldexpf(v[r], (int)CF::clamp_shift(rel[r] - sn));
        }
        if (lane == 0) p.eA[b * p.eA_stride + n] = zeroA ? 0.0 : e0 + smax + (double)sn;
    }
}

// St = identity (first d rows and columns), exponents 0.  grid (rows_padded, chains), 256 threads.
__global__ __launch_bounds__(256) void state_identity_kernel(float *St, double *expo, int rows_padded, int len, int d)
{
    const int n = blockIdx.x;
    const long long chain = blockIdx.y;
    float *row = St + ((size_t)chain * rows_padded + n) * len;
    for (int i = threadIdx.x; i < len; i += 256) row[i] = (i == n && n < d) ? 1.0f : 0.0f;
    if (threadIdx.x == 0) expo[(size_t)chain * rows_padded + n] = 0.0;
}

// out[b][j][i] = in[b][i][j], square dp x dp.  grid (dp / 32, dp / 32, batch), block 32 x 8.
__global__ __launch_bounds__(256) void transpose_kernel(const float *__restrict__ in, long long in_stride, float *__restrict__ out, long long out_stride,
                                                        int dp)
{
    __shared__ float tile[32][33];
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
__global__ __launch_bounds__(256) void chain_store_kernel(const float *__restrict__ St, const double *__restrict__ expo, float2 *__restrict__ P,
                                                          ChainGeom q, long long s, int m, int rows_padded, long long slots, long long fixed_slot)
{
    __shared__ float tile[32][33];
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
            const float x = tile[tx][ty + 8 * r];
            float2 o;
            o.x = x != 0.0f ? CF::out_re((float)x, 0.0f, expo[(size_t)chain * rows_padded + n]) : -__builtin_huge_valf();
            o.y = x < 0.0f ? CF::pi() : 0.0f;
            P[(((size_t)item * slots + slot) * q.d + i) * m + n] = o;
        }
    }
}

inline int pad_to(int v, int a) { return (v + a - 1) / a * a; }

} // namespace

namespace goom {

// workspace: X [batch][Np][Kp], row shifts [batch][Np], Y [batch][Mp][Kp], column shifts [batch][Mp], Ct [batch][Mp][Np]
size_t lmme_large_workspace_bytes(long long batch, int n, int d, int m)
{
    const size_t Np = pad_to(n, 128), Mp = pad_to(m, 128), Kp = pad_to(d, 16);
    return align_up((size_t)batch * Np * Kp * 4, 256) + align_up((size_t)batch * Np * 4, 256) + align_up((size_t)batch * Mp * Kp * 4, 256) +
           align_up((size_t)batch * Mp * 4, 256) + align_up((size_t)batch * Mp * Np * 4, 256);
}

int launch_lmme_large(goom_ctx *ctx, const void *A, const void *B, void *C, long long batch, int n, int d, int m, void *ws)
{
    const int Np = pad_to(n, 128), Mp = pad_to(m, 128), Kp = pad_to(d, 16);
    if (batch > 65535) return fail(ctx, GOOM_EUNSUPPORTED, "at most 65535 pairs per call for shapes above 128 (batch=%lld)", batch);
    unsigned char *w = static_cast<unsigned char *>(ws);
    float *X = reinterpret_cast<float *>(w);
    w += align_up((size_t)batch * Np * Kp * 4, 256);
    float *rs = reinterpret_cast<float *>(w);
    w += align_up((size_t)batch * Np * 4, 256);
    float *Y = reinterpret_cast<float *>(w);
    w += align_up((size_t)batch * Mp * Kp * 4, 256);
    float *cs = reinterpret_cast<float *>(w);
    w += align_up((size_t)batch * Mp * 4, 256);
    float *Ct = reinterpret_cast<float *>(w);
    const unsigned nb = (unsigned)batch;
    prof_begin(ctx, "lmme_large_scale_operands");
    hipLaunchKernelGGL(convert_left_kernel, dim3(Np, nb), dim3(256), 0, ctx->stream, static_cast<const float2 *>(A), X, rs, n, d, Np, Kp);
    hipLaunchKernelGGL(column_shift_kernel<float>, dim3(Mp / 64, nb), dim3(256), 0, ctx->stream, static_cast<const float2 *>(B), cs, d, m, Mp);
    hipLaunchKernelGGL(convert_right_kernel<float>, dim3(Mp / 32, (Kp + 31) / 32, nb), dim3(256), 0, ctx->stream, static_cast<const float2 *>(B), cs, Y,
                       d, m, Mp, Kp);
    prof_end(ctx);
    if (int s = check_hip(ctx, hipGetLastError(), "launch LMME operand kernels")) return s;
    prof_begin(ctx, "lmme_large_gemm");
    hipLaunchKernelGGL(gemm_nt_kernel, dim3(Np / BN, Mp / BM, nb), dim3(256), 0, ctx->stream, Y, X, Ct, Mp, Np, Kp, (long long)Mp * Kp,
                       (long long)Np * Kp, (long long)Mp * Np);
    prof_end(ctx);
    if (int s = check_hip(ctx, hipGetLastError(), "launch gemm_nt_kernel")) return s;
    prof_begin(ctx, "lmme_large_log_store");
    hipLaunchKernelGGL(lmme_store_kernel, dim3((n + 31) / 32, (m + 31) / 32, nb), dim3(256), 0, ctx->stream, Ct, rs, cs,
                       static_cast<float2 *>(C), n, m, Np, Mp);
    prof_end(ctx);
    return check_hip(ctx, hipGetLastError(), "launch lmme_store_kernel");
}

} // namespace goom

// ------------------------------------------------------------------------------------------------
// Scan / reduction driver for matrices above 128 x 128: the three phases of the chunked scan, every
// phase advancing all of its chains by one step per round of launches.
// ------------------------------------------------------------------------------------------------
namespace {

struct LargePlan {
    long long L, C, C1; // chunk length, chunks per item, chunks whose products phase 1 forms
    int dp, mp;
    size_t off_atil, off_na, off_s1, off_e1, off_s3, off_e3, off_cbuf, off_yt, off_ey, off_trow, off_nrow, off_x2, off_ey2, total;
    bool resident; // 128 < d <= 256 and m <= 256: the chains run with register-resident states
};

LargePlan plan_large(long long T, int d, int m, long long batch, long long requested, bool final_only)
{
    LargePlan p;
    p.dp = pad_to(d, 128);
    p.mp = pad_to(m, 128);
    const long long tiles = (long long)(p.dp / 128) * (p.dp / 128);
    const size_t per_chain = ((size_t)4 * p.dp * p.dp + (size_t)2 * p.mp * p.dp) * 4;
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
    p.off_atil = take(chains * p.dp * p.dp * 4);
    p.off_na = take(chains * p.dp * 8);
    p.off_s1 = take((size_t)batch * p.C1 * p.dp * p.dp * 4);
    p.off_e1 = take((size_t)batch * p.C1 * p.dp * 8);
    p.off_s3 = take(final_only ? 0 : chains * p.mp * p.dp * 4);
    p.off_e3 = take(final_only ? 0 : chains * p.mp * 8);
    p.off_cbuf = take(chains * (size_t)(p.mp > p.dp ? p.mp : p.dp) * p.dp * 4);
    p.off_yt = take((size_t)batch * p.mp * p.dp * 4);
    p.off_ey = take((size_t)batch * p.mp * 8);
    p.off_trow = take((size_t)batch * (p.C1 > 0 ? p.C1 : 1) * p.dp * p.dp * 4); // chunk products, transposed back
    p.off_x2 = take((size_t)batch * p.mp * p.dp * 4); // carry phase: the operand of the next product and its exponents
    p.off_ey2 = take((size_t)batch * p.mp * 8);
    p.resident = p.dp == 256 && p.mp <= 256;
    p.off_nrow = take(p.resident ? (size_t)batch * T * 256 * 4 : 0);
    p.total = off;
    return p;
}

} // namespace

namespace goom {

size_t scan_large_workspace_bytes(long long T, int d, int m, long long batch, long long requested_chunk, bool final_only)
{
    return plan_large(T, d, m, batch, requested_chunk, final_only).total;
}

int run_scan_large(goom_ctx *ctx, const void *M, const void *init, void *P, long long T, int d, int m, long long batch,
                   long long requested_chunk, void *ws, bool final_only)
{
    const LargePlan p = plan_large(T, d, m, batch, requested_chunk, final_only);
    const long long chains_all = batch * p.C;
    if (chains_all > 65535) return fail(ctx, GOOM_EUNSUPPORTED, "too many chains (%lld) for matrices above %d", chains_all, GOOM_MAX_DIM);
    unsigned char *w = static_cast<unsigned char *>(ws);
    float *atil = reinterpret_cast<float *>(w + p.off_atil);
    double *na = reinterpret_cast<double *>(w + p.off_na);
    float *s1 = reinterpret_cast<float *>(w + p.off_s1);
    double *e1 = reinterpret_cast<double *>(w + p.off_e1);
    float *s3 = reinterpret_cast<float *>(w + p.off_s3);
    double *e3 = reinterpret_cast<double *>(w + p.off_e3);
    float *cbuf = reinterpret_cast<float *>(w + p.off_cbuf);
    float *yt = reinterpret_cast<float *>(w + p.off_yt);
    double *ey = reinterpret_cast<double *>(w + p.off_ey);
    float *trow = reinterpret_cast<float *>(w + p.off_trow);
    float *cbuf2 = reinterpret_cast<float *>(w + p.off_x2);
    double *ey2 = reinterpret_cast<double *>(w + p.off_ey2);
    const float2 *Mg = static_cast<const float2 *>(M);
    const int dp = p.dp, mp = p.mp;
    hipStream_t st = ctx->stream;
    auto ok = [&](const char *what) { return check_hip(ctx, hipGetLastError(), what); };

    // one step of all chains of a launch: state[chain] (rows x dp) <- state A~^T, rescaled
    auto advance = [&](float *state, double *expo, int rows, const ChainGeom &q, long long chains, long long s) {
        hipLaunchKernelGGL(chain_convert_left_kernel, dim3(dp / 4, (unsigned)chains), dim3(256), 0, st, Mg, atil, na, q, s);
        hipLaunchKernelGGL(gemm_nt_kernel, dim3(dp / BN, rows / BM, (unsigned)chains), dim3(256), 0, st, state, atil, cbuf, rows, dp, dp,
                           (long long)rows * dp, (long long)dp * dp, (long long)rows * dp);
        hipLaunchKernelGGL(rescale_rows_kernel, dim3(rows / 4, (unsigned)chains), dim3(256), 0, st, cbuf, state, na, (long long)dp, expo, rows, dp);
    };

    float *nrow = reinterpret_cast<float *>(w + p.off_nrow);
    if (p.resident) {
        prof_begin(ctx, "scan_large_row_shifts");
        const int e = launch_row_shifts256(ctx, M, nrow, d, batch * T);
        prof_end(ctx);
        if (e) return e;
    }

    // ---- phase 1: chunk products
    if (p.C1 > 0) {
        ChainGeom q{T, p.L, p.C1, d, dp};
        const long long chains = batch * p.C1;
        prof_begin(ctx, "scan_large_phase1_chunk_products");
        if (p.resident) {
            if (int e = launch_chain256(ctx, M, nrow, T, p.L, p.C1, batch, d, d, nullptr, nullptr, s1, e1, nullptr)) return e;
        } else {
            hipLaunchKernelGGL(state_identity_kernel, dim3(dp, (unsigned)chains), dim3(256), 0, st, s1, e1, dp, dp, d);
            for (long long s = 0; s < p.L; ++s) advance(s1, e1, dp, q, chains, s);
        }
        prof_end(ctx);
        if (int e = ok("scan_large phase 1")) return e;
    }

    // ---- phase 2: prefixes at the chunk boundaries (and, for a reduction, the final product)
    prof_begin(ctx, "scan_large_phase2_carries");
    if (init) {
        hipLaunchKernelGGL(column_shift_kernel<double>, dim3(mp / 64, (unsigned)batch), dim3(256), 0, st, static_cast<const float2 *>(init), ey, d, m, mp);
        hipLaunchKernelGGL(convert_right_kernel<double>, dim3(mp / 32, dp / 32, (unsigned)batch), dim3(256), 0, st, static_cast<const float2 *>(init),
                           ey, yt, d, m, mp, dp);
    } else {
        hipLaunchKernelGGL(state_identity_kernel, dim3(mp, (unsigned)batch), dim3(256), 0, st, yt, ey, mp, dp, d);
    }
    // Y <- T_c Y for c = 0, 1, ...: the exponents of T_c's columns go onto Y's rows, T_c (held transposed, as a
    // state) is turned K-contiguous again; two launches per chunk.  The scan keeps every Y (the carry into chunk c).
    if (p.C1 > 0)
        hipLaunchKernelGGL(transpose_kernel, dim3(dp / 32, dp / 32, (unsigned)(batch * p.C1)), dim3(256), 0, st, s1, (long long)dp * dp, trow,
                           (long long)dp * dp, dp);
    auto pass = [&](const float *in, const double *ein, long long c_next) {
        // from `in`: the carry into chunk c_next (kept, for a scan) and the operand of the product with T_c_next
        CarryPass cp;
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
        if (cp.outA || cp.outB) hipLaunchKernelGGL(carry_pass_kernel, dim3(mp / 4, (unsigned)batch), dim3(256), 0, st, cp);
    };
    pass(yt, ey, 0);
    for (long long c = 0; c < p.C1; ++c) {
        hipLaunchKernelGGL(gemm_nt_kernel, dim3(dp / BN, mp / BM, (unsigned)batch), dim3(256), 0, st, cbuf2, trow + (size_t)c * dp * dp, cbuf, mp, dp, dp,
                           (long long)mp * dp, (long long)p.C1 * dp * dp, (long long)mp * dp);
        pass(cbuf, ey2, c + 1);
    }
    if (final_only && p.C1 > 0) {
        ChainGeom q{T, p.L, 1, d, dp};
        hipLaunchKernelGGL(chain_store_kernel, dim3((d + 31) / 32, (m + 31) / 32, (unsigned)batch), dim3(256), 0, st, yt, ey, static_cast<float2 *>(P), q,
                           0LL, m, mp, 1LL, 0LL);
    }
    prof_end(ctx);
    if (int e = ok("scan_large phase 2")) return e;
    if (final_only && p.C1 > 0) return GOOM_OK;

    // ---- phase 3: every chunk from its incoming prefix, all prefixes stored (a single chunk runs only this)
    {
        ChainGeom q{T, p.L, p.C, d, dp};
        float *state = final_only ? yt : s3; // a reduction of a single chunk walks it here
        double *expo = final_only ? ey : e3;
        prof_begin(ctx, final_only ? "scan_large_single_chunk" : "scan_large_phase3_outputs");
        if (p.resident) {
            // (a reduction of a single chunk leaves its product in the state, stored below)
            const int e = final_only ? launch_chain256(ctx, M, nrow, T, p.L, p.C, batch, d, m, state, expo, state, expo, nullptr)
                                     : launch_chain256(ctx, M, nrow, T, p.L, p.C, batch, d, m, state, expo, nullptr, nullptr, P);
            if (e) return e;
        }
        for (long long s = 0; s < (p.resident ? 0 : p.L); ++s) {
            advance(state, expo, mp, q, chains_all, s);
            if (!final_only)
                hipLaunchKernelGGL(chain_store_kernel, dim3((d + 31) / 32, (m + 31) / 32, (unsigned)chains_all), dim3(256), 0, st, state, expo,
                                   static_cast<float2 *>(P), q, s, m, mp, T, -1LL);
        }
        if (final_only) {
            ChainGeom q1{T, p.L, 1, d, dp};
            hipLaunchKernelGGL(chain_store_kernel, dim3((d + 31) / 32, (m + 31) / 32, (unsigned)batch), dim3(256), 0, st, state, expo,
                               static_cast<float2 *>(P), q1, 0LL, m, mp, 1LL, 0LL);
        }
        prof_end(ctx);
    }
    return ok("scan_large phase 3");
}

} // namespace goom
