// LMME for shapes above 128 with double components (complex128 GOOMs; the paper's appendix compares
// LMME on 1024 x 1024 matrices in both formats): the scaled real product of Section 3.2 (eqs. 10-11,
// shifts by the identity of eq. 12) as separate passes through the caller's workspace, like the float path:
//   1. rows of A' -> reals scaled by the row's power of two (K-contiguous, zero padded);
//   2. columns of B' -> reals scaled by the column's power of two, written transposed;
//   3. C~^T = B~^T A~^T on the double-precision matrix instruction (16 x 16 x 4): 128 x 128 tile per
//      workgroup, 64 x 64 per wave, K in steps of 16 through double-buffered LDS;
//   4. signed logarithm, shifts re-added, transposed back on the way out.
// Scans and reductions of such matrices (Section 4.1) run through the shared driver with this file's GEMM.
#include <cmath>

#include "goom_large_scan.h"

namespace {

using goom_chain::Comp;
using goom_chain::d4;
using goom_chain::kLog2e;
typedef Comp<double> CD;
typedef double d2 __attribute__((ext_vector_type(2)));

__device__ inline double neg_inf() { return -__builtin_huge_val(); }

__device__ inline double signed_scaled(double re, double im, double shift)
{
    return CD::apply_sign(CD::exp2_shifted(re, shift), im);
}

// ---- 1. rows of the left operand.  grid (rows_padded, batch), 256 threads.
__global__ __launch_bounds__(256) void convert_left_f64_kernel(const double2 *__restrict__ A, double *__restrict__ X, double *__restrict__ shifts,
                                                               int n, int d, int rows_padded, int k_padded)
{
    __shared__ double red[4];
    const int row = blockIdx.x;
    const long long b = blockIdx.y;
    const int tid = threadIdx.x;
    double *xrow = X + ((size_t)b * rows_padded + row) * k_padded;
    if (row >= n) { // padding rows
        for (int j = tid; j < k_padded; j += 256) xrow[j] = 0.0;
        if (tid == 0) shifts[(size_t)b * rows_padded + row] = 0.0;
        return;
    }
    const double2 *arow = A + ((size_t)b * n + row) * d;
    double mx = neg_inf();
    for (int j = tid; j < d; j += 256) mx = fmax(mx, arow[j].x);
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) mx = fmax(mx, __shfl_xor(mx, s, 64));
    if ((tid & 63) == 0) red[tid >> 6] = mx;
    __syncthreads();
    mx = fmax(fmax(red[0], red[1]), fmax(red[2], red[3]));
    const bool zero_row = !(mx > neg_inf());
    const double sh = zero_row ? 0.0 : ceil(mx * kLog2e);
    for (int j = tid; j < k_padded; j += 256) {
        double v = 0.0;
        if (j < d && !zero_row) {
            const double2 e = arow[j];
            v = signed_scaled(e.x, e.y, sh);
        }
        xrow[j] = v;
    }
    if (tid == 0) shifts[(size_t)b * rows_padded + row] = sh;
}

// ---- 2a. column maxima of the right operand.  grid (ceil(m / 64), batch), block 64 x 4.
__global__ __launch_bounds__(256) void column_shift_f64_kernel(const double2 *__restrict__ B, double *__restrict__ shifts, int d, int m, int cols_padded)
{
    __shared__ double red[4][64];
    const int cx = threadIdx.x & 63, ry = threadIdx.x >> 6;
    const int col = blockIdx.x * 64 + cx;
    const long long b = blockIdx.y;
    double mx = neg_inf();
    if (col < m) {
        double part[8]; // eight independent loads in flight per thread
#pragma unroll
        for (int u = 0; u < 8; ++u) part[u] = neg_inf();
        const double2 *base = B + (size_t)b * d * m + col;
        int j = ry;
        for (; j + 28 < d; j += 32) {
#pragma unroll
            for (int u = 0; u < 8; ++u) part[u] = fmax(part[u], base[(size_t)(j + 4 * u) * m].x);
        }
        for (; j < d; j += 4) part[0] = fmax(part[0], base[(size_t)j * m].x);
#pragma unroll
        for (int u = 0; u < 8; ++u) mx = fmax(mx, part[u]);
    }
    red[ry][cx] = mx;
    __syncthreads();
    if (ry == 0 && col < cols_padded) {
        mx = fmax(fmax(red[0][cx], red[1][cx]), fmax(red[2][cx], red[3][cx]));
        shifts[(size_t)b * cols_padded + col] = (col < m && mx > neg_inf()) ? ceil(mx * kLog2e) : 0.0;
    }
}

// ---- 2b. right operand scaled and transposed: Y[b][col][j] = (+-) 2^(log2|B_j,col| - shift_col).
// grid (cols_padded / 32, k_padded / 32 rounded up, batch), block 32 x 8.
__global__ __launch_bounds__(256) void convert_right_f64_kernel(const double2 *__restrict__ B, const double *__restrict__ shifts,
                                                                double *__restrict__ Y, int d, int m, int cols_padded, int k_padded)
{
    __shared__ double tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int c0 = blockIdx.x * 32, j0 = blockIdx.y * 32;
    const long long b = blockIdx.z;
    const int col = c0 + tx;
    const double sh = col < cols_padded ? shifts[(size_t)b * cols_padded + col] : 0.0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int j = j0 + ty + 8 * r;
        double v = 0.0;
        if (j < d && col < m) {
            const double2 e = B[((size_t)b * d + j) * m + col];
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
// grid (N / 128, M / 128, batch), 256 threads = 2 x 2 waves of 64 x 64.  One matrix instruction contracts
// four values of K, one per group of sixteen lanes; lane group g takes K = 4 g + v in instruction v, so
// that its four values are adjacent in LDS.  Rows are 18 doubles apart: the sixteen rows that sixteen
// lanes read at once then start in sixteen different groups of four banks.
constexpr int BM = 128, BN = 128, BK = 16, LDK = BK + 2;

// WT = 4: 128 x 128 tiles; WT = 2: 64 x 64 tiles, for products with too few of the large ones to fill the chip
template <int WT>
__global__ __launch_bounds__(256, 2) void gemm_nt_f64_kernel(const double *__restrict__ X, const double *__restrict__ Y, double *__restrict__ Cout,
                                                              int M, int N, int K, long long sx, long long sy, long long sc)
{
    constexpr int TM = 32 * WT;      // tile edge
    constexpr int NL = TM * 4 / 256; // 32-byte pieces of a TM x 16 tile per thread
    extern __shared__ __align__(16) unsigned char smem_raw[];
    double *xs = reinterpret_cast<double *>(smem_raw);          // [2][TM * LDK]
    double *ys = xs + 2 * TM * LDK;                             // [2][TM * LDK]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 4, c = lane & 15;
    const int wm = wave >> 1, wn = wave & 1;
    // workgroups go to the eight XCDs in turn: renumber them so that one XCD works on a contiguous range of
    // tiles and shares their operand panels in its L2
    const unsigned tiles_x = gridDim.x, tiles_y = gridDim.y;
    const unsigned long long nwg = (unsigned long long)tiles_x * tiles_y * gridDim.z;
    unsigned long long lin = ((unsigned long long)blockIdx.z * tiles_y + blockIdx.y) * tiles_x + blockIdx.x;
    if (nwg % 8 == 0) lin = (lin % 8) * (nwg / 8) + lin / 8;
    const unsigned bx = (unsigned)(lin % tiles_x), by = (unsigned)((lin / tiles_x) % tiles_y);
    const long long b = (long long)(lin / ((unsigned long long)tiles_x * tiles_y));
    const double *Xb = X + b * sx + (size_t)by * TM * K;
    const double *Yb = Y + b * sy + (size_t)bx * TM * K;
    // global -> registers: a TM x 16 tile is TM * 4 pieces of four doubles; a thread takes NL of each operand
    const int r0 = tid >> 2, kq = (tid & 3) * 4;
    d2 xr[2 * NL], yr[2 * NL];
    auto load_tiles = [&](int k0) {
#pragma unroll
        for (int u = 0; u < NL; ++u) {
            const d2 *p = reinterpret_cast<const d2 *>(Xb + (size_t)(r0 + 64 * u) * K + k0 + kq);
            xr[2 * u] = p[0]; xr[2 * u + 1] = p[1];
            p = reinterpret_cast<const d2 *>(Yb + (size_t)(r0 + 64 * u) * K + k0 + kq);
            yr[2 * u] = p[0]; yr[2 * u + 1] = p[1];
        }
    };
    auto store_tiles = [&](int buf) {
#pragma unroll
        for (int u = 0; u < NL; ++u) {
            d2 *q = reinterpret_cast<d2 *>(&xs[buf * TM * LDK + (r0 + 64 * u) * LDK + kq]);
            q[0] = xr[2 * u]; q[1] = xr[2 * u + 1];
            q = reinterpret_cast<d2 *>(&ys[buf * TM * LDK + (r0 + 64 * u) * LDK + kq]);
            q[0] = yr[2 * u]; q[1] = yr[2 * u + 1];
        }
    };
    d4 acc[WT][WT];
#pragma unroll
    for (int i = 0; i < WT; ++i)
#pragma unroll
        for (int j = 0; j < WT; ++j) acc[i][j] = d4{0.0, 0.0, 0.0, 0.0};
    const int nk = K / BK;
    load_tiles(0);
    store_tiles(0);
    __syncthreads();
    int buf = 0;
    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk) load_tiles((kt + 1) * BK);
        const double *xb = xs + buf * TM * LDK, *yb = ys + buf * TM * LDK;
#pragma unroll
        for (int h = 0; h < 2; ++h) { // K = 4 g + 2 h, 4 g + 2 h + 1
            d2 av[WT], bv[WT];
#pragma unroll
            for (int i = 0; i < WT; ++i) {
                av[i] = *reinterpret_cast<const d2 *>(&xb[(wm * 16 * WT + 16 * i + c) * LDK + 4 * g + 2 * h]);
                bv[i] = *reinterpret_cast<const d2 *>(&yb[(wn * 16 * WT + 16 * i + c) * LDK + 4 * g + 2 * h]);
            }
#pragma unroll
            for (int v = 0; v < 2; ++v)
#pragma unroll
                for (int i = 0; i < WT; ++i)
#pragma unroll
                    for (int j = 0; j < WT; ++j) acc[i][j] = CD::mfma(av[i][v], bv[j][v], acc[i][j]);
        }
        if (kt + 1 < nk) store_tiles(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }
    // register v of lane group g holds row 4 v + g of a 16 x 16 tile
    double *Cb = Cout + b * sc + ((size_t)by * TM + wm * 16 * WT) * N + (size_t)bx * TM + wn * 16 * WT;
#pragma unroll
    for (int i = 0; i < WT; ++i)
#pragma unroll
        for (int j = 0; j < WT; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) Cb[(size_t)(16 * i + CD::row_of(g, v)) * N + 16 * j + c] = acc[i][j][v];
}

constexpr size_t kGemmLds = (size_t)2 * (BM + BN) * LDK * sizeof(double); // of the 128 x 128 variant

inline int prepare_gemm_f64(goom_ctx *ctx)
{
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(gemm_nt_f64_kernel<4>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)kGemmLds);
    return e == hipSuccess ? GOOM_OK : goom::check_hip(ctx, e, "hipFuncSetAttribute(gemm_nt_f64_kernel)");
}

// gx, gy: the grid in 128 x 128 tiles
inline void launch_gemm_nt_f64(hipStream_t st, const double *X, const double *Y, double *C, unsigned gx, unsigned gy, unsigned gz, int M, int N,
                               int K, long long sx, long long sy, long long sc)
{
    if ((unsigned long long)gx * gy * gz < 128)
        hipLaunchKernelGGL(gemm_nt_f64_kernel<2>, dim3(2 * gx, 2 * gy, gz), dim3(256), kGemmLds / 2, st, X, Y, C, M, N, K, sx, sy, sc);
    else
        hipLaunchKernelGGL(gemm_nt_f64_kernel<4>, dim3(gx, gy, gz), dim3(256), kGemmLds, st, X, Y, C, M, N, K, sx, sy, sc);
}

// ---- 4. C'[b][i][k] = GOOM of Ct[b][k][i] 2^(row_shift_i + col_shift_k).
// grid (ceil(n / 32), ceil(m / 32), batch), block 32 x 8.
__global__ __launch_bounds__(256) void lmme_store_f64_kernel(const double *__restrict__ Ct, const double *__restrict__ row_shift,
                                                             const double *__restrict__ col_shift, double2 *__restrict__ Cg, int n, int m,
                                                             int rows_padded, int cols_padded)
{
    __shared__ double tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int i0 = blockIdx.x * 32, k0 = blockIdx.y * 32;
    const long long b = blockIdx.z;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int k = k0 + ty + 8 * r, i = i0 + tx; // inside the padded array always (multiples of 128)
        tile[ty + 8 * r][tx] = Ct[((size_t)b * cols_padded + k) * rows_padded + i];
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int i = i0 + ty + 8 * r, k = k0 + tx;
        if (i < n && k < m) {
            const double x = tile[tx][ty + 8 * r];
            double2 o;
            o.x = CD::out_re(x, row_shift[(size_t)b * rows_padded + i], col_shift[(size_t)b * cols_padded + k]);
            o.y = x < 0.0 ? CD::pi() : 0.0;
            Cg[((size_t)b * n + i) * m + k] = o;
        }
    }
}

using goom_large::pad_to;

} // namespace

namespace goom {

// workspace: X [batch][Np][Kp], row shifts [batch][Np], Y [batch][Mp][Kp], column shifts [batch][Mp], Ct [batch][Mp][Np]
size_t lmme_large_f64_workspace_bytes(long long batch, int n, int d, int m)
{
    const size_t Np = pad_to(n, 128), Mp = pad_to(m, 128), Kp = pad_to(d, 16);
    return align_up((size_t)batch * Np * Kp * 8, 256) + align_up((size_t)batch * Np * 8, 256) + align_up((size_t)batch * Mp * Kp * 8, 256) +
           align_up((size_t)batch * Mp * 8, 256) + align_up((size_t)batch * Mp * Np * 8, 256);
}

int launch_lmme_large_f64(goom_ctx *ctx, const void *A, const void *B, void *C, long long batch, int n, int d, int m, void *ws)
{
    const int Np = pad_to(n, 128), Mp = pad_to(m, 128), Kp = pad_to(d, 16);
    if (batch > 65535) return fail(ctx, GOOM_EUNSUPPORTED, "at most 65535 pairs per call for shapes above 128 (batch=%lld)", batch);
    unsigned char *w = static_cast<unsigned char *>(ws);
    double *X = reinterpret_cast<double *>(w);
    w += align_up((size_t)batch * Np * Kp * 8, 256);
    double *rs = reinterpret_cast<double *>(w);
    w += align_up((size_t)batch * Np * 8, 256);
    double *Y = reinterpret_cast<double *>(w);
    w += align_up((size_t)batch * Mp * Kp * 8, 256);
    double *cs = reinterpret_cast<double *>(w);
    w += align_up((size_t)batch * Mp * 8, 256);
    double *Ct = reinterpret_cast<double *>(w);
    const unsigned nb = (unsigned)batch;
    if (int e = prepare_gemm_f64(ctx)) return e;
    prof_begin(ctx, "lmme_large_scale_operands");
    hipLaunchKernelGGL(convert_left_f64_kernel, dim3(Np, nb), dim3(256), 0, ctx->stream, static_cast<const double2 *>(A), X, rs, n, d, Np, Kp);
    hipLaunchKernelGGL(column_shift_f64_kernel, dim3(Mp / 64, nb), dim3(256), 0, ctx->stream, static_cast<const double2 *>(B), cs, d, m, Mp);
    hipLaunchKernelGGL(convert_right_f64_kernel, dim3(Mp / 32, (Kp + 31) / 32, nb), dim3(256), 0, ctx->stream, static_cast<const double2 *>(B), cs,
                       Y, d, m, Mp, Kp);
    prof_end(ctx);
    if (int s = check_hip(ctx, hipGetLastError(), "launch LMME operand kernels")) return s;
    prof_begin(ctx, "lmme_large_gemm");
    launch_gemm_nt_f64(ctx->stream, Y, X, Ct, Np / BN, Mp / BM, nb, Mp, Np, Kp, (long long)Mp * Kp, (long long)Np * Kp, (long long)Mp * Np);
    prof_end(ctx);
    if (int s = check_hip(ctx, hipGetLastError(), "launch gemm_nt_f64_kernel")) return s;
    prof_begin(ctx, "lmme_large_log_store");
    hipLaunchKernelGGL(lmme_store_f64_kernel, dim3((n + 31) / 32, (m + 31) / 32, nb), dim3(256), 0, ctx->stream, Ct, rs, cs,
                       static_cast<double2 *>(C), n, m, Np, Mp);
    prof_end(ctx);
    return check_hip(ctx, hipGetLastError(), "launch lmme_store_f64_kernel");
}

} // namespace goom

// ------------------------------------------------------------------------------------------------
// Scans and reductions of complex128 matrices above 128 x 128
// ------------------------------------------------------------------------------------------------
namespace {

struct OpsF64 {
    static constexpr bool kResident = false;
    static int prepare(goom_ctx *ctx) { return prepare_gemm_f64(ctx); }
    static void gemm(hipStream_t st, const double *X, const double *Y, double *C, unsigned gx, unsigned gy, unsigned gz, int M, int N, int K,
                     long long sx, long long sy, long long sc)
    {
        launch_gemm_nt_f64(st, X, Y, C, gx, gy, gz, M, N, K, sx, sy, sc);
    }
    static void init_state(hipStream_t st, const void *init, double *ey, double *yt, int d, int m, int mp, int dp, unsigned batch)
    {
        hipLaunchKernelGGL(column_shift_f64_kernel, dim3(mp / 64, batch), dim3(256), 0, st, static_cast<const double2 *>(init), ey, d, m, mp);
        hipLaunchKernelGGL(convert_right_f64_kernel, dim3(mp / 32, dp / 32, batch), dim3(256), 0, st, static_cast<const double2 *>(init), ey, yt, d, m,
                           mp, dp);
    }
};

} // namespace

namespace goom {

size_t scan_large_f64_workspace_bytes(long long T, int d, int m, long long batch, long long requested_chunk, bool final_only)
{
    return goom_large::plan_large(T, d, m, batch, requested_chunk, final_only, sizeof(double), false).total;
}

int run_scan_large_f64(goom_ctx *ctx, const void *M, const void *init, void *P, long long T, int d, int m, long long batch,
                       long long requested_chunk, void *ws, bool final_only)
{
    return goom_large::run_scan_large_t<double, OpsF64>(ctx, M, init, P, T, d, m, batch, requested_chunk, ws, final_only);
}

} // namespace goom
