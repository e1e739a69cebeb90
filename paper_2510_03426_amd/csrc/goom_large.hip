// LMME for shapes beyond the register-resident kernels (any of n, d, m above 128, up to 1024; float
// components): the same scaled real product (paper Section 3.2, eqs. 10-11; shifts by the identity of eq. 12), but as
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

#include "goom_large_scan.h"

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
// grid (N / T, M / T, batch), 256 threads = 2 x 2 waves of (T / 2) x (T / 2), T = 32 WT: 128 x 128 tiles
// (WT = 4) for throughput, 64 x 64 tiles (WT = 2) where a product has too few of the large ones to fill the
// chip and its latency is what counts (the carry phase of a scan: one 256 x 256 product after the other).
constexpr int BM = 128, BN = 128, BK = 16, LDK = BK + 4;

// The matrix instruction is the 32 x 32 x 2 form: twice the work per operand fetch of the 16 x 16 x 4 form, which
// matters when several waves of a SIMD take turns (measured with instruction-only kernels: 138 against 104
// TFLOP/s at two waves per SIMD).  Lane l supplies row (or column) l % 32 and one of two K values, l / 32; of
// the sixteen K values of a step, instruction (t, v) contracts 8 t + v and 8 t + 4 + v, so that a lane's four
// values per t are adjacent in LDS.  Register r of the result holds row 8 (r / 4) + 4 (l / 32) + r % 4 of
// column l % 32.
typedef float f16v __attribute__((ext_vector_type(16)));

template <int WT>
__global__ __launch_bounds__(256, 2) void gemm_nt_kernel(const float *__restrict__ X, const float *__restrict__ Y, float *__restrict__ Cout, int M,
                                                          int N, int K, long long sx, long long sy, long long sc)
{
    constexpr int TM = 32 * WT;      // tile edge
    constexpr int NL = TM * 4 / 256; // 16-byte pieces of a TM x 16 tile per thread
    constexpr int WB = WT / 2;       // 32 x 32 blocks per wave and dimension
    __shared__ __align__(16) float xs[2][TM * LDK];
    __shared__ __align__(16) float ys[2][TM * LDK];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = lane >> 5, c = lane & 31;
    const int wm = wave >> 1, wn = wave & 1;
    // Workgroups are handed to the eight XCDs in turn, each with its own L2: renumber them so that one
    // XCD works on a contiguous range of tiles, whose operand panels it then shares in its L2.
    const unsigned tiles_x = gridDim.x, tiles_y = gridDim.y;
    const unsigned long long nwg = (unsigned long long)tiles_x * tiles_y * gridDim.z;
    unsigned long long lin = ((unsigned long long)blockIdx.z * tiles_y + blockIdx.y) * tiles_x + blockIdx.x;
    if (nwg % 8 == 0) lin = (lin % 8) * (nwg / 8) + lin / 8;
    const unsigned bx = (unsigned)(lin % tiles_x), by = (unsigned)((lin / tiles_x) % tiles_y);
    const long long b = (long long)(lin / ((unsigned long long)tiles_x * tiles_y));
    const float *Xb = X + b * sx + (size_t)by * TM * K;
    const float *Yb = Y + b * sy + (size_t)bx * TM * K;
    // global -> registers: the TM x 16 tile is TM * 4 pieces of four floats; a thread takes NL of each operand
    const int r0 = tid >> 2, kq = (tid & 3) * 4;
    f4 xr[NL], yr[NL];
    auto load_tiles = [&](int k0) {
#pragma unroll
        for (int u = 0; u < NL; ++u) {
            xr[u] = *reinterpret_cast<const f4 *>(Xb + (size_t)(r0 + 64 * u) * K + k0 + kq);
            yr[u] = *reinterpret_cast<const f4 *>(Yb + (size_t)(r0 + 64 * u) * K + k0 + kq);
        }
    };
    auto store_tiles = [&](int buf) {
#pragma unroll
        for (int u = 0; u < NL; ++u) {
            *reinterpret_cast<f4 *>(&xs[buf][(r0 + 64 * u) * LDK + kq]) = xr[u];
            *reinterpret_cast<f4 *>(&ys[buf][(r0 + 64 * u) * LDK + kq]) = yr[u];
        }
    };
    f16v acc[WB][WB];
#pragma unroll
    for (int i = 0; i < WB; ++i)
#pragma unroll
        for (int j = 0; j < WB; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    const int nk = K / BK;
    load_tiles(0);
    store_tiles(0);
    __syncthreads();
    int buf = 0;
    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk) load_tiles((kt + 1) * BK);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            f4 av[WB], bv[WB];
#pragma unroll
            for (int i = 0; i < WB; ++i) {
                av[i] = *reinterpret_cast<const f4 *>(&xs[buf][(wm * 16 * WT + 32 * i + c) * LDK + 8 * t + 4 * h]);
                bv[i] = *reinterpret_cast<const f4 *>(&ys[buf][(wn * 16 * WT + 32 * i + c) * LDK + 8 * t + 4 * h]);
            }
#pragma unroll
            for (int v = 0; v < 4; ++v)
#pragma unroll
                for (int i = 0; i < WB; ++i)
#pragma unroll
                    for (int j = 0; j < WB; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i][v], bv[j][v], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) store_tiles(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }
    float *Cb = Cout + b * sc + ((size_t)by * TM + wm * 16 * WT) * N + (size_t)bx * TM + wn * 16 * WT;
#pragma unroll
    for (int i = 0; i < WB; ++i)
#pragma unroll
        for (int j = 0; j < WB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) Cb[(size_t)(32 * i + 8 * (r / 4) + 4 * h + r % 4) * N + 32 * j + c] = acc[i][j][r];
}

// gx, gy: the grid in 128 x 128 tiles
inline void launch_gemm_nt(hipStream_t st, const float *X, const float *Y, float *C, unsigned gx, unsigned gy, unsigned gz, int M, int N, int K,
                           long long sx, long long sy, long long sc)
{
    if ((unsigned long long)gx * gy * gz < 128)
        hipLaunchKernelGGL(gemm_nt_kernel<2>, dim3(2 * gx, 2 * gy, gz), dim3(256), 0, st, X, Y, C, M, N, K, sx, sy, sc);
    else
        hipLaunchKernelGGL(gemm_nt_kernel<4>, dim3(gx, gy, gz), dim3(256), 0, st, X, Y, C, M, N, K, sx, sy, sc);
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


using goom_large::pad_to;

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
    launch_gemm_nt(ctx->stream, Y, X, Ct, Np / BN, Mp / BM, nb, Mp, Np, Kp, (long long)Mp * Kp, (long long)Np * Kp, (long long)Mp * Np);
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
// Scans and reductions of complex64 matrices above 128 x 128: the shared driver with this file's GEMM, the
// conversion of an initial state, and the register-resident kernels for 128 < d <= 256.
// ------------------------------------------------------------------------------------------------
namespace {

struct OpsF32 {
    static constexpr bool kResident = true;
    static int prepare(goom_ctx *) { return GOOM_OK; }
    static void gemm(hipStream_t st, const float *X, const float *Y, float *C, unsigned gx, unsigned gy, unsigned gz, int M, int N, int K,
                     long long sx, long long sy, long long sc)
    {
        launch_gemm_nt(st, X, Y, C, gx, gy, gz, M, N, K, sx, sy, sc);
    }
    static void init_state(hipStream_t st, const void *init, double *ey, float *yt, int d, int m, int mp, int dp, unsigned batch)
    {
        hipLaunchKernelGGL(column_shift_kernel<double>, dim3(mp / 64, batch), dim3(256), 0, st, static_cast<const float2 *>(init), ey, d, m, mp);
        hipLaunchKernelGGL(convert_right_kernel<double>, dim3(mp / 32, dp / 32, batch), dim3(256), 0, st, static_cast<const float2 *>(init), ey, yt, d,
                           m, mp, dp);
    }
    static int row_shifts(goom_ctx *ctx, const void *M, float *nrow, int d, long long nmat) { return goom::launch_row_shifts256(ctx, M, nrow, d, nmat); }
    static int chains(goom_ctx *ctx, const void *M, const float *nrow, long long T, long long L, long long chunks, long long batch, int d, int m,
                      const float *init, const double *einit, float *fin, double *efin, void *P)
    {
        return goom::launch_chain256(ctx, M, nrow, T, L, chunks, batch, d, m, init, einit, fin, efin, P);
    }
};

} // namespace

namespace goom {

size_t scan_large_workspace_bytes(long long T, int d, int m, long long batch, long long requested_chunk, bool final_only)
{
    return goom_large::plan_large(T, d, m, batch, requested_chunk, final_only, sizeof(float), true).total;
}

int run_scan_large(goom_ctx *ctx, const void *M, const void *init, void *P, long long T, int d, int m, long long batch,
                   long long requested_chunk, void *ws, bool final_only)
{
    return goom_large::run_scan_large_t<float, OpsF32>(ctx, M, init, P, T, d, m, batch, requested_chunk, ws, final_only);
}

} // namespace goom
