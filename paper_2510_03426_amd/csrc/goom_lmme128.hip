// Batched LMME of 128 x 128 x 128 operands (paper Section 3.2, eqs. 10-12: the scaled product, its shifts, the scaling identity), float or double components:
// the inner index is walked in tiles of 32 with a running rescale, so that nothing has to be known
// about a whole row or column in advance and neither operand is read twice.
//
// The scaling identity (eq. 12) lets every row of A' and every column of B' be shifted by any amount.  Here the shifts grow as
// the tiles arrive: after tile q the accumulators hold the partial product scaled by 2^-(n_i + e_k), with
// n_i (e_k) a whole number near the largest log2 magnitude seen so far in row i of A' (column k of B').
// When tile q + 1 raises a maximum, the accumulators of that row (column) are scaled down by the
// difference, an exact power of two, before its terms are added.  The state per workgroup is small
// (a 128 x 32 tile of A~ in LDS, a 32 x 16 slice of B~ and a 128 x 16 slice of the result in the
// registers of each wave), which leaves room for the next tile's operands to be in flight during the
// products, and keeps the double-precision variant out of register spills.
//
// One workgroup (8 waves) per pair; wave w owns result columns 16 w .. 16 w + 15.
#include "goom_chain_kernel.h"

namespace {

using goom_chain::Comp;
using goom_chain::Item;
using goom_chain::f4;
using goom_chain::d4;
using goom_chain::kLog2e;

constexpr int kD = 128;     // all three dimensions
constexpr int kKQ = 32;     // inner indices per tile
constexpr int kNQ = kD / kKQ;
constexpr int kThreads = 512;

struct Lmme128Args {
    const void *A, *B;
    void *C;
    void *shifts; // NULL, or per pair the 128 row shifts n_i then the 128 column shifts e_k (for the repair pass)
    // backward modes: the addend Z [pair, 128, 128] GOOMs, the shift of the transposed operand's log-magnitudes along the inner
    // index and that of the addend along the output's rows (MODE 1) or columns (MODE 2), 128 reals per pair each
    const void *Z, *in_shift, *out_shift;
};

constexpr double kInvPi = 0.318309886183790671538;
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

// MODE 0: C' = LMME(A', B') as GOOMs.
// MODE 1, 2 (the two products of the backward pass): the result leaves as reals, C[i, k] = +- exp(Re Z'[i, k] - s + Re P'[i, k]),
// P the product, s = out_shift[i] (MODE 1) or out_shift[k] (MODE 2); and one operand is read transposed from its array with
// in_shift taken from its log-magnitudes along the inner index:
//   MODE 1: right operand (j, k) = B[k][j] e^(-in_shift[j])      MODE 2: left operand (i, j) = A[j][i] e^(-in_shift[j])
// (MODE 1 with float components is held to four waves per SIMD, i.e. 128 registers a lane: two workgroups per compute unit as in the
// other modes; left alone it takes 156 registers, one workgroup per compute unit, and 1.4 ms in place of 1.1)
template <typename R, int MODE> __global__ __launch_bounds__(kThreads, (sizeof(R) == 4 && MODE == 1) ? 4 : 1) void lmme_ktile_kernel(Lmme128Args a)
{
    typedef Comp<R> CR;
    typedef typename CR::vec4 vec4;
    constexpr int LDQ = kKQ + CR::kPad;
    constexpr int LPR = kKQ / 2;             // producer lanes per row: two adjacent entries each
    constexpr int RPP = kThreads / LPR;      // rows per pass
    constexpr int QA = kD / RPP;             // passes = items per thread
    constexpr size_t kTileBytes = (size_t)kD * LDQ * sizeof(R);
    constexpr size_t kBufBytes = kTileBytes + 2 * (size_t)kD * sizeof(R);
    extern __shared__ __align__(16) unsigned char smem[];
    auto tile_of = [&](int b) { return reinterpret_cast<R *>(smem + (size_t)b * kBufBytes); };
    auto nsh_of = [&](int b) { return reinterpret_cast<R *>(smem + (size_t)b * kBufBytes + kTileBytes); };          // row shifts so far
    auto dsh_of = [&](int b) { return reinterpret_cast<R *>(smem + (size_t)b * kBufBytes + kTileBytes) + kD; };     // their change in this tile

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, c = lane & 15;
    const int col = wave * 16 + c;
    const long long pair = blockIdx.x;
    const R *Ap = static_cast<const R *>(a.A) + (size_t)pair * kD * kD * 2;
    const R *Bp = static_cast<const R *>(a.B) + (size_t)pair * kD * kD * 2;
    R *Cp = static_cast<R *>(a.C) + (size_t)pair * kD * kD * (MODE == 0 ? 2 : 1);
    [[maybe_unused]] const R *ins = MODE != 0 ? static_cast<const R *>(a.in_shift) + (size_t)pair * kD : nullptr;
    const R kNone = (R)-1.0e30; // "no finite entry seen yet"

    // producer side: this thread's rows and column pair inside a tile
    const int prow = tid / LPR, pcj = 2 * (tid % LPR);
    auto load_a = [&](int q, Item<R> (&it)[QA]) {
#pragma unroll
        for (int p = 0; p < QA; ++p) {
            if (MODE == 2) { // entries (row, k), (row, k + 1) of the transpose: two loads a row of the array apart
                const int k = q * kKQ + pcj;
                const R *gp = Ap + ((size_t)k * kD + prow + p * RPP) * 2;
                it[p].re0 = gp[0] - ins[k]; it[p].im0 = gp[1];
                it[p].re1 = gp[2 * kD] - ins[k + 1]; it[p].im1 = gp[2 * kD + 1];
            } else {
                const R *gp = Ap + ((size_t)(prow + p * RPP) * kD + q * kKQ + pcj) * 2;
                const vec4 w = *reinterpret_cast<const vec4 *>(gp);
                it[p].re0 = w[0]; it[p].im0 = w[1]; it[p].re1 = w[2]; it[p].im1 = w[3];
            }
        }
    };
    // consumer side: rows 32 q + 16 kt + row_of(g, v) of column col
    auto load_b = [&](int q, R (&bre)[2][4], R (&bim)[2][4]) {
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                // MODE 1: a lane's four inner indices of a 16-tile are neighbours, 4 g + v (32 contiguous bytes of the array's row `col`);
                // the tile of the left operand is then laid out in plain order (see convert_a)
                const int k = q * kKQ + 16 * kt + (MODE == 1 ? 4 * g + v : CR::row_of(g, v));
                if (MODE == 1) { // entry (k, col) of the transpose
                    const R *gp = Bp + ((size_t)col * kD + k) * 2;
                    bre[kt][v] = gp[0] - ins[k];
                    bim[kt][v] = gp[1];
                } else {
                    const R *gp = Bp + ((size_t)k * kD + col) * 2;
                    bre[kt][v] = gp[0];
                    bim[kt][v] = gp[1];
                }
            }
    };

    R nprev[QA];
#pragma unroll
    for (int p = 0; p < QA; ++p) nprev[p] = kNone;
    // tile q of A~ into buffer buf, with the running row shifts
    auto convert_a = [&](const Item<R> (&it)[QA], int buf) {
        R *tile = tile_of(buf);
        R *nsh = nsh_of(buf), *dsh = dsh_of(buf);
#pragma unroll
        for (int p = 0; p < QA; ++p) {
            const int row = prow + p * RPP;
            const R mx = CR::template group_allmax<LPR>(it[p].re0, it[p].re1);
            const R cand = mx > CR::neg_inf() ? CR::ceil_(mx * (R)kLog2e) : kNone;
            const R nnew = cand > nprev[p] ? cand : nprev[p];
            const R x0 = CR::apply_sign(CR::exp2_shifted(it[p].re0, nnew), it[p].im0);
            const R x1 = CR::apply_sign(CR::exp2_shifted(it[p].re1, nnew), it[p].im1);
            tile[row * LDQ + (MODE == 1 ? pcj : CR::phys(pcj))] = x0;
            tile[row * LDQ + (MODE == 1 ? pcj + 1 : CR::phys(pcj + 1))] = x1;
            nsh[CR::phys(row)] = nnew;
            dsh[CR::phys(row)] = nprev[p] - nnew; // <= 0; hugely negative the first time a row gets entries
            nprev[p] = nnew;
        }
    };

    vec4 acc[kD / 16];
#pragma unroll
    for (int mt = 0; mt < kD / 16; ++mt) acc[mt] = vec4{0, 0, 0, 0};
    R ecol = kNone;

    Item<R> ait[QA];
    R bre[2][4], bim[2][4];
    load_a(0, ait);
    load_b(0, bre, bim);
    convert_a(ait, 0);
    if (kNQ > 1) load_a(1, ait);
    __syncthreads();

    for (int q = 0; q < kNQ; ++q) {
        const int buf = q & 1;
        const R *tile = tile_of(buf);
        const R *dsh = dsh_of(buf);
        // ---- this tile's slice of B~ and the column's running shift
        R cmax = CR::neg_inf();
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int v = 0; v < 4; ++v) cmax = CR::max_(cmax, bre[kt][v]);
        cmax = CR::xor16_32_max(cmax);
        const R cand = cmax > CR::neg_inf() ? CR::ceil_(cmax * (R)kLog2e) : kNone;
        const R enew = cand > ecol ? cand : ecol;
        const R de = ecol - enew;
        ecol = enew;
        R bq[2][4];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int v = 0; v < 4; ++v) bq[kt][v] = CR::apply_sign(CR::exp2_shifted(bre[kt][v], enew), bim[kt][v]);
        if (q + 1 < kNQ) load_b(q + 1, bre, bim);
        // ---- accumulators onto the new shifts (exact powers of two)
        if (q > 0) {
#pragma unroll
            for (int mt = 0; mt < kD / 16; ++mt) {
                const vec4 dn = *reinterpret_cast<const vec4 *>(&dsh[16 * mt + 4 * g]);
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[mt][v] = CR::ldexp_(acc[mt][v], (int)CR::clamp_shift(dn[v] + de));
            }
        }
        // ---- products
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            vec4 av[kD / 16];
#pragma unroll
            for (int mt = 0; mt < kD / 16; ++mt) av[mt] = *reinterpret_cast<const vec4 *>(&tile[(16 * mt + c) * LDQ + 16 * kt + 4 * g]);
#pragma unroll
            for (int v = 0; v < 4; ++v)
#pragma unroll
                for (int mt = 0; mt < kD / 16; ++mt) acc[mt] = CR::mfma(av[mt][v], bq[kt][v], acc[mt]);
        }
        // ---- next tile of A~ into the other buffer, the one after that on its way
        if (q + 1 < kNQ) {
            convert_a(ait, buf ^ 1);
            if (q + 2 < kNQ) load_a(q + 2, ait);
        }
        __syncthreads();
    }

    // ---- signed logarithm, shifts re-added
    const R *nsh = nsh_of((kNQ - 1) & 1);
#pragma unroll
    for (int mt = 0; mt < kD / 16; ++mt) {
        const vec4 nv = *reinterpret_cast<const vec4 *>(&nsh[16 * mt + 4 * g]);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const R x = acc[mt][v];
            const int i = 16 * mt + CR::row_of(g, v);
            if (MODE == 0) {
                R *op = Cp + ((size_t)i * kD + col) * 2;
                const bool zero = x == (R)0;
                op[0] = zero ? CR::neg_inf() : CR::out_re(x, nv[v], (double)ecol);
                op[1] = x < (R)0 ? CR::pi() : (R)0;
            } else {
                const R *zp = static_cast<const R *>(a.Z) + ((size_t)pair * kD * kD + (size_t)i * kD + col) * 2;
                const R zre = zp[0], zim = zp[1];
                const R osh = static_cast<const R *>(a.out_shift)[(size_t)pair * kD + (MODE == 1 ? i : col)];
                double val = 0.0;
                if (x != (R)0 && zre != CR::neg_inf()) val = exp_for<R>(((double)zre - (double)osh) + (double)CR::out_re(x, nv[v], (double)ecol));
                Cp[(size_t)i * kD + col] = (R)((x < (R)0) != odd_phase<R>(zim) ? -val : val);
            }
        }
    }
    // the final shifts (whole numbers of log2 units; -1e30 for a row or column without a finite entry), by row and column
    if (a.shifts) {
        R *sh = static_cast<R *>(a.shifts) + (size_t)pair * 2 * kD;
        if (tid < kD) sh[tid] = nsh[CR::phys(tid)];
        if (g == 0) sh[kD + col] = ecol;
    }
}

template <typename R, int MODE> int launch_ktile(goom_ctx *ctx, const Lmme128Args &args, long long batch)
{
    constexpr int LDQ = kKQ + Comp<R>::kPad;
    const size_t lds = 2 * ((size_t)kD * LDQ * sizeof(R) + 2 * (size_t)kD * sizeof(R));
    auto kern = lmme_ktile_kernel<R, MODE>;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return goom::check_hip(ctx, e, "hipFuncSetAttribute(lmme_ktile_kernel)");
    }
    if (batch > 0x7fffffffLL) return goom::fail(ctx, GOOM_EUNSUPPORTED, "too many pairs for one launch");
    goom::prof_begin(ctx, "lmme");
    hipLaunchKernelGGL(kern, dim3((unsigned)batch), dim3(kThreads), lds, ctx->stream, args);
    goom::prof_end(ctx);
    return goom::check_hip(ctx, hipGetLastError(), "launch lmme_ktile_kernel");
}

} // namespace

namespace goom {

int launch_lmme128(goom_ctx *ctx, const void *A, const void *B, void *C, long long batch, int dtype, void *shifts)
{
    Lmme128Args args{A, B, C, shifts, nullptr, nullptr, nullptr};
    return dtype == GOOM_C64 ? launch_ktile<float, 0>(ctx, args, batch) : launch_ktile<double, 0>(ctx, args, batch);
}

// The two products of the backward pass of a 128 x 128 x 128 LMME, their results as real gradients (see the kernel's modes):
// mode 1: grad[i, j] = +- exp(Re Z'[i, j] - out_shift[i] + log|sum_k left[i, k] right[j, k] e^(-in_shift[k])|)
// mode 2: grad[j, k] = +- exp(Re Z'[j, k] - out_shift[k] + log|sum_i left[i, j] e^(-in_shift[i]) right[i, k]|)
int launch_lmme128_backward(goom_ctx *ctx, int mode, const void *left, const void *right, const void *Z, const void *in_shift, const void *out_shift,
                            void *grad, long long batch, int dtype)
{
    Lmme128Args args{left, right, grad, nullptr, Z, in_shift, out_shift};
    if (mode == 1) return dtype == GOOM_C64 ? launch_ktile<float, 1>(ctx, args, batch) : launch_ktile<double, 1>(ctx, args, batch);
    return dtype == GOOM_C64 ? launch_ktile<float, 2>(ctx, args, batch) : launch_ktile<double, 2>(ctx, args, batch);
}

} // namespace goom
