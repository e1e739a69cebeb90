// LMME of tall operands (paper Section 3.2, the scaled product of eq. 10): C'[b] = LMME(A'[b], B'[b]) with A' [n, d] of many rows
// and B' [d, m] small, d, m <= 64, float components.  This is the shape of the state-space layer's input term (Section 4.3):
// bias_t = B u_t for all steps t at once, the rows being the steps.
//
// B~ = (+-) 2^(log2|B_jk| - e_k), e_k a whole number near the column's largest log2 magnitude, is formed once per wave and stays in
// registers in the matrix instruction's operand order; the rows of A' stream through, sixteen at a time per wave: each lane reads a
// contiguous quarter of a row, the row shift n_i is a maximum over four lanes, A~ = (+-) 2^(log2|A_ij| - n_i) goes straight into the
// instruction (16 x 16 x 4, float), and the store pass writes log|acc| + (n_i + e_k) ln 2 with the sign.  Every byte is read and
// written once; nothing passes through LDS.
//
// Inner index order: lane group g of the instruction's four supplies inner index g KD / 4 + t at step t (KD: d padded to 16, 32 or
// 64), for both operands, so that a lane's part of a row of A' is contiguous in memory.
#include "goom_chain_kernel.h"

namespace {

using goom_chain::Comp;
using goom_chain::f4;

struct TallArgs {
    const float2 *A, *B;
    float2 *C;
    int n, d, m;
    int blocks_per_item; // sixteen-row blocks per batch item
    int wgs_per_item;    // workgroups per batch item; workgroup w takes blocks 4 w', 4 w' + 1, ... by wave, stride 4 wgs_per_item
};

template <int KD, int MS> __global__ __launch_bounds__(256) void lmme_tall_kernel(TallArgs a)
{
    typedef Comp<float> C;
    constexpr int KS = KD / 4; // steps of the instruction = inner indices per lane
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, c = lane & 15;
    const size_t item = blockIdx.x / a.wgs_per_item;
    const int wg = (int)(blockIdx.x - item * a.wgs_per_item);
    const float2 *Ap = a.A + item * (size_t)a.n * a.d;
    const float2 *Bp = a.B + item * (size_t)a.d * a.m;
    float2 *Cp = a.C + item * (size_t)a.n * a.m;
    const float kNegInf = C::neg_inf();
    const int d = a.d, m = a.m, n = a.n;

    // ---- B~ in registers: bt[s][t] = entry (g KS + t, 16 s + c), scaled by the column's shift
    float bt[MS][KS], ecol[MS];
#pragma unroll
    for (int s = 0; s < MS; ++s) {
        const int col = 16 * s + c;
        float re[KS], im[KS];
        float top = kNegInf;
#pragma unroll
        for (int t = 0; t < KS; ++t) {
            const int k = g * KS + t;
            float2 v = float2{kNegInf, 0.0f};
            if (k < d && col < m) v = Bp[(size_t)k * m + col];
            re[t] = v.x;
            im[t] = v.y;
            top = C::max_(top, v.x);
        }
        top = C::xor16_32_max(top); // over the four lane groups: the whole column
        const float e = C::row_shift(top);
        ecol[s] = e;
#pragma unroll
        for (int t = 0; t < KS; ++t) bt[s][t] = re[t] > kNegInf ? C::apply_sign(C::exp2_shifted(re[t], e), im[t]) : 0.0f;
    }

    // ---- rows of A', sixteen at a time
    const int k0 = g * KS; // this lane's first inner index
    for (int blk = wg * 4 + wave; blk < a.blocks_per_item; blk += 4 * a.wgs_per_item) {
        const int row = blk * 16 + c;
        float re[KS], im[KS];
        if (row < n) {
            const float2 *rp = Ap + (size_t)row * d + k0;
#pragma unroll
            for (int t = 0; t < KS; t += 2) { // (d is a multiple of four: pairs of entries lie on 16-byte boundaries)
                if (k0 + t < d) {
                    const f4 w = *reinterpret_cast<const f4 *>(rp + t);
                    re[t] = w[0];
                    im[t] = w[1];
                    re[t + 1] = w[2];
                    im[t + 1] = w[3];
                } else {
                    re[t] = re[t + 1] = kNegInf;
                    im[t] = im[t + 1] = 0.0f;
                }
            }
        } else {
#pragma unroll
            for (int t = 0; t < KS; ++t) {
                re[t] = kNegInf;
                im[t] = 0.0f;
            }
        }
        float top = re[0];
#pragma unroll
        for (int t = 1; t < KS; ++t) top = C::max_(top, re[t]);
        top = C::xor16_32_max(top); // the row's other three quarters
        const float nrow = C::row_shift(top);
        f4 acc[MS];
#pragma unroll
        for (int s = 0; s < MS; ++s) acc[s] = f4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int t = 0; t < KS; ++t) {
            const float av = re[t] > kNegInf ? C::apply_sign(C::exp2_shifted(re[t], nrow), im[t]) : 0.0f;
#pragma unroll
            for (int s = 0; s < MS; ++s) acc[s] = C::mfma(av, bt[s][t], acc[s]);
        }
        // ---- signed logarithm, shifts re-added: register v of lane group g is row 4 g + v of the block, column 16 s + c
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const float nr = __shfl(nrow, 4 * g + v, 64); // lane 4 g + v (group 0) holds that row's shift
            const int orow = blk * 16 + 4 * g + v;
#pragma unroll
            for (int s = 0; s < MS; ++s) {
                const int col = 16 * s + c;
                const float x = acc[s][v];
                if (orow < n && col < m) {
                    float2 o;
                    o.x = x == 0.0f ? kNegInf : C::out_re_f(x, nr + ecol[s]);
                    o.y = x < 0.0f ? C::pi() : 0.0f;
                    Cp[(size_t)orow * m + col] = o;
                }
            }
        }
    }
}

template <int KD, int MS> int launch_t(goom_ctx *ctx, const TallArgs &args, long long batch)
{
    const long long grid = batch * args.wgs_per_item;
    if (grid > 0x7fffffffLL) return goom::fail(ctx, GOOM_EUNSUPPORTED, "too many row blocks for one launch");
    goom::prof_begin(ctx, "lmme");
    hipLaunchKernelGGL((lmme_tall_kernel<KD, MS>), dim3((unsigned)grid), dim3(256), 0, ctx->stream, args);
    goom::prof_end(ctx);
    return goom::check_hip(ctx, hipGetLastError(), "launch lmme_tall_kernel");
}

template <int KD> int launch_ms(goom_ctx *ctx, const TallArgs &args, long long batch, int ms)
{
    switch (ms) {
    case 1: return launch_t<KD, 1>(ctx, args, batch);
    case 2: return launch_t<KD, 2>(ctx, args, batch);
    case 3: return launch_t<KD, 3>(ctx, args, batch);
    default: return launch_t<KD, 4>(ctx, args, batch);
    }
}

} // namespace

namespace goom {

// many rows against a small right operand: float components, d a multiple of four, d and m at most 64
bool lmme_tall_applies(int n, int d, int m, int dtype) { return dtype == GOOM_C64 && d <= 64 && m <= 64 && d % 4 == 0 && n >= 2 * (d > m ? d : m); }

int launch_lmme_tall(goom_ctx *ctx, const void *A, const void *B, void *Cm, long long batch, int n, int d, int m)
{
    TallArgs args;
    args.A = static_cast<const float2 *>(A);
    args.B = static_cast<const float2 *>(B);
    args.C = static_cast<float2 *>(Cm);
    args.n = n;
    args.d = d;
    args.m = m;
    args.blocks_per_item = (n + 15) / 16;
    // a workgroup forms B~ once and then takes at least sixteen row blocks when there are that many; enough workgroups to fill the chip
    int wgs = (args.blocks_per_item + 63) / 64;
    while (wgs * batch < 2048 && wgs * 4 < args.blocks_per_item) wgs *= 2;
    args.wgs_per_item = wgs;
    const int ms = (m + 15) / 16;
    if (d <= 16) return launch_ms<16>(ctx, args, batch, ms);
    if (d <= 32) return launch_ms<32>(ctx, args, batch, ms);
    return launch_ms<64>(ctx, args, batch, ms);
}

} // namespace goom
