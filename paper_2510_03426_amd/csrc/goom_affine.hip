// Linear recurrence with bias, h_t = A_t h_{t-1} + b_t over GOOMs (paper Section 4.3), float
// components: the two kernels its long batched form spends its time in.
//
//   * chunk products of the augmented matrices [A | b] (last row implicit): the hot chain
//     kernel with one more wave for the bias column;
//   * the walk that turns the carried vectors into all states: per chunk, h <- A_t h + b_t as a
//     matrix-vector product.  One wave owns one chunk.  A lane loads adjacent entries of a
//     row of A_t (four lanes share a row, sixteen rows are handled per pass), scales
//     them by the row's power-of-two shift, multiplies by the vector's mantissas and adds up
//     across the row's lanes.  The vector is kept as float mantissas with one exponent for
//     the whole vector; it goes from the lanes that own rows to the lanes that own columns
//     through a few words of LDS private to the wave.  Nothing but A_t, b_t (read once) and
//     h_t (written once) touches HBM, which bounds this kernel.
#include "goom_chain_fast.h"

namespace goom_chain {

namespace {



constexpr int kWalkWaves = 4; // chunks per workgroup

// TI: the same matrix at every step (a time-invariant recurrence): it is loaded and scaled once,
// and a step is a few multiply-adds per lane on registers.
//
// Four lanes share a row (eight adjacent entries each at d = 32, four at d = 16), so sixteen rows
// are handled per pass and the work that is done once per row (its shift, the bias, the new
// exponent) is repeated by few lanes.  Outputs leave through the transposed vector: after its trip
// through LDS lane i < d holds entry i and one store instruction writes the whole state.
template <int DP, bool TI> __global__ __launch_bounds__(kWalkWaves * 64) void affine_walk_kernel(ChainArgs a, long long nchains)
{
    typedef Comp<float> C;
    constexpr int EPL = DP >= 32 ? 8 : 4; // entries of a row per lane
    constexpr int LPR = DP / EPL;         // lanes that share a row
    constexpr int RPP = 64 / LPR;         // rows per pass
    constexpr int Q = DP / RPP;           // passes
    constexpr int NV = EPL / 2;           // 16-byte pieces (two entries each) of a lane's part of a row
    static_assert(LPR == 4 && Q >= 1 && Q * RPP == DP, "a row is shared by the four lanes of a quad");
    __shared__ __align__(16) float hvec_all[kWalkWaves][DP];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long long chain = (long long)blockIdx.x * kWalkWaves + wave;
    if (chain >= nchains) return; // whole wave; the kernel has no workgroup barrier
    float *hvec = hvec_all[wave];
    const int rsub = lane / LPR;
    const int c0 = EPL * (lane % LPR);
    const bool row_owner = (lane % LPR) == 0;
    const bool entry_owner = lane < DP; // after the transposition lane i < d also holds entry i

    const long long item = chain / a.chunks_launched;
    const long long chunk = chain % a.chunks_launched;
    const long long t0 = chunk * a.chunk_len;
    long long len = a.steps - t0;
    if (len > a.chunk_len) len = a.chunk_len;
    if (len <= 0) return;
    // wave-uniform bases plus 32-bit lane offsets
    const unsigned char *left0 = a.left + item * a.left_batch_stride + t0 * a.left_step_stride;
    const unsigned char *bias0 = a.bias + (size_t)(item * a.steps + t0) * DP * 8;
    unsigned char *out0 = a.out_goom ? a.out_goom + (size_t)(item * a.steps + t0) * DP * 8 : nullptr;
    float *scaled0 = a.out_scaled ? a.out_scaled + (size_t)(item * a.steps + t0) * DP : nullptr;
    float *logscale0 = a.out_logscale ? a.out_logscale + (size_t)(item * a.steps + t0) : nullptr;
    const unsigned mat_off = (unsigned)(rsub * DP + c0) * 8u; // bytes: the lane's part of row rsub
    const unsigned bias_off = (unsigned)rsub * 8u;
    const unsigned ent_off = (unsigned)(lane & (DP - 1));

    // starting vector: zero, or column 0 of a factored carry
    float hm[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) hm[e] = 0.0f;
    double eh = 0.0;
    if (a.init_mode == 1) {
        long long iidx = item * a.chunks_per_item + chunk;
        if (a.init_group > 0) {
            long long grp = chunk / a.init_group;
            if (grp >= a.init_ngroups) grp = a.init_ngroups - 1;
            iidx = (item * a.init_ngroups + grp) * (a.init_group + 1) + (chunk - grp * a.init_group);
        }
        const unsigned char *ip = a.init + iidx * a.init_stride;
        const float *mp = reinterpret_cast<const float *>(ip);
        eh = *reinterpret_cast<const double *>(ip + (size_t)DP * a.fact_cols * sizeof(float));
        bool nz = false;
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            hm[e] = mp[(size_t)(c0 + e) * a.fact_cols];
            nz = nz || hm[e] != 0.0f;
        }
        // a zero vector carries no meaningful exponent
        if (__builtin_amdgcn_ballot_w64(nz) == 0 || !(__builtin_fabs(eh) < 1.0e15)) eh = 0.0;
    }

    f4 cur[Q][NV], nxt[Q][NV];
    float2 bcur[Q], bnxt[Q];
    auto load_matrix = [&](long long t, f4 (&it)[Q][NV]) {
        const unsigned char *src = left0 + t * a.left_step_stride;
#pragma unroll
        for (int q = 0; q < Q; ++q)
#pragma unroll
            for (int v = 0; v < NV; ++v)
                it[q][v] = *reinterpret_cast<const f4 *>(src + (mat_off + (unsigned)(q * RPP * DP * 8 + 16 * v)));
    };
    auto load_bias = [&](long long t, float2 (&bb)[Q]) {
        const unsigned char *bsrc = bias0 + (size_t)t * DP * 8;
#pragma unroll
        for (int q = 0; q < Q; ++q) bb[q] = *reinterpret_cast<const float2 *>(bsrc + (bias_off + (unsigned)(q * RPP * 8)));
    };
    const float kHi = 1.44269502162933349609375f; // float nearest log2(e)
    const float kLo = 1.925963033500011e-8f;      // log2(e) - kHi
    // the lane's entries of every row, scaled by the row's power of two and signed; the row shifts
    float sv[Q][EPL], nrow[Q];
    auto scale_rows = [&](const f4 (&it)[Q][NV]) {
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            float re[EPL], im[EPL];
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                re[2 * v] = it[q][v][0];
                im[2 * v] = it[q][v][1];
                re[2 * v + 1] = it[q][v][2];
                im[2 * v + 1] = it[q][v][3];
            }
            // row shift: a whole number near the row's largest log2|A_ij|
            float u = re[0];
#pragma unroll
            for (int e = 1; e < EPL; ++e) u = vmax_raw(u, re[e]);
            int key = C::key_of(u * kHi);
            key = C::imax(key, C::dpp<0xB1>(key));
            key = C::imax(key, C::dpp<0x4E>(key));
            const float mx = C::of_key(key);
            const bool zero_row = !(mx > -1.0e30f);
            const float n = zero_row ? 0.0f : __builtin_ceilf(mx);
            const float nsub = zero_row ? __builtin_huge_valf() : n;
            nrow[q] = n;
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                // exponent argument with one rounding at its own (small) magnitude, then the low part of log2(e)
                float t = __builtin_fmaf(re[e], kHi, -nsub);
                t = __builtin_fmaf(re[e], kLo, t);
                const float v = __builtin_amdgcn_exp2f(t); // 2^-inf = 0 covers zero entries and zero rows
                const float kf = __builtin_fmaf(im[e], 0.318309886183790671538f, 12582912.0f);
                sv[q][e] = __builtin_bit_cast(float, __builtin_bit_cast(int, v) ^ (__builtin_bit_cast(int, kf) << 31));
            }
        }
    };
    load_matrix(0, cur);
    load_bias(0, bcur);
    if (TI) scale_rows(cur);

    // A step's outputs are stored at the top of the next step, behind that step's loads: the wait for
    // those loads then finds the stores a whole step old, not just issued (loads and stores share
    // one counter of outstanding operations).
    float2 pend_goom = {0.0f, 0.0f};
    float pend_scaled = 0.0f, pend_logscale = 0.0f;
    auto store_outputs = [&](long long t) {
        if (out0 && entry_owner) *reinterpret_cast<float2 *>(out0 + (size_t)t * DP * 8 + ent_off * 8u) = pend_goom;
        if (scaled0 && entry_owner) scaled0[(size_t)t * DP + ent_off] = pend_scaled;
        if (logscale0 && lane == 0) logscale0[t] = pend_logscale;
    };
    for (long long t = 0; t < len; ++t) {
        const long long tn = t + 1 < len ? t + 1 : len - 1;
        if (!TI) load_matrix(tn, nxt);
        load_bias(tn, bnxt);
        if (t > 0) store_outputs(t - 1);
        if (!TI) scale_rows(cur);
        const float eh_f = (float)eh;
        float val[Q], barg[Q];
        bool big = false;
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            float part = 0.0f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) part = __builtin_fmaf(sv[q][e], hm[e], part);
            part = add_dpp<0xB1>(part);
            part = add_dpp<0x4E>(part);
            // the row's entry of A_t h is part 2^(n + eh); the bias joins it on that scale
            float x = __builtin_fmaf(bcur[q].x, kHi, -(nrow[q] + eh_f));
            x = __builtin_fmaf(bcur[q].x, kLo, x);
            val[q] = part;
            barg[q] = x;
            big = big || x > 64.0f;
        }
        // should the vector have shrunk so far below the bias that the bias would overflow on
        // its scale, the vector is scaled down first (to nothing, if need be)
        float down = 0.0f;
        if (__builtin_amdgcn_ballot_w64(big) != 0) {
            float bmax = barg[0];
#pragma unroll
            for (int q = 1; q < Q; ++q) bmax = C::max_(bmax, barg[q]);
            bmax = C::template group_allmax<64>(bmax, bmax);
            down = C::max_(0.0f, __builtin_ceilf(bmax) - 64.0f);
            const int idown = -(int)C::clamp_shift(down);
#pragma unroll
            for (int q = 0; q < Q; ++q) val[q] = __builtin_ldexpf(val[q], idown);
        }
        float xmax = -1.0e30f;
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            const float bv = C::apply_sign(__builtin_amdgcn_exp2f(barg[q] - down), bcur[q].y);
            val[q] += bv;
            const float ex = val[q] != 0.0f ? C::exponent_of(val[q]) + nrow[q] : -1.0e30f;
            xmax = C::max_(xmax, ex);
        }
        // new exponent of the vector: the largest entry's; mantissas at most 1 in magnitude
        {
            int key = C::key_of(xmax);
            key = C::imax(key, C::dpp<0x141>(key));
            key = C::imax(key, C::dpp<0x140>(key));
            key = C::xor16_imax(key);
            key = C::xor32_imax(key);
            xmax = C::of_key(key);
        }
        const bool all_zero = !(xmax > -1.0e29f);
        const float xm = all_zero ? 0.0f : xmax;
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            const float m = __builtin_ldexpf(val[q], (int)C::clamp_shift(nrow[q] - xm));
            if (row_owner) hvec[q * RPP + rsub] = m;
        }
        eh = all_zero ? 0.0 : eh + (double)down + (double)xm;
        // rows to columns through the wave's own LDS words (a wave's LDS operations complete in order)
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int v = 0; v < EPL / 4; ++v) {
            const f4 h4 = *reinterpret_cast<const f4 *>(&hvec[c0 + 4 * v]);
#pragma unroll
            for (int e = 0; e < 4; ++e) hm[4 * v + e] = h4[e];
        }
        const float mine = hvec[ent_off];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        // the state is mantissas 2^eh
        if (out0) pend_goom = float2{C::out_re_f(mine, (float)eh), mine < 0.0f ? C::pi() : 0.0f};
        if (scaled0) {
            // eq. 21 on the factored vector: with c = log of the largest magnitude, exp(z_i - c + 2) is the
            // mantissa over the largest mantissa, times e^2; the vector's exponent only enters c
            float am = __builtin_fabsf(mine);
            am = C::template group_allmax<64>(am, am);
            pend_scaled = am > 0.0f ? mine * (7.38905609893065022723f / am) : 0.0f;
            if (logscale0) pend_logscale = am > 0.0f ? (float)(((double)C::log2_abs(am) + eh) * kLn2) : -__builtin_huge_valf();
        }
#pragma unroll
        for (int q = 0; q < Q; ++q) {
#pragma unroll
            for (int v = 0; v < NV; ++v)
                if (!TI) cur[q][v] = nxt[q][v];
            bcur[q] = bnxt[q];
        }
    }
    store_outputs(len - 1);

    if (a.out_fact_final) {
        // the chunk's vector as column bias_col of the chunk's factored total, with its own exponent
        unsigned char *dst = a.out_fact_final + (item * a.chunks_per_item + chunk) * a.fact_stride;
        float *mp = reinterpret_cast<float *>(dst);
        double *ep = reinterpret_cast<double *>(dst + (size_t)DP * a.fact_cols * sizeof(float));
        if (rsub == 0) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) mp[(size_t)(c0 + e) * a.fact_cols + a.bias_col] = hm[e];
        }
        if (lane == 0) ep[a.bias_col] = eh;
    }
}

// Time-invariant recurrence: every chunk's total is [A^L | b*_c].  A^L has been written to the first
// chunk's slot of each batch item; this copies it to the other chunks and clears the padding columns
// (column d, the bias, is written by the walk kernel).
__global__ __launch_bounds__(256) void replicate_power_kernel(unsigned char *totals, long long stride, int fact_cols, int dp, int d,
                                                              long long chunks, long long chunks_per_item)
{
    const long long item = blockIdx.x / chunks, chunk = blockIdx.x % chunks;
    const unsigned char *src = totals + (item * chunks_per_item) * stride;
    unsigned char *dst = totals + (item * chunks_per_item + chunk) * stride;
    const float *sm = reinterpret_cast<const float *>(src);
    float *dm = reinterpret_cast<float *>(dst);
    const size_t mant = (size_t)dp * fact_cols * sizeof(float);
    const double *se = reinterpret_cast<const double *>(src + mant);
    double *de = reinterpret_cast<double *>(dst + mant);
    for (int e = threadIdx.x; e < dp * fact_cols; e += 256) {
        const int col = e % fact_cols;
        if (col < d) {
            if (chunk != 0) dm[e] = sm[e];
        } else if (col > d) {
            dm[e] = 0.0f;
        }
    }
    for (int col = threadIdx.x; col < fact_cols; col += 256) {
        if (col < d) {
            if (chunk != 0) de[col] = se[col];
        } else if (col > d) {
            de[col] = 0.0;
        }
    }
}

template <int DP, bool TI> int launch_walk(goom_ctx *ctx, const ChainArgs &args, long long nchains, const char *label)
{
    const long long grid = (nchains + kWalkWaves - 1) / kWalkWaves;
    if (grid <= 0) return GOOM_OK;
    if (grid > 0x7fffffffLL) return goom::fail(ctx, GOOM_EUNSUPPORTED, "too many chains for one launch (%lld)", nchains);
    goom::prof_begin(ctx, label);
    hipLaunchKernelGGL((affine_walk_kernel<DP, TI>), dim3((unsigned)grid), dim3(kWalkWaves * 64), 0, ctx->stream, args, nchains);
    goom::prof_end(ctx);
    return goom::check_hip(ctx, hipGetLastError(), "launch affine_walk_kernel");
}

} // namespace

// chunk products with the bias wave: the factor fills its tile, the state is [A* | b*] with the
// bias in column d, starting from the identity, and only the chunk's factored product is wanted
bool affine_chunk_applies(const ChainArgs &args, int dp)
{
    return (dp == 16 || dp == 32 || dp == 64) && args.n == dp && args.d == dp && args.m == dp + 1 && args.bias_mode == 1 &&
           args.bias_col == dp && args.init_mode == 0 && args.out_goom == nullptr && args.out_fact_steps == nullptr &&
           args.out_fact_final != nullptr && args.fact_cols == dp + 16;
}

int dispatch_affine_chunk(goom_ctx *ctx, const ChainArgs &args, int dp, long long grid, const char *label)
{
    switch (dp) {
    case 16: return launch_fast<16, 1, true>(ctx, args, grid, label);
    case 32: return launch_fast<32, 2, true>(ctx, args, grid, label);
    default: return launch_fast<64, 4, true>(ctx, args, grid, label);
    }
}

// the walk: a single state column that receives the bias, started from factored carries (or from
// zero), every state stored as GOOMs and / or the last one as a column of the chunk's factored total
bool affine_walk_applies(const ChainArgs &args, int dp)
{
    return (dp == 16 || dp == 32) && args.n == dp && args.d == dp && args.m == 1 && args.bias_mode == 1 &&
           (args.init_mode == 1 || args.init_mode == 3) &&
           (args.out_goom != nullptr || args.out_fact_final != nullptr || args.out_scaled != nullptr) &&
           !args.out_goom_last_only && args.out_fact_steps == nullptr &&
           ((args.out_goom == nullptr && args.out_scaled == nullptr) || args.bias_col == 0);
}

int dispatch_affine_walk(goom_ctx *ctx, const ChainArgs &args, int dp, long long nchains, const char *label)
{
    const bool ti = args.left_step_stride == 0;
    if (dp == 16) return ti ? launch_walk<16, true>(ctx, args, nchains, label) : launch_walk<16, false>(ctx, args, nchains, label);
    return ti ? launch_walk<32, true>(ctx, args, nchains, label) : launch_walk<32, false>(ctx, args, nchains, label);
}

int launch_replicate_power(goom_ctx *ctx, void *totals, long long stride, int fact_cols, int dp, int d, long long batch,
                           long long chunks, long long chunks_per_item)
{
    const long long grid = batch * chunks;
    if (grid <= 0) return GOOM_OK;
    if (grid > 0x7fffffffLL) return goom::fail(ctx, GOOM_EUNSUPPORTED, "too many chunks for one launch");
    hipLaunchKernelGGL(replicate_power_kernel, dim3((unsigned)grid), dim3(256), 0, ctx->stream, static_cast<unsigned char *>(totals), stride,
                       fact_cols, dp, d, chunks, chunks_per_item);
    return goom::check_hip(ctx, hipGetLastError(), "launch replicate_power_kernel");
}

} // namespace goom_chain
