// Chains of 8 x 8 and 16 x 16 matrices (float components, left factors as GOOMs; the small end of the
// sizes the paper scans in Section 4.1).  A factor is 512 bytes or 2 KB: what a step costs here is
// instructions, not bytes or matrix-unit time, so this kernel is the hot chain kernel stripped to its
// arithmetic for one 16 x 16 tile:
//   * one wave per workgroup and no workgroup barrier: the wave converts the factor into a 16 x 20 LDS
//     tile of its own, reads it back as the A operands of four 16 x 16 x 4 matrix instructions, and keeps
//     the state in the four accumulator registers that are the next step's B operands;
//   * a lane converts four adjacent entries of a row (four lanes share a row: two lane exchanges for the
//     row's maximum); pointers advance by a constant per step;
//   * 8 x 8 chains travel in pairs: the tile is block diagonal, chain 2 w in rows and columns 0..7 and
//     chain 2 w + 1 in 8..15, and so is the state, so one wave's instructions serve both;
//   * as in the larger kernel the product is not rescaled after a step: the row exponents go into the
//     next factor's exponent arguments, columns are renormalised every fourth step.
// Starts from the identity or from factored states, writes every prefix as GOOMs and / or the chain's
// factored product; other combinations stay with the general kernels.
#include "goom_chain_fast.h"

namespace goom_chain {

namespace {

constexpr int kSmallLDA = 20;

template <int D, bool OUT> __global__ __launch_bounds__(64, 6) void small_chain_kernel(ChainArgs a, long long nchains)
{
    typedef Comp<float> C;
    constexpr int PACK = D == 8 ? 2 : 1;
    __shared__ __align__(16) float tile[16 * kSmallLDA];
    __shared__ __align__(16) float nsh[16];

    const int lane = threadIdx.x;
    const int g = lane >> 4, c = lane & 15;
    const int crow = lane >> 2, c4 = 4 * (lane & 3); // the lane's part of the tile when converting
    const long long chain0 = (long long)blockIdx.x * PACK;

    // ---- the chain this lane converts for (rows 8..15 of a packed tile belong to the second chain)
    const int csel = PACK == 2 ? crow >> 3 : 0;
    const bool cvalid = PACK == 1 || (c4 >> 3) == csel; // inside the diagonal block
    const int lrow = crow - 8 * csel, lcol = c4 - 8 * csel;
    const long long cchain = chain0 + csel;
    const bool cexists = cchain < nchains;
    long long clen = 0;
    const unsigned char *src = a.left;
    if (cexists) {
        const long long item = cchain / a.chunks_launched, chunk = cchain % a.chunks_launched;
        const long long t0 = chunk * a.chunk_len;
        clen = a.steps - t0;
        if (clen > a.chunk_len) clen = a.chunk_len;
        src = a.left + item * a.left_batch_stride + t0 * a.left_step_stride + ((size_t)lrow * D + lcol) * 8;
    }
    // ---- the chain whose state this lane holds: rows 4 g + v, column c of the tile
    const int ssel = PACK == 2 ? c >> 3 : 0;
    const bool svalid = PACK == 1 || (g >> 1) == ssel;
    const int scol = c - 8 * ssel, srow0 = 4 * g - 8 * ssel; // local column, first local row (valid lanes)
    const long long schain = chain0 + ssel;
    const bool sexists = schain < nchains;
    long long sitem = 0, schunk = 0, st0 = 0, slen = 0;
    if (sexists) {
        sitem = schain / a.chunks_launched;
        schunk = schain % a.chunks_launched;
        st0 = schunk * a.chunk_len;
        slen = a.steps - st0;
        if (slen > a.chunk_len) slen = a.chunk_len;
    }
    const long long sglobal = sitem * a.chunks_per_item + schunk;
    // steps of the wave: the longer of its chains (a shorter one is fed identity blocks at the end)
    long long len = clen;
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) {
        const long long o = __shfl_xor(len, s, 64);
        len = o > len ? o : len;
    }
    if (len <= 0) return;

    // ---- initial state
    float st[4];
    double ecol = 0.0;
    const size_t fact_mant_bytes = (size_t)16 * a.fact_cols * sizeof(float);
    // row of the chain's own 16 x 16 (padded) factored matrix that tile row 4 g + v maps to
    auto slot_row = [&](int v) { return (4 * g + v + 8 * ssel) & 15; };
    if (a.init_mode == 1 && sexists) {
        long long iidx = sglobal;
        if (a.init_group > 0) {
            long long grp = schunk / a.init_group;
            if (grp >= a.init_ngroups) grp = a.init_ngroups - 1;
            iidx = (sitem * a.init_ngroups + grp) * (a.init_group + 1) + (schunk - grp * a.init_group);
        }
        const unsigned char *ip = a.init + iidx * a.init_stride;
        const float *mp = reinterpret_cast<const float *>(ip);
#pragma unroll
        for (int v = 0; v < 4; ++v) st[v] = svalid ? mp[(size_t)slot_row(v) * a.fact_cols + scol] : 0.0f;
        ecol = reinterpret_cast<const double *>(ip + fact_mant_bytes)[scol];
    } else {
#pragma unroll
        for (int v = 0; v < 4; ++v) st[v] = (4 * g + v == c) ? 1.0f : 0.0f; // identity (block diagonal as it is)
    }

    float2 *outp = nullptr;
    if (OUT && sexists && svalid) outp = reinterpret_cast<float2 *>(a.out_goom) + ((size_t)(sitem * a.steps + st0) * D + srow0) * D + scol;

    // Factors wait in registers kAhead steps before they are used: with so little to do per step it is the
    // number of loads in flight, not their size, that hides the memory latency.  A load is issued only by
    // lanes that have one; what the others (outside the diagonal blocks, or past the end of a chain that is
    // shorter than its partner: the identity) contribute is substituted when the value is used, so no lane
    // writes a register that a load is still due to fill.
    constexpr int kAhead = 4;
    f4 xa[kAhead], xb[kAhead];
    auto load = [&](long long t, f4 &x0, f4 &x1) {
        if (cvalid && t < clen) {
            const f4 *p = reinterpret_cast<const f4 *>(src);
            x0 = p[0];
            x1 = p[1];
            src += a.left_step_stride;
        }
    };
    const float ninf = -__builtin_huge_valf();
    const bool mine = cvalid && cexists;
    const float syn[4] = {(mine && lrow == lcol) ? 0.0f : ninf, (mine && lrow == lcol + 1) ? 0.0f : ninf,
                          (mine && lrow == lcol + 2) ? 0.0f : ninf, (mine && lrow == lcol + 3) ? 0.0f : ninf};
#pragma unroll
    for (int s = 0; s < kAhead; ++s) {
        xa[s] = f4{0.f, 0.f, 0.f, 0.f};
        xb[s] = f4{0.f, 0.f, 0.f, 0.f};
        load(s, xa[s], xb[s]);
    }
    f4 rj = {0.f, 0.f, 0.f, 0.f}; // row exponents the state still carries, for this lane's four columns
    const float kHi = 1.44269502162933349609375f; // float nearest log2(e)
    const float kLo = 1.925963033500011e-8f;      // log2(e) - kHi
    f4 acc = {0.f, 0.f, 0.f, 0.f};
    f4 nv = {0.f, 0.f, 0.f, 0.f};

    for (long long tb = 0; tb < len; tb += kAhead) {
#pragma unroll
    for (int slot = 0; slot < kAhead; ++slot) { // (unrolled: the register slot of a step is known at compile time)
        const long long t = tb + slot;
        if (t >= len) break;
        // ---------------------------------------------------------------- factor -> tile
        const bool live = cvalid && t < clen;
        const float re[4] = {live ? xa[slot][0] : syn[0], live ? xa[slot][2] : syn[1], live ? xb[slot][0] : syn[2], live ? xb[slot][2] : syn[3]};
        const float im[4] = {live ? xa[slot][1] : 0.0f, live ? xa[slot][3] : 0.0f, live ? xb[slot][1] : 0.0f, live ? xb[slot][3] : 0.0f};
        load(t + kAhead, xa[slot], xb[slot]);
        float u = __builtin_fmaf(re[0], kHi, rj[0]);
#pragma unroll
        for (int e = 1; e < 4; ++e) u = vmax_raw(u, __builtin_fmaf(re[e], kHi, rj[e]));
        int key = C::key_of(u);
        key = C::imax(key, C::dpp<0xB1>(key));
        key = C::imax(key, C::dpp<0x4E>(key));
        const float mx = C::of_key(key);
        const bool zero_row = !(mx > -1.0e30f);
        const float n = zero_row ? -1.0e30f : __builtin_ceilf(mx);
        const float nsub = zero_row ? __builtin_huge_valf() : n;
        f4 y;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float tt = __builtin_fmaf(re[e], kHi, rj[e] - nsub);
            tt = __builtin_fmaf(re[e], kLo, tt);
            const float v = __builtin_amdgcn_exp2f(tt);
            const float kf = __builtin_fmaf(im[e], 0.318309886183790671538f, 12582912.0f);
            y[e] = __builtin_bit_cast(float, __builtin_bit_cast(int, v) | (__builtin_bit_cast(int, kf) << 31));
        }
        *reinterpret_cast<f4 *>(&tile[crow * kSmallLDA + c4]) = y;
        nsh[crow] = n;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        // ---------------------------------------------------------------- product
        const f4 av = *reinterpret_cast<const f4 *>(&tile[c * kSmallLDA + 4 * g]);
        nv = *reinterpret_cast<const f4 *>(&nsh[4 * g]);
        rj = *reinterpret_cast<const f4 *>(&nsh[c4]);
        acc = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int v = 0; v < 4; ++v) acc = C::mfma(av[v], st[v], acc);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        // ---------------------------------------------------------------- outputs: entry (i, col) is acc 2^(n_i + ecol)
        if (OUT && outp && t < slen) {
            const float ecol_f = (float)ecol;
#pragma unroll
            for (int v = 0; v < 4; ++v) outp[v * D] = float2{C::out_re_f(acc[v], nv[v] + ecol_f), acc[v] < 0.0f ? C::pi() : 0.0f};
            outp += D * D;
        }
        // ---------------------------------------------------------------- state: raw; columns renormalised now and then
#pragma unroll
        for (int v = 0; v < 4; ++v) st[v] = acc[v];
        if (slot == kAhead - 1 && t + 1 < len) {
            float cm = -300.0f;
#pragma unroll
            for (int v = 0; v < 4; ++v) cm = C::max_(cm, C::exponent_of(st[v]));
            cm = C::xor16_32_max(cm);
            const int sh = -(int)cm;
#pragma unroll
            for (int v = 0; v < 4; ++v) st[v] = __builtin_ldexpf(st[v], sh);
            ecol += (double)cm;
        }
    }
    }

    if (a.out_fact_final) {
        // row exponents of the last step folded in; all columns of a chain on one exponent (the product
        // becomes a left factor); the padding of the chain's 16 x 16 slot is written as zeros
        float cm = C::neg_inf();
#pragma unroll
        for (int v = 0; v < 4; ++v) cm = C::max_(cm, C::exponent_of(st[v]) + nv[v]);
        cm = C::xor16_32_max(cm);
        float amax = 0.0f;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            st[v] = __builtin_ldexpf(st[v], (int)C::clamp_shift(nv[v] - cm));
            amax = C::max_(amax, __builtin_fabsf(st[v]));
        }
        amax = C::xor16_32_max(amax);
        ecol += (double)cm;
        double ev = amax > 0.0f ? ecol : kNegBig;
#pragma unroll
        for (int s = 1; s < (PACK == 2 ? 8 : 16); s <<= 1) {
            const double o = shfl_xor_double(ev, s);
            ev = o > ev ? o : ev;
        }
        const double emax = ev == kNegBig ? 0.0 : ev;
        double dsh = ecol - emax;
        dsh = dsh > -4000.0 ? dsh : -4000.0;
        const int shift = amax > 0.0f ? (int)dsh : 0;
        if (sexists) {
            unsigned char *dst = a.out_fact_final + sglobal * a.fact_stride;
            float *mp = reinterpret_cast<float *>(dst);
            double *ep = reinterpret_cast<double *>(dst + fact_mant_bytes);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                mp[(size_t)slot_row(v) * a.fact_cols + scol] = __builtin_ldexpf(st[v], shift);
                if (PACK == 2) mp[(size_t)slot_row(v) * a.fact_cols + scol + 8] = 0.0f;
            }
            if (g == 0) {
                ep[scol] = emax;
                if (PACK == 2) ep[scol + 8] = 0.0;
            }
        }
    }
}

template <int D, bool OUT> int launch_small(goom_ctx *ctx, const ChainArgs &args, long long nchains, const char *label)
{
    constexpr int PACK = D == 8 ? 2 : 1;
    const long long grid = (nchains + PACK - 1) / PACK;
    if (grid <= 0) return GOOM_OK;
    if (grid > 0x7fffffffLL) return goom::fail(ctx, GOOM_EUNSUPPORTED, "too many chains for one launch (%lld)", nchains);
    goom::prof_begin(ctx, label);
    hipLaunchKernelGGL((small_chain_kernel<D, OUT>), dim3((unsigned)grid), dim3(64), 0, ctx->stream, args, nchains);
    goom::prof_end(ctx);
    return goom::check_hip(ctx, hipGetLastError(), "launch small_chain_kernel");
}

} // namespace

bool small_applies(const ChainArgs &args, int dp)
{
    // (dp above 16: a wider state elsewhere in the same scan fixes the layout of the factored matrices)
    return dp == 16 && (args.d == 8 || args.d == 16) && args.n == args.d && args.m == args.d && args.bias_mode == 0 && args.out_fact_steps == nullptr &&
           (args.init_mode == 0 || args.init_mode == 1) && !args.out_goom_last_only && args.out_scaled == nullptr && !args.left_real &&
           (args.out_goom != nullptr || args.out_fact_final != nullptr) && (args.out_fact_final == nullptr || args.fact_cols >= 16);
}

int dispatch_small(goom_ctx *ctx, const ChainArgs &args, long long nchains, const char *label)
{
    if (args.d == 8) return args.out_goom ? launch_small<8, true>(ctx, args, nchains, label) : launch_small<8, false>(ctx, args, nchains, label);
    return args.out_goom ? launch_small<16, true>(ctx, args, nchains, label) : launch_small<16, false>(ctx, args, nchains, label);
}

} // namespace goom_chain
