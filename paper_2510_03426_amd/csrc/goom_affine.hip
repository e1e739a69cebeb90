// Linear recurrence with bias, h_t = A_t h_{t-1} + b_t over GOOMs (paper Section 4.3), float
// components: the two kernels its long batched form spends its time in.
//
//   * chunk products of the augmented matrices [A | b] (last row implicit): the hot chain
//     kernel with one more wave for the bias column; for d = 16 and 32 in a variant whose running
//     product is held in double and multiplied on the double-precision matrix instruction.  A
//     product of many matrices is all but rank one, and a float product carries its rounding
//     error relative to its norm: applied to a carried vector that happens to lie nearly
//     orthogonal to the product's dominant input direction, that error is magnified without
//     bound.  With double products (and double carries) what reaches the states is the rounding
//     of the last walk alone, as in a sequential float evaluation;
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
// ADJ: the adjoint recurrence's factors, read from the forward pass's matrices: step s takes the transpose of matrix
// steps - s (eight 8-byte loads a pass instead of four 16-byte ones; a load instruction of the wave still covers
// whole 128-byte lines) and adds left_shift[s] to its log-magnitudes.
// IOS (with TI): io_shift[s], a whole number c_s per step: the bias enters as bias[s] e^(-c_s) and the state leaves as h_s e^(c_s),
// both formed in double beside the vector's exponent (an adjoint recurrence, whose states are e^-1000 and below, fed and
// read through float GOOMs of ordinary size).
template <int DP, bool TI, bool ADJ = false, bool IOS = false> __global__ __launch_bounds__(kWalkWaves * 64) void affine_walk_kernel(ChainArgs a, long long nchains)
{
    typedef Comp<float> C;
    constexpr int EPL = DP / 4;           // entries of a row per lane (d = 64: one matrix for all steps only, it stays in registers)
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
    [[maybe_unused]] const float *ios0 = IOS ? a.io_shift + (item * a.steps + t0) : nullptr;
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
    bool vec_zero = true; // wave-uniform: every mantissa is zero
    if (a.init_mode == 1) {
        long long iidx = item * a.chunks_per_item + chunk;
        if (a.init_group > 0) {
            long long grp = chunk / a.init_group;
            if (grp >= a.init_ngroups) grp = a.init_ngroups - 1;
            iidx = (item * a.init_ngroups + grp) * (a.init_group + 1) + (chunk - grp * a.init_group);
        }
        const unsigned char *ip = a.init + iidx * a.init_stride;
        bool nz = false;
        if (a.fact_f64) { // carries with double mantissas (scaled to at most 1 in magnitude, so the conversion is safe)
            const double *mp = reinterpret_cast<const double *>(ip);
            eh = *reinterpret_cast<const double *>(ip + (size_t)DP * a.fact_cols * sizeof(double));
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                hm[e] = (float)mp[(size_t)(c0 + e) * a.fact_cols];
                nz = nz || hm[e] != 0.0f;
            }
        } else {
            const float *mp = reinterpret_cast<const float *>(ip);
            eh = *reinterpret_cast<const double *>(ip + (size_t)DP * a.fact_cols * sizeof(float));
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                hm[e] = mp[(size_t)(c0 + e) * a.fact_cols];
                nz = nz || hm[e] != 0.0f;
            }
        }
        // a zero vector carries no meaningful exponent
        vec_zero = __builtin_amdgcn_ballot_w64(nz) == 0;
        if (vec_zero || !(__builtin_fabs(eh) < 1.0e15)) eh = 0.0;
    }

    f4 cur[Q][NV], nxt[Q][NV];
    float2 bcur[Q], bnxt[Q];
    [[maybe_unused]] float shift_cur = 0.0f, shift_nxt = 0.0f;
    [[maybe_unused]] const unsigned char *adj0 = a.left + item * a.left_batch_stride;
    [[maybe_unused]] const float *shift0 = ADJ ? a.left_shift + item * a.steps : nullptr;
    [[maybe_unused]] const unsigned adj_off = (unsigned)(c0 * DP + rsub) * 8u; // bytes: entry (c0, rsub) of the source matrix
    auto load_matrix = [&](long long t, f4 (&it)[Q][NV], float &shift) {
        if constexpr (ADJ) {
            const long long s = t0 + t, k = s > 0 ? a.steps - s : a.steps - 1; // (step 0: any matrix, shifted to nothing)
            const unsigned char *src = adj0 + k * a.left_step_stride;
            shift = shift0[s];
#pragma unroll
            for (int q = 0; q < Q; ++q)
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    // entries (row, c0 + 2 v) and (row, c0 + 2 v + 1) of the transpose, row = q RPP + rsub
                    const float2 x = *reinterpret_cast<const float2 *>(src + (adj_off + (unsigned)(((2 * v) * DP + q * RPP) * 8)));
                    const float2 y = *reinterpret_cast<const float2 *>(src + (adj_off + (unsigned)(((2 * v + 1) * DP + q * RPP) * 8)));
                    it[q][v] = f4{x.x, x.y, y.x, y.y};
                }
        } else {
            const unsigned char *src = left0 + t * a.left_step_stride;
#pragma unroll
            for (int q = 0; q < Q; ++q)
#pragma unroll
                for (int v = 0; v < NV; ++v)
                    it[q][v] = *reinterpret_cast<const f4 *>(src + (mat_off + (unsigned)(q * RPP * DP * 8 + 16 * v)));
        }
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
    auto scale_rows = [&](const f4 (&it)[Q][NV], float shift) {
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            float re[EPL], im[EPL];
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                re[2 * v] = ADJ ? it[q][v][0] + shift : it[q][v][0];
                im[2 * v] = it[q][v][1];
                re[2 * v + 1] = ADJ ? it[q][v][2] + shift : it[q][v][2];
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
                float v;
                if (TI) {
                    // converted once and applied at every step: its rounding is the same at every step and adds up
                    // along the chain, so the one conversion is made in double and rounded once
                    v = zero_row ? 0.0f : (float)Comp<double>::exp2_shifted((double)re[e], (double)n);
                } else {
                    float t = __builtin_fmaf(re[e], kHi, -nsub);
                    t = __builtin_fmaf(re[e], kLo, t);
                    v = __builtin_amdgcn_exp2f(t); // 2^-inf = 0 covers zero entries and zero rows
                }
                const float kf = __builtin_fmaf(im[e], 0.318309886183790671538f, 12582912.0f);
                sv[q][e] = __builtin_bit_cast(float, __builtin_bit_cast(int, v) | (__builtin_bit_cast(int, kf) << 31));
            }
        }
    };
    load_matrix(0, cur, shift_cur);
    load_bias(0, bcur);
    if (TI) scale_rows(cur, 0.0f);

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
        if (!TI) load_matrix(tn, nxt, shift_nxt);
        load_bias(tn, bnxt);
        if (t > 0) store_outputs(t - 1);
        if (!TI) scale_rows(cur, shift_cur);
        [[maybe_unused]] const double cs = IOS ? (double)ios0[t] * 1.44269504088896340736 : 0.0; // c_s in powers of two
        if (vec_zero) {
            // a zero vector has no scale of its own: it takes the bias's, whatever its magnitude (an adjoint
            // recurrence starts at e^-1000 and below), instead of flushing the bias on the scale 2^0
            float m = -__builtin_huge_valf();
#pragma unroll
            for (int q = 0; q < Q; ++q) m = C::max_(m, __builtin_fmaf(bcur[q].x, kHi, -nrow[q]));
            m = C::template group_allmax<64>(m, m);
            if (IOS)
                eh = (m > -1.0e30f && m < 1.0e30f) ? __builtin_ceil((double)m - cs) : 0.0; // (the vector's exponent stays a whole number)
            else
                eh = (m > -1.0e30f && m < 1.0e30f) ? (double)__builtin_ceilf(m) : 0.0;
        }
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
            float x;
            if (IOS) { // the shift and the vector's exponent are large and nearly cancel: in double
                x = (float)__builtin_fma((double)bcur[q].x, 1.44269504088896340736, -(cs + (double)nrow[q] + eh));
            } else {
                x = __builtin_fmaf(bcur[q].x, kHi, -(nrow[q] + eh_f));
                x = __builtin_fmaf(bcur[q].x, kLo, x);
            }
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
        vec_zero = all_zero;
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
        if (out0) pend_goom = float2{C::out_re_f(mine, IOS ? (float)(eh + cs) : (float)eh), mine < 0.0f ? C::pi() : 0.0f};
        if (scaled0) {
            // the scaled exponentiation (Section 4.3, eq. 27) on the factored vector: with c = log of the largest magnitude, exp(z_i - c + 2) is the
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
        shift_cur = shift_nxt;
    }
    store_outputs(len - 1);

    if (a.out_fact_final) {
        // the chunk's vector as column bias_col of the chunk's factored total, with its own exponent
        unsigned char *dst = a.out_fact_final + (item * a.chunks_per_item + chunk) * a.fact_stride;
        if (a.fact_f64) {
            double *mp = reinterpret_cast<double *>(dst);
            double *ep = reinterpret_cast<double *>(dst + (size_t)DP * a.fact_cols * sizeof(double));
            if (rsub == 0) {
#pragma unroll
                for (int e = 0; e < EPL; ++e) mp[(size_t)(c0 + e) * a.fact_cols + a.bias_col] = (double)hm[e];
            }
            if (lane == 0) ep[a.bias_col] = eh;
        } else {
            float *mp = reinterpret_cast<float *>(dst);
            double *ep = reinterpret_cast<double *>(dst + (size_t)DP * a.fact_cols * sizeof(float));
            if (rsub == 0) {
#pragma unroll
                for (int e = 0; e < EPL; ++e) mp[(size_t)(c0 + e) * a.fact_cols + a.bias_col] = hm[e];
            }
            if (lane == 0) ep[a.bias_col] = eh;
        }
    }
}


// Chunk products [A* | b*] with the running product in double (float GOOM factors, double factored result).
// The factor is exponentiated into a float LDS tile exactly as in the hot kernel; A operands are widened when
// they are read.  The double-precision 16 x 16 x 4 instruction leaves rows 4 v + g of a column in register v of
// lane group g and takes row g of its B operand from lane group g, so the accumulators are again the next
// step's B operands if contraction index 16 kt + 4 v + g sits at position 16 kt + 4 g + v of a tile row
// (Comp<double>::phys); the row exponents and the bias wave's column are stored in the same order.
// a.bias == NULL: no bias is added (the column stays zero), which gives plain matrix powers and products.
// PRECISE: every entry of the tile is exponentiated in double and rounded once (for one matrix applied at every
// step, whose conversion error would otherwise be the same at every step and add up along the chain).
// ADJ: as in the matrix-vector walk above (the factor of step s is the transpose of matrix steps - s, shifted).
template <int DP, int NW, bool PRECISE, bool ADJ = false>
__global__ __launch_bounds__((NW + 1) * 64, 4) void affine_chunk_f64_kernel(ChainArgs a)
{
    typedef Comp<float> C;
    typedef Comp<double> CD;
    constexpr int KT = DP / 16;
    constexpr int LDA = DP + 4;
    constexpr int NWT = NW + 1;
    constexpr int NT = NW * 64;  // threads that convert the factor
    constexpr int LPR = DP / 4;  // lanes per row of the factor
    constexpr int NITEMS = DP * LPR;
    constexpr int Q = NITEMS / NT;
    constexpr int kRenormEvery = 4;
    static_assert(NITEMS % NT == 0 && NT % LPR == 0 && NW == KT, "tile does not divide among the threads");
    constexpr size_t kTileBytes = (size_t)DP * LDA * sizeof(float);
    constexpr size_t kBufBytes = kTileBytes + (size_t)DP * sizeof(float);

    extern __shared__ __align__(16) unsigned char smem[];
    auto tile_of = [&](int b) { return reinterpret_cast<float *>(smem + (size_t)b * kBufBytes); };
    auto nsh_of = [&](int b) { return reinterpret_cast<float *>(smem + (size_t)b * kBufBytes + kTileBytes); };
    double *wave_red = reinterpret_cast<double *>(smem + 2 * kBufBytes);
    double *wvec = reinterpret_cast<double *>(smem + 2 * kBufBytes + 128); // the bias wave's column, in tile column order

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4;
    const int c = lane & 15;
    const int col = wave * 16 + c;
    const int c4 = 4 * (tid % LPR);                      // first of this lane's four factor columns
    const int p4 = (c4 & ~15) | ((c4 >> 2) & 3);         // position of column c4 in a tile row; c4 + e sits 4 e further on
    const bool bias_wave = wave == NW;
    const bool converter = !bias_wave;
    const bool has_bias = a.bias != nullptr;
    constexpr int LPRB = 64 / DP; // bias wave: lanes per row
    constexpr int CPLB = DP / LPRB;
    const int brow = lane / LPRB;
    const int bc0 = CPLB * (lane % LPRB);

    const long long chain = blockIdx.x;
    const long long item = chain / a.chunks_launched;
    const long long chunk = chain % a.chunks_launched;
    const long long t0 = chunk * a.chunk_len;
    long long len = a.steps - t0;
    if (len > a.chunk_len) len = a.chunk_len;
    const long long chain_global = item * a.chunks_per_item + chunk;
    const unsigned char *left0 = a.left + item * a.left_batch_stride + t0 * a.left_step_stride;

    [[maybe_unused]] const unsigned char *adj0 = a.left + item * a.left_batch_stride;
    [[maybe_unused]] const float *shift0 = ADJ ? a.left_shift + item * a.steps : nullptr;
    [[maybe_unused]] float pre_shift = 0.0f; // the shift of the step whose entries wait in `pre`
    auto load_items = [&](long long t, Item4 (&it)[Q]) {
        if constexpr (ADJ) {
            const long long s = t0 + t, k = s > 0 ? a.steps - s : a.steps - 1; // (step 0: any matrix, shifted to nothing)
            const float *src = reinterpret_cast<const float *>(adj0 + k * a.left_step_stride);
            pre_shift = shift0[s];
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                const int row = (tid + q * NT) / LPR; // entries (row, c4 .. c4 + 3) of the transpose
                float2 x[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) x[e] = *reinterpret_cast<const float2 *>(src + ((size_t)(c4 + e) * DP + row) * 2);
                it[q].a = f4{x[0].x, x[0].y, x[1].x, x[1].y};
                it[q].b = f4{x[2].x, x[2].y, x[3].x, x[3].y};
            }
        } else {
            const float *src = reinterpret_cast<const float *>(left0 + t * a.left_step_stride);
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                const int row = (tid + q * NT) / LPR;
                const f4 *gp = reinterpret_cast<const f4 *>(src + ((size_t)row * DP + c4) * 2);
                it[q].a = gp[0];
                it[q].b = gp[1];
            }
        }
    };
    // tile[i][phys(j)] = (+-) 2^(log2|A_ij| + r_j - n_i), n_i = ceil(max_j (log2|A_ij| + r_j)); r_j: the row
    // exponents still attached to the running product (zero at the start)
    auto convert_items = [&](const Item4 (&it)[Q], int buf, const float *rsrc) {
        const float kHi = 1.44269502162933349609375f;
        const float kLo = 1.925963033500011e-8f;
        float *tile = tile_of(buf);
        float *nsh = nsh_of(buf);
        float rj[4] = {0.f, 0.f, 0.f, 0.f};
        if (rsrc) {
#pragma unroll
            for (int e = 0; e < 4; ++e) rj[e] = rsrc[p4 + 4 * e];
        }
        const float sh = ADJ ? pre_shift : 0.0f;
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            const int row = (tid + q * NT) / LPR;
            const float re[4] = {ADJ ? it[q].a[0] + sh : it[q].a[0], ADJ ? it[q].a[2] + sh : it[q].a[2], ADJ ? it[q].b[0] + sh : it[q].b[0],
                                 ADJ ? it[q].b[2] + sh : it[q].b[2]};
            const float im[4] = {it[q].a[1], it[q].a[3], it[q].b[1], it[q].b[3]};
            float u = __builtin_fmaf(re[0], kHi, rj[0]);
#pragma unroll
            for (int e = 1; e < 4; ++e) u = vmax_raw(u, __builtin_fmaf(re[e], kHi, rj[e]));
            int key = C::key_of(u);
            key = C::imax(key, C::dpp<0xB1>(key));
            if (LPR >= 4) key = C::imax(key, C::dpp<0x4E>(key));
            if (LPR >= 8) key = C::imax(key, C::dpp<0x141>(key));
            const float mx = C::of_key(key);
            const bool zero_row = !(mx > -1.0e30f);
            const float n = zero_row ? 0.0f : __builtin_ceilf(mx); // (the bias is scaled by the shift: it stays small for a zero row)
            const float nsub = zero_row ? __builtin_huge_valf() : n;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float v;
                if (PRECISE) {
                    v = zero_row ? 0.0f : (float)CD::exp2_shifted((double)re[e], (double)(n - rj[e]));
                } else {
                    float t = __builtin_fmaf(re[e], kHi, rj[e] - nsub);
                    t = __builtin_fmaf(re[e], kLo, t);
                    v = __builtin_amdgcn_exp2f(t);
                }
                const float kf = __builtin_fmaf(im[e], 0.318309886183790671538f, 12582912.0f);
                tile[row * LDA + p4 + 4 * e] = __builtin_bit_cast(float, __builtin_bit_cast(int, v) | (__builtin_bit_cast(int, kf) << 31));
            }
            nsh[CD::phys(row)] = n; // every lane of the row writes the same value
        }
    };

    // state: st[kt][v] = W[16 kt + 4 v + g][col]; identity at the start, the bias column zero
    double st[KT][4];
    double ecol = 0.0;
#pragma unroll
    for (int kt = 0; kt < KT; ++kt)
#pragma unroll
        for (int v = 0; v < 4; ++v) st[kt][v] = (a.init_mode == 0 && 16 * kt + 4 * v + g == col) ? 1.0 : 0.0;

    Item4 pre[Q];
    if (len > 0 && converter) {
        load_items(0, pre);
        convert_items(pre, 0, nullptr);
        if (len > 1) load_items(1, pre);
    }
    float2 bpre = {-__builtin_huge_valf(), 0.0f};
    auto load_bias = [&](long long t) {
        if (has_bias) bpre = *reinterpret_cast<const float2 *>(a.bias + ((size_t)(item * a.steps + t0 + t) * DP + brow) * 8);
    };
    if (bias_wave && lane < DP) wvec[lane] = 0.0;
    if (bias_wave && len > 0) load_bias(0);
    __syncthreads();

    for (long long t = 0; t < len; ++t) {
        const int cur = (int)(t & 1);
        const float *tile = tile_of(cur);
        const float *nsh = nsh_of(cur);
        const bool last = t == len - 1;

        d4 acc[KT];
        double accb = 0.0;
        if (bias_wave) {
            // column d of the product: row brow of the tile times the column, on the vector ALU
#pragma unroll
            for (int k = 0; k < CPLB / 4; ++k) {
                const f4 av = *reinterpret_cast<const f4 *>(&tile[brow * LDA + bc0 + 4 * k]);
#pragma unroll
                for (int e = 0; e < 4; ++e) accb = __builtin_fma((double)av[e], wvec[bc0 + 4 * k + e], accb);
            }
#pragma unroll
            for (int s = 1; s < LPRB; s <<= 1) accb += __shfl_xor(accb, s, 64);
        } else {
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) acc[mt] = d4{0, 0, 0, 0};
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) {
                f4 av[KT];
#pragma unroll
                for (int mt = 0; mt < KT; ++mt)
                    av[mt] = *reinterpret_cast<const f4 *>(&tile[(16 * mt + c) * LDA + 16 * kt + 4 * g]);
#pragma unroll
                for (int v = 0; v < 4; ++v)
#pragma unroll
                    for (int mt = 0; mt < KT; ++mt) acc[mt] = CD::mfma((double)av[mt][v], st[kt][v], acc[mt]);
            }
        }
        if (converter && !last) {
            convert_items(pre, cur ^ 1, nsh);
            load_items(t + 2 < len ? t + 2 : len - 1, pre);
        }
        float nrb = 0.0f;
        if (bias_wave) {
            // b_i enters entry (i, d) of the product, held as accb 2^(n_i + ecol): add (+-) 2^(log2|b_i| - n_i - ecol).
            // Should the column have shrunk so far below the bias that this would overflow, it is scaled down first.
            nrb = nsh[CD::phys(brow)];
            double xd = __builtin_fma((double)bpre.x, kLog2e, -((double)nrb + ecol)); // -inf for a zero entry or no bias
            if (__builtin_amdgcn_ballot_w64(accb != 0.0) == 0) {
                // a zero column has no scale of its own: it takes the bias's, whatever its magnitude
                float m = (float)xd;
                m = C::template group_allmax<64>(m, m);
                const double sh = (m > -1.0e30f && m < 1.0e30f) ? (double)__builtin_ceilf(m) : 0.0;
                ecol += sh;
                xd -= sh;
            }
            const float x = (float)xd;
            float down = 0.0f;
            if (__builtin_amdgcn_ballot_w64(x > 64.0f) != 0) {
                const float amax = C::template group_allmax<64>(x, x);
                down = C::max_(0.0f, __builtin_ceilf(amax) - 64.0f);
                accb = __builtin_ldexp(accb, -(int)C::clamp_shift(down));
                ecol += (double)down;
            }
            accb += (double)C::apply_sign(__builtin_amdgcn_exp2f(x - down), bpre.y);
            load_bias(t + 1 < len ? t + 1 : len - 1);
        }

        // state for the next step: the raw product (its row exponents n_i go to the next factor's columns),
        // columns renormalised every few steps; after the last step the row exponents are folded in
        if (bias_wave) {
            if (!last) {
                if ((t % kRenormEvery) == kRenormEvery - 1) {
                    float cm = accb != 0.0 ? (float)CD::frexp_exp(accb) : -1.0e30f;
                    cm = C::template group_allmax<64>(cm, cm);
                    if (!(cm > -1.0e29f)) cm = 0.0f; // a zero column keeps its exponent
                    accb = __builtin_ldexp(accb, -(int)cm);
                    ecol += (double)cm;
                }
            } else {
                float cm = accb != 0.0 ? (float)CD::frexp_exp(accb) + nrb : -1.0e30f;
                cm = C::template group_allmax<64>(cm, cm);
                if (!(cm > -1.0e29f)) cm = 0.0f; // a zero column
                accb = __builtin_ldexp(accb, (int)C::clamp_shift(nrb - cm));
                ecol += (double)cm;
            }
            if (lane % LPRB == 0) wvec[CD::phys(brow)] = accb;
        } else if (!last) {
#pragma unroll
            for (int mt = 0; mt < KT; ++mt)
#pragma unroll
                for (int v = 0; v < 4; ++v) st[mt][v] = acc[mt][v];
            if ((t % kRenormEvery) == kRenormEvery - 1) {
                float cm = -1.0e30f;
#pragma unroll
                for (int mt = 0; mt < KT; ++mt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) cm = C::max_(cm, st[mt][v] != 0.0 ? (float)CD::frexp_exp(st[mt][v]) : -1.0e30f);
                cm = C::xor16_32_max(cm);
                if (!(cm > -1.0e29f)) cm = 0.0f;
                const int sh = -(int)cm;
#pragma unroll
                for (int mt = 0; mt < KT; ++mt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) st[mt][v] = __builtin_ldexp(st[mt][v], sh);
                ecol += (double)cm;
            }
        } else {
            float cm = -1.0e30f;
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) {
                const f4 nv = *reinterpret_cast<const f4 *>(&nsh[16 * mt + 4 * g]); // nv[v]: row 16 mt + 4 v + g
#pragma unroll
                for (int v = 0; v < 4; ++v) cm = C::max_(cm, acc[mt][v] != 0.0 ? (float)CD::frexp_exp(acc[mt][v]) + nv[v] : -1.0e30f);
            }
            cm = C::xor16_32_max(cm);
            if (!(cm > -1.0e29f)) cm = 0.0f;
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) {
                const f4 nv = *reinterpret_cast<const f4 *>(&nsh[16 * mt + 4 * g]);
#pragma unroll
                for (int v = 0; v < 4; ++v) st[mt][v] = __builtin_ldexp(acc[mt][v], (int)C::clamp_shift(nv[v] - cm));
            }
            ecol += (double)cm;
        }
        __syncthreads();
    }

    if (a.out_fact_final) {
        // factored product of the chunk: double mantissas [DP][fact_cols], the columns of A* on one exponent (it
        // becomes a left factor), the bias column on its own
        unsigned char *dst = a.out_fact_final + chain_global * a.fact_stride;
        double *mp = reinterpret_cast<double *>(dst);
        double *ep = reinterpret_cast<double *>(dst + (size_t)DP * a.fact_cols * sizeof(double));
        double cmx = 0.0;
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int v = 0; v < 4; ++v) cmx = CD::max_(cmx, __builtin_fabs(st[kt][v]));
        cmx = CD::xor16_32_max(cmx);
        double ev = (cmx > 0.0 && !bias_wave) ? ecol : kNegBig;
#pragma unroll
        for (int s = 1; s < 16; s <<= 1) {
            const double o = shfl_xor_double(ev, s);
            ev = o > ev ? o : ev;
        }
        if (lane == 0) wave_red[wave] = ev;
        __syncthreads();
        double emax = kNegBig;
        for (int w = 0; w < NWT; ++w) emax = wave_red[w] > emax ? wave_red[w] : emax;
        if (emax == kNegBig) emax = 0.0;
        double dsh = ecol - emax;
        dsh = dsh > -4000.0 ? dsh : -4000.0;
        const int shift = (cmx > 0.0 && !bias_wave) ? (int)dsh : 0;
        if (bias_wave) {
            if (lane % LPRB == 0) mp[(size_t)brow * a.fact_cols + DP] = wvec[CD::phys(brow)];
            for (int idx = lane; idx < DP * 15; idx += 64) mp[(size_t)(idx / 15) * a.fact_cols + DP + 1 + idx % 15] = 0.0;
        } else {
#pragma unroll
            for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    mp[(size_t)(16 * kt + 4 * v + g) * a.fact_cols + col] = __builtin_ldexp(st[kt][v], shift);
        }
        if (g == 0) ep[col] = bias_wave ? ecol : emax;
    }
}

template <int DP, int NW, bool PRECISE, bool ADJ = false> int launch_chunk_f64(goom_ctx *ctx, const ChainArgs &args, long long grid, const char *label)
{
    constexpr int LDA = DP + 4;
    const size_t lds = 2 * ((size_t)DP * LDA * sizeof(float) + (size_t)DP * sizeof(float)) + 128 + DP * sizeof(double);
    if (grid <= 0) return GOOM_OK;
    if (grid > 0x7fffffffLL) return goom::fail(ctx, GOOM_EUNSUPPORTED, "too many chains for one launch (%lld)", grid);
    goom::prof_begin(ctx, label);
    hipLaunchKernelGGL((affine_chunk_f64_kernel<DP, NW, PRECISE, ADJ>), dim3((unsigned)grid), dim3((NW + 1) * 64), lds, ctx->stream, args);
    goom::prof_end(ctx);
    return goom::check_hip(ctx, hipGetLastError(), "launch affine_chunk_f64_kernel");
}

// Time-invariant recurrence: every chunk's total is [A^L | b*_c].  A^L has been written to the first
// chunk's slot of each batch item; this copies it to the other chunks and clears the padding columns
// (column d, the bias, is written by the walk kernel).
template <typename R> __global__ __launch_bounds__(256) void replicate_power_kernel(unsigned char *totals, long long stride, int fact_cols, int dp, int d,
                                                              long long chunks, long long chunks_per_item)
{
    const long long item = blockIdx.x / chunks, chunk = blockIdx.x % chunks;
    const unsigned char *src = totals + (item * chunks_per_item) * stride;
    unsigned char *dst = totals + (item * chunks_per_item + chunk) * stride;
    const R *sm = reinterpret_cast<const R *>(src);
    R *dm = reinterpret_cast<R *>(dst);
    const size_t mant = (size_t)dp * fact_cols * sizeof(R);
    const double *se = reinterpret_cast<const double *>(src + mant);
    double *de = reinterpret_cast<double *>(dst + mant);
    for (int e = threadIdx.x; e < dp * fact_cols; e += 256) {
        const int col = e % fact_cols;
        if (col < d) {
            if (chunk != 0) dm[e] = sm[e];
        } else if (col > d) {
            dm[e] = (R)0;
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

template <int DP, bool TI, bool ADJ = false, bool IOS = false> int launch_walk(goom_ctx *ctx, const ChainArgs &args, long long nchains, const char *label)
{
    const long long grid = (nchains + kWalkWaves - 1) / kWalkWaves;
    if (grid <= 0) return GOOM_OK;
    if (grid > 0x7fffffffLL) return goom::fail(ctx, GOOM_EUNSUPPORTED, "too many chains for one launch (%lld)", nchains);
    goom::prof_begin(ctx, label);
    hipLaunchKernelGGL((affine_walk_kernel<DP, TI, ADJ, IOS>), dim3((unsigned)grid), dim3(kWalkWaves * 64), 0, ctx->stream, args, nchains);
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
           args.out_fact_final != nullptr && args.fact_cols == dp + 16 && args.io_shift == nullptr; // (a rescaled bias: the general kernel)
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
    return (dp == 16 || dp == 32 || (dp == 64 && !args.left_shift)) && args.n == dp && args.d == dp && args.m == 1 &&
           args.bias_mode == 1 && (args.init_mode == 1 || args.init_mode == 3) &&
           (args.out_goom != nullptr || args.out_fact_final != nullptr || args.out_scaled != nullptr) &&
           !args.out_goom_last_only && args.out_fact_steps == nullptr &&
           ((args.out_goom == nullptr && args.out_scaled == nullptr) || args.bias_col == 0);
}

int dispatch_affine_walk(goom_ctx *ctx, const ChainArgs &args, int dp, long long nchains, const char *label)
{
    const bool ti = args.left_step_stride == 0;
    if (args.left_shift) { // the adjoint recurrence: transposed factors in reverse order (a step stride of 0: one matrix, shifted anew every step)
        return dp == 16 ? launch_walk<16, false, true>(ctx, args, nchains, label) : launch_walk<32, false, true>(ctx, args, nchains, label);
    }
    if (args.io_shift) { // bias and states rescaled step by step: over one matrix, GOOM or factored outputs
        if (!ti || args.out_scaled) return goom::fail(ctx, GOOM_EUNSUPPORTED, "rescaled bias and states in the matrix-vector walk: one matrix for all steps only");
        if (dp == 64) return launch_walk<64, true, false, true>(ctx, args, nchains, label);
        return dp == 16 ? launch_walk<16, true, false, true>(ctx, args, nchains, label) : launch_walk<32, true, false, true>(ctx, args, nchains, label);
    }
    if (dp == 64) return ti ? launch_walk<64, true>(ctx, args, nchains, label) : launch_walk<64, false>(ctx, args, nchains, label);
    if (dp == 16) return ti ? launch_walk<16, true>(ctx, args, nchains, label) : launch_walk<16, false>(ctx, args, nchains, label);
    return ti ? launch_walk<32, true>(ctx, args, nchains, label) : launch_walk<32, false>(ctx, args, nchains, label);
}

// the double-state chunk products: same conditions as affine_chunk_applies, the result in double (d = 16, 32)
int dispatch_affine_chunk_f64(goom_ctx *ctx, const ChainArgs &args, int dp, long long grid, const char *label)
{
    if (!((dp == 16 || dp == 32) && args.n == dp && args.d == dp && args.m == dp + 1 && args.init_mode == 0 && args.out_goom == nullptr &&
          args.out_fact_steps == nullptr && args.out_fact_final != nullptr && args.fact_cols == dp + 16))
        return goom::fail(ctx, GOOM_EUNSUPPORTED, "double-state chunk products are built for d = 16 and 32");
    if (args.left_shift) { // the adjoint recurrence: transposed factors in reverse order (a step stride of 0: one matrix, shifted anew every step)
        return dp == 16 ? launch_chunk_f64<16, 1, false, true>(ctx, args, grid, label) : launch_chunk_f64<32, 2, false, true>(ctx, args, grid, label);
    }
    if (args.left_step_stride == 0) // one matrix at every step
        return dp == 16 ? launch_chunk_f64<16, 1, true>(ctx, args, grid, label) : launch_chunk_f64<32, 2, true>(ctx, args, grid, label);
    return dp == 16 ? launch_chunk_f64<16, 1, false>(ctx, args, grid, label) : launch_chunk_f64<32, 2, false>(ctx, args, grid, label);
}

int launch_replicate_power(goom_ctx *ctx, void *totals, long long stride, int fact_cols, int dp, int d, long long batch,
                           long long chunks, long long chunks_per_item, bool f64)
{
    const long long grid = batch * chunks;
    if (grid <= 0) return GOOM_OK;
    if (grid > 0x7fffffffLL) return goom::fail(ctx, GOOM_EUNSUPPORTED, "too many chunks for one launch");
    if (f64)
        hipLaunchKernelGGL(replicate_power_kernel<double>, dim3((unsigned)grid), dim3(256), 0, ctx->stream, static_cast<unsigned char *>(totals),
                           stride, fact_cols, dp, d, chunks, chunks_per_item);
    else
        hipLaunchKernelGGL(replicate_power_kernel<float>, dim3((unsigned)grid), dim3(256), 0, ctx->stream, static_cast<unsigned char *>(totals),
                           stride, fact_cols, dp, d, chunks, chunks_per_item);
    return goom::check_hip(ctx, hipGetLastError(), "launch replicate_power_kernel");
}

} // namespace goom_chain
